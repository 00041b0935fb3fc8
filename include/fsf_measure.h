/*
 * fsf_measure.h - measurement and introspection aids of libfsf.so, apart from the product ABI in
 * fsf.h: per-kernel timing with HIP events, the device's measured ceilings, and a host-only view
 * of how a pass's prompt chunks would be cut into workgroups.  None of them is needed to run a
 * pass.  fsf_profile_* keeps process-global host state and is not thread safe.
 */
#ifndef FSF_MEASURE_H
#define FSF_MEASURE_H

#include "fsf.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Profiling aid (host state, not thread safe; off by default).  While enabled, every
 * kernel the library launches is bracketed by a pair of HIP events on the caller's
 * stream.  fsf_profile_read() waits for the recorded events, adds the elapsed
 * milliseconds and launch counts per phase into ms_out[FSF_N_PHASES] /
 * launches_out[FSF_N_PHASES] (host arrays, overwritten), and clears the record.
 * Events are ordinary host-side HIP objects; no device memory is allocated.
 */
typedef enum {
  FSF_PHASE_APPEND = 0,  /* fsf_kv_append kernel                                  */
  FSF_PHASE_PLAN = 1,    /* work planning (prefix sums over the descriptors)      */
  FSF_PHASE_PREFILL = 2, /* prompt-chunk attention (matrix cores)                 */
  FSF_PHASE_DECODE = 3,  /* generation-row split-KV attention                     */
  FSF_PHASE_MERGE = 4,   /* merge of split partial results                        */
  FSF_PHASE_GENERIC = 5, /* generic fp32 attention kernel                         */
  FSF_PHASE_FUSED = 6,   /* prompt-chunk + generation-row attention in one launch  */
  FSF_PHASE_LINEAR = 7,  /* fsf_linear                                             */
  FSF_N_PHASES = 8
} fsf_phase;
int fsf_profile_enable(int on);
int fsf_profile_read(double* ms_out, int64_t* launches_out);

/*
 * Measurement aids: what the device sustains with nothing else in the way, to set beside the
 * published peaks the roofline fractions use.  Both run synchronously (they time themselves with
 * HIP events on hip_stream and wait) and write only to `scratch` (device, >= 4096 bytes).
 *   fsf_ceiling_mfma_bf16  a register-resident loop of 32x32x16 bf16 MFMAs, two waves per SIMD;
 *                          `operands` (device, >= 16 MiB, read once) supplies the fragment values:
 *                          the rate depends on them, because the clock the chip holds does.
 *                          iters: MFMAs per wave / 8.  Outputs (host): TFLOP/s and the shader clock
 *                          in MHz seen inside the kernel.
 *   fsf_ceiling_mfma_bf16_16x16x32  the same loop, same flops per iteration, on 16x16x32 MFMAs
 *                          (the power limit leaves that instruction about a tenth more flops).
 *   fsf_ceiling_hbm_read   every wave streams 32 scattered 16 KB tiles of `buf` (device, `bytes`
 *                          long, >= 512 KiB; the largest power-of-two tile count that fits is
 *                          used), with non-temporal loads if nontemporal != 0.  Output: GB/s.
 * Return FSF_ERR_INVALID_ARG on null or too small buffers, FSF_ERR_HIP on a runtime error.
 */
int fsf_ceiling_mfma_bf16(const void* operands, int64_t operand_bytes, int32_t iters, void* scratch,
                          double* tflops_out, double* mhz_out, void* hip_stream);
int fsf_ceiling_mfma_bf16_16x16x32(const void* operands, int64_t operand_bytes, int32_t iters, void* scratch,
                                   double* tflops_out, double* mhz_out, void* hip_stream);
int fsf_ceiling_hbm_read(const void* buf, int64_t bytes, int32_t nontemporal, void* scratch,
                         double* gbs_out, void* hip_stream);

/*
 * Introspection (host only, no device call): how fsf_ragged_attention would cut the prompt
 * chunks of a pass into workgroups on a device with compute_units_assumed compute units.  A
 * chunk is tiled 256 rows at a time (tiles are numbered in descriptor order); a tile may be
 * cut into parts along its keys (a tile that would outlast the rest of the pass, or the tiles
 * of a last round of workgroups that is at most half full).  Writes up to cap entries of
 * (tile, part, n_parts, slab) in start order (slab: number of the (tile, part) in the
 * partial-result buffer, -1 for an unsplit tile); one workgroup per entry and query head.
 * Returns the number of entries, or -1 on invalid arguments.
 */
int32_t fsf_plan_prefill_groups(const fsf_attn_cfg* cfg, const fsf_seq_desc* descs_host, int32_t n_seqs,
                                int32_t compute_units_assumed, int32_t* groups_out, int32_t cap);

#ifdef __cplusplus
}
#endif
#endif /* FSF_MEASURE_H */

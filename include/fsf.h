/*
 * fsf.h - C ABI of the Dynamic SplitFuse attention step for AMD MI355X (gfx950).
 *
 * One forward pass of the serving loop hands the model a ragged batch: for each
 * sequence n_new tokens to process now and n_cached tokens already in the KV cache.
 * A prompt pass brings many tokens, a generation pass exactly one (paper Sec. 2, the
 * two phases of text generation).  Dynamic SplitFuse cuts prompts into chunks and fuses
 * them with running generations so that every pass carries a fixed token budget
 * (Sec. 3.2).  The cache is a pool of fixed-size blocks that a sequence owns in any
 * order (Sec. 2.1, blocked KV caching).
 *
 * The library covers the per-layer attention part of such a pass
 *     fsf_kv_append        new K/V rows -> cache blocks (bit-exact copy)
 *     fsf_ragged_attention causal attention of every new row over its sequence's
 *                          cached + new tokens, read through the block table
 * and the host-side decision that precedes it
 *     fsf_compose_batch    pick generations and prompt chunks that fill the budget and
 *                          hand out cache blocks.
 * Beside them: the position rotation fused into the append (fsf_kv_append_rotary,
 * fsf_rotary_q), the layer's linear maps (fsf_linear, fsf_linear_ws), a host-side check of a
 * pass (fsf_validate_pass) and the pass for callers that may not allocate
 * (fsf_ragged_attention_static).
 *
 * Conventions
 *   - All functions return FSF_OK (0) or a negative fsf_status; none throws, aborts or
 *     prints.  fsf_strerror() names a status.
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are
 *     ordinary host memory.  The library allocates no device memory and keeps no device
 *     state between calls (fsf_ragged_attention_static alone works in a fixed array that is
 *     part of the library's image, see there).  Device work is enqueued on the given hipStream_t (passed as
 *     void*, NULL = default stream) and is asynchronous; host arrays may be reused as
 *     soon as a call returns.
 *   - Token tensors are row-major [T, H, d], sequences back to back in descriptor
 *     order; q_offset of a descriptor is the running sum of n_new.
 *   - Caches: K and V separate, each row-major [num_blocks, n_kv_heads, block_size, d].
 *   - Block table: int32 [n_seqs, max_blocks]; entry b of row s is the physical block
 *     holding positions [b*block_size, (b+1)*block_size) of sequence s; unused entries
 *     are -1 and never dereferenced.  Block ids are trusted (not range-checked on device).
 *   - Query head hq reads KV head hq / (n_q_heads / n_kv_heads).
 *   - fsf_kv_append for a pass must be enqueued before fsf_ragged_attention of the same
 *     pass: attention reads this pass's tokens from the cache, n_cached counts tokens
 *     present before the pass.
 */
#ifndef FSF_H
#define FSF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  FSF_OK = 0,
  FSF_ERR_INVALID_ARG = -1, /* null pointer, bad shape, inconsistent descriptors           */
  FSF_ERR_UNSUPPORTED = -2, /* dtype / head_dim / group size no kernel is built for        */
  FSF_ERR_WORKSPACE = -3,   /* workspace missing or smaller than ..._workspace_bytes()      */
  FSF_ERR_NO_BLOCKS = -4,   /* composer: requests wait but no KV block is free             */
  FSF_ERR_HIP = -5          /* a HIP runtime call failed (launch error)                    */
} fsf_status;

typedef enum { FSF_F32 = 0, FSF_BF16 = 1, FSF_F16 = 2 } fsf_dtype;

/* fsf_attn_cfg.flags */
#define FSF_FLAG_FORCE_GENERIC 1    /* run the generic fp32 kernel even where a fast path exists     */
#define FSF_FLAG_FUSED_LAUNCH 2     /* matrix-core path: launch prompt-chunk and generation-row work  */
                                    /* as one fused grid instead of two kernels.  Needs cache blocks  */
                                    /* of 32 tokens or more (ignored otherwise), and a fused pass     */
                                    /* never cuts prompt-chunk tiles along their keys                 */

/*
 * Tuning of fsf_ragged_attention's work partition, passed by value through fsf_attn_cfg.tuning
 * (NULL: every default).  It is read during the call and may be freed or changed afterwards.  A
 * field that is 0 takes its default; the defaults suit MI355X.  Results stay within the stated
 * tolerance for every setting; the partition (and with it the summation order) changes.
 * struct_bytes = sizeof(fsf_tuning) as the caller compiled it; fields beyond it take defaults.
 */
typedef struct {
  int32_t struct_bytes;
  int32_t decode_target_waves;     /* about how many streaming wave units a pass is at least cut into   */
                                   /* (default 4096 = two rounds of the chip's wave slots; by default a  */
                                   /* pass whose units nearly all come from cut rows is then cut a little */
                                   /* coarser until its units fill whole rounds, a given value is kept)   */
  int32_t decode_min_item_blocks;  /* no cut of a row's keys leaves fewer cache blocks than this per     */
                                   /* unit (default 16, or 1024 tokens' worth for blocks below 64        */
                                   /* tokens; a quarter of that in passes with fewer units than compute   */
                                   /* units, unless set here)                                            */
  int32_t decode_hold;             /* -1: store every unit's result as it finishes; default (0, 1): with */
                                   /* more units than wave slots, one round of waves (eight to a          */
                                   /* workgroup, one workgroup per compute unit) keep finished rows in LDS */
                                   /* and store them at the end; 2: the same with single-wave workgroups   */
  int32_t prefill_split;           /* -1: never cut prompt-chunk tiles along their keys; default: cut    */
                                   /* tiles that would outlast the pass or sit in a half-empty last round */
  int32_t compute_units;           /* compute units the cutting rules assume (default: the device's)     */
  int32_t max_decode_items_extra;  /* bounds the workspace: streaming units beyond one per sequence and  */
                                   /* KV head that may hold partial results (default 8192)               */
  int32_t max_prefill_split_units; /* bounds the workspace: (tile, head, part) workgroups with partial    */
                                   /* results, 139 KB each (default 512)                                 */
  int32_t overlap;                 /* 1: in passes with both kinds of work, more streaming units than     */
                                   /* wave slots and little prompt-chunk work, the prompt-chunk tiles run  */
                                   /* beside the streaming kernel on a second stream the library keeps per */
                                   /* device, on 8 or 16 compute units the streaming kernel leaves empty;  */
                                   /* forked from and joined to the caller's stream inside the call.       */
                                   /* 8 or more: the same on exactly this many units (a multiple of 8, at  */
                                   /* most half the chip), whatever the share of the prompt-chunk work.    */
                                   /* Default (0) and -1: one kernel after the other, which measured       */
                                   /* faster on most passes                                               */
  int32_t stream_chunk_slices;     /* a prompt chunk of at most this many slices of 16 / (query heads    */
                                   /* per KV head) rows runs on the streaming kernel like generation      */
                                   /* rows, every slice reading the chunk's K/V once (default 2, at most  */
                                   /* 16; -1: only one-token sequences stream)                            */
} fsf_tuning;

/* One sequence of the pass (paper Sec. 2: tokens processed now vs tokens in the cache). */
typedef struct {
  int32_t n_new;    /* tokens processed in this pass, >= 1                                  */
  int32_t n_cached; /* tokens in the cache BEFORE this pass, >= 0                          */
  int32_t q_offset; /* first row of this sequence in the [T, H, d] token tensors           */
  int32_t seq_id;   /* caller's tag; not interpreted by the kernels                        */
} fsf_seq_desc;

typedef struct {
  int32_t n_q_heads;
  int32_t n_kv_heads; /* divides n_q_heads                                                  */
  int32_t head_dim;
  int32_t block_size; /* tokens per cache block                                             */
  int32_t window;     /* 0: row at position p sees keys 0..p; W>0: keys j with 0 <= p-j < W */
  float scale;        /* multiplies q.k before the softmax, normally 1/sqrt(head_dim)      */
  int32_t dtype;      /* fsf_dtype of q, k_new, v_new, both caches and out                  */
  int32_t flags;      /* 0, or FSF_FLAG_* bits                                              */
  int64_t num_blocks; /* physical blocks in each cache                                      */
  const fsf_tuning* tuning; /* host; NULL = defaults (see fsf_tuning)                        */
} fsf_attn_cfg;

const char* fsf_strerror(int status);

/* Library version as major*10000 + minor*100 + patch. */
int fsf_version(void);

/*
 * KV-cache append (paper Sec. 2: a pass adds its tokens to the sequence's cache;
 * Sec. 2.1: storage is block granular).  For token i of sequence s (position
 * p = n_cached + i) and every KV head h, copies k_new[q_offset+i, h, :] to
 * k_cache[block_tables[s, p / block_size], h, p % block_size, :], same for V.
 * Bit-exact; no other cache byte is written.
 *   k_new, v_new        device, [n_tokens, n_kv_heads, d]
 *   k_cache, v_cache    device, [num_blocks, n_kv_heads, block_size, d]
 *   descs_dev           device, [n_seqs]
 *   block_tables_dev    device, [n_seqs, max_blocks]
 * n_seqs == 0 or n_tokens == 0 is a no-op.  Requires head_dim * sizeof(element) % 4 == 0 and
 * 4-byte aligned tensors (16-byte aligned ones are copied in 16-byte units).
 * This call sees only the device copies of the descriptors and block tables and trusts them:
 * n_tokens must equal the sum of n_new, and every position must have its table entry.  A
 * caller that cannot vouch for them runs fsf_validate_pass on its host copies first.
 */
int fsf_kv_append(const fsf_attn_cfg* cfg, const void* k_new, const void* v_new, void* k_cache,
                  void* v_cache, const fsf_seq_desc* descs_dev, const int32_t* block_tables_dev,
                  int32_t n_seqs, int32_t max_blocks, int32_t n_tokens, void* hip_stream);

/*
 * Host-side check of a pass before it is enqueued (optional; the device calls trust block ids,
 * because checking them on the device would cost a synchronisation).  Verifies on the host
 * copies what fsf_ragged_attention verifies (n_new >= 1, n_cached >= 0, q_offsets the running
 * sum of n_new ending at n_tokens, ceil((n_cached + n_new) / block_size) <= max_blocks) and, for
 * every table entry the pass will dereference (columns 0 .. ceil((n_cached+n_new)/block_size)-1 of
 * each row), that 0 <= id < num_blocks and that no block is named twice in the pass (paper
 * Sec. 2.1: a block belongs to one sequence).  Returns FSF_OK, or FSF_ERR_INVALID_ARG with the
 * first offending sequence and table column in *bad_seq_out / *bad_column_out (either may be
 * NULL; -1 where the fault is not tied to one).  O(table entries) time, num_blocks bits of host
 * memory; no device call.
 */
int fsf_validate_pass(const fsf_attn_cfg* cfg, const fsf_seq_desc* descs_host,
                      const int32_t* block_tables_host, int32_t n_seqs, int32_t max_blocks,
                      int32_t n_tokens, int32_t* bad_seq_out, int32_t* bad_column_out);

/*
 * As fsf_kv_append, with the rotary position embedding of the served model family (paper
 * Sec. 4.1: Llama-2) applied to K on the way into the cache.  For the row at position p and
 * every head, element i < d/2 pairs with element i + d/2:
 *     k'[i]       = k[i] * cos(p, i) - k[i + d/2] * sin(p, i)
 *     k'[i + d/2] = k[i + d/2] * cos(p, i) + k[i] * sin(p, i)
 * cos_sin_dev: device, float32 [table_positions, d/2, 2] (cos, sin), supplied by the caller;
 * every position of the pass must be below table_positions (checked on descs_host).  The
 * arithmetic is fixed, so that the cache contents remain reproducible bit for bit: the four
 * products and the sum and the difference are float32 operations rounded to nearest even,
 * never fused, and the result is rounded once to the storage type.  V is copied bit for bit.
 * head_dim must be even.  Errors as fsf_kv_append.
 */
int fsf_kv_append_rotary(const fsf_attn_cfg* cfg, const void* k_new, const void* v_new, void* k_cache,
                         void* v_cache, const fsf_seq_desc* descs_dev, const fsf_seq_desc* descs_host,
                         const int32_t* block_tables_dev, int32_t n_seqs, int32_t max_blocks,
                         int32_t n_tokens, const float* cos_sin_dev, int32_t table_positions,
                         void* hip_stream);

/*
 * The rotation of fsf_kv_append_rotary applied in place to the pass's query rows
 * (device, [n_tokens, n_q_heads, d]): row i of a sequence by the angles of position
 * n_cached + i, the position its key is stored at; same pairing, same fixed arithmetic, same
 * table.  Scores of rotated queries against rotated keys then depend on the distance between
 * the two positions only (the property the Llama family's attention relies on, paper Sec. 4.1).
 * Errors as fsf_kv_append_rotary (block tables are not needed).
 */
int fsf_rotary_q(const fsf_attn_cfg* cfg, void* q, const fsf_seq_desc* descs_dev,
                 const fsf_seq_desc* descs_host, int32_t n_seqs, int32_t n_tokens,
                 const float* cos_sin_dev, int32_t table_positions, void* hip_stream);

/*
 * A linear layer over the tokens of a pass (the projections and MLP products on either side of
 * attention; paper Sec. 3.1: they make a pass weight-bound at few tokens and compute-bound at
 * many, which is what a token budget is chosen against):
 *     y[t, o] = sum_k x[t, k] * w[o, k]
 *   x  device, [n_tokens, k]      tokens of the ragged batch, row-major
 *   w  device, [n_out, k]         one output feature per row (k contiguous)
 *   y  device, [n_tokens, n_out]
 * bf16 or f16 operands on the matrix cores, fp32 accumulation, the result rounded once to the
 * storage type (nearest even).  Any n_tokens >= 0 (0 is a no-op).  Requires n_out % 256 == 0,
 * k % 64 == 0, 16-byte aligned tensors and x, w below 2 GiB each; FSF_ERR_UNSUPPORTED otherwise
 * and for FSF_F32.  Allocates nothing, asynchronous on hip_stream.
 */
int fsf_linear(int32_t dtype, const void* x, const void* w, void* y, int32_t n_tokens, int32_t n_out,
               int32_t k, void* hip_stream);

/*
 * The same product with a device workspace, which lets the library cut k into parts where the
 * output tiles alone would leave compute units idle (few tokens and a narrow output: a pass in
 * the weight-bound regime of paper Sec. 3.1 is then bound by how fast the few busy units pull
 * the weights from HBM).  Each part leaves an fp32 partial result in the workspace and a second
 * kernel sums them in a fixed order and rounds once, so results are deterministic and within
 * fsf_linear's tolerance (not bit-equal to it: another summation order).
 * fsf_linear_workspace_bytes: bytes that let every cut the library would choose for this shape
 * happen (0: it would not cut; also 0 for shapes fsf_linear refuses).  A smaller or NULL
 * workspace means fewer parts or none, never an error; a workspace that is not 16-byte aligned
 * is FSF_ERR_WORKSPACE.  The workspace is scratch: nothing is kept in it between calls.
 */
size_t fsf_linear_workspace_bytes(int32_t n_tokens, int32_t n_out, int32_t k);
int fsf_linear_ws(int32_t dtype, const void* x, const void* w, void* y, int32_t n_tokens, int32_t n_out,
                  int32_t k, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Bytes of device workspace fsf_ragged_attention needs for a pass of at most n_seqs
 * sequences, n_tokens tokens and max_blocks table columns.  Never zero (a small plan
 * area is always used); 256-byte aligned sizes.  Returns 0 on invalid cfg.  On the
 * matrix-core path it holds the work tables, the partial results of generation rows whose
 * keys were split (at most n_seqs + 8192 units) and of prompt-chunk tiles whose keys were
 * split (at most 512 units of 256 rows, 71 MB).
 */
size_t fsf_ragged_attention_workspace_bytes(const fsf_attn_cfg* cfg, int32_t n_seqs,
                                            int32_t n_tokens, int32_t max_blocks);

/*
 * Ragged blocked-KV causal attention (paper Sec. 2 and 3.2: prompt chunks attend to
 * their own earlier chunks in the cache, generations to their whole history, all in one
 * pass).  For row i of sequence s (p = n_cached + i), query head hq, KV head hk:
 *     J = { j : 0 <= j <= p and (window == 0 or p - j < window) }
 *     out[q_offset+i, hq, :] = sum_{j in J} softmax_J(scale * q.k_j)_j * v_j
 * with k_j, v_j read from the caches through the block table.  Scores, softmax and
 * accumulation are fp32; bf16/f16 inputs use matrix cores with the softmax weights
 * rounded to the storage type for the second product; the result is rounded to the
 * storage type (nearest even).  Cache slots beyond a row's visible set never influence
 * the result, whatever bits they hold.
 *   q, out              device, [n_tokens, n_q_heads, d]
 *   descs_dev           device copy of the descriptors
 *   descs_host          host copy of the same descriptors (validated, sizes the launch)
 *   workspace           device, >= fsf_ragged_attention_workspace_bytes(...), 256-aligned;
 *                       contents are scratch, not preserved, no initialisation needed
 * Validation (host side): n_new >= 1, n_cached >= 0, q_offsets are the running sum of
 * n_new and end at n_tokens, ceil((n_cached+n_new)/block_size) <= max_blocks.
 * The work partition is tuned through cfg->tuning (fsf_tuning); the library reads no
 * environment variable.
 * Fast paths: bf16/f16 with head_dim 128, block_size 16 * 2^k and at most 16 query heads per KV
 * head; every other supported shape (any dtype, head_dim <= 256 and a multiple of
 * 4/sizeof-ratio, any block_size) runs a generic fp32 kernel, one wavefront per (row, head)
 * with scalar dot products: correct, and meant for small or odd shapes only (the 194-token
 * fp32 example pass takes about 0.1 ms; at benchmark sizes it is two to three orders of
 * magnitude below either roofline).
 */
int fsf_ragged_attention(const fsf_attn_cfg* cfg, const void* q, const void* k_cache,
                         const void* v_cache, const fsf_seq_desc* descs_dev,
                         const fsf_seq_desc* descs_host, const int32_t* block_tables_dev,
                         int32_t n_seqs, int32_t max_blocks, int32_t n_tokens, void* out,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * fsf_ragged_attention for callers that cannot allocate device memory or pass a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments without the workspace, same kernels, same results to the same tolerance.  The work
 * tables and partial results live in a fixed array of FSF_STATIC_SCRATCH_BYTES (64 MiB) of device
 * memory that is part of the library image: every GPU the library runs on holds it from the
 * first call on that GPU until the process ends, and the call allocates and frees nothing.
 * The cutting of generation rows and prompt-chunk tiles into units with partial results is
 * limited to what fits the array (at most 1024 extra row units and 64 tile units, fewer for
 * passes with many heads); a pass whose work tables alone exceed the array (millions of
 * tokens) is refused with FSF_ERR_WORKSPACE and nothing is launched.  All calls on one GPU share
 * the array: calls that overlap on one GPU (two streams, two threads) race and give wrong
 * results; calls on one stream, or ordered by events, are safe.  The first call on a device looks the array's address up and should be
 * made outside a graph capture.  Errors otherwise as fsf_ragged_attention.
 */
#define FSF_STATIC_SCRATCH_BYTES (64u << 20)
int fsf_ragged_attention_static(const fsf_attn_cfg* cfg, const void* q, const void* k_cache,
                                const void* v_cache, const fsf_seq_desc* descs_dev,
                                const fsf_seq_desc* descs_host, const int32_t* block_tables_dev,
                                int32_t n_seqs, int32_t max_blocks, int32_t n_tokens, void* out,
                                void* hip_stream);

/*
 * Host-side Dynamic SplitFuse scheduler with a block allocator (paper Sec. 2.2: one
 * batch decision per forward pass; Sec. 3.2: long prompts are split over passes with
 * only the last chunk generating, and prompts are fused with generations to meet the
 * token budget exactly when enough tokens wait).  Policy where the paper is silent:
 * generations first, one token each, least recently scheduled first; prompts first come
 * first served, a partly processed prompt continues before a new one starts; a chunk
 * takes min(remaining prompt, remaining budget); blocks are popped from the front of
 * the free list and returned to its back when a sequence retires; without free blocks
 * a generation is skipped for the pass and a prompt chunk shrinks to what fits, after
 * which no later prompt is started; nothing is evicted unless fsf_sched_set_exhaustion says so.
 */
typedef struct fsf_sched fsf_sched;

/* free_list_order: NULL (blocks 0..num_blocks-1) or a permutation of them (host). */
int fsf_sched_create(fsf_sched** out, int32_t token_budget, int32_t max_seqs, int32_t block_size,
                     int64_t num_blocks, const int32_t* free_list_order);
void fsf_sched_destroy(fsf_sched* s);

/*
 * Composition policy, to be chosen before the first request (default Dynamic SplitFuse).
 * The other two are the batch decisions the paper contrasts it with (Sec. 2.2, Sec. 3,
 * Sec. 4.4), for the scheduling simulator; neither splits a prompt:
 *   FSF_POLICY_PROMPT_FIRST        while prompts wait, a pass holds whole prompts only (first
 *                                  come first served, as many as fit token_budget, the first
 *                                  even if longer) and generations wait; else all generations
 *   FSF_POLICY_WHOLE_PROMPT_JOINS  every pass runs the generations (at most token_budget and
 *                                  max_seqs of them) and waiting prompts join whole while
 *                                  sequences and blocks allow; no token budget for prompts
 * Generations keep their descriptors ahead of the prompts in every policy.
 * Returns FSF_ERR_INVALID_ARG for an unknown policy or once requests exist.
 */
typedef enum {
  FSF_POLICY_SPLITFUSE = 0,
  FSF_POLICY_PROMPT_FIRST = 1,
  FSF_POLICY_WHOLE_PROMPT_JOINS = 2
} fsf_policy;
int fsf_sched_set_policy(fsf_sched* s, int32_t policy);

/*
 * What fsf_compose_batch does when requests wait but nothing can be scheduled because the
 * block pool is used up (the paper describes the blocked cache, Sec. 2.1, but no policy for a
 * full pool).  To be chosen before the first request.
 *   FSF_EXHAUST_STALL           (default) report FSF_ERR_NO_BLOCKS and change nothing
 *   FSF_EXHAUST_PREEMPT_NEWEST  the sequence that arrived last among those holding blocks gives
 *                               them back (to the end of the free list, in logical order) and
 *                               starts over: its n_cached processed tokens plus the generated
 *                               token it was about to feed become a prompt of n_cached + 1
 *                               tokens, queued by its arrival order; emitted tokens stay
 *                               emitted.  The decision is taken again until something can be
 *                               scheduled.  The caller sees the restart as a descriptor with
 *                               n_cached = 0 for a known seq_id and must feed that sequence's
 *                               tokens from its beginning again.  FSF_ERR_NO_BLOCKS remains for
 *                               the case that fewer than two sequences hold blocks (a sequence
 *                               that alone exceeds the pool).  Preemptions made before an
 *                               error is returned are not undone.
 * fsf_sched_preemptions reports how many sequences were restarted so far and how many cached
 * tokens that discarded.
 */
typedef enum { FSF_EXHAUST_STALL = 0, FSF_EXHAUST_PREEMPT_NEWEST = 1 } fsf_exhaustion;
int fsf_sched_set_exhaustion(fsf_sched* s, int32_t mode);
int fsf_sched_preemptions(const fsf_sched* s, int64_t* n_preemptions_out, int64_t* tokens_discarded_out);

/* Queue a request: prompt_len >= 1 tokens to read, max_new_tokens >= 1 tokens to emit.
 * The sequence emits its first token in the pass that consumes its last prompt token,
 * then runs as a generation until max_new_tokens are emitted; the last emitted token
 * is never fed back, so the cache ends at prompt_len + max_new_tokens - 1 tokens. */
int fsf_sched_add_request(fsf_sched* s, int32_t seq_id, int32_t prompt_len, int32_t max_new_tokens);

/*
 * Compose the next pass.  All outputs are host arrays:
 *   descs_out         [max_seqs]               descriptors, generations first
 *   block_tables_out  [max_seqs, max_blocks]   every block of each scheduled sequence, -1 padded
 *   emits_token_out   [max_seqs]               1 if the sequence produces a token in this pass
 * Blocks are allocated here; the pass stays pending until fsf_sched_step_done().
 * Returns FSF_ERR_INVALID_ARG if a pass is already pending or a sequence would need more
 * than max_blocks blocks (state unchanged), FSF_ERR_NO_BLOCKS if requests exist but
 * nothing can be scheduled.  With no requests at all: FSF_OK and *n_seqs_out = 0.
 */
int fsf_compose_batch(fsf_sched* s, fsf_seq_desc* descs_out, int32_t* block_tables_out,
                      int32_t max_blocks, int32_t* n_seqs_out, int32_t* n_tokens_out,
                      int32_t* emits_token_out);

/* Commit the pending pass: advance n_cached, turn finished prompts into generations,
 * retire sequences that emitted max_new_tokens and free their blocks. */
int fsf_sched_step_done(fsf_sched* s);

/* Introspection (host): free blocks, live sequences (waiting prompts + generations). */
int64_t fsf_sched_free_blocks(const fsf_sched* s);
int32_t fsf_sched_live_seqs(const fsf_sched* s);

#ifdef __cplusplus
}
#endif
#endif /* FSF_H */

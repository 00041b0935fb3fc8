"""Benchmark: one Dynamic SplitFuse forward step (KV append + ragged attention) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2]

A "step" is one pass of the whole hot path over one ragged batch of synthetic input:
fsf_kv_append followed by fsf_ragged_attention for one layer.  The default workload is the
Llama-2-7B-shaped batch with a 2048-token budget (one 1792-token prompt chunk plus 256
generation rows).  Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line.  `value` is tokens/s of the whole step.  `roofline` prices the
dominant kernel (generation-row attention, HBM bound) by its algorithmic bytes and its
average duration measured with HIP events on the launch stream inside the timed region.
`cpu_baseline` times the fp64 oracle on the host cores for a bounded sample of the batch.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2401_08671_amd import fsf  # noqa: E402
from paper_2401_08671_amd import workloads as wl  # noqa: E402
from paper_2401_08671_amd.harness import DeviceStep, StreamRunner, algorithmic_work  # noqa: E402

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix rate


def cpu_baseline(ds: DeviceStep, k_cache0: np.ndarray, v_cache0: np.ndarray, n_decode_sample: int = 256):
    """Time the fp64 oracle (as it stands) on every prompt chunk plus a seeded sample of generation rows."""
    from oracle import attention as oa
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = 1
    spec = ds.spec
    rng = np.random.default_rng(spec.seed + 99)
    dec = [s for s, (n, _) in enumerate(spec.seqs) if n == 1]
    pre = [s for s, (n, _) in enumerate(spec.seqs) if n > 1]
    sample = sorted(rng.choice(dec, size=min(n_decode_sample, len(dec)), replace=False).tolist()) if dec else []
    q = wl.to_numpy_storage(ds.q)
    k_new, v_new = wl.to_numpy_storage(ds.k_new), wl.to_numpy_storage(ds.v_new)
    t0 = time.perf_counter()
    oa.kv_append(k_cache0, v_cache0, k_new, v_new, ds.descs, ds.block_tables, spec.block_size)
    t_app = time.perf_counter() - t0
    t0 = time.perf_counter()
    out_pre = oa.ragged_attention(q, k_cache0, v_cache0, ds.descs, ds.block_tables, block_size=spec.block_size,
                                  scale=spec.scale, window=spec.window, dtype=spec.dtype, seq_subset=pre)
    t_pre = time.perf_counter() - t0
    t0 = time.perf_counter()
    out_dec = oa.ragged_attention(q, k_cache0, v_cache0, ds.descs, ds.block_tables, block_size=spec.block_size,
                                  scale=spec.scale, window=spec.window, dtype=spec.dtype, seq_subset=sample)
    t_dec = time.perf_counter() - t0
    # generation rows cost in proportion to the keys they read
    keys = lambda idx: sum(min(spec.seqs[s][1] + 1, spec.window) if spec.window else spec.seqs[s][1] + 1 for s in idx)
    t_dec_full = t_dec * keys(dec) / max(keys(sample), 1) if sample else 0.0
    t_full = t_app + t_pre + t_dec_full
    ref = np.where(np.isnan(out_pre), out_dec, out_pre)
    return dict(value=spec.n_tokens / t_full, unit="tokens/s", cores=int(threads), kind="oracle",
                sample=(f"append of all {spec.n_tokens} tokens ({t_app:.2f}s) + all {len(pre)} prompt chunks ({t_pre:.2f}s) + "
                        f"{len(sample)} of {len(dec)} generation rows ({t_dec:.2f}s), generation time scaled to the "
                        f"full batch by visible keys; numpy fp64")), ref


def stream_bench(args):
    """Benchmark shape 5: 200 consecutive passes of the long-prompt stream, batches from fsf_compose_batch."""
    n_steps = 200
    run = StreamRunner(n_steps=n_steps, rate=1.0)
    # one fixed set of new-token tensors, sliced per pass (values do not affect timing)
    q_all, k_all, v_all = run.new_tokens(0, run.budget)
    warm = DeviceStep(wl.config(2, n_decodes=8))          # load the kernels before timing
    for _ in range(max(1, args.warmup)):
        warm.step()
    torch.cuda.synchronize()
    del warm
    fsf.profile_enable(True)
    fsf.profile_read()
    per_step = []
    t_compose = 0.0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for step in range(n_steps):
        tc = time.perf_counter()
        descs, tables, _ = run.compose()
        t_compose += time.perf_counter() - tc
        T = int(descs[:, 0].sum()) if len(descs) else 0
        run.run_pass(descs, tables, q_all[:T], k_all[:T], v_all[:T])
        run.commit()
        spec = wl.BatchSpec(f"pass{step}", run.Hq, run.Hkv, run.d, run.B, run.dtype,
                            [(int(n), int(c)) for n, c, _, _ in descs])
        per_step.append((T, algorithmic_work(spec) if T else None))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = fsf.profile_read()
    fsf.profile_enable(False)
    total_tokens = sum(t for t, _ in per_step)
    gpu_ms = sum(v[0] for v in prof.values())
    fused_ms = prof["decode"][0] + prof["prefill"][0]      # the two attention kernels of every pass
    bytes_ = sum(w["decode_bytes"] + w["prefill_bytes"] for _, w in per_step if w)
    flops = sum(w["decode_flops"] + w["prefill_flops"] for _, w in per_step if w)
    t_hbm = sum((w["decode_bytes"] + w["prefill_bytes"]) / (HBM_PEAK_GBS * 1e9) for _, w in per_step if w)
    t_mfma = sum((w["decode_flops"] + w["prefill_flops"]) / (MFMA_BF16_PEAK_TFLOPS * 1e12) for _, w in per_step if w)
    # ideal time of the stream = sum over passes of max(bytes / HBM peak, flops / MFMA peak)
    t_ideal = sum(max((w["decode_bytes"] + w["prefill_bytes"]) / (HBM_PEAK_GBS * 1e9),
                      (w["decode_flops"] + w["prefill_flops"]) / (MFMA_BF16_PEAK_TFLOPS * 1e12)) for _, w in per_step if w)
    hbm_bound = t_hbm >= t_mfma
    wall_ms = (t1 - t0) * 1e3
    line = {
        "metric": "ragged SplitFuse attn tokens/s per step + % HBM/MFMA roofline, 1 GPU",
        "value": total_tokens / (t1 - t0), "unit": "tokens/s", "n_gpus": 1, "steps": n_steps, "warmup": args.warmup,
        "ms_per_step": wall_ms / n_steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": run.dtype, "data": "synthetic",
        "config": {"workload": f"cfg5-13b-stream: Hq={run.Hq} Hkv={run.Hkv} d={run.d} block={run.B} budget={run.budget}, "
                               f"{n_steps} consecutive passes composed by fsf_compose_batch, {len(run.requests)} requests "
                               "(log-normal prompts, Poisson(1.0) arrivals per pass), one layer; wall clock includes "
                               "host composition and descriptor upload",
                   "total_tokens": total_tokens, "kv_pool_blocks": run.num_blocks},
        "roofline": ({"bound": "hbm", "kernel": "attn_decode_kernel + attn_prefill_kernel", "achieved": bytes_ / (fused_ms * 1e-3) / 1e9,
                      "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": bytes_ / (fused_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                      "traffic": None, "algorithmic_bytes_all_launches": bytes_, "total_launch_ms": fused_ms}
                     if hbm_bound else
                     {"bound": "mfma", "kernel": "attn_decode_kernel + attn_prefill_kernel", "achieved": flops / (fused_ms * 1e-3) / 1e12,
                      "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                      "frac": flops / (fused_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                      "algorithmic_flops_all_launches": flops, "total_launch_ms": fused_ms}),
        "stream": {"gpu_kernel_ms_total": gpu_ms, "gpu_tokens_per_s": total_tokens / (gpu_ms * 1e-3),
                   "host_compose_ms_total": t_compose * 1e3, "wall_ms_total": wall_ms,
                   "ideal_ms_total_max_of_rooflines": t_ideal * 1e3,
                   "frac_of_per_pass_roofline": t_ideal * 1e3 / fused_ms,
                   "phases_ms_total": {k: v[0] for k, v in prof.items()},
                   "tokens_per_pass_min_median_max": [int(np.min([t for t, _ in per_step])),
                                                      int(np.median([t for t, _ in per_step])),
                                                      int(np.max([t for t, _ in per_step]))]},
    }
    print(json.dumps(line))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, choices=[2, 3, 4, 5, 6])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the measurement of the device's ceilings")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (the attention step shards by KV head with no "
              "exchange inside it); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    if args.config == 5:
        return stream_bench(args)
    spec = wl.config(args.config)
    ds = DeviceStep(spec)
    work = algorithmic_work(spec)
    torch.cuda.synchronize()
    k0 = v0 = None
    if not args.no_cpu_baseline:
        k0, v0 = wl.to_numpy_storage(ds.k_cache), wl.to_numpy_storage(ds.v_cache)

    for _ in range(args.warmup):
        ds.step()
    torch.cuda.synchronize()

    fsf.profile_enable(True)
    fsf.profile_read()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ds.step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = fsf.profile_read()
    fsf.profile_enable(False)

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = spec.n_tokens / (ms_per_step * 1e-3)
    phase_ms = {k: (v[0] / v[1] if v[1] else 0.0) for k, v in prof.items()}

    # Dominant kernel of the timed region: generation-row attention (HBM bound) or prompt-chunk
    # attention (matrix-core bound), whichever ran longer.
    dec_ms, pre_ms = phase_ms["decode"], phase_ms["prefill"]
    hbm_bound = dec_ms >= pre_ms
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"bench_cfg{args.config}_hbm_traffic.md")
    if os.path.exists(tpath):
        for ln in open(tpath):
            if ln.startswith("hbm_bytes_per_launch:"):
                traffic = float(ln.split(":")[1])
    if hbm_bound:
        achieved = work["decode_bytes"] / (dec_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "attn_decode_kernel", "achieved": achieved, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                    "algorithmic_bytes_per_launch": work["decode_bytes"], "avg_launch_ms": dec_ms}
    else:
        achieved = work["prefill_flops"] / (pre_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "kernel": "attn_prefill_kernel", "achieved": achieved,
                    "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                    "traffic": traffic, "algorithmic_flops_per_launch": work["prefill_flops"],
                    "avg_launch_ms": pre_ms}
    line = {
        "metric": "ragged SplitFuse attn tokens/s per step + % HBM/MFMA roofline, 1 GPU",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": spec.dtype, "data": "synthetic",
        "config": {"workload": f"{spec.name}: Hq={spec.n_q_heads} Hkv={spec.n_kv_heads} d={spec.head_dim} "
                               f"block={spec.block_size} window={spec.window} budget={spec.n_tokens} "
                               f"({sum(1 for n, _ in spec.seqs if n > 1)} prompt chunks, "
                               f"{sum(1 for n, _ in spec.seqs if n == 1)} generation rows), one layer",
                   "n_seqs": spec.n_seqs, "n_tokens": spec.n_tokens, "kv_pool_blocks": ds.num_blocks},
        "roofline": roofline,
        "phases_ms": phase_ms,
        "step_roofline": {"algorithmic_bytes": work["total_bytes"],
                          "achieved_GBs": work["total_bytes"] / (ms_per_step * 1e-3) / 1e9,
                          "frac_hbm": work["total_bytes"] / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "decode_only": {"bytes": work["decode_bytes"], "ms": dec_ms,
                        "GBs": work["decode_bytes"] / (dec_ms * 1e-3) / 1e9 if dec_ms else 0.0,
                        "frac_hbm": work["decode_bytes"] / (dec_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if dec_ms else 0.0},
        "prefill_only": {"flops": work["prefill_flops"], "ms": pre_ms,
                         "TFLOPs": work["prefill_flops"] / (pre_ms * 1e-3) / 1e12 if pre_ms else 0.0,
                         "frac_mfma": work["prefill_flops"] / (pre_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS if pre_ms else 0.0},
    }
    if not args.no_ceilings:
        # what the device sustains with nothing else in the way (scattered 16 KB tiles streamed with
        # non-temporal loads; a register-resident bf16 MFMA loop on normally distributed operands)
        from paper_2401_08671_amd import ceilings
        c = ceilings.measure(hbm_bytes=4 << 30)
        ceil = (c["hbm_read_scattered_16KB_tiles_nontemporal_loads"]["GBs"] if hbm_bound
                else c["mfma_bf16_normal_operands"]["TFLOPs"])
        line["roofline"]["measured_ceiling"] = ceil
        line["roofline"]["frac_of_measured_ceiling"] = achieved / ceil
        line["measured_ceilings"] = c
    if not args.no_cpu_baseline:
        base, ref = cpu_baseline(ds, k0, v0)
        line["cpu_baseline"] = base
        got = ds.out.to(torch.float64).cpu().numpy()
        m = ~np.isnan(ref)
        err = np.abs(got[m] - ref[m])
        line["check_vs_oracle"] = {"max_abs": float(err.max()), "mean_abs": float(err.mean()), "elements": int(m.sum())}
    print(json.dumps(line))


if __name__ == "__main__":
    main()

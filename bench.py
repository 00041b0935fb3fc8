"""Benchmark: Dynamic SplitFuse forward steps (KV append + ragged attention) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3]

A "step" is one pass of the whole hot path over one ragged batch of synthetic input:
fsf_kv_append followed by fsf_ragged_attention for one layer.  Inputs are resident in HBM
before the timed region starts.  Prints ONE JSON line.

Headline (`value`, `roofline`, `cpu_baseline`): the Mistral-7B-shaped batch with a 4096-token
budget, 32 query / 8 KV heads, sliding window 4096 (two 1024-token prompt chunks over long
prefixes plus 2048 generation rows; the largest of the benchmark shapes that is a single step:
19 GB of K/V per step out of a 33 GB pool).  `roofline` prices the dominant kernel by its
algorithmic bytes (or flops) and its average duration measured with HIP events on the launch
stream inside the timed region.  `cpu_baseline` times the fp64 oracle on the host cores for a
bounded sample of the same batch.  `sustained` repeats the timed steps after ten seconds of
continuous stepping, with the shader clock the device's matrix-core probe sees before and after.

Without --config the same line also carries `per_config`: the Llama-2-7B shape (budget 2048),
the Llama-2-70B one-GPU share (decode dominated), the 200-pass long-prompt stream composed by
fsf_compose_batch, and the heaviest kind of step of that stream (one 4096-token chunk 8192
tokens into its prompt; matrix-core bound), each with step time, tokens/s, its kernels against
their rooflines and its own comparison with the oracle.  With --config K only shape K is run,
as the headline (this is what the profiles under profiles/ are collected on).

Every comparison with the oracle is asserted: a result outside the tolerance ends the run
with a non-zero exit code and no JSON line.
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
METRIC = "ragged SplitFuse attn tokens/s per step + % HBM/MFMA roofline, 1 GPU"
DENSE_PAIR_LIMIT = 12_000_000   # chunks with more (row, key) pairs than this are checked on sampled rows


def host_threads():
    """(cores this process may run on, threads of numpy's BLAS pool)."""
    cores = len(os.sched_getaffinity(0))
    try:
        from threadpoolctl import threadpool_info
        blas = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        blas = 1
    return cores, int(blas)


def pick_sequences(spec: wl.BatchSpec, n_decode: int):
    """All prompt chunks plus a seeded sample of generation rows that always holds the shortest and
    the longest and rows on both sides of block and window boundaries."""
    rng = np.random.default_rng(spec.seed + 99)
    B, W = spec.block_size, spec.window
    dec = [(s, c) for s, (n, c) in enumerate(spec.seqs) if n == 1]
    chosen = [s for s, (n, _) in enumerate(spec.seqs) if n > 1]
    if dec:
        by_c = sorted(dec, key=lambda t: t[1])
        must = {by_c[0][0], by_c[-1][0]}
        for rem in (0, B - 1):                      # one row on either side of a block boundary
            must |= set([s for s, c in dec if c % B == rem][:1])
        if W:
            must |= {s for s, _ in sorted(dec, key=lambda t: abs(t[1] + 1 - W))[:2]}
        rest = [s for s, _ in dec if s not in must]
        extra = rng.choice(rest, size=min(len(rest), max(0, n_decode - len(must))), replace=False).tolist()
        chosen += sorted(must | set(extra))
    return chosen


def host_subset(ds: DeviceStep, seqs):
    """Host copies (numpy storage arrays) of the cache blocks of the given sequences, renumbered
    0..n-1, with their descriptors, block tables and token rows: input preparation for the oracle
    (results do not depend on physical block ids)."""
    bt = ds.block_tables[seqs]
    used = np.unique(bt[bt >= 0])
    remap = -np.ones(ds.num_blocks, dtype=np.int64)
    remap[used] = np.arange(len(used))
    idx = torch.from_numpy(used.astype(np.int64)).to(ds.k_cache.device)
    k_small = wl.to_numpy_storage(ds.k_cache.index_select(0, idx))
    v_small = wl.to_numpy_storage(ds.v_cache.index_select(0, idx))
    bt_small = np.where(bt >= 0, remap[np.maximum(bt, 0)], -1).astype(np.int32)
    descs = ds.descs[seqs].copy()
    rows = np.concatenate([np.arange(o, o + n) for n, _, o, _ in descs])
    descs[:, 2] = np.concatenate([[0], np.cumsum(descs[:-1, 0])])
    rows_t = torch.from_numpy(rows).to(ds.q.device)
    take = lambda t: wl.to_numpy_storage(t.index_select(0, rows_t))
    return dict(k=k_small, v=v_small, bt=bt_small, descs=descs, rows=rows, rows_t=rows_t,
                q=take(ds.q), k_new=take(ds.k_new), v_new=take(ds.v_new))


def oracle_compare(ds: DeviceStep, n_decode: int, what: str):
    """Run the fp64 oracle (as it stands) on every prompt chunk and a sample of generation rows of
    the batch, compare the device's outputs of those rows and the appended cache of those
    sequences, and time the oracle.  Call BEFORE the first device step (the cache state before the
    pass is taken from the device pool).  Returns a function to call after the device has run."""
    from oracle import attention as oa
    from tests.gpu_util import LAST_MARGINS, assert_outputs_close
    spec = ds.spec
    seqs = pick_sequences(spec, n_decode)
    sub = host_subset(ds, seqs)
    pre = [k for k, s in enumerate(seqs) if spec.seqs[s][0] > 1]
    dec = [k for k, s in enumerate(seqs) if spec.seqs[s][0] == 1]

    def after_device_run():
        t0 = time.perf_counter()
        oa.kv_append(sub["k"], sub["v"], sub["k_new"], sub["v_new"], sub["descs"], sub["bt"], spec.block_size)
        t_app = time.perf_counter() - t0
        kw = dict(block_size=spec.block_size, scale=spec.scale, window=spec.window, dtype=spec.dtype)
        ref = np.full(sub["q"].shape, np.nan)
        # prompt chunks: whole where the dense score matrix is small, else sampled rows, each as a
        # one-row pass over the same history (the oracle's "generation row = last prompt row" pin)
        t0 = time.perf_counter()
        pre_pairs_done = pre_pairs_all = 0
        rng = np.random.default_rng(spec.seed + 7)
        for k in pre:
            n, c, off, _ = (int(x) for x in sub["descs"][k])
            vis = lambda i: min(c + i + 1, spec.window) if spec.window else c + i + 1
            pairs = sum(vis(i) for i in range(n))
            pre_pairs_all += pairs
            if n * (c + n) <= DENSE_PAIR_LIMIT:
                ref[off:off + n] = oa.ragged_attention(sub["q"], sub["k"], sub["v"], sub["descs"], sub["bt"], seq_subset=[k], **kw)[off:off + n]
                pre_pairs_done += pairs
            else:
                for i in sorted({0, 1, 63, 64, n // 2, n - 2, n - 1} | set(rng.integers(0, n, size=17).tolist())):
                    one = np.array([[1, c + i, 0, 0]], np.int32)
                    ref[off + i] = oa.ragged_attention(sub["q"][off + i:off + i + 1], sub["k"], sub["v"], one, sub["bt"][k:k + 1], **kw)[0]
                    pre_pairs_done += vis(i)
        t_pre = time.perf_counter() - t0
        t0 = time.perf_counter()
        if dec:
            out_dec = oa.ragged_attention(sub["q"], sub["k"], sub["v"], sub["descs"], sub["bt"], seq_subset=dec, **kw)
            ref = np.where(np.isnan(ref), out_dec, ref)
        t_dec = time.perf_counter() - t0
        got = ds.out.index_select(0, sub["rows_t"]).to(torch.float64).cpu().numpy()
        mx, mean = assert_outputs_close(got, ref, spec.dtype, what)          # raises: the run ends without a JSON line
        used = np.unique(ds.block_tables[seqs][ds.block_tables[seqs] >= 0])
        idx = torch.from_numpy(used.astype(np.int64)).to(ds.k_cache.device)
        assert np.array_equal(wl.to_numpy_storage(ds.k_cache.index_select(0, idx)), sub["k"]), f"{what}: K cache differs"
        assert np.array_equal(wl.to_numpy_storage(ds.v_cache.index_select(0, idx)), sub["v"]), f"{what}: V cache differs"
        check = {"max_abs": mx, "mean_abs": mean, "worst_row_max_err_over_max_ref": LAST_MARGINS["rel_max"],
                 "worst_row_mean_err_over_mean_ref": LAST_MARGINS["rel_mean"],
                 "rows": int((~np.isnan(ref).any(axis=(1, 2))).sum()), "sequences": len(seqs), "kv_bit_exact": True,
                 "asserted": "max-abs <= 2e-2, mean-abs <= 2e-3, per row and head max-abs <= 2e-2 of max |ref|, per row mean-abs <= 6e-3 of mean |ref|"}
        # oracle time for the whole batch: append by tokens, chunks by (row, key) pairs, generation rows by visible keys
        keys = lambda ks: sum(min(spec.seqs[seqs[k]][1] + 1, spec.window) if spec.window else spec.seqs[seqs[k]][1] + 1 for k in ks)
        all_dec = [s for s, (n, _) in enumerate(spec.seqs) if n == 1]
        keys_all = sum(min(spec.seqs[s][1] + 1, spec.window) if spec.window else spec.seqs[s][1] + 1 for s in all_dec)
        t_full = (t_app * spec.n_tokens / max(len(sub["rows"]), 1)
                  + (t_pre * pre_pairs_all / pre_pairs_done if pre_pairs_done else 0.0)
                  + (t_dec * keys_all / keys(dec) if dec else 0.0))
        cores, blas = host_threads()
        base = dict(value=spec.n_tokens / t_full, unit="tokens/s", cores=cores, blas_threads=blas, kind="oracle",
                    seconds_measured=t_app + t_pre + t_dec,
                    sample=(f"append of {len(sub['rows'])} of {spec.n_tokens} tokens ({t_app:.2f}s) + "
                            f"{pre_pairs_done} of {pre_pairs_all} (row, key) pairs of the {len(pre)} prompt chunks ({t_pre:.2f}s) + "
                            f"{len(dec)} of {len(all_dec)} generation rows ({t_dec:.2f}s); each part scaled to the whole batch "
                            f"(by tokens, pairs, visible keys); numpy fp64, python loops over tokens and heads mostly on one core"))
        return check, base
    return after_device_run


def time_steps(ds: DeviceStep, steps: int, warmup: int):
    """(ms per step by wall clock, average ms per kernel by HIP events inside the timed region)."""
    for _ in range(warmup):
        ds.step()
    torch.cuda.synchronize()
    fsf.profile_enable(True)
    fsf.profile_read()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        ds.step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = fsf.profile_read()
    fsf.profile_enable(False)
    return (t1 - t0) * 1e3 / steps, {k: (v[0] / v[1] if v[1] else 0.0) for k, v in prof.items()}


def committed_traffic(config: int, kernel: str, live_ms: float):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary of
    this workload (profiles/, written by paper_2401_08671_amd.profile_summary), or None if there
    is none or its kernel duration is not the one measured now (a stale profile)."""
    path = os.path.join(ROOT, "profiles", f"bench_cfg{config}_hbm_traffic.md")
    if not os.path.exists(path):
        return None, None
    traffic = ms = None
    for ln in open(path):
        if ln.startswith("hbm_bytes_per_launch:"):
            traffic = float(ln.split(":")[1])
        if ln.startswith("kernel_avg_ms_in_that_run:"):
            ms = float(ln.split(":")[1])
    if traffic is None or ms is None or abs(ms - live_ms) > 0.08 * live_ms:
        return None, None
    return traffic, os.path.relpath(path, ROOT)


def shape_report(config: int, steps: int, warmup: int, n_decode_check: int, with_baseline: bool):
    """Time one benchmark shape and compare it with the oracle.  Returns (report, DeviceStep)."""
    spec = wl.config(config)
    ds = DeviceStep(spec)
    work = algorithmic_work(spec)
    torch.cuda.synchronize()
    finish_check = oracle_compare(ds, n_decode_check, spec.name) if with_baseline else None
    ms_per_step, phase_ms = time_steps(ds, steps, warmup)
    dec_ms, pre_ms = phase_ms["decode"], phase_ms["prefill"]
    hbm_bound = dec_ms >= pre_ms
    if hbm_bound:
        achieved = work["decode_bytes"] / (dec_ms * 1e-3) / 1e9
        traffic, src = committed_traffic(config, "attn_decode_kernel", dec_ms)
        roofline = {"bound": "hbm", "kernel": "attn_decode_kernel", "achieved": achieved, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                    "traffic_from_committed_profile": src,
                    "algorithmic_bytes_per_launch": work["decode_bytes"], "avg_launch_ms": dec_ms}
    else:
        achieved = work["prefill_flops"] / (pre_ms * 1e-3) / 1e12
        traffic, src = committed_traffic(config, "attn_prefill_kernel", pre_ms)
        roofline = {"bound": "mfma", "kernel": "attn_prefill_kernel", "achieved": achieved,
                    "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                    "traffic": traffic, "traffic_from_committed_profile": src,
                    "algorithmic_flops_per_launch": work["prefill_flops"], "avg_launch_ms": pre_ms}
    rep = {
        "workload": (f"{spec.name}: Hq={spec.n_q_heads} Hkv={spec.n_kv_heads} d={spec.head_dim} "
                     f"block={spec.block_size} window={spec.window} budget={spec.n_tokens} "
                     f"({sum(1 for n, _ in spec.seqs if n > 1)} prompt chunks, "
                     f"{sum(1 for n, _ in spec.seqs if n == 1)} generation rows), one layer"),
        "n_seqs": spec.n_seqs, "n_tokens": spec.n_tokens, "kv_pool_blocks": ds.num_blocks,
        "ms_per_step": ms_per_step, "tokens_per_s": spec.n_tokens / (ms_per_step * 1e-3),
        "roofline": roofline, "phases_ms": phase_ms,
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
    if finish_check:
        rep["check_vs_oracle"], rep["cpu_baseline"] = finish_check()
    return rep, ds


def stream_report(warmup: int, check: bool, rate: float = 1.0, warm_passes: int = 0):
    """Benchmark shape 5: 200 consecutive passes of the long-prompt stream, batches from fsf_compose_batch.
    rate: mean arrivals per pass (Poisson).  warm_passes: that many passes are run, untimed, before
    the 200 timed ones, so that the timed ones see the generations of a stream in progress instead
    of the ramp from an empty server."""
    n_steps = 200
    run = StreamRunner(n_steps=n_steps + warm_passes, rate=rate)
    # one fixed set of new-token tensors, sliced per pass (values do not affect timing)
    q_all, k_all, v_all = run.new_tokens(0, run.budget)
    warm = DeviceStep(wl.config(2, n_decodes=8))          # load the kernels before timing
    for _ in range(max(1, warmup)):
        warm.step()
    torch.cuda.synchronize()
    del warm
    for _ in range(warm_passes):                       # untimed: the stream before the timed window
        descs, tables, _ = run.compose()
        T = int(descs[:, 0].sum()) if len(descs) else 0
        run.run_pass(descs, tables, q_all[:T], k_all[:T], v_all[:T])
        run.commit()
    fsf.profile_enable(True)
    fsf.profile_read()
    per_step = []
    t_compose = 0.0
    last = None
    n_rows_max = 0
    spans = []                                          # events around every pass, on the launch stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for step in range(n_steps):
        tc = time.perf_counter()
        descs, tables, _ = run.compose()
        t_compose += time.perf_counter() - tc
        T = int(descs[:, 0].sum()) if len(descs) else 0
        ev = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
        ev[0].record()
        run.run_pass(descs, tables, q_all[:T], k_all[:T], v_all[:T])
        ev[1].record()
        spans.append(ev)
        run.commit()
        spec = wl.BatchSpec(f"pass{step}", run.Hq, run.Hkv, run.d, run.B, run.dtype,
                            [(int(n), int(c)) for n, c, _, _ in descs])
        per_step.append((T, algorithmic_work(spec) if T else None))
        n_rows_max = max(n_rows_max, sum(1 for n, _, _, _ in descs if n == 1))
        last = (descs, tables, T)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = fsf.profile_read()
    fsf.profile_enable(False)
    total_tokens = sum(t for t, _ in per_step)
    gpu_ms = sum(a.elapsed_time(b) for a, b in spans)     # GPU time of the passes (their kernels may overlap)
    attn_ms = gpu_ms - prof["append"][0]                  # ... without the appends: planning, both attention kernels, merges
    bytes_ = sum(w["decode_bytes"] + w["prefill_bytes"] for _, w in per_step if w)
    flops = sum(w["decode_flops"] + w["prefill_flops"] for _, w in per_step if w)
    # ideal time of the stream = sum over passes of max(bytes / HBM peak, flops / MFMA peak)
    t_ideal = sum(max((w["decode_bytes"] + w["prefill_bytes"]) / (HBM_PEAK_GBS * 1e9),
                      (w["decode_flops"] + w["prefill_flops"]) / (MFMA_BF16_PEAK_TFLOPS * 1e12)) for _, w in per_step if w)
    wall_ms = (t1 - t0) * 1e3
    rep = {
        "workload": (f"cfg5-13b-stream: Hq={run.Hq} Hkv={run.Hkv} d={run.d} block={run.B} budget={run.budget}, "
                     f"{n_steps} consecutive passes composed by fsf_compose_batch"
                     + (f" after {warm_passes} untimed passes of the same stream" if warm_passes else "") +
                     f", {len(run.requests)} requests (log-normal prompts, Poisson({rate}) arrivals per pass), one layer; "
                     "wall clock includes host composition and descriptor upload"),
        "arrival_rate_per_pass": rate, "warm_passes": warm_passes, "generation_rows_per_pass_max": n_rows_max,
        "total_tokens": total_tokens, "kv_pool_blocks": run.num_blocks, "passes": n_steps,
        "ms_per_step": wall_ms / n_steps, "tokens_per_s": total_tokens / (t1 - t0),
        "gpu_kernel_ms_total": gpu_ms, "gpu_tokens_per_s": total_tokens / (gpu_ms * 1e-3),
        "host_compose_ms_total": t_compose * 1e3, "wall_ms_total": wall_ms,
        "attention_ms_total": attn_ms, "algorithmic_bytes": bytes_, "algorithmic_flops": flops,
        "achieved_GBs": bytes_ / (attn_ms * 1e-3) / 1e9, "achieved_TFLOPs": flops / (attn_ms * 1e-3) / 1e12,
        "ideal_ms_total_max_of_rooflines": t_ideal * 1e3, "frac_of_per_pass_roofline": t_ideal * 1e3 / attn_ms,
        "phases_ms_total": {k: v[0] for k, v in prof.items()},
        "tokens_per_pass_min_median_max": [int(np.min([t for t, _ in per_step])), int(np.median([t for t, _ in per_step])),
                                           int(np.max([t for t, _ in per_step]))],
    }
    if check and last and last[2]:
        # the last pass once more with known inputs, sampled rows against the oracle (each as a
        # one-row pass over the same history, read back from the device pool the stream wrote)
        from oracle import attention as oa
        from tests.gpu_util import LAST_MARGINS, assert_outputs_close
        descs, tables, T = last
        q = q_all[:T]
        batch = fsf.DeviceBatch(descs, tables, run.device)
        out = run.out[:T]
        out.fill_(float("nan"))
        fsf.ragged_attention(run.cfg, q, run.k_cache, run.v_cache, batch, out, run.ws)
        torch.cuda.synchronize()
        rng = np.random.default_rng(5)
        picks = []
        for s in rng.permutation(len(descs))[:40].tolist():
            n = int(descs[s][0])
            picks += [(s, i) for i in sorted({0, n - 1, n // 2})]
        got_all = out.to(torch.float64).cpu().numpy()
        qn = wl.to_numpy_storage(q)
        worst = dict(max_abs=0.0, rel_max=0.0, rel_mean=0.0)
        for s, i in picks:
            n, c, off, _ = (int(x) for x in descs[s])
            used = tables[s][tables[s] >= 0]
            idx = torch.from_numpy(used.astype(np.int64)).to(run.device)
            k_s = wl.to_numpy_storage(run.k_cache.index_select(0, idx))
            v_s = wl.to_numpy_storage(run.v_cache.index_select(0, idx))
            bt = np.arange(len(used), dtype=np.int32)[None, :]
            one = np.array([[1, c + i, 0, 0]], np.int32)
            ref = oa.ragged_attention(qn[off + i:off + i + 1], k_s, v_s, one, bt, block_size=run.B, scale=run.d ** -0.5, dtype=run.dtype)
            mx, _ = assert_outputs_close(got_all[off + i:off + i + 1], ref, run.dtype, f"stream last pass seq {s} row {i}")
            worst["max_abs"] = max(worst["max_abs"], mx)
            worst["rel_max"] = max(worst["rel_max"], LAST_MARGINS["rel_max"])
            worst["rel_mean"] = max(worst["rel_mean"], LAST_MARGINS["rel_mean"])
        rep["check_vs_oracle"] = {"rows": len(picks), "pass": n_steps - 1, "max_abs": worst["max_abs"],
                                  "worst_row_max_err_over_max_ref": worst["rel_max"],
                                  "worst_row_mean_err_over_mean_ref": worst["rel_mean"],
                                  "note": "attention of the last pass repeated on the pool the 200 passes wrote; K/V history read back from the device"}
    return rep


def sustained_report(ds: DeviceStep, steps: int, burst_ms: float, seconds: float = 10.0):
    """The same step after `seconds` of continuous stepping, and the shader clock the matrix-core
    probe sees right before and right after (the chip lowers its clock under sustained load)."""
    from paper_2401_08671_amd import ceilings
    before = ceilings.mfma_probe(iters=20_000)
    n = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(50):
            ds.step()
        torch.cuda.synchronize()
        n += 50
    soak_s = time.perf_counter() - t0
    ms, phases = time_steps(ds, steps, 0)
    after = ceilings.mfma_probe(iters=20_000)
    return {"soak_seconds": soak_s, "soak_steps": n, "soak_ms_per_step": soak_s * 1e3 / n,
            "ms_per_step_after_soak": ms, "burst_ms_per_step": burst_ms, "slowdown": ms / burst_ms,
            "dominant_kernel_ms_after_soak": max(phases["decode"], phases["prefill"]),
            "mfma_probe_before": before, "mfma_probe_after": after}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=None, choices=[2, 3, 4, 5, 6],
                    help="run only this shape, as the headline (default: shape 3 as the headline plus per_config)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle (no check, no cpu_baseline)")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the measurement of the device's ceilings")
    ap.add_argument("--no-sustained", action="store_true", help="skip the ten seconds of continuous stepping")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (the attention step shards by KV head with no "
              "exchange inside it); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    with_oracle = not args.no_cpu_baseline
    t_start = time.perf_counter()

    if args.config == 5:
        rep = stream_report(args.warmup, with_oracle)
        hbm = rep["algorithmic_bytes"] / (HBM_PEAK_GBS * 1e9) >= rep["algorithmic_flops"] / (MFMA_BF16_PEAK_TFLOPS * 1e12)
        line = {"metric": METRIC, "value": rep["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": rep["passes"],
                "warmup": args.warmup, "ms_per_step": rep["ms_per_step"], "higher_is_better": True, "scaling": "weak",
                "vs_baseline": None, "dtype": "bf16", "data": "synthetic", "config": {"workload": rep["workload"]},
                "roofline": ({"bound": "hbm", "kernel": "attn_decode_kernel + attn_prefill_kernel", "achieved": rep["achieved_GBs"],
                              "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": rep["achieved_GBs"] / HBM_PEAK_GBS, "traffic": None}
                             if hbm else
                             {"bound": "mfma", "kernel": "attn_decode_kernel + attn_prefill_kernel", "achieved": rep["achieved_TFLOPs"],
                              "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": rep["achieved_TFLOPs"] / MFMA_BF16_PEAK_TFLOPS,
                              "traffic": None}),
                "stream": rep}
        print(json.dumps(line))
        return

    head_cfg = args.config or 3
    rep, ds = shape_report(head_cfg, args.steps, args.warmup, n_decode_check=400, with_baseline=with_oracle)
    line = {
        "metric": METRIC, "value": rep["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": rep["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": ds.spec.dtype, "data": "synthetic",
        "config": {"workload": rep["workload"], "n_seqs": rep["n_seqs"], "n_tokens": rep["n_tokens"],
                   "kv_pool_blocks": rep["kv_pool_blocks"]},
        "roofline": rep["roofline"], "phases_ms": rep["phases_ms"], "step_roofline": rep["step_roofline"],
        "decode_only": rep["decode_only"], "prefill_only": rep["prefill_only"],
    }
    if with_oracle:
        line["cpu_baseline"] = rep["cpu_baseline"]
        line["check_vs_oracle"] = rep["check_vs_oracle"]
    if not args.no_sustained:
        line["sustained"] = sustained_report(ds, args.steps, rep["ms_per_step"])
    del ds
    torch.cuda.empty_cache()
    if not args.no_ceilings:
        # what the device sustains with nothing else in the way (scattered 16 KB tiles streamed with
        # non-temporal loads; a register-resident bf16 MFMA loop on normally distributed operands)
        from paper_2401_08671_amd import ceilings
        c = ceilings.measure(hbm_bytes=4 << 30)
        ceil = (c["hbm_read_scattered_16KB_tiles_nontemporal_loads"]["GBs"] if rep["roofline"]["bound"] == "hbm"
                else c["mfma_bf16_normal_operands"]["TFLOPs"])
        line["roofline"]["measured_ceiling"] = ceil
        line["roofline"]["frac_of_measured_ceiling"] = rep["roofline"]["achieved"] / ceil
        line["measured_ceilings"] = c
    if args.config is None:
        per = {}
        for k in (2, 4, 6):
            r, d = shape_report(k, args.steps, args.warmup, n_decode_check=24, with_baseline=with_oracle)
            r.pop("cpu_baseline", None)              # one oracle timing per line: the headline's
            per[f"cfg{k}"] = r
            del d
            torch.cuda.empty_cache()
        per["cfg5_stream"] = stream_report(args.warmup, with_oracle)
        # the same stream at half and at saturating load, and 200 passes of a stream in progress
        slim = lambda r: {k: r[k] for k in ("workload", "total_tokens", "ms_per_step", "tokens_per_s", "gpu_tokens_per_s",
                                             "frac_of_per_pass_roofline", "achieved_GBs", "achieved_TFLOPs",
                                             "generation_rows_per_pass_max", "tokens_per_pass_min_median_max")}
        per["cfg5_stream_rate_0.5"] = slim(stream_report(args.warmup, False, rate=0.5))
        per["cfg5_stream_rate_1.4"] = slim(stream_report(args.warmup, False, rate=1.4))
        per["cfg5_stream_in_progress"] = slim(stream_report(args.warmup, False, rate=1.0, warm_passes=300))
        line["per_config"] = per
    line["bench_seconds"] = time.perf_counter() - t_start
    print(json.dumps(line))


if __name__ == "__main__":
    main()

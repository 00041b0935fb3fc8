"""Turn raw rocprofv3 output into the short text summaries kept under profiles/.

    python -m paper_2401_08671_amd.profile_summary RAW_DIR [--out profiles] [--configs 2 3 4 6]

RAW_DIR holds what these commands wrote (run from the repository root on the MI355X machine, each
profiler pass a run of its own; K = benchmark shape):

    rocprofv3 --kernel-trace --stats --output-format csv -d RAW_DIR/prof_cfgK -o cfgK -- \\
        python3 bench.py --config K --no-cpu-baseline --no-ceilings --no-sustained --steps 50 --warmup 5 \\
        > RAW_DIR/prof_cfgK_bench.json
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d RAW_DIR/pmc_FETCH_SIZE_cfgK -o bench -- \\
        python3 bench.py --config K --no-cpu-baseline --no-ceilings --no-sustained --steps 5 --warmup 2
    rocprofv3 --pmc WRITE_SIZE ...                      (the same with WRITE_SIZE)
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d RAW_DIR/pmc_FETCH_SIZE_copy -o copy -- \\
        python3 -m paper_2401_08671_amd.hbm_counter_calibration 2
    rocprofv3 --pmc WRITE_SIZE ...                      (the same with WRITE_SIZE)
    rocprofv3 --pmc SQ_BUSY_CYCLES SQ_VALU_MFMA_BUSY_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_INSTS_VALU \\
        SQ_LDS_BANK_CONFLICT SQ_WAIT_INST_LDS --output-format csv -d RAW_DIR/pmc_mfma_cfgK -o bench -- \\
        python3 bench.py --config K --no-cpu-baseline --no-ceilings --no-sustained --steps 5 --warmup 2

Writes bench_cfgK_kernel_trace.md, bench_cfgK_hbm_traffic.md and bench_cfgK_mfma.md for every K
whose raw files exist.  HBM bytes = counter (KiB per dispatch) x 1024 x scale, where scale is
what the same counter reads on a plain 2 GiB device copy against the bytes that copy is known
to move.  bench.py reads `hbm_bytes_per_launch` and `kernel_avg_ms_in_that_run` from the
traffic summary for its `roofline.traffic` field.
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import os

KERNELS = ("attn_decode_single_kernel", "attn_decode_kernel", "attn_prefill_kernel", "attn_fused_kernel", "kv_append_kernel",
           "prefill_merge_kernel", "merge_kernel", "plan_kernel", "attn_generic_kernel", "linear_sum_kernel", "linear_kernel")
BENCH_ARGS = "--no-cpu-baseline --no-ceilings --no-sustained"


def short(name: str):
    for k in KERNELS:
        if k in name:
            return k
    return None


def load_counters(path):
    """{kernel name: {counter: [value per dispatch]}}"""
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(path)):
        agg[r["Kernel_Name"]][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return agg


def mean(v):
    return sum(v) / len(v)


def calibration(raw):
    scale, notes = {}, []
    for c in ("FETCH_SIZE", "WRITE_SIZE"):
        path = os.path.join(raw, f"pmc_{c}_copy", "copy_counter_collection.csv")
        if not os.path.exists(path):
            return None, []
        v = [x for k, cs in load_counters(path).items() if "copyBuffer" in k or "copy" in k.lower() for x in cs[c]]
        avg = mean(v)
        scale[c] = (2 * 1024 * 1024) / avg
        notes.append(f"Calibration: a 2 GiB device copy (reads 2097152 KiB, writes 2097152 KiB) shows {c} = {avg:.1f} KiB "
                     f"per launch -> scale {scale[c]:.4f}")
    return scale, notes


def kernel_trace(raw, cfg, out_dir):
    stats = os.path.join(raw, f"prof_cfg{cfg}", f"cfg{cfg}_kernel_stats.csv")
    bj = os.path.join(raw, f"prof_cfg{cfg}_bench.json")
    if not (os.path.exists(stats) and os.path.exists(bj)):
        return None
    bench = json.loads([l for l in open(bj) if l.startswith("{")][-1])
    rows = list(csv.DictReader(open(stats)))
    out = [f"# rocprofv3 kernel trace: bench.py --config {cfg}", "", bench["config"]["workload"], "",
           "Command (run from the repository root on the MI355X box):", "",
           f"    rocprofv3 --kernel-trace --stats --output-format csv -d RAW/prof_cfg{cfg} -o cfg{cfg} -- python3 bench.py "
           f"--config {cfg} {BENCH_ARGS} --steps 50 --warmup 5", "",
           "| kernel | calls | avg ns | min ns | max ns | % of GPU time |", "|---|---|---|---|---|---|"]
    avg_ns = {}
    for r in rows:
        s = short(r["Name"])
        if s:
            avg_ns[s] = float(r["AverageNs"])
            out.append(f"| {s} | {r['Calls']} | {float(r['AverageNs']):.0f} | {r['MinNs']} | {r['MaxNs']} | {float(r['Percentage']):.2f} |")
    out += ["", "bench.py output of the same run (HIP-event averages per kernel inside the timed region, ms):", "",
            "    " + json.dumps({k: round(v, 5) for k, v in bench["phases_ms"].items()}), "",
            f"    roofline: {json.dumps(bench['roofline'])}", "",
            f"    value: {bench['value']:.0f} tokens/s, ms_per_step {bench['ms_per_step']:.4f}", ""]
    open(os.path.join(out_dir, f"bench_cfg{cfg}_kernel_trace.md"), "w").write("\n".join(out))
    return bench, avg_ns


def hbm_traffic(raw, cfg, out_dir, bench, avg_ns, scale, notes):
    f_path = os.path.join(raw, f"pmc_FETCH_SIZE_cfg{cfg}", "bench_counter_collection.csv")
    w_path = os.path.join(raw, f"pmc_WRITE_SIZE_cfg{cfg}", "bench_counter_collection.csv")
    if scale is None or not (os.path.exists(f_path) and os.path.exists(w_path)):
        return
    out = [f"# rocprofv3 HBM traffic counters: bench.py --config {cfg}", "", bench["config"]["workload"], "",
           "Commands (one counter per run; the calibration copy is run the same way):", "",
           f"    rocprofv3 --pmc FETCH_SIZE --output-format csv -d RAW/pmc_FETCH_SIZE_cfg{cfg} -o bench -- python3 bench.py --config {cfg} {BENCH_ARGS} --steps 5 --warmup 2",
           f"    rocprofv3 --pmc WRITE_SIZE --output-format csv -d RAW/pmc_WRITE_SIZE_cfg{cfg} -o bench -- python3 bench.py --config {cfg} {BENCH_ARGS} --steps 5 --warmup 2",
           "    rocprofv3 --pmc FETCH_SIZE --output-format csv -d RAW/pmc_FETCH_SIZE_copy -o copy -- python3 -m paper_2401_08671_amd.hbm_counter_calibration 2",
           "    rocprofv3 --pmc WRITE_SIZE --output-format csv -d RAW/pmc_WRITE_SIZE_copy -o copy -- python3 -m paper_2401_08671_amd.hbm_counter_calibration 2",
           ""] + notes
    out += ["", "| kernel | FETCH_SIZE KiB | WRITE_SIZE KiB | HBM read bytes (scaled) | HBM write bytes (scaled) |", "|---|---|---|---|---|"]
    f, w = load_counters(f_path), load_counters(w_path)
    tot = {}
    for k in f:
        s = short(k)
        if not s or k not in w:
            continue
        fa, wa = mean(f[k]["FETCH_SIZE"]), mean(w[k]["WRITE_SIZE"])
        rb, wb = fa * 1024 * scale["FETCH_SIZE"], wa * 1024 * scale["WRITE_SIZE"]
        tot[s] = rb + wb
        out.append(f"| {s} | {fa:.1f} | {wa:.1f} | {rb:.4g} | {wb:.4g} |")
    dom = bench["roofline"]["kernel"]
    work = bench["roofline"].get("algorithmic_bytes_per_launch")
    out += ["", f"Dominant kernel {dom}: algorithmic bytes per launch {work}, measured HBM traffic per launch, and its",
            "average duration in the kernel-trace run of the same shape (bench.py drops the traffic figure when the",
            "duration it measures differs by more than 8 %):", "",
            f"hbm_bytes_per_launch: {tot[dom]:.0f}", f"kernel_avg_ms_in_that_run: {avg_ns[dom] * 1e-6:.5f}", ""]
    if work:
        out += [f"ratio traffic / algorithmic = {tot[dom] / work:.4f}", ""]
    open(os.path.join(out_dir, f"bench_cfg{cfg}_hbm_traffic.md"), "w").write("\n".join(out))


MFMA_COUNTERS = ("SQ_BUSY_CYCLES", "SQ_VALU_MFMA_BUSY_CYCLES", "SQ_INSTS_VALU_MFMA_MOPS_BF16", "SQ_INSTS_VALU",
                 "SQ_LDS_BANK_CONFLICT", "SQ_WAIT_INST_LDS")


N_SE, N_SIMD = 32, 1024      # MI355X: 8 dies x 4 shader engines; 256 compute units x 4 SIMDs


def mfma_counters(raw, cfg, out_dir, bench, avg_ns):
    path = os.path.join(raw, f"pmc_mfma_cfg{cfg}", "bench_counter_collection.csv")
    if not os.path.exists(path):
        return
    agg = load_counters(path)
    out = [f"# rocprofv3 matrix-core and LDS counters: bench.py --config {cfg}", "", bench["config"]["workload"], "",
           "Command:", "",
           f"    rocprofv3 --pmc {' '.join(MFMA_COUNTERS)} --output-format csv -d RAW/pmc_mfma_cfg{cfg} -o bench -- "
           f"python3 bench.py --config {cfg} {BENCH_ARGS} --steps 5 --warmup 2", "",
           "Averages per dispatch, summed over the chip as rocprofv3 reports them: SQ_BUSY_CYCLES counts once per",
           f"shader engine ({N_SE} of them), the matrix-pipe counter once per SIMD ({N_SIMD}).  So cycles of the launch =",
           f"SQ_BUSY_CYCLES / {N_SE}, matrix-pipe busy cycles per SIMD = SQ_VALU_MFMA_BUSY_CYCLES / {N_SIMD}, and their",
           "ratio is the share of the launch in which a SIMD's matrix pipe was busy, at the clock the chip held",
           "(cycles of the launch / kernel duration); share x clock / 2.4 GHz is the fraction of the published peak.", "",
           "| kernel | " + " | ".join(MFMA_COUNTERS) + " | launch cycles | pipe busy share | clock GHz (cycles / avg duration) |",
           "|---|" + "---|" * (len(MFMA_COUNTERS) + 3)]
    for k, cs in agg.items():
        s = short(k)
        if s not in ("attn_prefill_kernel", "attn_decode_kernel", "attn_fused_kernel", "linear_kernel"):
            continue
        vals = [mean(cs[c]) if cs.get(c) else float("nan") for c in MFMA_COUNTERS]
        busy, mfma, mops = vals[0], vals[1], vals[2]
        cycles = busy / N_SE
        ghz = cycles / avg_ns[s] if avg_ns.get(s) else float("nan")
        out.append(f"| {s} | " + " | ".join(f"{v:.4g}" for v in vals) + f" | {cycles:.4g} | {mfma / N_SIMD / cycles:.3f} | {ghz:.2f} |")
    out += ["", "SQ_INSTS_VALU_MFMA_MOPS_BF16 counts matrix work in units of 512 flops (a 32x32x16 instruction is 64 of",
            "them and keeps the pipe busy for 32 cycles); SQ_INSTS_VALU counts all vector instructions per wave, MFMAs",
            "included; SQ_LDS_BANK_CONFLICT counts cycles lost to LDS bank conflicts; the kernel durations are those of",
            "the kernel-trace run of the same shape.", ""]
    open(os.path.join(out_dir, f"bench_cfg{cfg}_mfma.md"), "w").write("\n".join(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("raw")
    ap.add_argument("--out", default=os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "profiles"))
    ap.add_argument("--configs", type=int, nargs="*", default=[2, 3, 4, 6])
    args = ap.parse_args()
    scale, notes = calibration(args.raw)
    for cfg in args.configs:
        kt = kernel_trace(args.raw, cfg, args.out)
        if kt is None:
            continue
        bench, avg_ns = kt
        hbm_traffic(args.raw, cfg, args.out, bench, avg_ns, scale, notes)
        mfma_counters(args.raw, cfg, args.out, bench, avg_ns)
        print(f"cfg{cfg}: summaries written to {args.out}")


if __name__ == "__main__":
    main()

"""The measurement tools around the library: the profile summariser's arithmetic on a made-up raw
directory (CPU), and one small point of the sweeps, of the layer model and of the ceilings (GPU)."""
import csv
import json
import os

import pytest

from paper_2401_08671_amd import profile_summary as ps


def _write_csv(path, header, rows):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(header)
        w.writerows(rows)


def test_profile_summaries_from_a_made_up_raw_directory(tmp_path):
    """counter x 1024 x (known copy bytes / copy's counter) = HBM bytes; busy cycles / 32 = launch
    cycles; matrix-pipe cycles / 1024 / launch cycles = busy share; cycles / duration = clock"""
    raw, out = str(tmp_path / "raw"), str(tmp_path / "out")
    os.makedirs(out)
    dec = "void fsf::(anonymous namespace)::attn_decode_kernel<1, fsf::bf16_t, false>(...)"
    bench = {"config": {"workload": "made up"}, "value": 1.0e6, "ms_per_step": 2.0,
             "phases_ms": {"decode": 1.9}, "roofline": {"kernel": "attn_decode_kernel", "algorithmic_bytes_per_launch": 8.0e9}}
    os.makedirs(raw)
    with open(os.path.join(raw, "prof_cfg3_bench.json"), "w") as f:
        f.write("noise\n" + json.dumps(bench) + "\n")
    _write_csv(os.path.join(raw, "prof_cfg3", "cfg3_kernel_stats.csv"),
               ["Name", "Calls", "TotalDurationNs", "AverageNs", "Percentage", "MinNs", "MaxNs", "StdDev"],
               [[dec, 50, 100_000_000, 2_000_000.0, 90.0, 1_900_000, 2_100_000, 10.0], ["some_other_kernel", 1, 5, 5.0, 0.1, 5, 5, 0]])
    hdr = ["Dispatch_Id", "Kernel_Name", "Counter_Name", "Counter_Value"]
    # the copy of 2 GiB reads as 1 GiB on FETCH_SIZE (scale 2) and as 2 GiB on WRITE_SIZE (scale 1)
    _write_csv(os.path.join(raw, "pmc_FETCH_SIZE_copy", "copy_counter_collection.csv"), hdr, [[1, "copyBuffer", "FETCH_SIZE", 1024 * 1024]])
    _write_csv(os.path.join(raw, "pmc_WRITE_SIZE_copy", "copy_counter_collection.csv"), hdr, [[1, "copyBuffer", "WRITE_SIZE", 2 * 1024 * 1024]])
    _write_csv(os.path.join(raw, "pmc_FETCH_SIZE_cfg3", "bench_counter_collection.csv"), hdr,
               [[1, dec, "FETCH_SIZE", 4_000_000], [2, dec, "FETCH_SIZE", 4_000_000]])
    _write_csv(os.path.join(raw, "pmc_WRITE_SIZE_cfg3", "bench_counter_collection.csv"), hdr, [[1, dec, "WRITE_SIZE", 100_000]])
    _write_csv(os.path.join(raw, "pmc_mfma_cfg3", "bench_counter_collection.csv"), hdr,
               [[1, dec, "SQ_BUSY_CYCLES", 32 * 4_000_000], [1, dec, "SQ_VALU_MFMA_BUSY_CYCLES", 1024 * 1_000_000],
                [1, dec, "SQ_INSTS_VALU_MFMA_MOPS_BF16", 1], [1, dec, "SQ_INSTS_VALU", 2], [1, dec, "SQ_LDS_BANK_CONFLICT", 0],
                [1, dec, "SQ_WAIT_INST_LDS", 3]])
    scale, notes = ps.calibration(raw)
    assert scale == {"FETCH_SIZE": 2.0, "WRITE_SIZE": 1.0} and len(notes) == 2
    b, avg_ns = ps.kernel_trace(raw, 3, out)
    assert avg_ns == {"attn_decode_kernel": 2_000_000.0}
    ps.hbm_traffic(raw, 3, out, b, avg_ns, scale, notes)
    ps.mfma_counters(raw, 3, out, b, avg_ns)
    text = open(os.path.join(out, "bench_cfg3_hbm_traffic.md")).read()
    want = 4_000_000 * 1024 * 2.0 + 100_000 * 1024 * 1.0
    assert f"hbm_bytes_per_launch: {want:.0f}" in text and "kernel_avg_ms_in_that_run: 2.00000" in text
    assert f"ratio traffic / algorithmic = {want / 8.0e9:.4f}" in text
    row = [l for l in open(os.path.join(out, "bench_cfg3_mfma.md")) if l.startswith("| attn_decode_kernel")][0].split("|")
    assert row[-4].strip() == "4e+06" and row[-3].strip() == "0.250" and row[-2].strip() == "2.00"   # cycles, share, GHz
    assert ps.kernel_trace(raw, 4, out) is None      # nothing collected for that shape: nothing written


def test_the_bench_reads_its_traffic_figure_from_such_a_summary():
    """every committed traffic summary carries the two lines bench.py looks for"""
    prof = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "profiles")
    names = [n for n in os.listdir(prof) if n.endswith("_hbm_traffic.md")]
    assert len(names) >= 4
    for n in names:
        text = open(os.path.join(prof, n)).read()
        assert "hbm_bytes_per_launch: " in text and "kernel_avg_ms_in_that_run: " in text, n


@pytest.mark.gpu
def test_one_point_of_each_sweep_and_of_the_layer_model():
    import torch
    from paper_2401_08671_amd import ceilings, layer_model, sweeps
    from paper_2401_08671_amd import workloads as wl
    from paper_2401_08671_amd.harness import algorithmic_work
    # 128 generation rows over 1024 cached tokens: no faster than its bytes at the HBM peak, no slower than 50 x that
    spec = sweeps.spec_of([(1, 1024)] * 128, "point")
    ms = sweeps.time_spec(spec, steps=5, warmup=2)
    floor_ms = algorithmic_work(spec)["total_bytes"] / 8e12 * 1e3
    assert floor_ms < ms < 50 * floor_ms
    # the layer's linear maps at 64 tokens: at least the weights' bytes at the HBM peak
    rows = layer_model.measure_linear(grid=(64,), reps=3)
    assert len(rows) == 1 and rows[0][0] == 64
    assert layer_model.layer_weight_bytes() / 8e12 < rows[0][1] < 5e-3
    # the matrix-core probe stays below the published peak
    probe = ceilings.mfma_probe(iters=20000)
    assert 100.0 < probe["TFLOPs"] < 2500.0
    # the 16x16x32 instruction sustains at least what 32x32x16 does under the power limit
    probe16 = ceilings.mfma_probe(iters=20000, shape=16)
    assert probe["TFLOPs"] * 0.97 < probe16["TFLOPs"] < 2500.0
    torch.cuda.synchronize()

"""Token-count sweeps of the attention step (the shape of the paper's two motivating figures).

The paper motivates Dynamic SplitFuse with two observations about a whole forward pass
(Sec. 3.1): (1) at a fixed number of forward tokens the pass time barely depends on how
the tokens are split into sequences, and (2) throughput rises with the token count until
it saturates.  Those are whole-model effects dominated by the weight GEMMs, which are not
part of this library; the sweeps below measure the same two questions for the attention
step alone (KV append + ragged attention, Llama-2-13B-shaped heads), where the context
length matters in addition to the token count:

  composition  fixed 2048 forward tokens as 1 x 2048, 2 x 1024, ... 2048 x 1 rows, every
               sequence with the same number of cached tokens
  budget       forward tokens 64 .. 8192 for (a) one prompt chunk at n_cached 0,
               (b) generation rows at n_cached 1024, (c) the half/half SplitFuse mix
  block_size   the cache block size (Sec. 2.1: non-contiguous fixed-size blocks) against the
               HBM rate of 512 generation rows over 2048 cached tokens and the matrix rate of
               one 4096-row chunk over 4096 cached tokens, physical blocks randomly permuted

    python -m paper_2401_08671_amd.sweeps [--only composition|budget|block_size]   # prints one JSON object
"""
from __future__ import annotations

import argparse
import json
import sys

import torch

from . import workloads as wl
from .harness import DeviceStep, algorithmic_work


def time_spec(spec: wl.BatchSpec, steps: int = 10, warmup: int = 2) -> float:
    """Milliseconds per step (CUDA events on torch's current stream, which the library launches on)."""
    ds = DeviceStep(spec)
    for _ in range(warmup):
        ds.step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        ds.step()
    e1.record()
    torch.cuda.synchronize()
    del ds
    return e0.elapsed_time(e1) / steps


def spec_of(seqs, name, block=64):
    return wl.BatchSpec(name, 40, 40, 128, block, "bf16", seqs, seed=4242)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--only", choices=["composition", "budget", "block_size"], default=None)
    only = ap.parse_args().only
    assert torch.cuda.is_available(), "sweeps need a GPU"
    out = {"shape": "Hq=40 Hkv=40 d=128 block=64 bf16, one layer", "composition": [], "budget": [], "block_size": []}
    T, ctx = 2048, 1024
    n_seq = 1
    while n_seq <= T and only in (None, "composition"):
        rows = T // n_seq
        ms = time_spec(spec_of([(rows, ctx)] * n_seq, f"comp-{n_seq}x{rows}"))
        out["composition"].append({"n_seqs": n_seq, "rows_per_seq": rows, "n_cached": ctx, "ms": ms,
                                   "tokens_per_s": T / (ms * 1e-3)})
        n_seq *= 4
    for budget in (64, 128, 256, 512, 1024, 2048, 4096, 8192) if only in (None, "budget") else ():
        row = {"forward_tokens": budget}
        for kind, seqs in (("one_chunk_ctx0", [(budget, 0)]),
                           ("decodes_ctx1024", [(1, 1024)] * budget),
                           ("half_chunk_half_decodes", [(budget // 2, 0)] + [(1, 1024)] * (budget - budget // 2))):
            ms = time_spec(spec_of(seqs, f"budget-{kind}-{budget}"))
            row[kind] = {"ms": ms, "tokens_per_s": budget / (ms * 1e-3)}
        out["budget"].append(row)
    for block in (16, 32, 64, 128, 256) if only in (None, "block_size") else ():
        dec = spec_of([(1, 2048)] * 512, f"block-{block}-decodes", block)
        pre = spec_of([(4096, 4096)], f"block-{block}-chunk", block)
        ms_d, ms_p = time_spec(dec), time_spec(pre)
        wd, wp = algorithmic_work(dec), algorithmic_work(pre)
        out["block_size"].append({"block_size": block, "decodes_ms": ms_d,
                                  "decodes_GBs": wd["total_bytes"] / (ms_d * 1e-3) / 1e9,
                                  "chunk_ms": ms_p, "chunk_TFLOPs": wp["prefill_flops"] / (ms_p * 1e-3) / 1e12})
    json.dump(out, sys.stdout)
    print()


if __name__ == "__main__":
    main()

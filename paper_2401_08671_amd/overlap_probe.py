"""Does matrix-core work anywhere on the chip slow the streaming kernel down?  (measurement aid)

A Dynamic SplitFuse pass holds HBM-bound work (generation rows) and matrix-bound work (prompt
chunks).  Running the two kernels side by side looks like free overlap; this probe measures what
the streaming kernel pays for company.  The main pass (the generation rows of the Llama-2-7B-shaped
benchmark batch, 8.7 GB of K/V) runs on one stream; on a second stream runs, at the same time,
one of

    none            nothing (the reference)
    tiles x N       N workgroups of the prompt-chunk kernel (a 256-row chunk over 60 000 cached
                    tokens, N query heads, tiles not cut): N compute units of MFMA work for longer
                    than the main pass lasts
    stream x N      N waves of the streaming kernel (one generation row over 20 000 cached tokens,
                    N heads, keys not cut): a little more HBM traffic from a second queue, no MFMA
                    work to speak of

Each case reports the main pass's attention time (events on its stream), alone and in company,
and the companion's own time.

    python -m paper_2401_08671_amd.overlap_probe          # prints one JSON object
"""
from __future__ import annotations

import json
import sys

import torch

from . import fsf
from . import workloads as wl
from .harness import DeviceStep


class _Side:
    def __init__(self, spec, tuning):
        self.ds = DeviceStep(spec)
        self.cfg = fsf.make_cfg(spec.n_q_heads, spec.n_kv_heads, spec.head_dim, spec.block_size, spec.dtype,
                                self.ds.num_blocks, tuning=tuning)
        self.ws = fsf.alloc_workspace(self.cfg, self.ds.batch.n_seqs, self.ds.batch.n_tokens, self.ds.batch.max_blocks)
        self.ds.step()                      # the chunk's own tokens into the cache

    def attention(self):
        d = self.ds
        fsf.ragged_attention(self.cfg, d.q, d.k_cache, d.v_cache, d.batch, d.out, self.ws)


def _timed(fn, stream):
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    with torch.cuda.stream(stream):
        e0.record()
        fn()
        e1.record()
    return e0, e1


def measure(reps: int = 7):
    main_spec = wl.config(2)
    main_spec.seqs = [s for s in main_spec.seqs if s[0] == 1]          # the generation rows only
    main = DeviceStep(main_spec)
    main.step()
    attn = lambda: fsf.ragged_attention(main.cfg, main.q, main.k_cache, main.v_cache, main.batch, main.out, main.ws)
    s_main, s_side = torch.cuda.Stream(), torch.cuda.Stream()
    sides = {"none": None}
    for n in (1, 8, 32):
        sides[f"tiles x {n}"] = _Side(wl.BatchSpec("side-tiles", n, n, 128, 64, "bf16", [(256, 60000)], seed=3),
                                      fsf.Tuning(prefill_split=-1, stream_chunk_slices=-1))
    for n in (1, 8):
        sides[f"stream x {n}"] = _Side(wl.BatchSpec("side-stream", n, n, 128, 64, "bf16", [(1, 20000)], seed=4),
                                       fsf.Tuning(decode_target_waves=1, decode_min_item_blocks=100000))
    torch.cuda.synchronize()
    out = {}
    for name, side in sides.items():
        alone, together, side_alone, side_together = [], [], [], []
        for _ in range(reps):
            e = _timed(attn, s_main)
            torch.cuda.synchronize()
            alone.append(e[0].elapsed_time(e[1]))
            if side is None:
                continue
            e = _timed(side.attention, s_side)
            torch.cuda.synchronize()
            side_alone.append(e[0].elapsed_time(e[1]))
            es = _timed(side.attention, s_side)          # the companion first, so that it is running
            em = _timed(attn, s_main)
            torch.cuda.synchronize()
            together.append(em[0].elapsed_time(em[1]))
            side_together.append(es[0].elapsed_time(es[1]))
        med = lambda v: sorted(v)[len(v) // 2] if v else None
        out[name] = dict(main_ms_alone=med(alone), main_ms_in_company=med(together),
                         companion_ms_alone=med(side_alone), companion_ms_in_company=med(side_together))
        if together:
            out[name]["main_slowdown"] = med(together) / med(alone)
    return out


def main():
    assert torch.cuda.is_available(), "needs a GPU"
    json.dump(measure(), sys.stdout)
    print()


if __name__ == "__main__":
    main()

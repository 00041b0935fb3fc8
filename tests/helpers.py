"""Test-side glue: build a ragged step (inputs + pre-filled cache) from a BatchSpec.

The cache state *before* the step is produced with the oracle's own append (oracle output
may feed the HIP path as an input; never the other way round).
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import attention as oa
from paper_2401_08671_amd import workloads as wl

NP_STORAGE = {"f32": np.float32, "f16": np.float16, "bf16": np.uint16}

# bit patterns used to poison unwritten cache slots
POISON = {
    "nan": {"f32": np.uint32(0x7FC00000), "bf16": np.uint16(0x7FC0), "f16": np.uint16(0x7E00)},
    "inf": {"f32": np.uint32(0x7F800000), "bf16": np.uint16(0x7F80), "f16": np.uint16(0x7C00)},
    "big": {"f32": np.uint32(0x7F000000), "bf16": np.uint16(0x7F00), "f16": np.uint16(0x7BFF)},
}


def poison_pool(shape, dtype: str, kind: str) -> np.ndarray:
    bits = POISON[kind][dtype]
    a = np.full(shape, bits, dtype=bits.dtype)
    return a.view(NP_STORAGE[dtype]) if dtype != "bf16" else a


class Step:
    """All arrays of one forward pass, as numpy storage arrays."""

    def __init__(self, spec: wl.BatchSpec, num_blocks: int | None = None, poison: str | None = None,
                 max_blocks: int | None = None, seed_shift: int = 0):
        self.spec = spec
        B, Hq, Hkv, d = spec.block_size, spec.n_q_heads, spec.n_kv_heads, spec.head_dim
        rng = np.random.default_rng(spec.seed + seed_shift)
        need = spec.blocks_needed()
        self.num_blocks = num_blocks if num_blocks is not None else need + max(4, need // 8)
        self.descs = wl.make_descs(spec.seqs)
        self.block_tables = wl.make_block_tables(spec.seqs, B, self.num_blocks, rng, max_blocks)
        T = spec.n_tokens
        sd = spec.seed + seed_shift
        self.q = wl.to_numpy_storage(wl.randn((T, Hq, d), spec.dtype, spec.value_mult, sd * 7 + 1))
        self.k_new = wl.to_numpy_storage(wl.randn((T, Hkv, d), spec.dtype, spec.value_mult, sd * 7 + 2))
        self.v_new = wl.to_numpy_storage(wl.randn((T, Hkv, d), spec.dtype, spec.value_mult, sd * 7 + 3))
        shape = (self.num_blocks, Hkv, B, d)
        if poison is None:
            self.k_cache0 = wl.to_numpy_storage(wl.randn(shape, spec.dtype, spec.value_mult, sd * 7 + 4))
            self.v_cache0 = wl.to_numpy_storage(wl.randn(shape, spec.dtype, spec.value_mult, sd * 7 + 5))
        else:
            self.k_cache0 = poison_pool(shape, spec.dtype, poison)
            self.v_cache0 = poison_pool(shape, spec.dtype, poison)
        # earlier tokens of every sequence: written through the oracle's append
        hist = [(c, 0) for _, c in spec.seqs if c > 0]
        if hist:
            idx = [s for s, (_, c) in enumerate(spec.seqs) if c > 0]
            hd = wl.make_descs(hist)
            Th = int(hd[:, 0].sum())
            kh = wl.to_numpy_storage(wl.randn((Th, Hkv, d), spec.dtype, spec.value_mult, sd * 7 + 6))
            vh = wl.to_numpy_storage(wl.randn((Th, Hkv, d), spec.dtype, spec.value_mult, sd * 7 + 7))
            oa.kv_append(self.k_cache0, self.v_cache0, kh, vh, hd, self.block_tables[idx], B)

    def oracle(self, seq_subset=None):
        """(k_cache_after, v_cache_after, out_f64) by the oracle."""
        sp = self.spec
        kc, vc = self.k_cache0.copy(), self.v_cache0.copy()
        oa.kv_append(kc, vc, self.k_new, self.v_new, self.descs, self.block_tables, sp.block_size)
        out = oa.ragged_attention(self.q, kc, vc, self.descs, self.block_tables,
                                  block_size=sp.block_size, scale=sp.scale, window=sp.window,
                                  dtype=sp.dtype, seq_subset=seq_subset)
        return kc, vc, out


def t2f64(t: torch.Tensor) -> np.ndarray:
    """Device/host tensor -> float64 numpy, exactly."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def plant_dominant_key(step: Step, s: int, row: int, q_head: int, position: int, logit: float = 34.0):
    """Make key ``position`` of sequence ``s`` dominate the softmax of (row ``row`` of that
    sequence, query head ``q_head``): its K row becomes a multiple of that query, scaled so that
    the logit is ``logit`` (random keys give logits of a few units at most).  The row's output is
    then that key's V row to ~1e-12, so a unit, part or split that drops or doubles the key moves
    the output by O(1).  Edits ``k_cache0`` (cached positions) or ``k_new`` (this pass's
    tokens) in place; returns the planted key's V row as float64 ``[d]``."""
    sp = step.spec
    n_new, n_cached, q_off, _ = (int(x) for x in step.descs[s])
    assert 0 <= row < n_new and 0 <= position <= n_cached + row
    hk = q_head // (sp.n_q_heads // sp.n_kv_heads)
    q = oa.to_f64(step.q[q_off + row, q_head], sp.dtype)
    k = (q * (logit / (sp.scale * float(q @ q)))).astype(np.float32)
    k_bits = oa.f32_to_storage(k, sp.dtype)
    if position < n_cached:
        blk = int(step.block_tables[s, position // sp.block_size])
        step.k_cache0[blk, hk, position % sp.block_size] = k_bits
        return oa.to_f64(step.v_cache0[blk, hk, position % sp.block_size], sp.dtype)
    step.k_new[q_off + position - n_cached, hk] = k_bits
    return oa.to_f64(step.v_new[q_off + position - n_cached, hk], sp.dtype)

"""Device-side harness shared by the benchmark and the GPU tests.

Builds the device buffers of one forward pass from a seeded BatchSpec, runs the pass
through the C-ABI binding, and counts the algorithmic bytes and flops of a batch.  No
attention or cache arithmetic lives here: every step of the path runs in libfsf.so.
"""
from __future__ import annotations

import numpy as np
import torch

from . import fsf
from . import workloads as wl


def algorithmic_work(spec: wl.BatchSpec):
    """Bytes and flops the method must move/compute, per kernel class, from the descriptors."""
    e = wl.DTYPE_BYTES[spec.dtype]
    d, Hq, Hkv = spec.head_dim, spec.n_q_heads, spec.n_kv_heads
    dec_bytes = pre_bytes = 0
    dec_flops = pre_flops = 0
    for n, c in spec.seqs:
        ps = np.arange(c, c + n, dtype=np.int64) + 1          # keys visible to each row without a window
        pairs = int(np.minimum(ps, spec.window).sum() if spec.window else ps.sum())
        vis_tokens = (c + n) if not spec.window else min(c + n, spec.window + n - 1)
        kv = 2 * Hkv * d * e * vis_tokens           # K+V read once per step
        qo = 2 * Hq * d * e * n                     # Q in, O out
        fl = 4 * d * pairs * Hq
        if n == 1:
            dec_bytes += kv + qo
            dec_flops += fl
        else:
            pre_bytes += kv + qo
            pre_flops += fl
    append_bytes = 4 * Hkv * d * e * spec.n_tokens   # read new K/V, write them to the cache
    return dict(decode_bytes=dec_bytes, prefill_bytes=pre_bytes, append_bytes=append_bytes,
                decode_flops=dec_flops, prefill_flops=pre_flops,
                total_bytes=dec_bytes + pre_bytes + append_bytes)


class DeviceStep:
    """All device buffers of one step, generated on the GPU with seeded generators."""

    def __init__(self, spec: wl.BatchSpec, device="cuda"):
        self.spec = spec
        B, Hq, Hkv, d = spec.block_size, spec.n_q_heads, spec.n_kv_heads, spec.head_dim
        need = spec.blocks_needed()
        self.num_blocks = need + max(16, need // 50)
        rng = np.random.default_rng(spec.seed)
        self.descs = wl.make_descs(spec.seqs)
        self.block_tables = wl.make_block_tables(spec.seqs, B, self.num_blocks, rng)
        self.batch = fsf.DeviceBatch(self.descs, self.block_tables, device)
        T = spec.n_tokens
        tdt = wl.TORCH_DTYPE[spec.dtype]
        self.q = wl.randn((T, Hq, d), spec.dtype, spec.value_mult, spec.seed * 7 + 1, device)
        self.k_new = wl.randn((T, Hkv, d), spec.dtype, spec.value_mult, spec.seed * 7 + 2, device)
        self.v_new = wl.randn((T, Hkv, d), spec.dtype, spec.value_mult, spec.seed * 7 + 3, device)
        self.k_cache = torch.empty((self.num_blocks, Hkv, B, d), dtype=tdt, device=device)
        self.v_cache = torch.empty_like(self.k_cache)
        wl.fill_pool_(self.k_cache, spec.value_mult, spec.seed * 7 + 4)
        wl.fill_pool_(self.v_cache, spec.value_mult, spec.seed * 7 + 5)
        self.out = torch.zeros((T, Hq, d), dtype=tdt, device=device)
        self.cfg = fsf.make_cfg(Hq, Hkv, d, B, spec.dtype, self.num_blocks, window=spec.window, scale=spec.scale)
        # same pass with prompt-chunk and generation-row work launched as two kernels (for per-kind timings)
        self.cfg_separate = fsf.make_cfg(Hq, Hkv, d, B, spec.dtype, self.num_blocks, window=spec.window,
                                         scale=spec.scale, flags=fsf.FSF_FLAG_SEPARATE_KERNELS)
        self.ws = fsf.alloc_workspace(self.cfg, self.batch.n_seqs, self.batch.n_tokens, self.batch.max_blocks, device)

    def step(self, separate: bool = False):
        cfg = self.cfg_separate if separate else self.cfg
        fsf.kv_append(cfg, self.k_new, self.v_new, self.k_cache, self.v_cache, self.batch)
        fsf.ragged_attention(cfg, self.q, self.k_cache, self.v_cache, self.batch, self.out, self.ws)

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

    def __init__(self, spec: wl.BatchSpec, device="cuda", tuning=None):
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
        self.cfg = fsf.make_cfg(Hq, Hkv, d, B, spec.dtype, self.num_blocks, window=spec.window, scale=spec.scale,
                                tuning=tuning)
        # same pass with prompt-chunk and generation-row work in one fused grid
        self.cfg_fused = fsf.make_cfg(Hq, Hkv, d, B, spec.dtype, self.num_blocks, window=spec.window,
                                      scale=spec.scale, flags=fsf.FSF_FLAG_FUSED_LAUNCH)
        self.ws = fsf.alloc_workspace(self.cfg, self.batch.n_seqs, self.batch.n_tokens, self.batch.max_blocks, device)

    def step(self, fused: bool = False):
        cfg = self.cfg_fused if fused else self.cfg
        fsf.kv_append(cfg, self.k_new, self.v_new, self.k_cache, self.v_cache, self.batch)
        fsf.ragged_attention(cfg, self.q, self.k_cache, self.v_cache, self.batch, self.out, self.ws)


class StreamRunner:
    """The long-prompt stream: requests arrive step by step, fsf_compose_batch builds every pass.

    Each pass: arrivals -> compose (host) -> descriptors and block tables to the device ->
    fsf_kv_append + fsf_ragged_attention -> step_done.  New-token tensors are drawn per pass
    from a seeded generator (there is no model: the "generated token" is just a counter).
    """

    def __init__(self, n_steps: int = 200, rate: float = 1.0, seed: int = 1005, device="cuda", tuning=None):
        shp = wl.stream_shape()
        self.Hq, self.Hkv, self.d, self.B = shp["n_q_heads"], shp["n_kv_heads"], shp["head_dim"], shp["block_size"]
        self.dtype, self.budget, self.n_steps = shp["dtype"], shp["token_budget"], n_steps
        self.device = device
        self.requests = wl.stream_requests(n_steps, rate, seed)
        self.arrivals = {}
        for step, sid, plen, gen in self.requests:
            self.arrivals.setdefault(step, []).append((sid, plen, gen))
        need = sum(-(-(p + g) // self.B) for _, _, p, g in self.requests)
        self.num_blocks = need + 64
        self.max_blocks = -(-(32768 + 600) // self.B)
        self.max_seqs = self.budget
        rng = np.random.default_rng(seed)
        self.sched = fsf.Scheduler(self.budget, self.max_seqs, self.B, self.num_blocks, self.max_blocks,
                                   rng.permutation(self.num_blocks))
        tdt = wl.TORCH_DTYPE[self.dtype]
        self.k_cache = torch.zeros((self.num_blocks, self.Hkv, self.B, self.d), dtype=tdt, device=device)
        self.v_cache = torch.zeros_like(self.k_cache)
        self.cfg = fsf.make_cfg(self.Hq, self.Hkv, self.d, self.B, self.dtype, self.num_blocks, tuning=tuning)
        self.ws = fsf.alloc_workspace(self.cfg, self.max_seqs, self.budget, self.max_blocks, device)
        self.out = torch.zeros((self.budget, self.Hq, self.d), dtype=tdt, device=device)
        self.step_index = 0

    def new_tokens(self, step: int, n_tokens: int):
        """Q, K, V rows of this pass (seeded by the step index)."""
        q = wl.randn((n_tokens, self.Hq, self.d), self.dtype, 1.0, 50_000 + 3 * step, self.device)
        k = wl.randn((n_tokens, self.Hkv, self.d), self.dtype, 1.0, 50_001 + 3 * step, self.device)
        v = wl.randn((n_tokens, self.Hkv, self.d), self.dtype, 1.0, 50_002 + 3 * step, self.device)
        return q, k, v

    def compose(self):
        """Arrivals + fsf_compose_batch for the next pass; returns (descs, block_tables, emits)."""
        for sid, plen, gen in self.arrivals.get(self.step_index, []):
            self.sched.add_request(sid, plen, gen)
        return self.sched.compose_batch()

    def run_pass(self, descs, tables, q, k_new, v_new):
        """Enqueue append + attention for a composed pass; returns the output view [T, Hq, d]."""
        batch = fsf.DeviceBatch(descs, tables, self.device)
        if batch.n_seqs == 0:
            return self.out[:0]
        out = self.out[:batch.n_tokens]
        fsf.kv_append(self.cfg, k_new, v_new, self.k_cache, self.v_cache, batch)
        fsf.ragged_attention(self.cfg, q, self.k_cache, self.v_cache, batch, out, self.ws)
        return out

    def commit(self):
        self.sched.step_done()
        self.step_index += 1

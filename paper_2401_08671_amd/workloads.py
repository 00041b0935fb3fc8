"""Seeded synthetic workloads: shapes, length mixes and random tensors only.

This module serves the tests, the smoke check and the benchmark.  It holds none of the
method's arithmetic (no attention, no cache indexing): it draws sequence lengths,
block-id permutations and Gaussian tensors, and describes the five benchmark shapes.
It imports neither the CPU oracle nor the HIP binding.

The paper's own workloads are synthetic length distributions fed to trained Llama-2
weights (Sec. 4.1-4.2: prompt and generation lengths drawn from a normal distribution).
Without those weights, the shapes below keep the models' attention geometry (heads,
head_dim, GQA ratio, sliding window) and draw Q/K/V i.i.d. Gaussian.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np
import torch

TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}
DTYPE_BYTES = {"f32": 4, "bf16": 2, "f16": 2}


@dataclass
class BatchSpec:
    """One forward pass over a ragged batch."""
    name: str
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    block_size: int
    dtype: str                      # "f32" | "bf16" | "f16"
    seqs: list                      # [(n_new, n_cached), ...] in batch order
    window: int = 0                 # 0 = plain causal
    value_mult: float = 1.0         # Q/K/V = N(0,1) * value_mult before rounding
    seed: int = 0
    scale: float = field(default=0.0)

    def __post_init__(self):
        if self.scale == 0.0:
            self.scale = 1.0 / math.sqrt(self.head_dim)

    @property
    def n_tokens(self) -> int:
        return sum(n for n, _ in self.seqs)

    @property
    def n_seqs(self) -> int:
        return len(self.seqs)

    def blocks_needed(self) -> int:
        return sum(-(-(n + c) // self.block_size) for n, c in self.seqs)


# --------------------------------------------------------------------------------------
# the benchmark shapes
# --------------------------------------------------------------------------------------
def config(k: int, n_decodes: int | None = None) -> BatchSpec:
    """Benchmark shape ``k`` (1..4).  ``n_decodes`` shrinks the generation count for tests."""
    seed = 1000 + k
    rng = np.random.default_rng(seed)
    if k == 1:
        return BatchSpec("cfg1-tiny-f32", 4, 4, 64, 16, "f32",
                         [(128, 0), (64, 256), (1, 100), (1, 517)], seed=seed)
    if k == 2:
        nd = 256 if n_decodes is None else n_decodes
        c = rng.integers(128, 4097, size=nd)
        return BatchSpec("cfg2-llama2-7b", 32, 32, 128, 64, "bf16",
                         [(1792, 0)] + [(1, int(x)) for x in c],
                         value_mult=1.0 / math.sqrt(128.0), seed=seed)
    if k == 3:
        nd = 2048 if n_decodes is None else n_decodes
        c = np.rint(np.exp(rng.uniform(math.log(256.0), math.log(16384.0), size=nd))).astype(np.int64)
        return BatchSpec("cfg3-mistral-7b-gqa-swa", 32, 8, 128, 64, "bf16",
                         [(1024, 2048), (1024, 6144)] + [(1, int(x)) for x in c],
                         window=4096, seed=seed)
    if k == 4:
        nd = 1984 if n_decodes is None else n_decodes
        c = rng.integers(512, 2049, size=nd)
        return BatchSpec("cfg4-llama2-70b-share", 64, 8, 128, 64, "bf16",
                         [(1, int(x)) for x in c] + [(64, 3000)], seed=seed)
    if k == 6:
        # the heaviest kind of step of the long-prompt stream: a full-budget chunk deep into a long prompt
        return BatchSpec("cfg5-step-13b-chunk4096-at-8192", 40, 40, 128, 64, "bf16", [(4096, 8192)], seed=seed)
    raise ValueError("config index must be 1..4 or 6 (config 5 is a request stream, see stream_requests)")


def stream_shape() -> dict:
    """Attention geometry of the long-prompt stream (benchmark shape 5)."""
    return dict(n_q_heads=40, n_kv_heads=40, head_dim=128, block_size=64, dtype="bf16",
                token_budget=4096, n_steps=200)


def stream_requests(n_steps: int = 200, rate: float = 1.0, seed: int = 1005):
    """Arrivals for the long-prompt stream: ``[(step, seq_id, prompt_len, max_new_tokens)]``.

    Prompt lengths are log-normal with arithmetic mean 2600 and sd 1500, clipped to
    [256, 32768]; output lengths uniform in [60, 600]; arrivals per step Poisson(rate).
    """
    rng = np.random.default_rng(seed)
    sigma2 = math.log(1.0 + (1500.0 / 2600.0) ** 2)
    mu = math.log(2600.0) - 0.5 * sigma2
    out, sid = [], 0
    for step in range(n_steps):
        for _ in range(int(rng.poisson(rate))):
            plen = int(np.clip(np.rint(rng.lognormal(mu, math.sqrt(sigma2))), 256, 32768))
            gen = int(rng.integers(60, 601))
            out.append((step, sid, plen, gen))
            sid += 1
    return out


def chat_requests(n_requests: int = 512, prompt_mean: float = 2600.0, gen_mean: float = 60.0,
                  rel_sd: float = 0.3, seed: int = 2024):
    """Requests of the paper's serving benchmarks (Sec. 4.1, figure captions): prompt and
    generation lengths normal with the given means and a standard deviation of 30 % of the
    mean, rounded, at least 1 token (prompts at least 16).  Returns ``[(prompt_len, gen_len)]``."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n_requests):
        p = int(max(16, round(rng.normal(prompt_mean, rel_sd * prompt_mean))))
        g = int(max(1, round(rng.normal(gen_mean, rel_sd * gen_mean))))
        out.append((p, g))
    return out


# --------------------------------------------------------------------------------------
# descriptors, block tables, tensors
# --------------------------------------------------------------------------------------
def make_descs(seqs) -> np.ndarray:
    """``int32 [S, 4]`` rows ``(n_new, n_cached, q_offset, seq_id)``; q_offset is the running sum."""
    d = np.zeros((len(seqs), 4), dtype=np.int32)
    off = 0
    for s, (n, c) in enumerate(seqs):
        d[s] = (n, c, off, s)
        off += n
    return d


def make_block_tables(seqs, block_size: int, num_blocks: int, rng, max_blocks: int | None = None) -> np.ndarray:
    """Hand each sequence distinct physical blocks drawn from a seeded permutation of the pool."""
    need = [-(-(n + c) // block_size) for n, c in seqs]
    if max_blocks is None:
        max_blocks = max(need) if need else 1
    assert sum(need) <= num_blocks, "pool too small"
    perm = rng.permutation(num_blocks).astype(np.int32)
    bt = np.full((len(seqs), max_blocks), -1, dtype=np.int32)
    pos = 0
    for s, nb in enumerate(need):
        bt[s, :nb] = perm[pos:pos + nb]
        pos += nb
    return bt


def randn(shape, dtype: str, mult: float, seed: int, device="cpu") -> torch.Tensor:
    """N(0,1)*mult rounded to the storage dtype, drawn with a seeded generator on ``device``."""
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    x = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    if mult != 1.0:
        x = x * mult
    return x.to(TORCH_DTYPE[dtype])


def fill_pool_(pool: torch.Tensor, mult: float, seed: int, chunk_blocks: int = 256) -> None:
    """Fill a ``[num_blocks, Hkv, B, d]`` pool in place with N(0,1)*mult, chunk by chunk."""
    g = torch.Generator(device=pool.device)
    g.manual_seed(seed)
    for b0 in range(0, pool.shape[0], chunk_blocks):
        view = pool[b0:b0 + chunk_blocks]
        x = torch.randn(view.shape, generator=g, device=pool.device, dtype=torch.float32)
        if mult != 1.0:
            x = x * mult
        view.copy_(x)


def to_numpy_storage(t: torch.Tensor) -> np.ndarray:
    """Torch tensor -> numpy array carrying the same bits (bf16 becomes uint16)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def from_numpy_storage(a: np.ndarray, dtype: str, device="cpu") -> torch.Tensor:
    """Inverse of :func:`to_numpy_storage`."""
    if dtype == "bf16":
        return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).to(device)
    return torch.from_numpy(a.copy()).to(device)

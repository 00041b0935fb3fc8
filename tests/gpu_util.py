"""Run a tests.helpers.Step through the HIP library (C ABI via the ctypes binding)."""
from __future__ import annotations

import numpy as np
import torch

from paper_2401_08671_amd import fsf
from paper_2401_08671_amd import workloads as wl

# tolerances: bf16/f16 as the task states; fp32 derived from fp32 accumulation over <= ~1e4 keys
TOL = {"bf16": (2e-2, 2e-3), "f16": (2e-2, 2e-3), "f32": (1e-4, 1e-5)}


def run_hip(step, flags: int = 0, return_cache: bool = True, repeat_append: int = 1, tuning=None,
            repeat_attention: int = 1):
    """Returns (k_cache_after, v_cache_after, out) as numpy storage arrays / float64 out."""
    sp = step.spec
    dev = "cuda"
    cfg = fsf.make_cfg(sp.n_q_heads, sp.n_kv_heads, sp.head_dim, sp.block_size, sp.dtype, step.num_blocks,
                       window=sp.window, scale=sp.scale, flags=flags, tuning=tuning)
    batch = fsf.DeviceBatch(step.descs, step.block_tables, dev)
    q = wl.from_numpy_storage(step.q, sp.dtype, dev)
    k_new = wl.from_numpy_storage(step.k_new, sp.dtype, dev)
    v_new = wl.from_numpy_storage(step.v_new, sp.dtype, dev)
    kc = wl.from_numpy_storage(step.k_cache0, sp.dtype, dev)
    vc = wl.from_numpy_storage(step.v_cache0, sp.dtype, dev)
    out = torch.full_like(q, float("nan"))
    ws = fsf.alloc_workspace(cfg, batch.n_seqs, batch.n_tokens, batch.max_blocks, dev)
    for _ in range(repeat_append):
        fsf.kv_append(cfg, k_new, v_new, kc, vc, batch)
    for _ in range(repeat_attention):          # back to back, no wait in between
        fsf.ragged_attention(cfg, q, kc, vc, batch, out, ws)
    torch.cuda.synchronize()
    out64 = out.to(torch.float64).cpu().numpy()
    if return_cache:
        return wl.to_numpy_storage(kc), wl.to_numpy_storage(vc), out64
    return None, None, out64


# Bounds relative to the size of the reference, which must hold besides the absolute ones (an
# absolute bound alone cannot fail where the outputs themselves are smaller than it: long rows,
# down-scaled values).  Where they come from: the device rounds the softmax weights to the
# storage type for the second product (relative error <= 2^-9 for bf16, rms 2^-9 / sqrt(3)) and
# the result once more, everything else is fp32.  With independent values the first error has
# the rms 1.1e-3 * rms(row of the reference), the second 2^-9 / sqrt(3) * |element|: together
# about 1.6e-3 of the row's rms, mean-abs about 1.6e-3 of the row's mean-abs, and the largest of
# 128 errors about 1.6e-3 of the row's largest element (a numpy model of exactly this rounding
# in tests/test_checker.py measures 1.8e-3..2.1e-3 for the mean and 2.5e-3..3.9e-3 for the
# maximum).  The bounds leave a factor of 3 on the mean (an average over n_q_heads * d
# elements) and of 5 on the maximum (a tail event over millions of rows); a lost or doubled
# unit of 1/64 of the keys moves a row by ~12 %.  f16 rounds four times finer; fp32 carries ~1e-6.
#   per (row, head):  max-abs error <= REL_MAX  * max |reference|
#   per row:          mean-abs error <= REL_MEAN * mean |reference|
REL_TOL = {"bf16": (2e-2, 6e-3), "f16": (2e-2, 6e-3), "f32": (1e-4, 2e-5)}


def assert_outputs_close(got64: np.ndarray, want64: np.ndarray, dtype: str, what: str = ""):
    """got, want: float64 [rows, heads, d]; rows the oracle was not asked for are NaN in want."""
    assert got64.shape == want64.shape and want64.ndim == 3
    rows = ~np.isnan(want64).any(axis=(1, 2))
    assert rows.any()
    got, want = got64[rows], want64[rows]
    assert np.isfinite(got).all(), f"{what}: non-finite outputs"
    err = np.abs(got - want)
    mx, mean = float(err.max()), float(err.mean())
    tol_max, tol_mean = TOL[dtype]
    assert mx <= tol_max and mean <= tol_mean, f"{what}: max-abs {mx:.3e} (<= {tol_max}), mean-abs {mean:.3e} (<= {tol_mean})"
    rel_max, rel_mean = REL_TOL[dtype]
    ref = np.abs(want)
    r_max = err.max(axis=2) / np.maximum(ref.max(axis=2), 1e-300)          # [rows, heads]
    r_mean = err.mean(axis=(1, 2)) / np.maximum(ref.mean(axis=(1, 2)), 1e-300)   # [rows]
    worst_max, worst_mean = float(r_max.max()), float(r_mean.max())
    assert worst_max <= rel_max, (f"{what}: a row's max-abs error is {worst_max:.3e} of its largest reference "
                                  f"element (<= {rel_max}); row {np.unravel_index(r_max.argmax(), r_max.shape)} of the checked rows")
    assert worst_mean <= rel_mean, (f"{what}: a row's mean-abs error is {worst_mean:.3e} of its mean-abs reference "
                                    f"(<= {rel_mean}); row {int(r_mean.argmax())} of the checked rows")
    LAST_MARGINS.update(what=what, rel_max=worst_max, rel_mean=worst_mean, max_abs=mx, mean_abs=mean)
    return mx, mean


LAST_MARGINS: dict = {}      # figures of the last passed comparison (for reports)


def assert_cache_bit_exact(got: np.ndarray, want: np.ndarray, what: str = ""):
    g = got.view(np.uint16 if got.dtype.itemsize == 2 else np.uint32)
    w = want.view(np.uint16 if want.dtype.itemsize == 2 else np.uint32)
    assert np.array_equal(g, w), f"{what}: cache differs in {(g != w).sum()} elements"

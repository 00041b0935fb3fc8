"""Measured ceilings of the device (fsf_ceiling_*): scattered-tile streaming reads and a
register-resident MFMA loop, to set beside the published peaks.

    python -m paper_2401_08671_amd.ceilings        # prints one JSON object
"""
from __future__ import annotations

import ctypes as C
import json
import sys

import torch

from . import fsf


def _mfma_fn(L, shape: int):
    fn = L.fsf_ceiling_mfma_bf16 if shape == 32 else L.fsf_ceiling_mfma_bf16_16x16x32
    fn.restype = C.c_int
    fn.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    return fn


def mfma_probe(device="cuda", iters: int = 20_000, seed: int = 11, shape: int = 32):
    """A short run of the register-resident bf16 MFMA loop (32x32x16, or 16x16x32 with shape=16) on
    normally distributed operands: ``{"TFLOPs", "shader_clock_MHz"}`` as the device holds them right now."""
    L = fsf.lib()
    n = 16 << 20
    g = torch.Generator(device=device).manual_seed(seed)
    ops = torch.randn(n // 2, generator=g, device=device).to(torch.bfloat16)
    scratch = torch.zeros(4096, dtype=torch.uint8, device=device)
    tf, mhz = C.c_double(0), C.c_double(0)
    fsf._check(_mfma_fn(L, shape)(ops.data_ptr(), n, iters, scratch.data_ptr(), C.byref(tf), C.byref(mhz),
                                  C.c_void_p(torch.cuda.current_stream().cuda_stream)), "fsf_ceiling_mfma_bf16")
    return {"TFLOPs": tf.value, "shader_clock_MHz": mhz.value}


def measure(device="cuda", hbm_bytes: int = 8 << 30, mfma_iters: int = 200_000):
    L = fsf.lib()
    L.fsf_ceiling_hbm_read.restype = C.c_int
    L.fsf_ceiling_hbm_read.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    scratch = torch.zeros(4096, dtype=torch.uint8, device=device)
    out = {}
    n = 16 << 20
    g = torch.Generator(device=device).manual_seed(11)
    for name, ops in (("ones", torch.ones(n // 2, dtype=torch.bfloat16, device=device)),
                      ("normal", torch.randn(n // 2, generator=g, device=device).to(torch.bfloat16))):
        tf, mhz = C.c_double(0), C.c_double(0)
        for shape, tag in ((32, ""), (16, "_16x16x32")):
            fsf._check(_mfma_fn(L, shape)(ops.data_ptr(), n, mfma_iters, scratch.data_ptr(),
                                          C.byref(tf), C.byref(mhz), stream), "fsf_ceiling_mfma_bf16")
            out[f"mfma_bf16{tag}_{name}_operands"] = {"TFLOPs": tf.value, "shader_clock_MHz": mhz.value}
    buf = torch.empty(hbm_bytes, dtype=torch.uint8, device=device)
    buf.fill_(1)
    for name, nt in (("plain", 0), ("nontemporal", 1)):
        gbs = C.c_double(0)
        fsf._check(L.fsf_ceiling_hbm_read(buf.data_ptr(), hbm_bytes, nt, scratch.data_ptr(), C.byref(gbs), stream),
                   "fsf_ceiling_hbm_read")
        out[f"hbm_read_scattered_16KB_tiles_{name}_loads"] = {"GBs": gbs.value}
    del buf
    return out


def main():
    assert torch.cuda.is_available(), "needs a GPU"
    json.dump(measure(), sys.stdout)
    print()


if __name__ == "__main__":
    main()

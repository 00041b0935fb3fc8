"""The C-ABI library loads on a machine without a GPU and exports what include/fsf.h declares."""
import ctypes
import os
import re

import pytest

from paper_2401_08671_amd import fsf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "fsf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(fsf_[a-z_0-9]+)\s*\(", text)
    return sorted(set(names))


def test_header_declares_the_three_named_calls():
    names = declared_functions()
    for need in ("fsf_kv_append", "fsf_ragged_attention", "fsf_compose_batch"):
        assert need in names


def test_library_exports_every_declared_symbol():
    L = fsf.lib()
    for name in declared_functions():
        assert hasattr(L, name), f"{name} declared in fsf.h but not exported"


def test_struct_layouts_match_header():
    assert ctypes.sizeof(fsf.SeqDesc) == 16
    assert ctypes.sizeof(fsf.AttnCfg) == 40
    assert fsf.AttnCfg.num_blocks.offset == 32


def test_strerror_and_version():
    assert fsf.strerror(0) == "ok"
    assert "block" in fsf.strerror(fsf.FSF_ERR_NO_BLOCKS)
    assert fsf.version() >= 100


def test_argument_validation_without_gpu():
    """Validation happens on the host before anything is launched."""
    L = fsf.lib()
    cfg = fsf.make_cfg(4, 3, 64, 16, "f32", 8)          # 3 does not divide 4
    st = L.fsf_kv_append(ctypes.byref(cfg), None, None, None, None, None, None, 1, 1, 1, None)
    assert st == fsf.FSF_ERR_INVALID_ARG
    assert L.fsf_ragged_attention_workspace_bytes(ctypes.byref(cfg), 1, 1, 1) == 0
    cfg = fsf.make_cfg(4, 4, 64, 16, "f32", 8)
    assert L.fsf_ragged_attention_workspace_bytes(ctypes.byref(cfg), 4, 194, 40) > 0
    # empty pass is a no-op, null pointers allowed
    assert L.fsf_kv_append(ctypes.byref(cfg), None, None, None, None, None, None, 0, 1, 0, None) == fsf.FSF_OK
    # null tensors with work to do
    st = L.fsf_ragged_attention(ctypes.byref(cfg), None, None, None, None, None, None, 1, 1, 1, None, None, 0, None)
    assert st == fsf.FSF_ERR_INVALID_ARG


def test_rotary_append_validation_without_gpu():
    """fsf_kv_append_rotary checks shapes, descriptors and the table length on the host and
    launches nothing when they are wrong (the device pointers here are never dereferenced)."""
    import numpy as np
    L = fsf.lib()
    fake = ctypes.c_void_p(0x1000)      # stands in for device memory; validation fails before any launch
    descs = np.array([[4, 0, 0, 0], [1, 9, 4, 1]], np.int32)
    host = ctypes.c_void_p(descs.ctypes.data)

    def call(cfg, table_positions, n_tokens=5, descs_host=host):
        return L.fsf_kv_append_rotary(ctypes.byref(cfg), fake, fake, fake, fake, fake, descs_host, fake,
                                      2, 4, n_tokens, fake, table_positions, None)
    cfg = fsf.make_cfg(2, 2, 64, 16, "f32", 8)
    assert call(cfg, 9) == fsf.FSF_ERR_INVALID_ARG            # position 9 needs a tenth table row
    assert call(cfg, -1) == fsf.FSF_ERR_INVALID_ARG
    assert call(cfg, 10, n_tokens=6) == fsf.FSF_ERR_INVALID_ARG   # descriptors do not add up to n_tokens
    assert call(cfg, 10, descs_host=None) == fsf.FSF_ERR_INVALID_ARG
    odd = fsf.make_cfg(2, 2, 63, 16, "f32", 8)
    assert call(odd, 10) in (fsf.FSF_ERR_UNSUPPORTED, fsf.FSF_ERR_INVALID_ARG)
    # an empty pass is a no-op whatever the pointers
    assert L.fsf_kv_append_rotary(ctypes.byref(cfg), None, None, None, None, None, None, None, 0, 1, 0, None, 0, None) == fsf.FSF_OK

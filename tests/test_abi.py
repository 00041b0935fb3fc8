"""The C-ABI library loads on a machine without a GPU and exports what include/fsf.h declares."""
import ctypes
import os
import re

import pytest

from paper_2401_08671_amd import fsf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


HEADERS = ("fsf.h", "fsf_measure.h")


def declared_functions(headers=HEADERS):
    names = set()
    for h in headers:
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(fsf_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_three_named_calls():
    names = declared_functions()
    for need in ("fsf_kv_append", "fsf_ragged_attention", "fsf_compose_batch"):
        assert need in names


def test_library_exports_every_declared_symbol():
    L = fsf.lib()
    for name in declared_functions():
        assert hasattr(L, name), f"{name} declared in fsf.h but not exported"


def struct_fields(name):
    """Field names of a struct typedef in fsf.h, in order."""
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "fsf.h")).read(), flags=re.S)
    body = re.search(r"typedef struct \{([^}]*)\}\s*" + name + ";", text).group(1)
    return [re.findall(r"(\w+)\s*$", decl.strip())[0] for decl in body.split(";") if decl.strip()]


def test_struct_layouts_match_header():
    assert ctypes.sizeof(fsf.SeqDesc) == 16
    assert ctypes.sizeof(fsf.AttnCfg) == 48
    assert fsf.AttnCfg.num_blocks.offset == 32 and fsf.AttnCfg.tuning.offset == 40
    assert [f[0] for f in fsf.AttnCfg._fields_] == struct_fields("fsf_attn_cfg")
    # the tuning struct: int32 fields in the header's order, its own size in the first
    assert [f[0] for f in fsf.Tuning._fields_] == struct_fields("fsf_tuning")
    assert all(f[1] is ctypes.c_int32 for f in fsf.Tuning._fields_)
    assert ctypes.sizeof(fsf.Tuning) == 4 * len(fsf.Tuning._fields_)
    assert fsf.Tuning(compute_units=7).struct_bytes == ctypes.sizeof(fsf.Tuning)


def test_the_product_header_holds_no_measurement_aid_and_the_library_reads_no_environment():
    names = declared_functions(("fsf.h",))
    assert not [n for n in names if n.startswith(("fsf_profile", "fsf_ceiling", "fsf_plan_"))]
    csrc = os.path.join(ROOT, "paper_2401_08671_amd", "csrc")
    for f in os.listdir(csrc):
        if f.endswith((".hip", ".cpp", ".h")):
            assert "getenv" not in open(os.path.join(csrc, f)).read(), f


def test_tuning_bounds_the_workspace():
    """max_decode_items_extra and max_prefill_split_units size the partial-result areas."""
    big = fsf.make_cfg(32, 8, 128, 64, "bf16", 1000)
    small = fsf.make_cfg(32, 8, 128, 64, "bf16", 1000,
                         tuning=fsf.Tuning(max_decode_items_extra=256, max_prefill_split_units=32))
    nb, ns = (fsf.ragged_attention_workspace_bytes(c, 300, 2048, 70) for c in (big, small))
    assert 0 < ns < nb and ns < 32 << 20 < nb
    # a caller compiled against a shorter struct: the missing fields take their defaults
    short = fsf.Tuning(max_decode_items_extra=256, max_prefill_split_units=32)
    short.struct_bytes = 8
    assert fsf.ragged_attention_workspace_bytes(fsf.make_cfg(32, 8, 128, 64, "bf16", 1000, tuning=short), 300, 2048, 70) == nb


def test_validate_pass_finds_bad_descriptors_and_block_ids():
    import numpy as np
    cfg = fsf.make_cfg(4, 2, 64, 16, "f32", 10)
    descs = np.array([[20, 0, 0, 0], [1, 31, 20, 1], [3, 5, 21, 2]], np.int32)
    bt = np.array([[4, 7, -1], [0, 1, -1], [9, -1, -1]], np.int32)
    assert fsf.validate_pass(cfg, descs, bt) is None
    bad = bt.copy(); bad[1, 1] = 10                       # beyond the pool
    assert fsf.validate_pass(cfg, descs, bad) == (1, 1)
    bad = bt.copy(); bad[0, 1] = -1                       # a position without its block
    assert fsf.validate_pass(cfg, descs, bad) == (0, 1)
    bad = bt.copy(); bad[2, 0] = 7                        # one block in two sequences
    assert fsf.validate_pass(cfg, descs, bad) == (2, 0)
    bad = bt.copy(); bad[2, 1] = 99                       # unused entries are never looked at
    assert fsf.validate_pass(cfg, descs, bad) is None
    d2 = descs.copy(); d2[2, 2] = 22                      # q_offset is not the running sum
    assert fsf.validate_pass(cfg, d2, bt) == (2, -1)
    d2 = descs.copy(); d2[1, 1] = 48                      # needs a fourth table column
    assert fsf.validate_pass(cfg, d2, bt) == (1, -1)
    d2 = descs.copy(); d2[0, 0] = 0
    assert fsf.validate_pass(cfg, d2, bt)[0] == 0


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


def test_static_entry_point_refuses_on_the_host_what_does_not_fit_its_array():
    """The work tables of three million one-token sequences exceed 64 MiB: the call is refused
    before any device call (the device pointers here are never dereferenced)."""
    import numpy as np
    L = fsf.lib()
    n = 3_000_000
    cfg = fsf.make_cfg(64, 8, 128, 64, "bf16", n)
    descs = np.stack([np.ones(n), np.zeros(n), np.arange(n), np.arange(n)], axis=1).astype(np.int32)
    fake = ctypes.c_void_p(0x1000)
    st = L.fsf_ragged_attention_static(ctypes.byref(cfg), fake, fake, fake, fake, ctypes.c_void_p(descs.ctypes.data),
                                       fake, n, 1, n, fake, None)
    assert st == fsf.FSF_ERR_WORKSPACE
    # and argument validation comes first
    st = L.fsf_ragged_attention_static(ctypes.byref(cfg), None, fake, fake, fake, ctypes.c_void_p(descs.ctypes.data),
                                       fake, n, 1, n, fake, None)
    assert st == fsf.FSF_ERR_INVALID_ARG
    assert L.fsf_ragged_attention_static(ctypes.byref(cfg), None, None, None, None, None, None, 0, 1, 0, None, None) == fsf.FSF_OK


def test_linear_workspace_query_without_gpu():
    """few tokens and a narrow output are cut along k (workspace = parts x fp32 result); wide outputs,
    many tokens and shapes the kernel refuses are not (0 bytes)"""
    small = fsf.linear_workspace_bytes(64, 5120, 5120)
    assert small >= 2 * 64 * 5120 * 4 and small % 256 == 0 and small <= 8 * 64 * 5120 * 4 + 256
    assert fsf.linear_workspace_bytes(64, 5120, 13824) >= small
    assert fsf.linear_workspace_bytes(4096, 15360, 5120) == 0      # the tiles fill the chip by themselves
    assert fsf.linear_workspace_bytes(16, 27648, 5120) == 0
    assert fsf.linear_workspace_bytes(16, 5120, 256) == 0          # too few k-steps to cut
    assert fsf.linear_workspace_bytes(16, 100, 5120) == 0 and fsf.linear_workspace_bytes(0, 5120, 5120) == 0

"""ctypes binding of libfsf.so: same names as the C ABI, argument marshalling only.

Every step of the path runs in the library's kernels; torch is used for device memory
and the current stream.  There is no CPU fallback: if the library is missing, loading
raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("FSF_LIB_PATH", os.path.join(_HERE, "libfsf.so"))

FSF_OK, FSF_ERR_INVALID_ARG, FSF_ERR_UNSUPPORTED, FSF_ERR_WORKSPACE, FSF_ERR_NO_BLOCKS, FSF_ERR_HIP = 0, -1, -2, -3, -4, -5
FSF_F32, FSF_BF16, FSF_F16 = 0, 1, 2
FSF_FLAG_FORCE_GENERIC = 1
FSF_FLAG_FUSED_LAUNCH = 2
DTYPE_CODE = {"f32": FSF_F32, "bf16": FSF_BF16, "f16": FSF_F16,
              torch.float32: FSF_F32, torch.bfloat16: FSF_BF16, torch.float16: FSF_F16}


class SeqDesc(C.Structure):
    _fields_ = [("n_new", C.c_int32), ("n_cached", C.c_int32), ("q_offset", C.c_int32), ("seq_id", C.c_int32)]


class Tuning(C.Structure):
    """fsf_tuning: 0 = default for every field (see include/fsf.h)."""
    _fields_ = [("struct_bytes", C.c_int32), ("decode_target_waves", C.c_int32),
                ("decode_min_item_blocks", C.c_int32), ("decode_hold", C.c_int32),
                ("prefill_split", C.c_int32), ("compute_units", C.c_int32),
                ("max_decode_items_extra", C.c_int32), ("max_prefill_split_units", C.c_int32),
                ("overlap", C.c_int32), ("stream_chunk_slices", C.c_int32)]

    def __init__(self, **kw):
        super().__init__(**kw)
        self.struct_bytes = C.sizeof(Tuning)


class AttnCfg(C.Structure):
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("block_size", C.c_int32), ("window", C.c_int32), ("scale", C.c_float),
                ("dtype", C.c_int32), ("flags", C.c_int32), ("num_blocks", C.c_int64),
                ("tuning", C.POINTER(Tuning))]


class FsfError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} ({status})")


_lib = None


def lib() -> C.CDLL:
    """Load libfsf.so once.  Raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not built: run `python -m paper_2401_08671_amd.build`")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    cfgp, descp, i32p = C.POINTER(AttnCfg), C.c_void_p, C.c_void_p
    L.fsf_strerror.restype = C.c_char_p
    L.fsf_strerror.argtypes = [C.c_int]
    L.fsf_version.restype = C.c_int
    L.fsf_kv_append.restype = C.c_int
    L.fsf_kv_append.argtypes = [cfgp, vp, vp, vp, vp, descp, i32p, i32, i32, i32, vp]
    L.fsf_validate_pass.restype = C.c_int
    L.fsf_validate_pass.argtypes = [cfgp, vp, vp, i32, i32, i32, C.POINTER(i32), C.POINTER(i32)]
    L.fsf_kv_append_rotary.restype = C.c_int
    L.fsf_kv_append_rotary.argtypes = [cfgp, vp, vp, vp, vp, descp, descp, i32p, i32, i32, i32, vp, i32, vp]
    L.fsf_rotary_q.restype = C.c_int
    L.fsf_rotary_q.argtypes = [cfgp, vp, descp, descp, i32, i32, vp, i32, vp]
    L.fsf_linear.restype = C.c_int
    L.fsf_linear.argtypes = [i32, vp, vp, vp, i32, i32, i32, vp]
    L.fsf_ragged_attention_workspace_bytes.restype = sz
    L.fsf_ragged_attention_workspace_bytes.argtypes = [cfgp, i32, i32, i32]
    L.fsf_ragged_attention.restype = C.c_int
    L.fsf_ragged_attention.argtypes = [cfgp, vp, vp, vp, descp, descp, i32p, i32, i32, i32, vp, vp, sz, vp]
    L.fsf_ragged_attention_static.restype = C.c_int
    L.fsf_ragged_attention_static.argtypes = [cfgp, vp, vp, vp, descp, descp, i32p, i32, i32, i32, vp, vp]
    L.fsf_sched_create.restype = C.c_int
    L.fsf_sched_create.argtypes = [C.POINTER(vp), i32, i32, i32, i64, vp]
    L.fsf_sched_destroy.restype = None
    L.fsf_sched_destroy.argtypes = [vp]
    L.fsf_sched_set_exhaustion.restype = C.c_int
    L.fsf_sched_set_exhaustion.argtypes = [vp, i32]
    L.fsf_sched_preemptions.restype = C.c_int
    L.fsf_sched_preemptions.argtypes = [vp, C.POINTER(i64), C.POINTER(i64)]
    L.fsf_sched_add_request.restype = C.c_int
    L.fsf_sched_add_request.argtypes = [vp, i32, i32, i32]
    L.fsf_compose_batch.restype = C.c_int
    L.fsf_compose_batch.argtypes = [vp, vp, vp, i32, C.POINTER(i32), C.POINTER(i32), vp]
    L.fsf_sched_step_done.restype = C.c_int
    L.fsf_sched_step_done.argtypes = [vp]
    L.fsf_sched_free_blocks.restype = i64
    L.fsf_sched_free_blocks.argtypes = [vp]
    L.fsf_sched_live_seqs.restype = i32
    L.fsf_sched_live_seqs.argtypes = [vp]
    _lib = L
    return L


def strerror(status: int) -> str:
    return lib().fsf_strerror(status).decode()


def version() -> int:
    return lib().fsf_version()


def make_cfg(n_q_heads, n_kv_heads, head_dim, block_size, dtype, num_blocks, window=0, scale=None, flags=0,
             tuning: Tuning | None = None) -> AttnCfg:
    if scale is None:
        scale = head_dim ** -0.5
    cfg = AttnCfg(n_q_heads, n_kv_heads, head_dim, block_size, window, scale, DTYPE_CODE[dtype], flags, num_blocks)
    if tuning is not None:
        cfg.tuning = C.pointer(tuning)
        cfg._tuning_ref = tuning          # the struct must outlive the calls that read it
    return cfg


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status: int, where: str):
    if status != FSF_OK:
        raise FsfError(status, where)


class DeviceBatch:
    """Descriptors and block tables of one pass, on the host (numpy) and on the device."""

    def __init__(self, descs: np.ndarray, block_tables: np.ndarray, device="cuda"):
        self.descs_host = np.ascontiguousarray(descs, dtype=np.int32).reshape(-1, 4)
        self.bt_host = np.ascontiguousarray(block_tables, dtype=np.int32)
        self.n_seqs = self.descs_host.shape[0]
        self.max_blocks = self.bt_host.shape[1] if self.bt_host.ndim == 2 else 1
        self.n_tokens = int(self.descs_host[:, 0].sum()) if self.n_seqs else 0
        self.descs_dev = torch.from_numpy(self.descs_host).to(device)
        self.bt_dev = torch.from_numpy(self.bt_host).to(device)


def validate_pass(cfg: AttnCfg, descs: np.ndarray, block_tables: np.ndarray):
    """fsf_validate_pass on host arrays: None if the pass is sound, else (bad sequence, bad table column)."""
    d = np.ascontiguousarray(descs, dtype=np.int32).reshape(-1, 4)
    bt = np.ascontiguousarray(block_tables, dtype=np.int32)
    bs, bc = C.c_int32(-2), C.c_int32(-2)
    st = lib().fsf_validate_pass(C.byref(cfg), C.c_void_p(d.ctypes.data), C.c_void_p(bt.ctypes.data), len(d),
                                 bt.shape[1] if bt.ndim == 2 else 1, int(d[:, 0].sum()) if len(d) else 0,
                                 C.byref(bs), C.byref(bc))
    return None if st == FSF_OK else (bs.value, bc.value)


def kv_append(cfg: AttnCfg, k_new, v_new, k_cache, v_cache, batch: DeviceBatch) -> None:
    """fsf_kv_append on torch's current stream."""
    st = lib().fsf_kv_append(C.byref(cfg), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                             _ptr(batch.descs_dev), _ptr(batch.bt_dev), batch.n_seqs, batch.max_blocks,
                             batch.n_tokens, _stream())
    _check(st, "fsf_kv_append")


def kv_append_rotary(cfg: AttnCfg, k_new, v_new, k_cache, v_cache, batch: DeviceBatch, cos_sin) -> None:
    """fsf_kv_append_rotary on torch's current stream; ``cos_sin`` is a float32 device tensor
    [table_positions, head_dim / 2, 2]."""
    assert cos_sin.dtype == torch.float32 and cos_sin.is_contiguous() and cos_sin.dim() == 3
    assert cos_sin.shape[1] * 2 == cfg.head_dim and cos_sin.shape[2] == 2
    st = lib().fsf_kv_append_rotary(C.byref(cfg), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                                    _ptr(batch.descs_dev), C.c_void_p(batch.descs_host.ctypes.data),
                                    _ptr(batch.bt_dev), batch.n_seqs, batch.max_blocks, batch.n_tokens,
                                    _ptr(cos_sin), cos_sin.shape[0], _stream())
    _check(st, "fsf_kv_append_rotary")


def rotary_q(cfg: AttnCfg, q, batch: DeviceBatch, cos_sin) -> None:
    """fsf_rotary_q on torch's current stream: q is rotated in place."""
    assert cos_sin.dtype == torch.float32 and cos_sin.is_contiguous() and cos_sin.shape[1] * 2 == cfg.head_dim
    st = lib().fsf_rotary_q(C.byref(cfg), _ptr(q), _ptr(batch.descs_dev), C.c_void_p(batch.descs_host.ctypes.data),
                            batch.n_seqs, batch.n_tokens, _ptr(cos_sin), cos_sin.shape[0], _stream())
    _check(st, "fsf_rotary_q")


def linear_workspace_bytes(n_tokens: int, n_out: int, k: int) -> int:
    L = lib()
    L.fsf_linear_workspace_bytes.restype = C.c_size_t
    L.fsf_linear_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
    return int(L.fsf_linear_workspace_bytes(n_tokens, n_out, k))


def linear(x, w, y, workspace=None) -> None:
    """fsf_linear on torch's current stream: y[t, o] = sum_k x[t, k] w[o, k]; x [T, K], w [N, K], y [T, N].
    With ``workspace`` (a uint8 device tensor, see linear_workspace_bytes): fsf_linear_ws."""
    assert x.dim() == 2 and w.dim() == 2 and y.dim() == 2 and x.is_contiguous() and w.is_contiguous() and y.is_contiguous()
    assert x.shape[1] == w.shape[1] and y.shape == (x.shape[0], w.shape[0]) and x.dtype == w.dtype == y.dtype
    L = lib()
    if workspace is None:
        st = L.fsf_linear(DTYPE_CODE[x.dtype], _ptr(x), _ptr(w), _ptr(y), x.shape[0], w.shape[0], x.shape[1], _stream())
        _check(st, "fsf_linear")
        return
    L.fsf_linear_ws.restype = C.c_int
    L.fsf_linear_ws.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                C.c_void_p, C.c_size_t, C.c_void_p]
    st = L.fsf_linear_ws(DTYPE_CODE[x.dtype], _ptr(x), _ptr(w), _ptr(y), x.shape[0], w.shape[0], x.shape[1],
                         _ptr(workspace), workspace.numel() * workspace.element_size(), _stream())
    _check(st, "fsf_linear_ws")


def ragged_attention_workspace_bytes(cfg: AttnCfg, n_seqs: int, n_tokens: int, max_blocks: int) -> int:
    return int(lib().fsf_ragged_attention_workspace_bytes(C.byref(cfg), n_seqs, n_tokens, max_blocks))


def ragged_attention(cfg: AttnCfg, q, k_cache, v_cache, batch: DeviceBatch, out, workspace) -> None:
    """fsf_ragged_attention on torch's current stream; ``workspace`` is a uint8 device tensor."""
    st = lib().fsf_ragged_attention(C.byref(cfg), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(batch.descs_dev),
                                    C.c_void_p(batch.descs_host.ctypes.data), _ptr(batch.bt_dev), batch.n_seqs,
                                    batch.max_blocks, batch.n_tokens, _ptr(out), _ptr(workspace),
                                    0 if workspace is None else workspace.numel() * workspace.element_size(),
                                    _stream())
    _check(st, "fsf_ragged_attention")


def ragged_attention_static(cfg: AttnCfg, q, k_cache, v_cache, batch: DeviceBatch, out) -> None:
    """fsf_ragged_attention_static on torch's current stream: no workspace, nothing allocated."""
    st = lib().fsf_ragged_attention_static(C.byref(cfg), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(batch.descs_dev),
                                           C.c_void_p(batch.descs_host.ctypes.data), _ptr(batch.bt_dev), batch.n_seqs,
                                           batch.max_blocks, batch.n_tokens, _ptr(out), _stream())
    _check(st, "fsf_ragged_attention_static")


def alloc_workspace(cfg: AttnCfg, n_seqs: int, n_tokens: int, max_blocks: int, device="cuda") -> torch.Tensor:
    n = ragged_attention_workspace_bytes(cfg, n_seqs, n_tokens, max_blocks)
    if n == 0:
        raise FsfError(FSF_ERR_INVALID_ARG, "fsf_ragged_attention_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


FSF_POLICY_SPLITFUSE, FSF_POLICY_PROMPT_FIRST, FSF_POLICY_WHOLE_PROMPT_JOINS = 0, 1, 2
FSF_EXHAUST_STALL, FSF_EXHAUST_PREEMPT_NEWEST = 0, 1


class Scheduler:
    """fsf_sched_* / fsf_compose_batch (host only)."""

    def __init__(self, token_budget: int, max_seqs: int, block_size: int, num_blocks: int,
                 max_blocks: int, free_list_order=None):
        self._h = C.c_void_p()
        order = None
        if free_list_order is not None:
            order = np.ascontiguousarray(free_list_order, dtype=np.int32)
        st = lib().fsf_sched_create(C.byref(self._h), token_budget, max_seqs, block_size, num_blocks,
                                    None if order is None else C.c_void_p(order.ctypes.data))
        _check(st, "fsf_sched_create")
        self.max_seqs, self.max_blocks = max_seqs, max_blocks
        self._descs = np.zeros((max_seqs, 4), dtype=np.int32)
        self._tables = np.zeros((max_seqs, max_blocks), dtype=np.int32)
        self._emits = np.zeros(max_seqs, dtype=np.int32)

    def set_policy(self, policy: int) -> None:
        _check(lib().fsf_sched_set_policy(self._h, policy), "fsf_sched_set_policy")

    def set_exhaustion(self, mode: int) -> None:
        _check(lib().fsf_sched_set_exhaustion(self._h, mode), "fsf_sched_set_exhaustion")

    def preemptions(self):
        """(sequences restarted so far, cached tokens that discarded)"""
        n, tok = C.c_int64(0), C.c_int64(0)
        _check(lib().fsf_sched_preemptions(self._h, C.byref(n), C.byref(tok)), "fsf_sched_preemptions")
        return int(n.value), int(tok.value)

    def add_request(self, seq_id: int, prompt_len: int, max_new_tokens: int) -> None:
        _check(lib().fsf_sched_add_request(self._h, seq_id, prompt_len, max_new_tokens), "fsf_sched_add_request")

    def compose_batch(self):
        """Returns (descs [S,4], block_tables [S,max_blocks], emits [S]) as fresh numpy arrays."""
        ns, nt = C.c_int32(0), C.c_int32(0)
        st = lib().fsf_compose_batch(self._h, C.c_void_p(self._descs.ctypes.data),
                                     C.c_void_p(self._tables.ctypes.data), self.max_blocks,
                                     C.byref(ns), C.byref(nt), C.c_void_p(self._emits.ctypes.data))
        _check(st, "fsf_compose_batch")
        S = ns.value
        return self._descs[:S].copy(), self._tables[:S].copy(), self._emits[:S].copy()

    def step_done(self) -> None:
        _check(lib().fsf_sched_step_done(self._h), "fsf_sched_step_done")

    def free_blocks(self) -> int:
        return int(lib().fsf_sched_free_blocks(self._h))

    def live_seqs(self) -> int:
        return int(lib().fsf_sched_live_seqs(self._h))

    def close(self) -> None:
        if self._h:
            lib().fsf_sched_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def plan_prefill_groups(cfg, descs: np.ndarray, compute_units: int = 256) -> np.ndarray:
    """fsf_plan_prefill_groups: ``int32 [G, 4]`` rows ``(tile, part, n_parts, slab)`` in start order (host only)."""
    L = lib()
    L.fsf_plan_prefill_groups.restype = C.c_int32
    d = np.ascontiguousarray(descs, dtype=np.int32)
    n = L.fsf_plan_prefill_groups(C.byref(cfg), C.c_void_p(d.ctypes.data), len(d), compute_units, None, 0)
    if n < 0:
        raise FsfError(FSF_ERR_INVALID_ARG, "fsf_plan_prefill_groups")
    out = np.zeros((n, 4), dtype=np.int32)
    L.fsf_plan_prefill_groups(C.byref(cfg), C.c_void_p(d.ctypes.data), len(d), compute_units,
                              C.c_void_p(out.ctypes.data), n)
    return out


# ------------------------------------------------------------------ per-kernel timing aid
PHASES = ("append", "plan", "prefill", "decode", "merge", "generic", "fused", "linear")


def profile_enable(on: bool) -> None:
    L = lib()
    L.fsf_profile_enable.restype = C.c_int
    L.fsf_profile_enable.argtypes = [C.c_int]
    _check(L.fsf_profile_enable(1 if on else 0), "fsf_profile_enable")


def profile_read():
    """{phase: (total_ms, launches)} since the last read; waits for the recorded events."""
    L = lib()
    L.fsf_profile_read.restype = C.c_int
    L.fsf_profile_read.argtypes = [C.c_void_p, C.c_void_p]
    ms = (C.c_double * len(PHASES))()
    n = (C.c_int64 * len(PHASES))()
    _check(L.fsf_profile_read(C.cast(ms, C.c_void_p), C.cast(n, C.c_void_p)), "fsf_profile_read")
    return {name: (ms[i], n[i]) for i, name in enumerate(PHASES)}

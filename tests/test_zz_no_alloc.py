"""fsf_ragged_attention_static (the entry point that allocates nothing; its work tables and
partial results live in a fixed array inside the library) against fsf_ragged_attention.

Given the same limits on cut units, both entry points plan the same partition and launch the
same kernels, so their outputs must be equal bit for bit; the first call is also checked
against the fp64 oracle.  Two calls in a row share the array: the second, smaller pass must not
see anything the first one left there.
"""
import numpy as np
import pytest
import torch

from paper_2401_08671_amd import fsf
from paper_2401_08671_amd import workloads as wl
from tests.gpu_util import assert_outputs_close
from tests.helpers import Step

pytestmark = pytest.mark.gpu

# the limits the static entry point applies to a pass that fits its array
STATIC_LIMITS = dict(max_decode_items_extra=1024, max_prefill_split_units=64)


def run_both(spec, tuning_kw):
    """(out of fsf_ragged_attention, out of fsf_ragged_attention_static, oracle out) for one pass."""
    st = Step(spec, poison="nan")
    dev = "cuda"
    batch = fsf.DeviceBatch(st.descs, st.block_tables, dev)
    q = wl.from_numpy_storage(st.q, spec.dtype, dev)
    k_new = wl.from_numpy_storage(st.k_new, spec.dtype, dev)
    v_new = wl.from_numpy_storage(st.v_new, spec.dtype, dev)
    kc = wl.from_numpy_storage(st.k_cache0, spec.dtype, dev)
    vc = wl.from_numpy_storage(st.v_cache0, spec.dtype, dev)
    mk = lambda **kw: fsf.make_cfg(spec.n_q_heads, spec.n_kv_heads, spec.head_dim, spec.block_size, spec.dtype,
                                   st.num_blocks, window=spec.window, scale=spec.scale, tuning=fsf.Tuning(**kw))
    cfg_ws = mk(**tuning_kw, **STATIC_LIMITS)
    cfg_static = mk(**tuning_kw)
    fsf.kv_append(cfg_ws, k_new, v_new, kc, vc, batch)
    out_ws = torch.full_like(q, float("nan"))
    ws = fsf.alloc_workspace(cfg_ws, batch.n_seqs, batch.n_tokens, batch.max_blocks, dev)
    fsf.ragged_attention(cfg_ws, q, kc, vc, batch, out_ws, ws)
    out_static = torch.full_like(q, float("nan"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    fsf.ragged_attention_static(cfg_static, q, kc, vc, batch, out_static)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return out_ws, out_static, st.oracle()[2]


def test_static_entry_point_equals_the_workspace_one_on_two_calls_in_a_row():
    # first pass: generation rows and a short chunk cut into many units (partial results + merge), a
    # chunk whose tiles are cut along their keys, short rows, a second chunk; 8 query heads on 2 KV heads
    big = wl.BatchSpec("static-big", 8, 2, 128, 64, "bf16",
                       [(1, 9000), (700, 1500), (1, 63), (1, 64), (300, 2100), (1, 2500), (1, 0), (40, 3), (7, 6000)], seed=51)
    tune = dict(decode_target_waves=1 << 20, decode_min_item_blocks=2, compute_units=64)
    a, b, ref = run_both(big, tune)
    assert torch.equal(a, b), "first call differs from fsf_ragged_attention"
    assert_outputs_close(b.to(torch.float64).cpu().numpy(), ref, "bf16", "static entry point, first call")
    # second pass, smaller: fewer sequences, fewer units, another head grouping and a window
    small = wl.BatchSpec("static-small", 4, 4, 128, 64, "bf16", [(1, 3000), (260, 700), (1, 5), (3, 2000)], window=1000, seed=52)
    a, b, ref = run_both(small, tune)
    assert torch.equal(a, b), "second call differs from fsf_ragged_attention"
    assert_outputs_close(b.to(torch.float64).cpu().numpy(), ref, "bf16", "static entry point, second call")


def test_static_entry_point_serves_the_generic_kernel():
    spec = wl.config(1)                    # fp32, head_dim 64: generic kernel, no work tables
    a, b, ref = run_both(spec, {})
    assert torch.equal(a, b)
    assert_outputs_close(b.to(torch.float64).cpu().numpy(), ref, "f32", "static entry point, fp32")

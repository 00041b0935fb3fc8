"""HIP path vs the fp64 oracle, element by element, at sizes the oracle finishes in seconds.

KV cache contents: bit-exact.  Outputs: max-abs <= 2e-2 and mean-abs <= 2e-3 for bf16/f16
(the stated bar), max-abs <= 1e-4 and mean-abs <= 1e-5 for fp32.
"""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from paper_2401_08671_amd import fsf
from paper_2401_08671_amd import workloads as wl
from tests.gpu_util import assert_cache_bit_exact, assert_outputs_close, run_hip
from tests.helpers import Step

pytestmark = pytest.mark.gpu


def check_step(step, flags=0, what=""):
    kc_o, vc_o, out_o = step.oracle()
    kc_h, vc_h, out_h = run_hip(step, flags=flags)
    assert_cache_bit_exact(kc_h, kc_o, what + " K")
    assert_cache_bit_exact(vc_h, vc_o, what + " V")
    return assert_outputs_close(out_h, out_o, step.spec.dtype, what)


# ------------------------------------------------------------------ benchmark shape 1 (tiny fp32)
@pytest.mark.parametrize("poison", [None, "nan", "inf", "big"])
def test_config1_full_parity(poison):
    check_step(Step(wl.config(1), num_blocks=128, poison=poison), what=f"cfg1 poison={poison}")


def test_config1_chunking_replay_on_device():
    """384-token prompt as 128+64+192 vs one shot: same KV bits, outputs within tolerance of the oracle's one shot."""
    L, Hq, Hkv, d, B, nb = 384, 4, 4, 64, 16, 64
    q = wl.randn((L, Hq, d), "f32", 1.0, 41, "cuda")
    k = wl.randn((L, Hkv, d), "f32", 1.0, 42, "cuda")
    v = wl.randn((L, Hkv, d), "f32", 1.0, 43, "cuda")
    perm = np.random.default_rng(1).permutation(nb).astype(np.int32)
    bt = perm[:L // B][None, :]
    cfg = fsf.make_cfg(Hq, Hkv, d, B, "f32", nb)

    def run(chunks):
        kc = torch.zeros((nb, Hkv, B, d), device="cuda")
        vc = torch.zeros_like(kc)
        outs, c = [], 0
        for n in chunks:
            batch = fsf.DeviceBatch(np.array([[n, c, 0, 0]], np.int32), bt)
            out = torch.empty((n, Hq, d), device="cuda")
            ws = fsf.alloc_workspace(cfg, 1, n, bt.shape[1])
            fsf.kv_append(cfg, k[c:c + n].contiguous(), v[c:c + n].contiguous(), kc, vc, batch)
            fsf.ragged_attention(cfg, q[c:c + n].contiguous(), kc, vc, batch, out, ws)
            outs.append(out)
            c += n
        torch.cuda.synchronize()
        return torch.cat(outs).double().cpu().numpy(), kc.cpu().numpy(), vc.cpu().numpy()

    one, kc1, vc1 = run([L])
    split, kc3, vc3 = run([128, 64, 192])
    assert np.array_equal(kc1, kc3) and np.array_equal(vc1, vc3)
    # oracle one-shot
    kco = np.zeros((nb, Hkv, B, d), np.float32)
    vco = np.zeros_like(kco)
    descs = np.array([[L, 0, 0, 0]], np.int32)
    oa.kv_append(kco, vco, k.cpu().numpy(), v.cpu().numpy(), descs, bt, B)
    ref = oa.ragged_attention(q.cpu().numpy(), kco, vco, descs, bt, block_size=B, scale=d ** -0.5, dtype="f32")
    assert np.array_equal(kc1, kco) and np.array_equal(vc1, vco)
    assert_outputs_close(one, ref, "f32", "one shot")
    assert_outputs_close(split, ref, "f32", "128+64+192")


# ------------------------------------------------------------------ generic kernel, other shapes and dtypes
@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("shape", [
    # Hq, Hkv, d, B, window, seqs
    (4, 2, 32, 8, 0, [(9, 0), (5, 11), (1, 13), (1, 0), (70, 3)]),
    (8, 2, 128, 64, 50, [(33, 100), (1, 63), (1, 64), (1, 65), (130, 0)]),
    (3, 3, 80, 16, 0, [(17, 5), (1, 300)]),
    (2, 1, 256, 4, 7, [(6, 6), (1, 1)]),
])
def test_generic_kernel_shapes(dtype, shape):
    Hq, Hkv, d, B, W, seqs = shape
    spec = wl.BatchSpec("g", Hq, Hkv, d, B, dtype, seqs, window=W, seed=77)
    check_step(Step(spec, poison="nan"), flags=fsf.FSF_FLAG_FORCE_GENERIC, what=f"generic {dtype} {shape[:5]}")


def test_append_is_idempotent_and_leaves_other_slots():
    spec = wl.BatchSpec("app", 8, 8, 128, 64, "bf16", [(200, 0), (3, 61), (1, 63), (1, 64), (1, 1000)], seed=5)
    st = Step(spec, poison="nan")
    kc_o, vc_o, _ = st.oracle(seq_subset=[])
    kc_h, vc_h, _ = run_hip(st, repeat_append=3)
    assert_cache_bit_exact(kc_h, kc_o, "K")
    assert_cache_bit_exact(vc_h, vc_o, "V")


# ------------------------------------------------------------------ argument errors reported, nothing launched
def test_bad_descriptors_are_rejected():
    spec = wl.BatchSpec("bad", 2, 2, 64, 16, "f32", [(4, 0), (1, 9)], seed=1)
    st = Step(spec)
    cfg = fsf.make_cfg(2, 2, 64, 16, "f32", st.num_blocks)
    q = torch.zeros((5, 2, 64), device="cuda")
    kc = torch.zeros((st.num_blocks, 2, 16, 64), device="cuda")
    out = torch.zeros_like(q)
    ws = fsf.alloc_workspace(cfg, 2, 5, st.block_tables.shape[1])
    for mutate in ("n_new0", "offset", "blocks", "total"):
        descs = st.descs.copy()
        bt = st.block_tables
        if mutate == "n_new0":
            descs[1, 0] = 0
        elif mutate == "offset":
            descs[1, 2] = 3
        elif mutate == "blocks":
            descs[1, 1] = 16 * bt.shape[1]
        elif mutate == "total":
            descs[0, 0] = 3
            descs[1, 2] = 3
        batch = fsf.DeviceBatch(descs, bt)
        batch.n_tokens = 5
        with pytest.raises(fsf.FsfError) as ei:
            fsf.ragged_attention(cfg, q, kc, kc, batch, out, ws)
        assert ei.value.status == fsf.FSF_ERR_INVALID_ARG, mutate
    batch = fsf.DeviceBatch(st.descs, st.block_tables)
    with pytest.raises(fsf.FsfError) as ei:
        fsf.ragged_attention(cfg, q, kc, kc, batch, out, None)
    assert ei.value.status == fsf.FSF_ERR_WORKSPACE
    torch.cuda.synchronize()


def test_empty_pass_is_a_noop():
    cfg = fsf.make_cfg(2, 2, 64, 16, "f32", 4)
    batch = fsf.DeviceBatch(np.zeros((0, 4), np.int32), np.zeros((0, 1), np.int32))
    fsf.kv_append(cfg, None, None, None, None, batch)
    fsf.ragged_attention(cfg, None, None, None, batch, None, None)
    torch.cuda.synchronize()


# ------------------------------------------------------------------ append with the rotary rotation fused in
def run_rotary(step, cos_sin, with_attention=False):
    sp = step.spec
    cfg = fsf.make_cfg(sp.n_q_heads, sp.n_kv_heads, sp.head_dim, sp.block_size, sp.dtype, step.num_blocks,
                       window=sp.window, scale=sp.scale)
    batch = fsf.DeviceBatch(step.descs, step.block_tables, "cuda")
    k_new = wl.from_numpy_storage(step.k_new, sp.dtype, "cuda")
    v_new = wl.from_numpy_storage(step.v_new, sp.dtype, "cuda")
    kc = wl.from_numpy_storage(step.k_cache0, sp.dtype, "cuda")
    vc = wl.from_numpy_storage(step.v_cache0, sp.dtype, "cuda")
    table = torch.from_numpy(cos_sin).cuda()
    fsf.kv_append_rotary(cfg, k_new, v_new, kc, vc, batch, table)
    out64 = None
    if with_attention:
        q = wl.from_numpy_storage(step.q, sp.dtype, "cuda")
        out = torch.full_like(q, float("nan"))
        ws = fsf.alloc_workspace(cfg, batch.n_seqs, batch.n_tokens, batch.max_blocks, "cuda")
        fsf.ragged_attention(cfg, q, kc, vc, batch, out, ws)
        out64 = out.to(torch.float64).cpu().numpy()
    torch.cuda.synchronize()
    return wl.to_numpy_storage(kc), wl.to_numpy_storage(vc), out64


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("shape", [
    # Hq, Hkv, d, B, seqs
    (8, 2, 128, 64, [(300, 0), (70, 130), (1, 63), (1, 64), (1, 1000), (5, 59)]),
    (4, 4, 64, 16, [(33, 7), (1, 0), (1, 95)]),
    (6, 3, 80, 8, [(9, 0), (1, 13)]),
])
def test_rotary_append_is_bit_exact(dtype, shape):
    Hq, Hkv, d, B, seqs = shape
    spec = wl.BatchSpec("rot", Hq, Hkv, d, B, dtype, seqs, seed=91)
    st = Step(spec, poison="nan")
    n_pos = max(c + n for n, c in seqs)
    table = oa.rotary_table(n_pos, d)                       # exactly as many rows as positions in use
    kc_o, vc_o = st.k_cache0.copy(), st.v_cache0.copy()
    oa.kv_append_rotary(kc_o, vc_o, st.k_new, st.v_new, st.descs, st.block_tables, B, table, dtype)
    kc_h, vc_h, _ = run_rotary(st, table)
    assert_cache_bit_exact(kc_h, kc_o, f"rotary K {dtype} {shape[:4]}")
    assert_cache_bit_exact(vc_h, vc_o, f"rotary V {dtype} {shape[:4]}")


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
def test_rotary_q_is_bit_exact(dtype):
    spec = wl.BatchSpec("rotq", 6, 3, 128 if dtype != "f32" else 80, 16, dtype, [(40, 100), (1, 0), (1, 511), (7, 3)], seed=93)
    st = Step(spec)
    table = oa.rotary_table(512, spec.head_dim)
    want = oa.rotate_queries(st.q, st.descs, table, dtype)
    cfg = fsf.make_cfg(spec.n_q_heads, spec.n_kv_heads, spec.head_dim, 16, dtype, st.num_blocks)
    batch = fsf.DeviceBatch(st.descs, st.block_tables, "cuda")
    q = wl.from_numpy_storage(st.q, dtype, "cuda")
    fsf.rotary_q(cfg, q, batch, torch.from_numpy(table).cuda())
    torch.cuda.synchronize()
    assert_cache_bit_exact(wl.to_numpy_storage(q), want, f"rotated Q {dtype}")
    with pytest.raises(fsf.FsfError):
        fsf.rotary_q(cfg, q, batch, torch.from_numpy(oa.rotary_table(512 - 1, spec.head_dim)).cuda())   # position 511 missing


def test_rotary_append_then_attention_matches_the_oracle():
    spec = wl.BatchSpec("rot-attn", 8, 2, 128, 64, "bf16", [(257, 0), (1, 190), (40, 90)], seed=92)
    st = Step(spec)
    table = oa.rotary_table(512, 128)
    kc_o, vc_o = st.k_cache0.copy(), st.v_cache0.copy()
    oa.kv_append_rotary(kc_o, vc_o, st.k_new, st.v_new, st.descs, st.block_tables, 64, table, "bf16")
    ref = oa.ragged_attention(st.q, kc_o, vc_o, st.descs, st.block_tables, block_size=64, scale=spec.scale,
                              window=0, dtype="bf16")
    kc_h, vc_h, out = run_rotary(st, table, with_attention=True)
    assert_cache_bit_exact(kc_h, kc_o, "K")
    assert_outputs_close(out, ref, "bf16", "attention over the rotated cache")


def test_rotary_append_rejects_a_table_that_is_too_short():
    spec = wl.BatchSpec("rot-bad", 2, 2, 64, 16, "f32", [(4, 0), (1, 9)], seed=1)
    st = Step(spec)
    table = oa.rotary_table(9, 64)      # position 9 has no row
    with pytest.raises(fsf.FsfError) as ei:
        run_rotary(st, table)
    assert ei.value.status == fsf.FSF_ERR_INVALID_ARG

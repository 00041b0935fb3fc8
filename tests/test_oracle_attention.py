"""Pins for oracle/attention.py: what the paper and the mathematics fix.

The paper prints no worked numeric example for the attention step, so every pin here is
mathematical: brute force, closed forms, invariants, and a library routine for the
special case it covers.  Each is chosen so that a plausible mistake (dropped scale, wrong
causal offset, transposed operand, wrong head mapping, wrong block/slot index, window
off by one) fails at least one of them.
"""
import math

import numpy as np
import pytest
import torch

from oracle import attention as oa
from paper_2401_08671_amd import workloads as wl
from tests.helpers import Step


# ----------------------------------------------------------------------------- helpers
def brute_force(q, k_cache, v_cache, descs, bt, B, scale, window, Hq, Hkv):
    """Scalar loops, python floats, own block-table walk (written independently)."""
    T, _, d = q.shape
    g = Hq // Hkv
    out = np.zeros((T, Hq, d))
    for s in range(len(descs)):
        n, c, off = int(descs[s][0]), int(descs[s][1]), int(descs[s][2])
        for i in range(n):
            pos = c + i
            for h in range(Hq):
                logits, keys = [], []
                for j in range(pos + 1):
                    if window > 0 and pos - j >= window:
                        continue
                    blk, slot = int(bt[s][j // B]), j % B
                    acc = 0.0
                    for t in range(d):
                        acc += float(q[off + i, h, t]) * float(k_cache[blk, h // g, slot, t])
                    logits.append(acc * scale)
                    keys.append((blk, slot))
                mx = max(logits)
                ws = [math.exp(x - mx) for x in logits]
                z = sum(ws)
                for t in range(d):
                    acc = 0.0
                    for w, (blk, slot) in zip(ws, keys):
                        acc += w * float(v_cache[blk, h // g, slot, t])
                    out[off + i, h, t] = acc / z
    return out


def tiny_spec(seqs, Hq=2, Hkv=1, d=4, B=3, window=0, seed=5, dtype="f32"):
    return wl.BatchSpec("tiny", Hq, Hkv, d, B, dtype, seqs, window=window, seed=seed)


# ----------------------------------------------------------------------------- P2 brute force
@pytest.mark.parametrize("B", [1, 2, 3])
@pytest.mark.parametrize("window", [0, 1, 3])
@pytest.mark.parametrize("heads", [(1, 1), (2, 1), (4, 2)])
def test_brute_force_tiny(B, window, heads):
    Hq, Hkv = heads
    spec = tiny_spec([(5, 0), (3, 4), (1, 7), (1, 0), (2, 5)], Hq=Hq, Hkv=Hkv, d=3, B=B, window=window)
    st = Step(spec)
    kc, vc, out = st.oracle()
    ref = brute_force(st.q, kc, vc, st.descs, st.block_tables, B, spec.scale, window, Hq, Hkv)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-13)


def test_hand_computed_two_keys():
    """One head, d=1: q=1, keys 0 and ln(3), values 0 and 1 -> weights 1/4, 3/4."""
    B = 2
    k_cache = np.zeros((2, 1, B, 1), np.float32)
    v_cache = np.zeros((2, 1, B, 1), np.float32)
    descs = np.array([[2, 0, 0, 0]], np.int32)
    bt = np.array([[1, 0]], np.int32)
    k_new = np.array([[[0.0]], [[math.log(3.0)]]], np.float32)
    v_new = np.array([[[0.0]], [[1.0]]], np.float32)
    q = np.ones((2, 1, 1), np.float32)
    oa.kv_append(k_cache, v_cache, k_new, v_new, descs, bt, B)
    # block table says the first logical block is physical block 1
    assert v_cache[1, 0, 1, 0] == 1.0 and v_cache[0].sum() == 0.0
    out = oa.ragged_attention(q, k_cache, v_cache, descs, bt, block_size=B, scale=1.0, dtype="f32")
    assert out[0, 0, 0] == 0.0                       # first row sees only itself
    k1 = float(np.float32(math.log(3.0)))
    expect = math.exp(k1) / (1.0 + math.exp(k1))     # ~0.75
    assert abs(out[1, 0, 0] - expect) < 1e-15
    assert abs(out[1, 0, 0] - 0.75) < 1e-7


# ----------------------------------------------------------------------------- P1 chunking invariance
def _run_chunked(chunks, q_all, k_all, v_all, B, num_blocks, perm, scale, window):
    """Feed one prompt as the given chunk sizes; return outputs and the logical KV."""
    L, Hkv, d = k_all.shape
    nblk = -(-L // B)
    bt = np.full((1, nblk), -1, np.int32)
    bt[0, :nblk] = perm[:nblk]
    kc = np.zeros((num_blocks, Hkv, B, d), np.float32)
    vc = np.zeros_like(kc)
    outs, c = [], 0
    for n in chunks:
        descs = np.array([[n, c, 0, 0]], np.int32)
        oa.kv_append(kc, vc, k_all[c:c + n], v_all[c:c + n], descs, bt, B)
        outs.append(oa.ragged_attention(q_all[c:c + n], kc, vc, descs, bt, block_size=B,
                                        scale=scale, window=window, dtype="f32"))
        c += n
    assert c == L
    return np.concatenate(outs), kc, vc


@pytest.mark.parametrize("window", [0, 100])
def test_chunking_invariance_384(window):
    """A 384-token prompt gives the same outputs and cache as 128+64+192, random cuts, or one shot.

    This is the claim that makes SplitFuse legal (Sec. 3.2): splitting moves tokens between
    forward passes and changes nothing the model computes.
    """
    L, Hq, Hkv, d, B = 384, 4, 4, 64, 16
    rng = np.random.default_rng(11)
    q = rng.standard_normal((L, Hq, d)).astype(np.float32)
    k = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    v = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    perm = rng.permutation(64).astype(np.int32)
    scale = 1 / math.sqrt(d)
    one, kc1, vc1 = _run_chunked([L], q, k, v, B, 64, perm, scale, window)
    cuts = sorted(rng.choice(np.arange(1, L), size=6, replace=False).tolist())
    rand_chunks = [b - a for a, b in zip([0] + cuts, cuts + [L])]
    for chunks in ([128, 64, 192], rand_chunks, [1] * 40 + [L - 40]):
        o, kc, vc = _run_chunked(chunks, q, k, v, B, 64, perm, scale, window)
        # same dense per-row computation on the same history; only the library matmul's
        # summation order may differ with the operand shapes
        np.testing.assert_allclose(o, one, rtol=0, atol=1e-13, err_msg=str(chunks))
        assert np.array_equal(kc, kc1) and np.array_equal(vc, vc1)


# ----------------------------------------------------------------------------- P3 normalisation
def test_softmax_rows_sum_to_one_and_constant_v():
    rng = np.random.default_rng(3)
    n, c, Hq, Hkv, d = 7, 9, 4, 2, 8
    q = rng.standard_normal((n, Hq, d)) * 3
    k = rng.standard_normal((n + c, Hkv, d)) * 3
    for window in (0, 1, 5, 100):
        w = oa.softmax_weights(q, k, c, 0.7, window, Hq // Hkv)
        np.testing.assert_allclose(w.sum(axis=2), 1.0, rtol=0, atol=1e-15)
        vis = oa.visible_mask(n, c, window)
        assert np.all(w[:, ~vis] == 0.0)
        assert np.all(w[:, vis] > 0.0)
    const = np.tile(rng.standard_normal((1, Hkv, d)), (n + c, 1, 1))
    out = oa.attention_one_sequence(q, k, const, c, 0.7, 0)
    for hq in range(Hq):
        np.testing.assert_allclose(out[:, hq], np.tile(const[0, hq // 2], (n, 1)), rtol=0, atol=1e-14)


# ----------------------------------------------------------------------------- P4 block permutation
def test_block_table_permutation_invariance():
    spec = wl.BatchSpec("perm", 4, 2, 16, 4, "f32", [(9, 0), (5, 11), (1, 13), (1, 3)], window=6, seed=21)
    st = Step(spec)
    kc, vc, out = st.oracle()
    rng = np.random.default_rng(99)
    perm = rng.permutation(st.num_blocks)            # old physical id -> new physical id
    kc2, vc2 = np.empty_like(kc), np.empty_like(vc)
    kc2[perm], vc2[perm] = kc, vc
    bt2 = np.where(st.block_tables >= 0, perm[np.maximum(st.block_tables, 0)], -1).astype(np.int32)
    out2 = oa.ragged_attention(st.q, kc2, vc2, st.descs, bt2, block_size=4, scale=spec.scale,
                               window=6, dtype="f32")
    assert np.array_equal(out, out2)
    # and the append itself follows the table: appending into the permuted pool gives the permuted pool
    k0, v0 = np.empty_like(kc), np.empty_like(vc)
    k0[perm], v0[perm] = st.k_cache0, st.v_cache0
    oa.kv_append(k0, v0, st.k_new, st.v_new, st.descs, bt2, 4)
    assert np.array_equal(k0, kc2) and np.array_equal(v0, vc2)


# ----------------------------------------------------------------------------- P5 closed forms
def _dense(n, c, Hq, Hkv, d, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((n, Hq, d)), rng.standard_normal((n + c, Hkv, d)),
            rng.standard_normal((n + c, Hkv, d)))


def test_single_key_returns_its_value():
    q, k, v = _dense(1, 0, 2, 2, 8, 0)
    out = oa.attention_one_sequence(q, k, v, 0, 0.3)
    assert np.array_equal(out[0], v[0])


def test_zero_query_gives_running_mean():
    n, c, d = 6, 5, 4
    q, k, v = _dense(n, c, 2, 1, d, 1)
    q[:] = 0.0
    out = oa.attention_one_sequence(q, k, v, c, 1.0, 0)
    for i in range(n):
        np.testing.assert_allclose(out[i, 0], v[:c + i + 1, 0].mean(axis=0), atol=1e-15)
    W = 3
    out = oa.attention_one_sequence(q, k, v, c, 1.0, W)
    for i in range(n):
        p = c + i
        np.testing.assert_allclose(out[i, 1], v[p - W + 1:p + 1, 0].mean(axis=0), atol=1e-15)


def test_equal_keys_give_running_mean():
    n, c = 4, 3
    q, k, v = _dense(n, c, 1, 1, 4, 2)
    k[:] = k[0]
    out = oa.attention_one_sequence(q, k, v, c, 0.9, 0)
    for i in range(n):
        np.testing.assert_allclose(out[i, 0], v[:c + i + 1, 0].mean(axis=0), atol=1e-14)


def test_window_conventions():
    n, c = 5, 7
    q, k, v = _dense(n, c, 2, 2, 4, 3)
    full = oa.attention_one_sequence(q, k, v, c, 0.5, 0)
    # a window at least as long as the history is no window
    assert np.array_equal(oa.attention_one_sequence(q, k, v, c, 0.5, n + c), full)
    assert not np.array_equal(oa.attention_one_sequence(q, k, v, c, 0.5, n + c - 1), full)
    # window 1: a row sees only its own position
    w1 = oa.attention_one_sequence(q, k, v, c, 0.5, 1)
    assert np.array_equal(w1, v[c:c + n])
    # a window of W shows exactly W keys once the history is long enough
    vis = oa.visible_mask(n, c, 4)
    assert np.all(vis.sum(axis=1) == 4)
    assert vis[0, c] and vis[0, c - 3] and not vis[0, c - 4] and not vis[0, c + 1]


def test_dominant_key_selects_its_value():
    n, c, d = 1, 9, 4
    q, k, v = _dense(n, c, 1, 1, d, 4)
    k[:] = 0.0
    k[6, 0] = q[0, 0] * 1e3 / np.dot(q[0, 0], q[0, 0])      # logit 1000 for key 6 only
    out = oa.attention_one_sequence(q, k, v, c, 1.0, 0)
    np.testing.assert_allclose(out[0, 0], v[6, 0], atol=1e-300, rtol=1e-15)


def test_scale_is_applied_to_logits():
    q, k, v = _dense(3, 2, 1, 1, 4, 8)
    a = oa.attention_one_sequence(q, k, v, 2, 0.25)
    b = oa.attention_one_sequence(q * 0.25, k, v, 2, 1.0)
    np.testing.assert_allclose(a, b, atol=1e-15)
    assert not np.allclose(a, oa.attention_one_sequence(q, k, v, 2, 1.0))


# ----------------------------------------------------------------------------- P6 library routine
def test_matches_torch_sdpa_causal_uncached():
    n, H, d = 37, 3, 16
    q, k, v = _dense(n, 0, H, H, d, 6)
    out = oa.attention_one_sequence(q, k, v, 0, 1 / math.sqrt(d), 0)
    tq, tk, tv = (torch.from_numpy(x).permute(1, 0, 2)[None] for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)
    np.testing.assert_allclose(out, ref[0].permute(1, 0, 2).numpy(), rtol=0, atol=1e-13)


def test_matches_torch_sdpa_with_cached_prefix_mask():
    """Cached prefix: library attention with an explicit bottom-right-aligned causal mask."""
    n, c, H, d = 5, 12, 2, 8
    q, k, v = _dense(n, c, H, H, d, 7)
    out = oa.attention_one_sequence(q, k, v, c, 0.2, 0)
    mask = torch.ones(n, n + c, dtype=torch.bool).tril(diagonal=c)
    tq, tk, tv = (torch.from_numpy(x).permute(1, 0, 2)[None] for x in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=0.2)
    np.testing.assert_allclose(out, ref[0].permute(1, 0, 2).numpy(), rtol=0, atol=1e-13)


# ----------------------------------------------------------------------------- P7 GQA
def test_gqa_equals_repeated_kv_mha():
    n, c, Hq, Hkv, d = 4, 6, 8, 2, 8
    q, k, v = _dense(n, c, Hq, Hkv, d, 9)
    a = oa.attention_one_sequence(q, k, v, c, 0.4, 5)
    b = oa.attention_one_sequence(q, np.repeat(k, Hq // Hkv, axis=1), np.repeat(v, Hq // Hkv, axis=1), c, 0.4, 5)
    assert np.array_equal(a, b)
    # interleaved (wrong) mapping must differ
    wrong = oa.attention_one_sequence(q, np.tile(k, (1, Hq // Hkv, 1)), np.tile(v, (1, Hq // Hkv, 1)), c, 0.4, 5)
    assert not np.allclose(a, wrong)


# ----------------------------------------------------------------------------- P8 decode = last row
def test_decode_equals_last_row_of_prefill():
    c, Hq, Hkv, d = 21, 4, 2, 8
    q, k, v = _dense(c + 1, 0, Hq, Hkv, d, 10)
    full = oa.attention_one_sequence(q, k, v, 0, 0.3, 0)
    dec = oa.attention_one_sequence(q[c:], k, v, c, 0.3, 0)
    np.testing.assert_allclose(dec[0], full[c], rtol=0, atol=1e-15)


# ----------------------------------------------------------------------------- append / storage
def test_append_touches_only_addressed_slots():
    spec = wl.BatchSpec("app", 2, 2, 4, 4, "bf16", [(6, 0), (3, 5), (1, 9), (1, 4)], seed=31)
    st = Step(spec, poison="nan")
    kc, vc, _ = st.oracle()
    touched = np.zeros(kc.shape[:1] + kc.shape[2:3], bool)          # [block, slot]
    for s, (n, c) in enumerate(spec.seqs):
        for i in range(n):
            p = c + i
            blk, slot = st.block_tables[s, p // 4], p % 4
            touched[blk, slot] = True
            off = st.descs[s, 2]
            assert np.array_equal(kc[blk, :, slot], st.k_new[off + i])
            assert np.array_equal(vc[blk, :, slot], st.v_new[off + i])
    same = (kc == st.k_cache0).all(axis=(1, 3)) & (vc == st.v_cache0).all(axis=(1, 3))
    assert np.all(same[~touched])


def test_bf16_and_f16_conversion_exact():
    bits = np.array([0x0000, 0x3F80, 0xBF80, 0x4049, 0x0001, 0x7F7F, 0x8000], np.uint16)
    want = np.array([0.0, 1.0, -1.0, 3.140625, 2.0 ** -133, (2 - 2.0 ** -7) * 2.0 ** 127, -0.0])
    got = oa.to_f64(bits, "bf16")
    assert np.array_equal(got, want) and np.signbit(got[-1])
    t = torch.tensor([0.1, -2.5, 1e-3, 300.0]).to(torch.bfloat16)
    assert np.array_equal(oa.to_f64(wl.to_numpy_storage(t), "bf16"), t.double().numpy())
    h = np.array([0.1, -2.5, 65504.0], np.float16)
    assert np.array_equal(oa.to_f64(h, "f16"), h.astype(np.float64))


def test_config1_oracle_runs_and_is_finite_under_poison():
    st = Step(wl.config(1), num_blocks=128, poison="nan")
    _, _, out = st.oracle()
    assert out.shape == (194, 4, 64) and np.isfinite(out).all()


# ---------------------------------------------------------------------------------------
# rotary append
def test_f32_to_bf16_rounding_matches_torch_and_ties_go_to_even():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(200000) * np.exp(rng.uniform(-8, 8, 200000))).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oa.f32_to_storage(x, "bf16"), want)
    # exact ties: 1 + 2^-8 (between 1 and 1 + 2^-7) -> even mantissa 1.0; 1 + 3 * 2^-8 -> 1 + 2^-6
    ties = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8], dtype=np.float32)
    assert oa.f32_to_storage(ties, "bf16").tolist() == [0x3F80, 0x3F82]


def test_f32_to_f16_rounding_matches_torch_ties_go_to_even_and_small_values_go_subnormal():
    rng = np.random.default_rng(4)
    x = (rng.standard_normal(200000) * np.exp(rng.uniform(-14, 9, 200000))).astype(np.float32)
    x = x[np.abs(x) < 65504.0]               # the kernels never produce values beyond the f16 range
    want = torch.from_numpy(x).to(torch.float16).numpy()
    got = oa.f32_to_storage(x, "f16")
    assert got.dtype == np.float16 and np.array_equal(got.view(np.uint16), want.view(np.uint16))
    # exact ties (f16 keeps 10 mantissa bits): 1 + 2^-11 lies between 1 and 1 + 2^-10 -> the even
    # mantissa 1.0 (0x3C00); 1 + 3 * 2^-11 between 1 + 2^-10 and 1 + 2^-9 -> 1 + 2^-9 (0x3C02)
    ties = np.array([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, -(1.0 + 2.0 ** -11)], dtype=np.float32)
    assert oa.f32_to_storage(ties, "f16").view(np.uint16).tolist() == [0x3C00, 0x3C02, 0xBC00]
    # just above a tie rounds up; subnormal range: 2^-24 is the smallest f16, half of it ties to zero
    more = np.array([1.0 + 2.0 ** -11 + 2.0 ** -20, 2.0 ** -24, 2.0 ** -25, 3 * 2.0 ** -25], dtype=np.float32)
    assert oa.f32_to_storage(more, "f16").view(np.uint16).tolist() == [0x3C01, 0x0001, 0x0000, 0x0002]


def test_rotary_table_and_rotation_closed_forms():
    tab = oa.rotary_table(64, 8, theta=10000.0)
    assert tab.shape == (64, 4, 2) and np.all(tab[0, :, 0] == 1.0) and np.all(tab[0, :, 1] == 0.0)
    assert tab[5, 0, 0] == np.float32(np.cos(5.0)) and tab[5, 1, 1] == np.float32(np.sin(5.0 * 10000.0 ** (-2 / 8)))
    k = np.random.default_rng(1).standard_normal((3, 8)).astype(np.float32)
    # position 0 is the identity, bit for bit
    assert np.array_equal(oa.rotate_row(k, tab[0], "f32"), k)
    # a rotation: every pair (i, i + d/2) keeps its length, and the result matches the
    # complex-number form computed in float64
    r = oa.rotate_row(k, tab[7], "f32").astype(np.float64)
    z = (k[:, :4] + 1j * k[:, 4:]) * (tab[7, :, 0] + 1j * tab[7, :, 1]).astype(np.complex128)[None, :]
    assert np.allclose(r[:, :4], z.real, atol=1e-6) and np.allclose(r[:, 4:], z.imag, atol=1e-6)
    assert np.allclose(r[:, :4] ** 2 + r[:, 4:] ** 2, k[:, :4].astype(np.float64) ** 2 + k[:, 4:] ** 2, rtol=1e-6)
    # dot products depend on the position difference only (what the embedding is for)
    q = np.random.default_rng(2).standard_normal((1, 8)).astype(np.float32)
    d1 = (oa.rotate_row(q, tab[20], "f32").astype(np.float64) * oa.rotate_row(k[:1], tab[13], "f32")).sum()
    d2 = (oa.rotate_row(q, tab[37], "f32").astype(np.float64) * oa.rotate_row(k[:1], tab[30], "f32")).sum()
    assert abs(d1 - d2) < 1e-5


def test_rotary_append_touches_k_only_and_only_addressed_slots():
    rng = np.random.default_rng(4)
    B, H, d = 4, 2, 8
    k_cache = np.full((6, H, B, d), 7, dtype=np.float32)
    v_cache = np.full((6, H, B, d), 9, dtype=np.float32)
    k_new = rng.standard_normal((5, H, d)).astype(np.float32)
    v_new = rng.standard_normal((5, H, d)).astype(np.float32)
    descs = np.array([[3, 2, 0, 0], [2, 0, 3, 1]], dtype=np.int32)
    tables = np.array([[4, 1], [0, -1]], dtype=np.int32)
    tab = oa.rotary_table(16, d)
    oa.kv_append_rotary(k_cache, v_cache, k_new, v_new, descs, tables, B, tab, "f32")
    # sequence 0: positions 2, 3 -> block 4 slots 2, 3; position 4 -> block 1 slot 0
    assert np.array_equal(v_cache[4, :, 2], v_new[0]) and np.array_equal(v_cache[1, :, 0], v_new[2])
    assert np.array_equal(k_cache[4, :, 3], oa.rotate_row(k_new[1], tab[3], "f32"))
    assert np.array_equal(k_cache[0, :, 0], k_new[3])                 # position 0: identity
    touched = {(4, 2), (4, 3), (1, 0), (0, 0), (0, 1)}
    for blk in range(6):
        for slot in range(B):
            if (blk, slot) not in touched:
                assert np.all(k_cache[blk, :, slot] == 7) and np.all(v_cache[blk, :, slot] == 9)


def test_rotated_queries_and_keys_score_by_distance_only():
    """End to end through the two rotating functions: with the same content in every row, the score
    of query row i of a chunk against the key at cache position j depends on (n_cached + i) - j
    only - which pins the position each query row is rotated by to n_cached + i."""
    d, B = 64, 4
    rng = np.random.default_rng(3)
    q_row = rng.standard_normal((1, d)).astype(np.float32)
    k_row = rng.standard_normal((1, d)).astype(np.float32)
    table = oa.rotary_table(64, d)
    descs = np.array([[5, 7, 0, 0], [3, 20, 5, 1]], np.int32)        # positions 7..11 and 20..22
    q = np.repeat(q_row[None], 8, axis=0)                              # [T=8, 1, d]
    qr = oa.rotate_queries(q, descs, table, "f32")
    keys = np.stack([oa.rotate_row(k_row, table[j], "f32") for j in range(23)])     # key content at every position
    score = lambda t, j: float(qr[t, 0].astype(np.float64) @ keys[j, 0].astype(np.float64))
    pos = [7, 8, 9, 10, 11, 20, 21, 22]
    for dist in (0, 1, 5):
        vals = [score(t, pos[t] - dist) for t in range(8)]
        assert np.allclose(vals, vals[0], rtol=0, atol=2e-4), (dist, vals)
    assert abs(score(0, 7) - score(0, 6)) > 1e-3                       # and it does depend on the distance
    assert np.array_equal(oa.rotate_queries(q[:1], np.array([[1, 0, 0, 0]], np.int32), table, "f32"), q[:1])  # position 0

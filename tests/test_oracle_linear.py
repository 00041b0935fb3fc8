"""Pins for oracle/linear.py: what the definition y[t, o] = sum_k x[t, k] w[o, k] fixes.

Chosen so that a plausible mistake (transposed weight, wrong axis, a dropped or doubled term,
a conversion that is not exact) fails at least one of them.
"""
import numpy as np
import torch

from oracle import attention as oa
from oracle.linear import linear


def test_hand_worked_example_and_weight_orientation():
    # two tokens, k = 3, two output features; w[o] is the weight row of output o
    x = np.array([[1.0, 2.0, 3.0], [0.5, -1.0, 4.0]], np.float32)
    w = np.array([[1.0, 0.0, -1.0], [2.0, 2.0, 0.25]], np.float32)
    y = linear(x, w, "f32")
    assert y.tolist() == [[1 - 3, 2 + 4 + 0.75], [0.5 - 4, 1 - 2 + 1]]
    assert y.shape == (2, 2)
    # not square: n_out differs from k, so a transposed weight cannot even be multiplied
    w3 = np.arange(12, dtype=np.float32).reshape(4, 3)
    assert linear(x, w3, "f32").shape == (2, 4)


def test_brute_force_scalar_loops():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 7)).astype(np.float32)
    w = rng.standard_normal((3, 7)).astype(np.float32)
    want = np.zeros((5, 3))
    for t in range(5):
        for o in range(3):
            acc = 0.0
            for k in range(7):
                acc += float(x[t, k]) * float(w[o, k])
            want[t, o] = acc
    np.testing.assert_allclose(linear(x, w, "f32"), want, rtol=0, atol=1e-14)


def test_closed_forms():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((6, 8)).astype(np.float32)
    # identity weight returns the tokens; a one-hot row picks a column; a row of ones sums a token
    assert np.array_equal(linear(x, np.eye(8, dtype=np.float32), "f32"), x.astype(np.float64))
    pick = np.zeros((1, 8), np.float32)
    pick[0, 5] = 1.0
    assert np.array_equal(linear(x, pick, "f32")[:, 0], x[:, 5].astype(np.float64))
    np.testing.assert_allclose(linear(x, np.ones((1, 8), np.float32), "f32")[:, 0], x.astype(np.float64).sum(axis=1), atol=1e-14)
    # linear in both arguments
    w = rng.standard_normal((4, 8)).astype(np.float32)
    np.testing.assert_allclose(linear((2 * x).astype(np.float32), w, "f32"), 2 * linear(x, w, "f32"), atol=1e-13)
    wa = rng.integers(-8, 9, size=(4, 8)).astype(np.float32)        # small integers: their sum is exact in float32
    wb = rng.integers(-8, 9, size=(4, 8)).astype(np.float32)
    np.testing.assert_allclose(linear(x, wa, "f32") + linear(x, wb, "f32"), linear(x, wa + wb, "f32"), atol=1e-12)


def test_tokens_are_independent_and_storage_types_convert_exactly():
    rng = np.random.default_rng(2)
    xb = oa.f32_to_storage(rng.standard_normal((9, 16)).astype(np.float32), "bf16")
    wb = oa.f32_to_storage(rng.standard_normal((5, 16)).astype(np.float32), "bf16")
    y = linear(xb, wb, "bf16")
    # a pass of 9 tokens equals 9 passes of one token (what lets a prompt be split over passes)
    for t in range(9):
        assert np.array_equal(linear(xb[t:t + 1], wb, "bf16")[0], y[t])
    # against a library routine on the same values (torch float64 matmul)
    xt = torch.from_numpy(xb.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64)
    wt = torch.from_numpy(wb.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64)
    np.testing.assert_allclose(y, (xt @ wt.T).numpy(), rtol=0, atol=1e-13)
    xh = rng.standard_normal((3, 4)).astype(np.float16)
    wh = rng.standard_normal((2, 4)).astype(np.float16)
    np.testing.assert_allclose(linear(xh, wh, "f16"), xh.astype(np.float64) @ wh.astype(np.float64).T, atol=0)

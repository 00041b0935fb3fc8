"""The output comparison of the GPU tests can fail where it matters (CPU only).

The absolute tolerance (2e-2 / 2e-3) is larger than the outputs themselves on long rows and on
down-scaled values, so `assert_outputs_close` also bounds the error relative to the reference.
Here a deliberately wrong *reference* (the oracle run on a history with keys missing) and wrong
results (zeros, one lost split) are shown to be rejected at those sizes, and a model of the
device's rounding (softmax weights and result rounded to the storage type, everything else
exact) is shown to pass with room to spare.  Everything runs on the oracle and numpy.
"""
import numpy as np
import pytest

from oracle import attention as oa
from tests.gpu_util import LAST_MARGINS, assert_outputs_close


def bf16_round(x64: np.ndarray) -> np.ndarray:
    return oa.to_f64(oa.f32_to_storage(x64.astype(np.float32), "bf16"), "bf16")


def one_row(n_keys: int, mult: float, seed: int, heads: int = 2, d: int = 128):
    """q [1, H, d], k, v [n_keys, H, d] as bf16-exact float64 values."""
    rng = np.random.default_rng(seed)
    draw = lambda *shape: bf16_round(rng.standard_normal(shape) * mult)
    return draw(1, heads, d), draw(n_keys, heads, d), draw(n_keys, heads, d)


def device_model(q, k, v, scale, keep=None):
    """One generation row the way the kernels round: exact scores and weights, weights rounded to
    bf16 for the second product, their sum taken before the rounding, result rounded to bf16."""
    out = np.empty_like(q)
    for h in range(q.shape[1]):
        s = scale * (k[:, h, :] @ q[0, h, :])
        if keep is not None:
            s = np.where(keep, s, -np.inf)
        p = np.exp(s - s.max())
        out[0, h] = bf16_round((bf16_round(p) @ v[:, h, :]) / p.sum())
    return out


CASES = [("200 000 keys, N(0,1)", 200_000, 1.0), ("config-2 scale, 3000 keys", 3000, 1.0 / np.sqrt(128.0))]


@pytest.mark.parametrize("name,n_keys,mult", CASES)
def test_device_rounding_passes_and_outputs_are_below_the_absolute_tolerance(name, n_keys, mult):
    q, k, v = one_row(n_keys, mult, seed=1)
    scale = 1.0 / np.sqrt(128.0)
    ref = oa.attention_one_sequence(q, k, v, n_keys - 1, scale)
    assert np.abs(ref).max() < 2e-2, "the case is meant to lie below the absolute tolerance"
    assert_outputs_close(device_model(q, k, v, scale), ref, "bf16", name)
    # room against the relative bounds (2e-2 per row and head, 6e-3 per row)
    assert LAST_MARGINS["rel_max"] < 7e-3 and LAST_MARGINS["rel_mean"] < 3e-3, LAST_MARGINS


@pytest.mark.parametrize("name,n_keys,mult", CASES)
def test_a_reference_with_an_eighth_of_the_keys_missing_is_rejected(name, n_keys, mult):
    q, k, v = one_row(n_keys, mult, seed=2)
    scale = 1.0 / np.sqrt(128.0)
    good = device_model(q, k, v, scale)
    cut = n_keys - n_keys // 8                   # the wrong reference never saw the last eighth
    wrong_ref = oa.attention_one_sequence(q, k[:cut], v[:cut], cut - 1, scale)
    with pytest.raises(AssertionError):
        assert_outputs_close(good, wrong_ref, "bf16", name)


@pytest.mark.parametrize("name,n_keys,mult", CASES)
def test_wrong_results_are_rejected(name, n_keys, mult):
    q, k, v = one_row(n_keys, mult, seed=3)
    scale = 1.0 / np.sqrt(128.0)
    ref = oa.attention_one_sequence(q, k, v, n_keys - 1, scale)
    with pytest.raises(AssertionError):          # all zeros
        assert_outputs_close(np.zeros_like(ref), ref, "bf16", name)
    keep = np.ones(n_keys, bool)
    keep[n_keys // 2: n_keys // 2 + n_keys // 64] = False       # one lost unit of 64
    with pytest.raises(AssertionError):
        assert_outputs_close(device_model(q, k, v, scale, keep), ref, "bf16", name)
    doubled = device_model(q, np.concatenate([k, k[:n_keys // 64]]), np.concatenate([v, v[:n_keys // 64]]), scale)
    with pytest.raises(AssertionError):          # one unit counted twice
        assert_outputs_close(doubled, ref, "bf16", name)


def test_rows_the_oracle_was_not_asked_for_are_skipped_and_nan_results_rejected():
    rng = np.random.default_rng(4)
    ref = rng.standard_normal((3, 2, 8))
    got = ref.copy()
    ref[1] = np.nan
    got[1] = 123.0
    assert_outputs_close(got, ref, "f32", "skip")
    got[2, 0, 0] = np.nan
    with pytest.raises(AssertionError):
        assert_outputs_close(got, ref, "f32", "nan")

"""fsf_linear (the projections of a layer at the ragged batch's token count) against the fp64 oracle.

Tolerance, derived from the arithmetic: products of bf16 / f16 values are exact in fp32, the
matrix core accumulates in fp32 (relative error of a k-term sum about sqrt(k) * 2^-24 of the
terms' size, below 1e-5 of the row's rms for k <= 27648), and the result is rounded once to the
storage type, half an ulp: 2^-9 of the value for bf16, 2^-12 for f16.  Asserted per element:
|y - ref| <= 2^-8 |ref| + 1e-4 rms(ref row)   (bf16; f16: 2^-11 |ref| + 1e-4 rms).
"""
import numpy as np
import pytest
import torch

from oracle.linear import linear as oracle_linear
from paper_2401_08671_amd import fsf
from paper_2401_08671_amd import workloads as wl

pytestmark = pytest.mark.gpu

REL = {"bf16": 2.0 ** -8, "f16": 2.0 ** -11}


def check(M, N, K, dtype, seed=0, w_mult=None, workspace_bytes=None):
    """workspace_bytes: None = fsf_linear; a number = fsf_linear_ws with a workspace of that size
    (-1: the size the library asks for)"""
    w_mult = K ** -0.5 if w_mult is None else w_mult
    x = wl.randn((M, K), dtype, 1.0, 9000 + seed, "cuda")
    w = wl.randn((N, K), dtype, w_mult, 9100 + seed, "cuda")
    guard = 3
    y_all = torch.full((M + guard, N), float("nan"), dtype=x.dtype, device="cuda")
    y = y_all[:M]
    print(f"fsf_linear M={M} N={N} K={K} {dtype} workspace {workspace_bytes}", flush=True)
    ws = None
    if workspace_bytes is not None:
        nbytes = fsf.linear_workspace_bytes(M, N, K) if workspace_bytes < 0 else workspace_bytes
        ws = torch.full((max(nbytes, 16),), 0xFF, dtype=torch.uint8, device="cuda")   # NaN bit patterns
    fsf.linear(x, w, y, ws)
    torch.cuda.synchronize()
    assert bool(torch.isnan(y_all[M:]).all()), "rows past the last token were written"
    got = y.to(torch.float64).cpu().numpy()
    ref = oracle_linear(wl.to_numpy_storage(x), wl.to_numpy_storage(w), dtype)
    assert np.isfinite(got).all()
    rms = np.sqrt((ref ** 2).mean(axis=1, keepdims=True))
    bound = REL[dtype] * np.abs(ref) + 1e-4 * rms
    err = np.abs(got - ref)
    worst = float((err / bound).max())
    assert worst <= 1.0, f"M={M} N={N} K={K} {dtype}: error {worst:.2f} x the bound at {np.unravel_index((err / bound).argmax(), err.shape)}"
    return worst


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("M", [1, 7, 128, 129, 300, 1024, 1025, 1300])
def test_token_counts_across_tile_boundaries(M, dtype):
    check(M, 512, 256, dtype, seed=M)


@pytest.mark.parametrize("K", [64, 128, 192, 256, 320, 1024 + 64])
@pytest.mark.parametrize("M", [5, 1100])
def test_short_and_odd_contraction_lengths(M, K):
    """k-steps fewer than, equal to and just above the depth of the copy ring."""
    check(M, 256, K, "bf16", seed=K)


@pytest.mark.parametrize("M,N,K", [(2048, 5120, 5120), (333, 15360, 5120), (4096, 5120, 13824), (64, 27648, 5120)])
def test_layer_shapes_of_a_13b_model(M, N, K):
    """The projections of a Llama-2-13B-shaped layer (query/key/value, output, MLP down and gate+up)."""
    check(M, N, K, "bf16", seed=1)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("M,N,K", [(1, 5120, 5120), (64, 5120, 13824), (130, 5120, 5120), (256, 2560, 1024),
                                   (300, 5120, 5120), (700, 1024, 4096), (64, 15360, 5120), (2048, 5120, 5120)])
def test_k_cut_into_parts_with_a_workspace(M, N, K, dtype):
    """fsf_linear_ws: narrow outputs at few tokens are cut along k (every part's partial result must
    count: a lost or doubled part moves the result by O(1) of the bound), wide or tall products are
    not; a workspace that holds only two parts, or none, still gives the result."""
    if (M, N, K) in ((1, 5120, 5120), (64, 5120, 13824), (300, 5120, 5120), (700, 1024, 4096)):
        assert fsf.linear_workspace_bytes(M, N, K) >= 2 * M * N * 4, "this product is one the library cuts"
    if (M, N) == (2048, 5120):
        assert fsf.linear_workspace_bytes(M, N, K) == 0
    check(M, N, K, dtype, seed=3, workspace_bytes=-1)
    if dtype == "bf16":
        check(M, N, K, dtype, seed=4, workspace_bytes=2 * M * N * 4)
        check(M, N, K, dtype, seed=5, workspace_bytes=16)


@pytest.mark.parametrize("M,N,K", [(384, 27648, 512), (768, 15360, 1024), (700, 15360, 1024), (4000, 5120, 1024)])
def test_token_counts_that_take_the_192_row_tile(M, N, K):
    """Shapes for which the library's cost model prefers tiles of 192 x 256 (a ragged last tile among them)."""
    check(M, N, K, "bf16", seed=7)
    check(M, N, K, "f16", seed=8)


@pytest.mark.parametrize("seed", range(16))
def test_random_shapes(seed):
    """Seeded random token counts, widths and contraction lengths, with and without a workspace of any size."""
    rng = np.random.default_rng(4000 + seed)
    M = int(rng.choice([int(rng.integers(1, 40)), int(rng.integers(40, 300)), int(rng.integers(300, 1100)), int(rng.integers(1100, 2600))]))
    N = 256 * int(rng.choice([1, 2, 3, 5, 8, 20]))
    K = 64 * int(rng.choice([1, 2, 3, 5, 9, 16, 33, 80]))
    if M * N * K > 2e10:
        K = 64 * 5
    ws = [None, -1, 16, 2 * M * N * 4, 3 * M * N * 4 + 16][int(rng.integers(0, 5))]
    check(M, N, K, "bf16" if seed % 3 else "f16", seed=seed, workspace_bytes=ws)


def test_structured_operands_catch_index_mistakes():
    """x = one-hot rows, w = distinct small integers: y[t, o] = w[o, k(t)] exactly."""
    M, N, K = 300, 512, 192
    rng = np.random.default_rng(3)
    kk = rng.integers(0, K, size=M)
    x = torch.zeros((M, K), dtype=torch.bfloat16)
    x[torch.arange(M), torch.from_numpy(kk)] = 1.0
    w = torch.from_numpy(rng.integers(-120, 121, size=(N, K)).astype(np.float32)).to(torch.bfloat16)
    y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    fsf.linear(x.cuda(), w.cuda(), y)
    torch.cuda.synchronize()
    want = w.to(torch.float32)[:, torch.from_numpy(kk)].T
    assert torch.equal(y.cpu().to(torch.float32), want)


def test_unsupported_shapes_are_refused():
    x = torch.zeros((4, 48), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((256, 48), dtype=torch.bfloat16, device="cuda")
    y = torch.zeros((4, 256), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fsf.FsfError) as e:
        fsf.linear(x, w, y)                      # k is not a multiple of 64
    assert e.value.status == fsf.FSF_ERR_UNSUPPORTED
    x = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((100, 64), dtype=torch.bfloat16, device="cuda")
    y = torch.zeros((4, 100), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fsf.FsfError) as e:
        fsf.linear(x, w, y)                      # n_out is not a multiple of 256
    assert e.value.status == fsf.FSF_ERR_UNSUPPORTED

"""The rest of a decoder layer at the ragged-batch shape: how long the weight GEMMs of a forward
pass take as a function of the number of forward tokens, measured on the GPU.

This library contains the attention step of a pass only.  The paper's two observations about a
whole pass (Sec. 3.1) are about the other part: with few tokens the pass is bound by reading the
weights, with many by their flops, and the transition fixes a sensible token budget.  To put the
attention step in that context, and to give the scheduling simulator a measured duration for
the linear part instead of a model, this module times the layer's linear maps (QKV, output
projection, gated MLP) with random bf16 weights of a Llama-2-13B-shaped layer through the
library's own matrix-core kernel (fsf_linear) for a grid of token counts, and, as context only,
through the vendor GEMM library (torch.matmul: hipBLASLt).  The gate of the MLP (silu(a) * b, an
element-wise step) is a torch expression in both cases; it is not part of this library.

`measure_layer` runs a whole layer of a Dynamic SplitFuse pass in order: the three projections,
the rotation of Q and of K (this library: in place, and fused into the append), the ragged attention, the
output projection and the gated MLP, for a grid of token budgets; the budget's tokens are a fixed
number of generation rows plus one prompt chunk that fills the rest (Sec. 3.2).

    python -m paper_2401_08671_amd.layer_model            # the linear maps alone (both backends); one JSON object
    python -m paper_2401_08671_amd.layer_model --layer    # the whole layer with attention
    python -m paper_2401_08671_amd.layer_model --gemm T N K   # one linear map 12 times through either backend (for profilers)
"""
from __future__ import annotations

import bisect
import json
import sys

import torch

SHAPE_13B = dict(hidden=5120, n_heads=40, head_dim=128, mlp=13824, n_layers=40)
TOKEN_GRID = (1, 16, 32, 64, 96, 128, 192, 256, 384, 512, 768, 1024, 1536, 2048, 3072, 4096, 8192, 16384)


def layer_gemm_flops(shape=SHAPE_13B) -> int:
    """flops of the layer's GEMMs per token"""
    h, qkv, mlp = shape["hidden"], 3 * shape["n_heads"] * shape["head_dim"], shape["mlp"]
    return 2 * (h * qkv + h * h + h * 2 * mlp + mlp * h)


def layer_weight_bytes(shape=SHAPE_13B) -> int:
    return layer_gemm_flops(shape)  # 2 bytes per weight, 2 flops per weight and token


def _linear(backend: str, x: torch.Tensor, w: torch.Tensor) -> torch.Tensor:
    """y[t, o] = sum_k x[t, k] w[o, k] through fsf_linear ("fsf") or the vendor library ("vendor")."""
    if backend == "vendor":
        return x @ w.T
    from . import fsf
    y = torch.empty((x.shape[0], w.shape[0]), dtype=x.dtype, device=x.device)
    fsf.linear(x, w, y, _workspace(fsf.linear_workspace_bytes(x.shape[0], w.shape[0], x.shape[1]), x.device))
    return y


_WORKSPACE = {}


def _workspace(nbytes: int, device):
    """one scratch buffer per device for fsf_linear_ws's partial results, grown as needed (None: not needed)"""
    if nbytes == 0:
        return None
    ws = _WORKSPACE.get(str(device))
    if ws is None or ws.numel() < nbytes:
        ws = _WORKSPACE[str(device)] = torch.empty(nbytes, dtype=torch.uint8, device=device)
    return ws


def _make_weights(shape, device, n_sets: int = 3, split_qkv: bool = False):
    """random bf16 weights [n_out, k] of n_sets layers (cycled, so that a pass never finds its weights in cache)"""
    h, mlp = shape["hidden"], shape["mlp"]
    qkv = 3 * shape["n_heads"] * shape["head_dim"]
    g = torch.Generator(device=device).manual_seed(5)
    mk = lambda *s: (torch.randn(*s, generator=g, device=device, dtype=torch.float32) * 0.02).to(torch.bfloat16)
    sets = []
    for _ in range(n_sets):
        w = dict(wo=mk(h, h), wgu=mk(2 * mlp, h), wd=mk(h, mlp))
        if split_qkv:
            w.update(wq=mk(h, h), wk=mk(h, h), wv=mk(h, h))
        else:
            w.update(wqkv=mk(qkv, h))
        sets.append(w)
    return sets, mk


def measure_linear(shape=SHAPE_13B, grid=TOKEN_GRID, reps: int = 5, device="cuda", backend: str = "fsf"):
    """[(tokens, seconds for the linear maps of ONE layer)], fastest of reps"""
    h, mlp = shape["hidden"], shape["mlp"]
    layers, mk = _make_weights(shape, device)
    out = []
    for T in grid:
        x = mk(T, h)
        best = float("inf")
        for r in range(reps + 2):
            w = layers[r % 3]
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            a = _linear(backend, x, w["wqkv"])
            b = _linear(backend, a[:, :h].contiguous(), w["wo"])
            c = _linear(backend, b, w["wgu"])
            d = _linear(backend, torch.nn.functional.silu(c[:, :mlp]) * c[:, mlp:], w["wd"])
            e1.record()
            torch.cuda.synchronize()
            if r >= 2:
                best = min(best, e0.elapsed_time(e1) * 1e-3)
        del a, b, c, d
        out.append((T, best))
    return out


def measure_layer(budgets=(128, 256, 512, 1024, 2048, 4096, 8192), n_generations: int = 64, context: int = 2048,
                  shape=SHAPE_13B, reps: int = 5, device="cuda", backend: str = "fsf"):
    """One Llama-2-13B-shaped layer of a SplitFuse pass per token budget: n_generations generation
    rows over `context` cached tokens plus one chunk of the remaining tokens of a prompt that has
    `context` tokens cached already.  Returns rows of dict(budget, layer_ms, gemm_ms, attention_ms)."""
    from . import fsf
    from . import workloads as wl
    from .harness import DeviceStep
    h, H, d, mlp = shape["hidden"], shape["n_heads"], shape["head_dim"], shape["mlp"]
    layers, mk = _make_weights(shape, device, split_qkv=True)
    n_pos = context + max(budgets) + 1
    # the caller of the rotary calls supplies the angle table; its values do not affect any timing,
    # so this measurement uses the identity rotation (cos 1, sin 0) at every position
    cos_sin = torch.zeros((n_pos, d // 2, 2), dtype=torch.float32, device=device)
    cos_sin[..., 0] = 1.0
    rows = []
    for T in budgets:
        n_dec = min(n_generations, T // 2)
        spec = wl.BatchSpec(f"layer-{T}", H, H, d, 64, "bf16", [(1, context)] * n_dec + [(T - n_dec, context)], seed=7)
        ds = DeviceStep(spec)
        x = mk(T, h)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        best = None
        for r in range(reps + 2):
            w = layers[r % 3]
            ev[0].record()
            q = _linear(backend, x, w["wq"]).view(T, H, d)
            k = _linear(backend, x, w["wk"]).view(T, H, d)
            v = _linear(backend, x, w["wv"]).view(T, H, d)
            ev[1].record()
            fsf.rotary_q(ds.cfg, q, ds.batch, cos_sin)
            fsf.kv_append_rotary(ds.cfg, k, v, ds.k_cache, ds.v_cache, ds.batch, cos_sin)
            fsf.ragged_attention(ds.cfg, q, ds.k_cache, ds.v_cache, ds.batch, ds.out, ds.ws)
            ev[2].record()
            o = _linear(backend, ds.out.view(T, h), w["wo"])
            gu = _linear(backend, o, w["wgu"])
            y = _linear(backend, torch.nn.functional.silu(gu[:, :mlp]) * gu[:, mlp:], w["wd"])
            ev[3].record()
            torch.cuda.synchronize()
            t = [ev[i].elapsed_time(ev[i + 1]) for i in range(3)]
            if r >= 2 and (best is None or sum(t) < sum(best)):
                best = t
        del ds, y, gu, o, q, k, v
        rows.append(dict(budget=T, generation_rows=n_dec, chunk_rows=T - n_dec, layer_ms=sum(best),
                         gemm_ms=best[0] + best[2], attention_ms=best[1],
                         tokens_per_s_whole_model=T / (sum(best) * 1e-3 * shape["n_layers"])))
    return rows


class MeasuredLinear:
    """seconds of the linear part of a pass of n tokens: table of measure_linear, interpolated"""

    def __init__(self, table, n_layers: int):
        self.tokens = [t for t, _ in table]
        self.secs = [s for _, s in table]
        self.n_layers = n_layers

    def __call__(self, n_tokens: int) -> float:
        i = bisect.bisect_left(self.tokens, n_tokens)
        if i == 0:
            per_layer = self.secs[0]
        elif i == len(self.tokens):  # beyond the grid: flops-bound, scale the last point
            per_layer = self.secs[-1] * n_tokens / self.tokens[-1]
        else:
            t0, t1, s0, s1 = self.tokens[i - 1], self.tokens[i], self.secs[i - 1], self.secs[i]
            per_layer = s0 + (s1 - s0) * (n_tokens - t0) / (t1 - t0)
        return self.n_layers * per_layer


def run_one_gemm(T: int, N: int, K: int, reps: int = 12, device="cuda"):
    """y = x w^T for x [T, K], w [N, K], `reps` times through fsf_linear and through the vendor library."""
    g = torch.Generator(device=device).manual_seed(1)
    mk = lambda *s: (torch.randn(*s, generator=g, device=device, dtype=torch.float32) * 0.05).to(torch.bfloat16)
    ws, x = [mk(N, K) for _ in range(3)], mk(T, K)
    for backend in ("fsf", "vendor"):
        for i in range(reps):
            _linear(backend, x, ws[i % 3])
    torch.cuda.synchronize()


def main():
    assert torch.cuda.is_available(), "needs a GPU"
    if "--gemm" in sys.argv[1:]:
        i = sys.argv.index("--gemm")
        run_one_gemm(*(int(a) for a in sys.argv[i + 1:i + 4]))
        print("done")
        return
    if "--layer" in sys.argv[1:]:
        json.dump(dict(shape=SHAPE_13B, rows=measure_layer(), rows_vendor_gemm=measure_layer(backend="vendor")), sys.stdout)
        print()
        return
    fl, by = layer_gemm_flops(), layer_weight_bytes()
    out = dict(shape=SHAPE_13B, gemm_flops_per_token_per_layer=fl, weight_bytes_per_layer=by)
    for backend in ("fsf", "vendor"):
        table = measure_linear(backend=backend)
        out["rows_" + backend] = [dict(tokens=T, layer_ms=s * 1e3, tflops=T * fl / s / 1e12, weight_gbs=by / s / 1e9,
                                       tokens_per_s_whole_model=T / (s * SHAPE_13B["n_layers"])) for T, s in table]
    json.dump(out, sys.stdout)
    print()


if __name__ == "__main__":
    main()

"""The long-prompt SplitFuse stream (benchmark shape 5): 200 passes composed by fsf_compose_batch.

Every pass appends on the device AND, independently, on a host shadow of the pool through the
oracle's append (the oracle never sees device-produced cache contents).  On passes 0, 1, 50
and 199 sampled rows (first/last/tile-boundary/random rows of every prompt chunk, and a
sample of generation rows) are checked against the fp64 oracle; a chunk row i is evaluated as
a one-row pass with n_cached = c + i over the same history (oracle pin "decode = last prefill
row"), which avoids dense 4096 x 30000 score matrices.  After the last pass the whole device
pool must equal the host shadow bit for bit.
"""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from paper_2401_08671_amd import workloads as wl
from paper_2401_08671_amd.harness import StreamRunner
from tests.gpu_util import assert_outputs_close

pytestmark = pytest.mark.gpu

CHECK_STEPS = (0, 1, 50, 199)


def sample_rows(descs, rng):
    """[(seq index, row i)] to check in this pass."""
    picks = []
    dec = [s for s in range(len(descs)) if descs[s][0] == 1]
    for s in (rng.choice(dec, size=min(24, len(dec)), replace=False).tolist() if dec else []):
        picks.append((s, 0))
    for s in range(len(descs)):
        n = int(descs[s][0])
        if n == 1:
            continue
        rows = {0, n - 1, min(n - 1, 127), min(n - 1, 128), n // 2}
        rows |= set(rng.integers(0, n, size=6).tolist())
        picks += [(s, i) for i in sorted(rows)]
    return picks


def test_stream_200_passes():
    run = StreamRunner(n_steps=200, rate=1.0)
    B = run.B
    shape = (run.num_blocks, run.Hkv, B, run.d)
    k_host = np.zeros(shape, np.uint16)
    v_host = np.zeros(shape, np.uint16)
    rng = np.random.default_rng(7)
    total_tokens = 0
    checked = 0
    worst = 0.0
    for step in range(200):
        descs, tables, emits = run.compose()
        T = int(descs[:, 0].sum()) if len(descs) else 0
        total_tokens += T
        assert T <= run.budget
        q, k_new, v_new = run.new_tokens(step, T)
        out = run.run_pass(descs, tables, q, k_new, v_new)
        kn, vn = wl.to_numpy_storage(k_new), wl.to_numpy_storage(v_new)
        oa.kv_append(k_host, v_host, kn, vn, descs, tables, B)              # host shadow, oracle code only
        if step in CHECK_STEPS and T:
            torch.cuda.synchronize()
            got = out.to(torch.float64).cpu().numpy()
            qn = wl.to_numpy_storage(q)
            for s, i in sample_rows(descs, rng):
                n, c, off, _ = (int(x) for x in descs[s])
                one = np.array([[1, c + i, 0, 0]], np.int32)
                ref = oa.ragged_attention(qn[off + i:off + i + 1], k_host, v_host, one, tables[s:s + 1],
                                          block_size=B, scale=run.d ** -0.5, dtype=run.dtype)
                mx, _ = assert_outputs_close(got[off + i:off + i + 1], ref, run.dtype, f"pass {step} seq {s} row {i}")
                worst = max(worst, mx)
                checked += 1
            # cache blocks of this pass's sequences: device == host shadow, bit for bit
            used = np.unique(tables[tables >= 0])
            idx = torch.from_numpy(used.astype(np.int64)).cuda()
            assert np.array_equal(wl.to_numpy_storage(run.k_cache.index_select(0, idx)), k_host[used]), f"K pass {step}"
            assert np.array_equal(wl.to_numpy_storage(run.v_cache.index_select(0, idx)), v_host[used]), f"V pass {step}"
            print(f"pass {step}: {len(descs)} sequences, {T} tokens, rows checked so far {checked}, worst max-abs {worst:.2e}")
        run.commit()
    torch.cuda.synchronize()
    assert total_tokens > 100 * run.budget          # arrivals (about 2900 tokens per pass) keep most of the budget busy
    # whole pool after 200 passes
    for dev, host, name in ((run.k_cache, k_host, "K"), (run.v_cache, v_host, "V")):
        for b0 in range(0, run.num_blocks, 1024):
            assert np.array_equal(wl.to_numpy_storage(dev[b0:b0 + 1024]), host[b0:b0 + 1024]), f"{name} blocks {b0}.."
    print(f"stream: {total_tokens} tokens in 200 passes, {checked} rows checked, worst max-abs {worst:.2e}")


def test_tight_pool_with_restarts_every_pass_checked():
    """A small closed loop on a pool two blocks larger than the largest request, with the
    preempt-newest policy: sequences are restarted, their blocks go to other sequences still
    holding the previous owner's data, and restarted sequences are processed again from an empty
    cache.  Every pass is checked in full against the oracle, the cache bit for bit."""
    from paper_2401_08671_amd import fsf
    Hq, Hkv, d, B, budget = 4, 2, 128, 64, 256
    rng = np.random.default_rng(11)
    reqs = [(int(rng.integers(100, 600)), int(rng.integers(5, 30))) for _ in range(10)]
    largest = max(-(-(p + g) // B) for p, g in reqs)
    num_blocks = largest + 2
    sched = fsf.Scheduler(budget, 6, B, num_blocks, largest, rng.permutation(num_blocks))
    sched.set_exhaustion(fsf.FSF_EXHAUST_PREEMPT_NEWEST)
    cfg = fsf.make_cfg(Hq, Hkv, d, B, "bf16", num_blocks)
    kc = wl.from_numpy_storage(np.full((num_blocks, Hkv, B, d), 0x7FC0, np.uint16), "bf16", "cuda")   # NaN everywhere
    vc = kc.clone()
    k_host, v_host = wl.to_numpy_storage(kc).copy(), wl.to_numpy_storage(vc).copy()
    nxt, emitted, passes, worst = 0, [0] * len(reqs), 0, 0.0
    for _ in range(4):
        sched.add_request(nxt, *reqs[nxt])
        nxt += 1
    while sched.live_seqs() > 0:
        descs, tables, emits = sched.compose_batch()
        T = int(descs[:, 0].sum())
        assert 0 < T <= budget
        q = wl.randn((T, Hq, d), "bf16", 1.0, 5000 + 3 * passes, "cuda")
        k_new = wl.randn((T, Hkv, d), "bf16", 1.0, 5001 + 3 * passes, "cuda")
        v_new = wl.randn((T, Hkv, d), "bf16", 1.0, 5002 + 3 * passes, "cuda")
        batch = fsf.DeviceBatch(descs, tables, "cuda")
        out = torch.full_like(q, float("nan"))
        ws = fsf.alloc_workspace(cfg, batch.n_seqs, batch.n_tokens, batch.max_blocks, "cuda")
        fsf.kv_append(cfg, k_new, v_new, kc, vc, batch)
        fsf.ragged_attention(cfg, q, kc, vc, batch, out, ws)
        oa.kv_append(k_host, v_host, wl.to_numpy_storage(k_new), wl.to_numpy_storage(v_new), descs, tables, B)
        ref = oa.ragged_attention(wl.to_numpy_storage(q), k_host, v_host, descs, tables, block_size=B,
                                  scale=d ** -0.5, dtype="bf16")
        torch.cuda.synchronize()
        mx, _ = assert_outputs_close(out.to(torch.float64).cpu().numpy(), ref, "bf16", f"pass {passes}: {descs.tolist()}")
        worst = max(worst, mx)
        assert np.array_equal(wl.to_numpy_storage(kc), k_host) and np.array_equal(wl.to_numpy_storage(vc), v_host)
        for dsc, em in zip(descs, emits):
            emitted[int(dsc[3])] += int(em)
        sched.step_done()
        passes += 1
        assert passes < 2000
        while nxt < len(reqs) and sched.live_seqs() < 4:
            sched.add_request(nxt, *reqs[nxt])
            nxt += 1
    restarted, discarded = sched.preemptions()
    sched.close()
    assert emitted == [g for _, g in reqs]
    assert restarted > 0
    print(f"tight pool: {passes} passes, {restarted} restarts ({discarded} cached tokens recomputed), worst max-abs {worst:.2e}")

"""The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only).

`python -m paper_2401_08671_amd.build --sanitize` compiles the host side of libfsf.so (composer,
block allocator, the attention call's planning, workspace sizing and pass validation) with both
sanitizers and builds tests/native/host_check.cpp against it.  Here that program replays random
request streams; any sanitizer report makes it exit non-zero, and the schedules it prints must
equal the oracle composer's.
"""
import os
import subprocess

import numpy as np
import pytest

from oracle.composer import NoBlocksError, SplitFuseComposer
from paper_2401_08671_amd import build as fsf_build

POLICIES = ["splitfuse", "prompt_first", "whole_prompt_joins"]


@pytest.fixture(scope="module")
def host_check():
    if not os.path.exists(fsf_build.HOST_CHECK):
        fsf_build.build_sanitized(verbose=False)          # host tool; compiles in about 20 s
    return fsf_build.HOST_CHECK


def run_host_check(exe, budget, max_seqs, B, num_blocks, max_blocks, policy, exhaustion, reqs):
    text = f"{budget} {max_seqs} {B} {num_blocks} {max_blocks} {POLICIES.index(policy)} {1 if exhaustion == 'preempt_newest' else 0} {len(reqs)}\n"
    text += "".join(f"{p} {i} {l} {g}\n" for p, i, l, g in reqs)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], input=text, capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, f"host_check exit {r.returncode}\n{r.stderr[-4000:]}"
    passes, cur, end = [], None, None
    for ln in r.stdout.splitlines():
        f = ln.split()
        if f[0] == "P":
            cur = []
            passes.append(cur)
        elif f[0] == "S":
            cur.append(tuple(int(x) for x in f[1:5]) + (tuple(int(x) for x in f[5:]),))
        elif f[0] == "X":
            passes.append(None)                            # nothing could be scheduled
        elif f[0] == "E":
            end = tuple(int(x) for x in f[1:])
    return passes, end


def oracle_passes(budget, max_seqs, B, num_blocks, policy, exhaustion, reqs):
    ref = SplitFuseComposer(budget, max_seqs, B, num_blocks, None, policy=policy, exhaustion=exhaustion)
    passes, nxt, step = [], 0, 0
    while True:
        while nxt < len(reqs) and reqs[nxt][0] <= step:
            ref.add_request(*reqs[nxt][1:])
            nxt += 1
        if ref.n_live() == 0 and nxt == len(reqs):
            break
        try:
            descs, tables, emits = ref.compose()
        except NoBlocksError:
            passes.append(None)
            break
        passes.append([(d[3], d[0], d[1], e, tuple(t)) for d, t, e in zip(descs, tables, emits)])
        ref.step_done()
        step += 1
    return passes, ref


@pytest.mark.parametrize("policy", POLICIES)
@pytest.mark.parametrize("seed", range(4))
def test_random_streams_under_sanitizers_equal_the_oracle(host_check, seed, policy):
    rng = np.random.default_rng(4100 + seed)
    budget = int(rng.integers(8, 400))
    B = int(rng.choice([16, 32, 64]))
    max_seqs = int(rng.integers(2, 60))
    reqs, tot, largest = [], 0, 1
    for step in range(80):
        for _ in range(rng.poisson(0.5)):
            plen, gen = int(rng.integers(1, 6 * budget)), int(rng.integers(1, 40))
            reqs.append((step, len(reqs), plen, gen))
            tot += -(-(plen + gen) // B)
            largest = max(largest, -(-(plen + gen) // B))
    tight = seed % 2 == 1
    num_blocks = max(largest + 3, tot // 8) if tight else max(tot, 1)
    exhaustion = "preempt_newest" if tight else "stall"
    got, end = run_host_check(host_check, budget, max_seqs, B, num_blocks, largest, policy, exhaustion, reqs)
    want, ref = oracle_passes(budget, max_seqs, B, num_blocks, policy, exhaustion, reqs)
    assert len(got) == len(want)
    for k, (g, w) in enumerate(zip(got, want)):
        assert g == w, f"pass {k}"
    if want and want[-1] is not None:
        assert end == (len(want), ref.n_free_blocks(), ref.n_preemptions)


def test_long_prompt_stream_under_sanitizers(host_check):
    """The benchmark's long-prompt stream (log-normal prompts up to 32768 tokens, budget 4096)."""
    from paper_2401_08671_amd import workloads as wl
    reqs = [(step, sid, plen, gen) for step, sid, plen, gen in wl.stream_requests(60, 1.0, 1005)]
    need = sum(-(-(p + g) // 64) for _, _, p, g in reqs)
    got, end = run_host_check(host_check, 4096, 4096, 64, need + 64, -(-(32768 + 600) // 64), "splitfuse", "stall", reqs)
    want, ref = oracle_passes(4096, 4096, 64, need + 64, "splitfuse", "stall", reqs)
    assert got == want and end == (len(want), ref.n_free_blocks(), 0)

"""Pins for oracle/composer.py: the properties the paper states for Dynamic SplitFuse.

Sec. 3.2 rule 1: a prompt's chunks run over several passes, only the last one generates.
Sec. 3.2 rule 2: the token budget is met exactly whenever enough tokens are waiting.
Sec. 3.2 (closing paragraph) / Sec. 2.2: generation is never stalled behind prompts.
Sec. 2.1: storage is fixed-size blocks; no block belongs to two live sequences.
"""
import numpy as np
import pytest

from oracle.composer import NoBlocksError, SplitFuseComposer


def test_hand_worked_schedule():
    """Budget 8, block 4: prompts of 10 and 5 tokens, 3 new tokens each.

    pass 0: A[0:8]                      (8 tokens, no generation)
    pass 1: A[8:10] emits, B[0:5] emits, budget under-filled (7) because nothing else waits
    pass 2: decode A (c=10), decode B (c=5)
    pass 3: decode A (c=11), decode B (c=6)  -> both have emitted 3 tokens and retire
    """
    comp = SplitFuseComposer(8, 16, 4, 8)
    comp.add_request(100, 10, 3)
    comp.add_request(200, 5, 3)
    d, t, e = comp.compose()
    assert d == [(8, 0, 0, 100)] and t == [[0, 1]] and e == [0]
    comp.step_done()
    d, t, e = comp.compose()
    assert d == [(2, 8, 0, 100), (5, 0, 2, 200)] and t == [[0, 1, 2], [3, 4]] and e == [1, 1]
    comp.step_done()
    d, t, e = comp.compose()
    assert d == [(1, 10, 0, 100), (1, 5, 1, 200)] and t == [[0, 1, 2], [3, 4]] and e == [1, 1]
    comp.step_done()
    d, t, e = comp.compose()
    assert d == [(1, 11, 0, 100), (1, 6, 1, 200)] and e == [1, 1]
    comp.step_done()
    assert comp.n_live() == 0 and comp.n_free_blocks() == 8
    assert list(comp.free) == [5, 6, 7, 0, 1, 2, 3, 4]          # freed blocks rejoin at the back
    assert comp.compose() == ([], [], [])


def test_fuses_short_prompts_to_fill_budget_exactly():
    comp = SplitFuseComposer(16, 16, 4, 64)
    for sid, plen in enumerate([5, 5, 5, 5]):
        comp.add_request(sid, plen, 2)
    d, _, e = comp.compose()
    assert [x[0] for x in d] == [5, 5, 5, 1] and e == [1, 1, 1, 0]       # 4th prompt is split
    comp.step_done()
    d, _, e = comp.compose()
    # three generations first, then the rest of prompt 3
    assert d == [(1, 5, 0, 0), (1, 5, 1, 1), (1, 5, 2, 2), (4, 1, 3, 3)] and e == [1, 1, 1, 1]


@pytest.mark.parametrize("seed", range(6))
def test_invariants_on_random_streams(seed):
    rng = np.random.default_rng(seed)
    budget = int(rng.integers(8, 200))
    B = int(rng.choice([1, 4, 16, 64]))
    max_seqs = int(rng.integers(4, 64))
    n_steps = 20000                 # upper bound; the loop stops once every request has retired
    arrivals, sid, req = {}, 0, {}
    for step in range(100):
        for _ in range(rng.poisson(0.4)):
            plen, gen = int(rng.integers(1, 4 * budget)), int(rng.integers(1, 40))
            arrivals.setdefault(step, []).append((sid, plen, gen))
            req[sid] = (plen, gen)
            sid += 1
    worst = max((-(-(p + g) // B) for p, g in req.values()), default=1)
    num_blocks = max(sum(-(-(p + g) // B) for p, g in req.values()), worst)   # never runs dry
    free_order = rng.permutation(num_blocks)
    comp = SplitFuseComposer(budget, max_seqs, B, num_blocks, free_order)

    cached = {}        # sid -> tokens in cache
    emitted = {}       # sid -> tokens generated
    owner = {}         # physical block -> sid
    prompt_order = []  # sids in order of first scheduling
    waiting_decodes_prev = set()

    def check(step, comp, descs, tables, emits):
        nonlocal waiting_decodes_prev
        total = sum(d[0] for d in descs)
        assert total <= budget and len(descs) <= max_seqs
        sids = [d[3] for d in descs]
        assert len(set(sids)) == len(sids)                          # each sequence at most once
        off = 0
        seen_prompt = False
        for (n, c, qo, s), tab, em in zip(descs, tables, emits):
            assert n >= 1 and qo == off
            off += n
            plen, gen = req[s]
            assert c == cached.get(s, 0)                            # n_cached = sum of earlier n_new
            if c >= plen:                                           # generation pass
                assert n == 1 and em == 1 and not seen_prompt       # generations come first
            else:
                seen_prompt = True
                assert c + n <= plen
                assert em == (1 if c + n == plen else 0)            # only the last chunk generates
                if s not in prompt_order:
                    prompt_order.append(s)
            assert len(tab) == -(-(c + n) // B)                     # exactly the blocks it needs
            for b in tab:
                assert owner.setdefault(b, s) == s                  # no block shared
        # budget met exactly unless supply or the sequence bound ran out
        supply = sum(p - cached.get(s, 0) for s, (p, g) in req.items()
                     if s in arrived and cached.get(s, 0) < p)
        n_dec = sum(1 for s in arrived if cached.get(s, 0) >= req[s][0] and not done(s))
        if len(descs) < max_seqs:
            assert total == min(budget, supply + n_dec), (step, total, supply, n_dec)
        # generation never stalls: every live generation runs unless the bound cuts it, and a
        # generation left out in one pass runs in the next (rotation)
        live_dec = {s for s in arrived if cached.get(s, 0) >= req[s][0] and not done(s)}
        sched_dec = {s for (n, c, qo, s) in descs if c >= req[s][0]}
        assert len(sched_dec) == min(len(live_dec), budget, max_seqs)
        assert waiting_decodes_prev & live_dec <= sched_dec or len(waiting_decodes_prev) > min(budget, max_seqs)
        waiting_decodes_prev = live_dec - sched_dec
        # bookkeeping for the next pass
        for (n, c, qo, s), em in zip(descs, emits):
            cached[s] = c + n
            emitted[s] = emitted.get(s, 0) + em
            if done(s):
                for b in [b for b, o in owner.items() if o == s]:
                    del owner[b]

    def done(s):
        return emitted.get(s, 0) >= req[s][1]

    arrived = set()
    history = []
    for step in range(n_steps):
        for a in arrivals.get(step, []):
            comp.add_request(*a)
            arrived.add(a[0])
        out = comp.compose()
        check(step, comp, *out)
        history.append(out)
        comp.step_done()
        if step > 100 and comp.n_live() == 0:
            break
    # every request ran to completion: chunks sum to the prompt, max_new tokens emitted
    assert comp.n_live() == 0
    for s, (plen, gen) in req.items():
        assert cached[s] == plen + gen - 1 and emitted[s] == gen
    assert prompt_order == sorted(prompt_order)                      # first come, first served
    assert comp.n_free_blocks() == num_blocks and sorted(comp.free) == list(range(num_blocks))


def test_consistent_forward_size_under_load():
    """With a backlog of long prompts every pass carries exactly the budget (Sec. 3.2)."""
    comp = SplitFuseComposer(512, 256, 64, 4096)
    for sid in range(12):
        comp.add_request(sid, 2600, 60)
    sizes = []
    for _ in range(40):
        d, _, _ = comp.compose()
        sizes.append(sum(x[0] for x in d))
        comp.step_done()
    assert sizes == [512] * 40


def test_block_shortage_shrinks_chunk_then_reports_no_blocks():
    comp = SplitFuseComposer(32, 8, 4, 3)            # 12 token slots in total
    comp.add_request(0, 20, 4)
    comp.add_request(1, 6, 2)
    d, t, e = comp.compose()
    assert d == [(12, 0, 0, 0)] and len(t[0]) == 3 and e == [0]     # shrunk to what fits; next prompt not started
    comp.step_done()
    with pytest.raises(NoBlocksError):
        comp.compose()


def test_generation_skipped_when_it_cannot_get_a_block():
    comp = SplitFuseComposer(8, 8, 4, 3)
    comp.add_request(0, 4, 5)       # one block, next token needs a second block
    comp.add_request(1, 8, 5)       # two blocks
    comp.compose(); comp.step_done()                 # pass 0: 4 + 4
    d, _, _ = comp.compose()                         # pass 1: decode 0 needs a block: 1 free -> ok; prompt 1 gets none
    assert d[0] == (1, 4, 0, 0) and len(d) == 1
    comp.step_done()
    d, _, _ = comp.compose()                         # pass 2: decode 0 (c=5) fits its block; prompt 1 still starved
    assert d == [(1, 5, 0, 0)]


def test_generations_hold_the_budget_before_new_prompts():
    """Budget 3: three running generations fill every pass; waiting prompts start only when one retires."""
    comp = SplitFuseComposer(3, 8, 4, 64)
    for sid in range(5):
        comp.add_request(sid, 1, 4)
    seen = []
    for _ in range(8):
        d, _, _ = comp.compose()
        seen.append([(x[3], x[1]) for x in d])
        comp.step_done()
    assert seen[0] == [(0, 0), (1, 0), (2, 0)]
    assert seen[1] == [(0, 1), (1, 1), (2, 1)] and seen[3] == [(0, 3), (1, 3), (2, 3)]
    assert seen[4] == [(3, 0), (4, 0)]                    # generations 0-2 retired after 4 tokens each
    assert seen[7] == [(3, 3), (4, 3)] and comp.n_live() == 0


# ---------------------------------------------------------------------------------------
# the two comparison policies of the scheduling simulator
def _run(policy, budget, max_seqs, B, num_blocks, arrivals, n_steps=400):
    c = SplitFuseComposer(budget, max_seqs, B, num_blocks, policy=policy)
    passes = []
    for step in range(n_steps):
        for r in arrivals.get(step, []):
            c.add_request(*r)
        if c.n_live() == 0 and step > max(arrivals):
            break
        descs, tables, emits = c.compose()
        passes.append((descs, emits))
        c.step_done()
    assert c.n_live() == 0 and c.n_free_blocks() == num_blocks
    return passes


def test_prompt_first_hand_worked_schedule():
    """budget 8: prompts of 5 and 6 tokens arrive together, each wants 2 tokens.  Pass 0 takes
    the first prompt only (5 + 6 > 8), pass 1 the second while sequence 0 waits, then both
    generate together once."""
    passes = _run("prompt_first", 8, 4, 4, 16, {0: [(0, 5, 2), (1, 6, 2)]})
    assert [[(n, c, sid) for n, c, _, sid in d] for d, _ in passes] == [
        [(5, 0, 0)], [(6, 0, 1)], [(1, 5, 0), (1, 6, 1)]]
    assert [e for _, e in passes] == [[1], [1], [1, 1]]


def test_whole_prompt_joins_hand_worked_schedule():
    """both prompts join the first pass whole (no token budget for prompts), a later prompt of
    20 tokens joins the running generations in pass 1"""
    passes = _run("whole_prompt_joins", 8, 4, 4, 32, {0: [(0, 5, 3), (1, 6, 3)], 1: [(2, 20, 1)]})
    assert [[(n, c, sid) for n, c, _, sid in d] for d, _ in passes] == [
        [(5, 0, 0), (6, 0, 1)], [(1, 5, 0), (1, 6, 1), (20, 0, 2)], [(1, 6, 0), (1, 7, 1)]]


@pytest.mark.parametrize("policy", ["prompt_first", "whole_prompt_joins"])
@pytest.mark.parametrize("seed", range(4))
def test_comparison_policies_invariants(policy, seed):
    rng = np.random.default_rng(500 + seed)
    budget, B = int(rng.integers(8, 200)), int(rng.choice([1, 4, 16]))
    arrivals, sid, blocks = {}, 0, 0
    for step in range(60):
        for _ in range(rng.poisson(0.4)):
            plen, gen = int(rng.integers(1, 3 * budget)), int(rng.integers(1, 30))
            arrivals.setdefault(step, []).append((sid, plen, gen))
            blocks += -(-(plen + gen) // B)
            sid += 1
    if not arrivals:
        arrivals = {0: [(0, 3, 2)]}
        blocks = 8
    prompt_len = {r[0]: r[1] for rs in arrivals.values() for r in rs}
    passes = _run(policy, budget, 64, B, blocks, arrivals, n_steps=5000)
    seen_prompt = set()
    for descs, emits in passes:
        gens = [d for d in descs if d[1] > 0]
        prompts = [d for d in descs if d[1] == 0]
        assert all(n == 1 for n, *_ in gens)
        for n, c, _, s in prompts:                       # never split, processed exactly once
            assert n == prompt_len[s] and s not in seen_prompt
            seen_prompt.add(s)
        assert all(emits)                                # every entry produces a token
        assert descs[:len(gens)] == gens                 # generations ahead of prompts
        if policy == "prompt_first":
            assert not (gens and prompts)                # a pass is one or the other
            if len(prompts) > 1:
                assert sum(n for n, *_ in prompts) <= budget
    assert seen_prompt == set(prompt_len)


# ------------------------------------------------------------------ pool exhaustion: preempt the newest (R9)
def test_preempt_newest_hand_worked_schedule():
    """Budget 8, blocks of 4 tokens, a pool of 4 blocks, requests A = (prompt 6, generate 6) and
    B = (6, 6).  Worked by hand:
      pass 1  A takes its 6 prompt tokens (blocks 0, 1) and emits; B gets the 2 tokens left (block 2)
      pass 2  A generates (position 6, no new block); B finishes its prompt (4 tokens, block 3), emits
      pass 3  both generate (positions 7 and 6)
      pass 4  A needs a third block for position 8, none is free: skipped; B generates (position 7)
      pass 5  A needs a block, B needs a block (position 8): nothing can run.  Stall: "no blocks".
              Preempt-newest: B arrived last, gives blocks 2, 3 back and restarts as a prompt of
              8 + 1 = 9 tokens (3 of its 6 tokens already emitted); A generates with block 2,
              B's first chunk is the 4 tokens that fit block 3
      pass 6, 7  A generates (positions 9, 10; no new block) and retires with 6 tokens emitted;
              B cannot get room for a single token
      pass 8  B takes its remaining 5 tokens with blocks 0, 1 and emits its 4th token
      pass 9, 10  B generates (positions 9, 10) and retires with 6 tokens emitted."""
    want = [
        ([(6, 0, 0, 0), (2, 0, 6, 1)], [[0, 1], [2]], [1, 0]),
        ([(1, 6, 0, 0), (4, 2, 1, 1)], [[0, 1], [2, 3]], [1, 1]),
        ([(1, 7, 0, 0), (1, 6, 1, 1)], [[0, 1], [2, 3]], [1, 1]),
        ([(1, 7, 0, 1)], [[2, 3]], [1]),
        ([(1, 8, 0, 0), (4, 0, 1, 1)], [[0, 1, 2], [3]], [1, 0]),
        ([(1, 9, 0, 0)], [[0, 1, 2]], [1]),
        ([(1, 10, 0, 0)], [[0, 1, 2]], [1]),
        ([(5, 4, 0, 1)], [[3, 0, 1]], [1]),
        ([(1, 9, 0, 1)], [[3, 0, 1]], [1]),
        ([(1, 10, 0, 1)], [[3, 0, 1]], [1]),
    ]
    c = SplitFuseComposer(8, 4, 4, 4, exhaustion="preempt_newest")
    c.add_request(0, 6, 6)
    c.add_request(1, 6, 6)
    for k, (descs, tables, emits) in enumerate(want):
        got = c.compose()
        assert got == (descs, tables, emits), f"pass {k + 1}: {got}"
        c.step_done()
    assert c.n_live() == 0 and c.n_free_blocks() == 4
    assert (c.n_preemptions, c.tokens_discarded) == (1, 8)
    # the default stalls at pass 5
    c = SplitFuseComposer(8, 4, 4, 4)
    c.add_request(0, 6, 6)
    c.add_request(1, 6, 6)
    for _ in range(4):
        c.compose()
        c.step_done()
    with pytest.raises(NoBlocksError):
        c.compose()


def test_preempt_newest_cannot_help_a_sequence_that_alone_exceeds_the_pool():
    c = SplitFuseComposer(8, 4, 4, 2, exhaustion="preempt_newest")     # 8 token slots in all
    c.add_request(0, 6, 6)                                               # needs 11
    for _ in range(3):
        c.compose()
        c.step_done()
    with pytest.raises(NoBlocksError):
        c.compose()
    assert c.n_preemptions == 0


@pytest.mark.parametrize("seed", range(12))
def test_preempt_newest_always_finishes_every_request(seed):
    """Any pool that can hold the largest single sequence serves every request to its last token:
    exactly max_new_tokens emissions each, within the budget in every pass, blocks never shared
    and all returned; a restarted sequence starts again from an empty cache and is otherwise
    consistent from pass to pass."""
    rng = np.random.default_rng(900 + seed)
    budget = int(rng.integers(4, 64))
    B = int(rng.choice([1, 4, 16]))
    reqs = [(int(rng.integers(1, 4 * budget)), int(rng.integers(1, 40))) for _ in range(int(rng.integers(2, 14)))]
    largest = max(-(-(p + g) // B) for p, g in reqs)
    num_blocks = largest + int(rng.integers(0, 3))
    c = SplitFuseComposer(budget, 8, B, num_blocks, rng.permutation(num_blocks), exhaustion="preempt_newest")
    for sid, (p, g) in enumerate(reqs):
        c.add_request(sid, p, g)
    emitted = [0] * len(reqs)
    cached = [0] * len(reqs)
    passes = 0
    while c.n_live() > 0:
        descs, tables, emits = c.compose()
        passes += 1
        assert passes < 100000
        assert descs and sum(d[0] for d in descs) <= budget
        held = [b for t in tables for b in t]
        assert len(held) == len(set(held))
        for (n_new, n_cached, _, sid), tab, em in zip(descs, tables, emits):
            assert n_cached in (cached[sid], 0)                  # continues, or restarted from nothing
            assert len(tab) == -(-(n_cached + n_new) // B)
            cached[sid] = n_cached + n_new
            emitted[sid] += em
        c.step_done()
    assert emitted == [g for _, g in reqs]
    assert c.n_free_blocks() == num_blocks
    if seed % 3 == 0:
        # with room for everything the policy never acts and the schedule is the default one
        roomy = sum(-(-(p + g) // B) for p, g in reqs)
        a = SplitFuseComposer(budget, 8, B, roomy, exhaustion="preempt_newest")
        b = SplitFuseComposer(budget, 8, B, roomy)
        for sid, (p, g) in enumerate(reqs):
            a.add_request(sid, p, g)
            b.add_request(sid, p, g)
        while b.n_live() > 0:
            assert a.compose() == b.compose()
            a.step_done()
            b.step_done()
        assert a.n_preemptions == 0

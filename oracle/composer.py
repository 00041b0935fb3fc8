"""Reference Dynamic SplitFuse batch composer with a block allocator (TEST INFRASTRUCTURE).

Follows the paper's description of the scheduling loop, in plain Python:

* a new batch decision is taken for every forward pass; sequences join and leave
  between passes and nothing is padded (Sec. 2.2, continuous batching);
* a long prompt is cut into chunks that run over several passes and only the pass that
  consumes its last token generates (Sec. 3.2, rule 1);
* prompts, cut where needed, are fused with the running generations so that the pass
  holds exactly ``token_budget`` tokens whenever enough tokens are waiting (rule 2);
* running generations are never stalled by prompts (Sec. 3.2, closing paragraph);
* cache storage is handed out in fixed-size blocks (Sec. 2.1).

Where the paper is silent this file takes the following readings:

R1  generations are placed first, one token each, in rotation order (least recently
    scheduled first); they move to the back of the rotation once scheduled.
R2  at most ``min(token_budget, max_seqs)`` generations per pass; the rest wait.
R3  prompts are first come, first served; a partly processed prompt continues before a
    new one starts; a chunk takes ``min(remaining prompt, remaining budget)`` tokens;
    chunks need not align to blocks and may be a single token.
R4  the pass that consumes the last prompt token emits the first generated token; from
    the next pass on the sequence is a generation with ``n_new = 1``.  A sequence retires
    once it has emitted ``max_new_tokens`` tokens; the last emitted token is never fed.
R5  a sequence needs ``ceil((c + n) / B) - ceil(c / B)`` new blocks; they are popped from
    the front of the free list; a retiring sequence pushes its blocks to the back, in
    logical order.
R6  out of blocks: a generation that cannot get its block is skipped this pass (it keeps
    its place in the rotation); a prompt chunk shrinks to what fits; when it shrinks, or
    nothing fits, no later prompt is started.  No eviction or swapping.
R7  descriptor order: generations (rotation order), then prompt chunks (arrival order);
    ``q_offset`` is the running sum of ``n_new``.
R8  if requests exist but nothing can be scheduled the composer reports "no blocks"
    (``exhaustion="stall"``, the default).
R9  ``exhaustion="preempt_newest"``: in the situation of R8 the sequence that arrived last
    among those holding blocks gives its blocks back (to the back of the free list, in
    logical order) and starts over: its cache is gone, so the ``n_cached`` tokens it had
    processed plus the generated token it was about to feed become a prompt of
    ``n_cached + 1`` tokens (a partly processed prompt simply restarts), queued by its
    arrival order; tokens it has emitted stay emitted.  The decision is then taken again,
    and again, until something can be scheduled.  If the only sequence holding blocks is
    stuck there is nothing to take from: "no blocks" as in R8.  (The paper does not say
    what happens when the pool runs dry; recomputation is the simplest policy that keeps
    a full pool from stopping the server, and the oldest sequence always makes progress.)

Two further policies serve the scheduling simulator as points of comparison.  They are the
batch decisions the paper sets Dynamic SplitFuse against (Sec. 2.2 continuous batching with
a bound on sequences; Sec. 3 and Sec. 4.4: prompt processing that preempts generation),
reduced to the decision itself; neither ever splits a prompt:

P1  ``prompt_first``: if any prompt waits, the pass holds whole prompts only, in arrival
    order, as long as their token sum stays within ``token_budget`` (the first prompt is
    taken even if it alone exceeds it) and sequences and blocks allow; generations wait.
    A prompt that cannot get its blocks waits and nothing behind it starts.  If no prompt
    could be placed, or none waits, the pass runs the generations as in R1, R2, R6.
P2  ``whole_prompt_joins``: every pass runs the generations (R1, R2, R6) and then lets
    waiting prompts join whole, in arrival order, while sequences and blocks allow; there
    is no token budget for prompts.
"""
from __future__ import annotations

from collections import deque
from dataclasses import dataclass, field


class NoBlocksError(RuntimeError):
    pass


@dataclass
class _Seq:
    seq_id: int
    prompt_len: int
    max_new_tokens: int
    n_cached: int = 0
    emitted: int = 0
    arrival: int = 0
    blocks: list = field(default_factory=list)


def _ceil_div(a: int, b: int) -> int:
    return -(-a // b)


POLICIES = ("splitfuse", "prompt_first", "whole_prompt_joins")
EXHAUSTION = ("stall", "preempt_newest")


class SplitFuseComposer:
    def __init__(self, token_budget: int, max_seqs: int, block_size: int, num_blocks: int,
                 free_list_order=None, policy: str = "splitfuse", exhaustion: str = "stall"):
        assert token_budget >= 1 and max_seqs >= 1 and block_size >= 1 and num_blocks >= 1
        assert policy in POLICIES and exhaustion in EXHAUSTION
        self.policy = policy
        self.exhaustion = exhaustion
        self.n_arrived = 0
        self.n_preemptions = 0          # R9 statistics
        self.tokens_discarded = 0
        self.token_budget = token_budget
        self.max_seqs = max_seqs
        self.block_size = block_size
        order = list(range(num_blocks)) if free_list_order is None else [int(b) for b in free_list_order]
        assert sorted(order) == list(range(num_blocks)), "free list must be a permutation"
        self.free = deque(order)
        self.prompts = deque()      # _Seq with prompt tokens left, arrival order
        self.decodes = []           # _Seq in rotation order
        self.pending = None         # batch composed but not yet committed

    # ------------------------------------------------------------------ requests
    def add_request(self, seq_id: int, prompt_len: int, max_new_tokens: int) -> None:
        assert prompt_len >= 1 and max_new_tokens >= 1
        self.prompts.append(_Seq(seq_id, prompt_len, max_new_tokens, arrival=self.n_arrived))
        self.n_arrived += 1

    def n_free_blocks(self) -> int:
        return len(self.free)

    def n_live(self) -> int:
        return len(self.prompts) + len(self.decodes)

    # ------------------------------------------------------------------ one pass
    def compose(self):
        """Return ``(descs, block_tables, emits)`` for the next forward pass.

        ``descs`` is a list of ``(n_new, n_cached, q_offset, seq_id)``; ``block_tables`` a
        list of block-id lists (all blocks of the sequence, including new ones);
        ``emits[k]`` is 1 if descriptor ``k`` produces a token in this pass.
        """
        assert self.pending is None, "previous pass not committed"
        while True:
            batch = self._decide()
            if batch or self.n_live() == 0:
                break
            if self.exhaustion == "stall" or not self._preempt_newest():      # R8, R9
                raise NoBlocksError("requests are waiting but no KV block is free")

        descs, tables, emits = [], [], []
        q_off = 0
        for seq, n_new, em, _ in batch:        # generations were placed before prompts (R7)
            descs.append((n_new, seq.n_cached, q_off, seq.seq_id))
            tables.append(list(seq.blocks))
            emits.append(em)
            q_off += n_new
        self.pending = batch
        return descs, tables, emits

    def _preempt_newest(self) -> bool:
        """R9.  False if there is nothing to take blocks from."""
        holders = [s for s in list(self.prompts) + self.decodes if s.blocks]
        if len(holders) < 2:
            return False
        victim = max(holders, key=lambda s: s.arrival)
        self.n_preemptions += 1
        self.tokens_discarded += victim.n_cached
        self._retire(victim)
        if any(s is victim for s in self.decodes):
            self.decodes = [s for s in self.decodes if s is not victim]
            victim.prompt_len = victim.n_cached + 1
            later = [i for i, s in enumerate(self.prompts) if s.arrival > victim.arrival]
            self.prompts.insert(later[0] if later else len(self.prompts), victim)
        victim.n_cached = 0
        return True

    def _decide(self):
        """One batch decision on the current state: list of (seq, n_new, emits, is_decode);
        blocks of the scheduled sequences are taken from the free list."""
        B = self.block_size
        batch = []
        budget_left = self.token_budget
        seqs_left = self.max_seqs

        def place_generations():
            nonlocal budget_left, seqs_left
            for seq in self.decodes:            # R1, R2, R6
                if budget_left == 0 or seqs_left == 0:
                    break
                need = _ceil_div(seq.n_cached + 1, B) - _ceil_div(seq.n_cached, B)
                if need > len(self.free):
                    continue
                for _ in range(need):
                    seq.blocks.append(self.free.popleft())
                batch.append((seq, 1, 1, True))
                budget_left -= 1
                seqs_left -= 1

        def place_whole_prompts(token_cap):
            """whole prompts in arrival order; token_cap None = no cap (P2), else P1's cap"""
            nonlocal seqs_left
            placed_tokens = 0
            for seq in self.prompts:
                if seqs_left == 0:
                    break
                assert seq.n_cached == 0
                if token_cap is not None and placed_tokens > 0 and placed_tokens + seq.prompt_len > token_cap:
                    break
                need = _ceil_div(seq.prompt_len, B)
                if need > len(self.free):
                    break
                for _ in range(need):
                    seq.blocks.append(self.free.popleft())
                batch.append((seq, seq.prompt_len, 1, False))
                placed_tokens += seq.prompt_len
                seqs_left -= 1
            return placed_tokens

        if self.policy == "prompt_first":
            if place_whole_prompts(self.token_budget) == 0:
                place_generations()
        elif self.policy == "whole_prompt_joins":
            place_generations()
            place_whole_prompts(None)
        else:
            place_generations()

        # Dynamic SplitFuse: prompt tokens fill what is left of the budget (R3, R6)
        for seq in (self.prompts if self.policy == "splitfuse" else ()):
            if budget_left == 0 or seqs_left == 0:
                break
            want = min(seq.prompt_len - seq.n_cached, budget_left)
            have_blocks = _ceil_div(seq.n_cached, B)
            room = (have_blocks + len(self.free)) * B - seq.n_cached
            take = min(want, room)
            if take == 0:
                break
            need = _ceil_div(seq.n_cached + take, B) - have_blocks
            for _ in range(need):
                seq.blocks.append(self.free.popleft())
            emits = 1 if seq.n_cached + take == seq.prompt_len else 0
            batch.append((seq, take, emits, False))
            budget_left -= take
            seqs_left -= 1
            if take < want:
                break

        return batch

    def step_done(self) -> None:
        """Commit the composed pass: advance caches, start/finish generations (R4, R5)."""
        assert self.pending is not None, "nothing composed"
        batch, self.pending = self.pending, None
        scheduled_decodes = [seq for seq, _, _, is_dec in batch if is_dec]
        scheduled_ids = {id(s) for s in scheduled_decodes}
        # rotation: unscheduled generations keep the front, scheduled ones go to the back
        self.decodes = [s for s in self.decodes if id(s) not in scheduled_ids] + scheduled_decodes
        for seq, n_new, em, is_dec in batch:
            seq.n_cached += n_new
            if em:
                seq.emitted += 1
            if is_dec:
                if seq.emitted == seq.max_new_tokens:
                    self.decodes.remove(seq)
                    self._retire(seq)
            elif seq.n_cached == seq.prompt_len:
                # prompt fully consumed: the head of the arrival queue is this sequence
                self.prompts.remove(seq)
                if seq.emitted == seq.max_new_tokens:
                    self._retire(seq)
                else:
                    self.decodes.append(seq)

    def _retire(self, seq: _Seq) -> None:
        self.free.extend(seq.blocks)
        seq.blocks = []

"""Scheduling simulator: Dynamic SplitFuse against two other batch-composition policies, on
the paper's serving metrics, with step times from this library's kernels.

The paper's claims are about serving behaviour (Sec. 4): throughput against latency,
effective throughput under a service-level agreement, and token-level tail latency.  They
follow from the batch decision taken before every forward pass (Sec. 3.2).  This module
replays that decision loop for closed-loop clients (Sec. 4.1) with the library's host
composer (``fsf_compose_batch``, policies of ``fsf_sched_set_policy``) and scores the
outcome:

* prompt latency = time from sending a request to its first token; target: at most
  ``prompt_len / 512`` seconds;
* generation latency = gaps between consecutive tokens of a request; target ``r`` tokens/s:
  the exponential moving average of the gaps (``alpha = 0.2``, started at the first gap)
  never exceeds ``1 / r`` seconds, for r = 2, 4, 6;
* effective throughput = requests per second that meet both targets;
* P50 / P90 / P95 over all generation gaps.

The duration of a pass is a callable.  ``ForwardModel`` is the one used for the published
runs: the attention part of every layer is either *measured* (``MeasuredAttention``: the
pass's KV append and ragged attention are executed on the GPU through the library on
buffers of the pass's real shape and block tables, and timed with events) or taken from the
rates the kernels reach; the rest of the layer (its linear maps) is either measured as well
(``layer_model``: the layer's linear maps through fsf_linear at the pass's token count) or a
two-regime model: reading the weights once, or the
flops of the forward tokens, whichever takes longer (Sec. 3.1: few tokens are bound by weight
reads, many by compute).

    python -m paper_2401_08671_amd.policy_sim [--clients 16] [--requests 128] [--analytic]
"""
from __future__ import annotations

import argparse
import json
import sys
from dataclasses import dataclass

import numpy as np

from . import fsf
from . import workloads as wl

POLICIES = {"splitfuse": fsf.FSF_POLICY_SPLITFUSE, "prompt_first": fsf.FSF_POLICY_PROMPT_FIRST,
            "whole_prompt_joins": fsf.FSF_POLICY_WHOLE_PROMPT_JOINS}
EMA_ALPHA = 0.2
PROMPT_TOKENS_PER_S = 512.0


class PoolStats:
    """Occupancy of the blocked KV cache over a run (paper Sec. 2.1: fixed-size blocks handed out on
    demand): blocks in use, tokens they hold, and how often a pass was cut short by the pool."""

    def __init__(self, block_size: int, num_blocks: int, token_budget: int):
        self.B, self.num_blocks, self.budget = block_size, num_blocks, token_budget
        self.cached = {}              # live sequence -> tokens in the cache
        self.passes = self.short_passes = 0
        self.preemptions = self.tokens_discarded = 0   # sequences restarted by the exhaustion policy
        self.sum_used = self.sum_tokens = self.peak_used = 0

    def on_pass(self, sched, descs, waiting_prompt_tokens: int):
        for n_new, n_cached, _, sid in descs:
            self.cached[int(sid)] = int(n_cached) + int(n_new)
        used = self.num_blocks - sched.free_blocks()
        self.passes += 1
        self.sum_used += used
        self.peak_used = max(self.peak_used, used)
        self.sum_tokens += sum(self.cached.values())
        n_tokens = int(sum(d[0] for d in descs))
        # tokens were waiting, the budget was not met: the pool had no block for them
        if n_tokens < self.budget and waiting_prompt_tokens > 0:
            self.short_passes += 1

    def retire(self, sid: int):
        self.cached.pop(sid, None)

    def summary(self):
        used = self.sum_used / max(self.passes, 1)
        return {"pool_blocks": self.num_blocks, "mean_blocks_in_use": used, "peak_blocks_in_use": self.peak_used,
                "mean_pool_utilisation": used / self.num_blocks,
                "tokens_per_allocated_slot": self.sum_tokens / max(self.sum_used * self.B, 1),
                "passes_cut_short_by_the_pool": self.short_passes / max(self.passes, 1),
                "sequences_restarted": self.preemptions, "cached_tokens_discarded": self.tokens_discarded}


def simulate(policy, requests, n_clients, step_time, token_budget, max_seqs, block_size, num_blocks,
             max_blocks=None, on_pass=None, pool_stats: PoolStats = None, exhaustion: int = fsf.FSF_EXHAUST_STALL):
    """Closed loop of ``n_clients`` clients over ``requests = [(prompt_len, gen_len)]``.

    ``step_time(descs)`` returns the seconds a pass with descriptors ``descs`` (rows
    ``(n_new, n_cached, q_offset, seq_id)``) takes; ``on_pass(descs, tables)`` is called for
    every pass if given.  Returns ``(sent [R], token_times list of arrays, total_time, n_passes)``.
    """
    if max_blocks is None:
        max_blocks = max(-(-(p + g) // block_size) for p, g in requests)
    sched = fsf.Scheduler(token_budget, max_seqs, block_size, num_blocks, max_blocks)
    sched.set_policy(POLICIES[policy])
    sched.set_exhaustion(exhaustion)
    R = len(requests)
    sent = np.zeros(R)
    tokens = [[] for _ in range(R)]
    nxt = 0
    for _ in range(min(n_clients, R)):
        sched.add_request(nxt, *requests[nxt])
        nxt += 1
    t, done, n_passes = 0.0, 0, 0
    while done < R:
        descs, tables, emits = sched.compose_batch()
        if len(descs) == 0:
            raise RuntimeError("closed loop: no request in flight")
        if on_pass is not None:
            on_pass(descs, tables)
        if pool_stats is not None:
            pool_stats.preemptions, pool_stats.tokens_discarded = sched.preemptions()
            in_pass = {int(d[3]): int(d[0]) + int(d[1]) for d in descs}
            waiting = sum(requests[i][0] - in_pass.get(i, pool_stats.cached.get(i, 0))
                          for i in range(nxt) if len(tokens[i]) == 0)
            pool_stats.on_pass(sched, descs, waiting)
        t = t + step_time([tuple(int(x) for x in d) for d in descs])
        n_passes += 1
        finished = 0
        for d, em in zip(descs, emits):
            if em:
                sid = int(d[3])
                tokens[sid].append(t)
                if len(tokens[sid]) == requests[sid][1]:
                    finished += 1
                    if pool_stats is not None:
                        pool_stats.retire(sid)
        sched.step_done()
        done += finished
        for _ in range(finished):
            if nxt < R:
                sent[nxt] = t
                sched.add_request(nxt, *requests[nxt])
                nxt += 1
    sched.close()
    return sent, [np.asarray(x) for x in tokens], t, n_passes


def metrics(requests, sent, tokens, total_time, rates=(2.0, 4.0, 6.0)):
    R = len(requests)
    first = np.array([tk[0] for tk in tokens])
    last = np.array([tk[-1] for tk in tokens])
    plen = np.array([p for p, _ in requests], dtype=np.float64)
    prompt_ok = (first - sent) <= plen / PROMPT_TOKENS_PER_S
    worst = np.zeros(R)
    gaps_all = []
    for i, tk in enumerate(tokens):
        gaps = np.diff(tk)
        gaps_all.append(gaps)
        ema = None
        for gap in gaps.tolist():
            ema = gap if ema is None else EMA_ALPHA * gap + (1.0 - EMA_ALPHA) * ema
            worst[i] = max(worst[i], ema)
    gaps_all = np.concatenate(gaps_all) if gaps_all else np.zeros(0)
    pct = (lambda q: float(np.percentile(gaps_all, q))) if len(gaps_all) else (lambda q: float("nan"))
    out = {
        "requests": R,
        "total_time_s": float(total_time),
        "throughput_rps": R / total_time,
        "mean_request_latency_s": float(np.mean(last - sent)),
        "prompt_sla_met": float(np.mean(prompt_ok)),
        "token_latency_p50_s": pct(50), "token_latency_p90_s": pct(90), "token_latency_p95_s": pct(95),
    }
    for r in rates:
        out[f"effective_throughput_rps_at_{r:g}_tok_s"] = float(np.sum(prompt_ok & (worst <= 1.0 / r))) / total_time
    return out


# ------------------------------------------------------------------ how long a pass takes
@dataclass
class ForwardModel:
    """Seconds of one forward pass of a dense decoder with this library's attention.

    Defaults: a 13B-parameter model in bf16 (40 layers, 40 heads of 128) on one MI355X; the
    linear part runs at the HBM rate the generation-row kernel reaches and at the matrix rate
    the prompt-chunk kernel reaches (both measured here); ``attention`` = None uses the same
    two rates for the attention part, else a callable ``descs -> seconds for ONE layer``."""
    n_layers: int = 40
    n_q_heads: int = 40
    n_kv_heads: int = 40
    head_dim: int = 128
    elem_bytes: int = 2
    weight_bytes: float = 26e9
    linear_flops_per_token: float = 2 * 13e9
    hbm_rate: float = 6.5e12
    matrix_rate: float = 1.05e15
    fixed_s: float = 100e-6          # launches and host work per pass
    attention: object = None
    linear: object = None            # None: the two-regime model; else a callable n_tokens -> seconds

    def linear_s(self, n_tokens: int) -> float:
        if self.linear is not None:
            return self.linear(n_tokens)
        return max(self.weight_bytes / self.hbm_rate, n_tokens * self.linear_flops_per_token / self.matrix_rate)

    def attention_layer_s(self, descs) -> float:
        if self.attention is not None:
            return self.attention(descs)
        d, e = self.head_dim, self.elem_bytes
        byt = flo = 0.0
        for n, c, _, _ in descs:
            byt += 4 * self.n_kv_heads * d * e * n                      # append
            if n == 1:
                byt += 2 * self.n_kv_heads * d * e * (c + 1) + 2 * self.n_q_heads * d * e
            else:
                pairs = n * c + n * (n + 1) // 2
                flo += 4.0 * d * self.n_q_heads * pairs
                byt += 2 * self.n_kv_heads * d * e * (c + n)
        return byt / self.hbm_rate + flo / self.matrix_rate

    def __call__(self, descs) -> float:
        n_tokens = sum(d[0] for d in descs)
        return self.fixed_s + self.linear_s(n_tokens) + self.n_layers * self.attention_layer_s(descs)


class MeasuredAttention:
    """One layer's KV append + ragged attention of a pass, executed and timed on the GPU.

    Buffers hold seeded random values (there is no model: only shapes, lengths and block
    tables matter for time); the composer's block tables are used as they are, so the
    gather pattern is the real one.  A pass is run ``repeats`` times and the fastest is taken."""

    def __init__(self, model: ForwardModel, block_size: int, num_blocks: int, max_blocks: int,
                 max_seqs: int, max_tokens: int, repeats: int = 2, device="cuda"):
        import torch
        self.torch = torch
        self.m, self.B, self.device, self.repeats = model, block_size, device, repeats
        tdt = torch.bfloat16
        self.num_blocks, self.max_blocks = num_blocks, max_blocks
        self.k_cache = torch.empty((num_blocks, model.n_kv_heads, block_size, model.head_dim), dtype=tdt, device=device)
        self.v_cache = torch.empty_like(self.k_cache)
        wl.fill_pool_(self.k_cache, 1.0, 71)
        wl.fill_pool_(self.v_cache, 1.0, 72)
        self.q = wl.randn((max_tokens, model.n_q_heads, model.head_dim), "bf16", 1.0, 73, device)
        self.k_new = wl.randn((max_tokens, model.n_kv_heads, model.head_dim), "bf16", 1.0, 74, device)
        self.v_new = wl.randn((max_tokens, model.n_kv_heads, model.head_dim), "bf16", 1.0, 75, device)
        self.out = torch.empty_like(self.q)
        self.cfg = fsf.make_cfg(model.n_q_heads, model.n_kv_heads, model.head_dim, block_size, "bf16", num_blocks)
        self.ws = fsf.alloc_workspace(self.cfg, max_seqs, max_tokens, max_blocks, device)
        self.tables = None
        self.total_gpu_s = 0.0

    def set_tables(self, descs, tables):
        self.tables = tables

    def __call__(self, descs) -> float:
        torch = self.torch
        d = np.asarray(descs, dtype=np.int32)
        batch = fsf.DeviceBatch(d, self.tables, self.device)
        T = batch.n_tokens
        best = float("inf")
        for _ in range(self.repeats):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fsf.kv_append(self.cfg, self.k_new[:T], self.v_new[:T], self.k_cache, self.v_cache, batch)
            fsf.ragged_attention(self.cfg, self.q[:T], self.k_cache, self.v_cache, batch, self.out[:T], self.ws)
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) * 1e-3)
        self.total_gpu_s += best
        return best


_LINEAR_TABLE = None


def run(policy: str, requests, n_clients: int, token_budget: int, measured: bool, block_size: int = 64):
    need = sum(-(-(p + g) // block_size) for p, g in sorted(requests, key=lambda r: -(r[0] + r[1]))[:n_clients])
    num_blocks = need + 64
    max_blocks = max(-(-(p + g) // block_size) for p, g in requests)
    model = ForwardModel()
    on_pass = None
    if measured:
        from . import layer_model
        global _LINEAR_TABLE
        if _LINEAR_TABLE is None:   # the layer's GEMMs, timed once per process
            _LINEAR_TABLE = layer_model.measure_linear()
        model.linear = layer_model.MeasuredLinear(_LINEAR_TABLE, model.n_layers)
        # whole-prompt policies can put every client's prompt into one pass
        max_tokens = max(token_budget, sum(sorted((p for p, _ in requests), reverse=True)[:n_clients]) + n_clients)
        att = MeasuredAttention(model, block_size, num_blocks, max_blocks, max_seqs=n_clients + 1,
                                max_tokens=max_tokens)
        model.attention = att
        on_pass = att.set_tables
    sent, tokens, total, n_passes = simulate(policy, requests, n_clients, model, token_budget,
                                             max_seqs=n_clients + 1, block_size=block_size,
                                             num_blocks=num_blocks, max_blocks=max_blocks, on_pass=on_pass)
    out = metrics(requests, sent, tokens, total)
    out.update(policy=policy, clients=n_clients, passes=n_passes,
               attention="measured on the GPU" if measured else "from the kernels' rates",
               linear_part="GEMMs measured on the GPU" if measured else "two-regime model")
    if measured:
        out["attention_gpu_s_one_layer_total"] = model.attention.total_gpu_s
    return out


def pool_sweep(requests, n_clients: int, token_budget: int, fractions=(1.0, 0.8, 0.6, 0.4, 0.3), block_size: int = 64,
               exhaustion: int = fsf.FSF_EXHAUST_STALL):
    """Dynamic SplitFuse with a KV pool of a fraction of what the clients' largest requests would
    need together: throughput, occupancy, and how often the pool cut a pass short (analytic times).
    ``exhaustion``: what the composer does when nothing can be scheduled (stall, or restart the
    newest sequence and recompute it)."""
    full = sum(-(-(p + g) // block_size) for p, g in sorted(requests, key=lambda r: -(r[0] + r[1]))[:n_clients])
    largest = max(-(-(p + g) // block_size) for p, g in requests)
    out = []
    for frac in fractions:
        num_blocks = max(int(full * frac), largest)
        stats = PoolStats(block_size, num_blocks, token_budget)
        try:
            sent, tokens, total, n_passes = simulate("splitfuse", requests, n_clients, ForwardModel(), token_budget,
                                                     max_seqs=n_clients + 1, block_size=block_size,
                                                     num_blocks=num_blocks, max_blocks=largest, pool_stats=stats,
                                                     exhaustion=exhaustion)
            m = metrics(requests, sent, tokens, total)
            row = {"pool_fraction": frac, "exhaustion": "preempt_newest" if exhaustion else "stall",
                   "throughput_rps": m["throughput_rps"],
                   "mean_request_latency_s": m["mean_request_latency_s"], "passes": n_passes}
        except fsf.FsfError as e:
            if e.status != fsf.FSF_ERR_NO_BLOCKS:
                raise
            # every block is held by sequences that all need one more: without eviction (the paper
            # describes none) the composer can schedule nothing
            row = {"pool_fraction": frac, "exhaustion": "preempt_newest" if exhaustion else "stall",
                   "stuck_without_free_blocks_after_passes": stats.passes}
        row.update(stats.summary())
        out.append(row)
    return out


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--clients", type=int, nargs="+", default=[4, 16])
    ap.add_argument("--requests", type=int, default=96)
    ap.add_argument("--budget", type=int, default=2048)
    ap.add_argument("--analytic", action="store_true", help="no GPU: attention time from the kernels' rates")
    ap.add_argument("--pool-sweep", action="store_true", help="SplitFuse under a shrinking KV pool (no GPU)")
    a = ap.parse_args(argv)
    if a.pool_sweep:
        rows = []
        for mode in (fsf.FSF_EXHAUST_STALL, fsf.FSF_EXHAUST_PREEMPT_NEWEST):
            rows += pool_sweep(wl.chat_requests(a.requests), a.clients[-1], a.budget,
                               fractions=(1.0, 0.8, 0.6, 0.4, 0.3, 0.2, 0.1), exhaustion=mode)
        for r in rows:
            print(json.dumps(r), flush=True)
        return rows
    if not a.analytic:
        import torch
        assert torch.cuda.is_available(), "measured attention needs a GPU (or pass --analytic)"
    requests = wl.chat_requests(a.requests)
    results = []
    for nc in a.clients:
        for policy in POLICIES:
            results.append(run(policy, requests, nc, a.budget, measured=not a.analytic))
            print(json.dumps(results[-1]), flush=True)
    return results


if __name__ == "__main__":
    main()

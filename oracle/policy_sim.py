"""Reference scheduling simulator (TEST INFRASTRUCTURE): closed-loop clients, one batch
decision per forward pass, the paper's service-level metrics.

Method, following the paper's benchmarking section (Sec. 4.1) in plain Python:

* ``n_clients`` clients each keep one request in flight: a client sends a request, waits
  for its last token, and sends its next one at once, until ``len(requests)`` requests
  have been sent in total (throughput-latency methodology);
* every forward pass is one decision of the batch composer (``oracle.composer``, any of
  its policies); the pass lasts ``step_time(descs)`` seconds, a function the caller
  passes in; every sequence whose descriptor emits gets its token at the end of the pass;
* a request's prompt latency is the time from sending it to its first token, and it meets
  the prompt target if that is at most ``prompt_len / 512`` seconds; its generation
  latencies are the gaps between consecutive tokens, and it meets the generation target
  ``r`` tokens/s if the exponential moving average of those gaps never exceeds ``1/r``
  seconds; effective throughput is the rate of requests that meet both (Sec. 4.1,
  effective throughput);
* token-level latency percentiles are taken over all generation gaps of all requests
  (Sec. 4.4).

Readings where the paper is silent: the moving average starts at the first gap and uses
``ema <- alpha * gap + (1 - alpha) * ema`` with ``alpha = 0.2``; a request that generates
one token has no gaps and meets every generation target; percentiles interpolate linearly
between order statistics (position ``q * (n - 1)``); requests are handed to clients in
list order; when several clients become free in the same pass they send in order of their
finished requests' positions in the pass.
"""
from __future__ import annotations

from oracle.composer import SplitFuseComposer

EMA_ALPHA = 0.2
PROMPT_TOKENS_PER_S = 512.0


def simulate(policy, requests, n_clients, step_time, token_budget, max_seqs, block_size, num_blocks,
             exhaustion="stall"):
    """requests: list of (prompt_len, gen_len).  Returns (log, total_time, n_passes) with
    log[i] = dict(sent=..., tokens=[time of every emitted token])."""
    comp = SplitFuseComposer(token_budget, max_seqs, block_size, num_blocks, policy=policy, exhaustion=exhaustion)
    log = [None] * len(requests)
    nxt = 0
    t = 0.0

    def send(now):
        nonlocal nxt
        i = nxt
        nxt += 1
        log[i] = {"sent": now, "tokens": []}
        comp.add_request(i, requests[i][0], requests[i][1])

    for _ in range(min(n_clients, len(requests))):
        send(0.0)
    done = 0
    n_passes = 0
    while done < len(requests):
        descs, _tables, emits = comp.compose()
        assert descs, "closed loop: some request is always in flight"
        t = t + step_time(descs)
        n_passes += 1
        finished = 0
        for (n_new, n_cached, q_off, sid), em in zip(descs, emits):
            if em:
                log[sid]["tokens"].append(t)
                if len(log[sid]["tokens"]) == requests[sid][1]:
                    finished += 1
        comp.step_done()
        done += finished
        for _ in range(finished):
            if nxt < len(requests):
                send(t)
    return log, t, n_passes


def _percentile(sorted_vals, q):
    if not sorted_vals:
        return float("nan")
    pos = q * (len(sorted_vals) - 1)
    lo = int(pos)
    hi = min(lo + 1, len(sorted_vals) - 1)
    frac = pos - lo
    return sorted_vals[lo] + (sorted_vals[hi] - sorted_vals[lo]) * frac


def metrics(requests, log, total_time, rates=(2.0, 4.0, 6.0)):
    gaps_all = []
    prompt_ok = []
    worst_ema = []
    latency = []
    for (plen, glen), rec in zip(requests, log):
        toks = rec["tokens"]
        assert len(toks) == glen
        prompt_ok.append(toks[0] - rec["sent"] <= plen / PROMPT_TOKENS_PER_S)
        latency.append(toks[-1] - rec["sent"])
        ema = None
        worst = 0.0
        for a, b in zip(toks, toks[1:]):
            gap = b - a
            gaps_all.append(gap)
            ema = gap if ema is None else EMA_ALPHA * gap + (1.0 - EMA_ALPHA) * ema
            worst = max(worst, ema)
        worst_ema.append(worst)
    gaps_all.sort()
    out = {
        "requests": len(requests),
        "total_time_s": total_time,
        "throughput_rps": len(requests) / total_time,
        "mean_request_latency_s": sum(latency) / len(latency),
        "prompt_sla_met": sum(prompt_ok) / len(prompt_ok),
        "token_latency_p50_s": _percentile(gaps_all, 0.50),
        "token_latency_p90_s": _percentile(gaps_all, 0.90),
        "token_latency_p95_s": _percentile(gaps_all, 0.95),
    }
    for r in rates:
        ok = sum(1 for p, w in zip(prompt_ok, worst_ema) if p and w <= 1.0 / r)
        out[f"effective_throughput_rps_at_{r:g}_tok_s"] = ok / total_time
    return out

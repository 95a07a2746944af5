"""TEST INFRASTRUCTURE -- not part of the product.

Oracle for the request scheduler (eMoE Section 3.5: Eq. 3 and Algorithm 1), plain Python in the
paper's order and notation; nothing here is shared with the HIP library.

Eq. 3, the expected latency of running request i if a new request is scheduled:
    t_i = dE + (W + n_i * G_i) * c + r_i
W input tokens of the new request, dE expert loading latency its scheduling causes, c latency per
token, G_i tokens request i still has to generate, r_i its run time so far, n_i the number of
running requests that will finish after request i.

Algorithm 1: waiting requests are tried in order of SLO stringency (how soon the first token is
due); a request is admitted if the engine's token limit allows it and no running request that
currently meets its SLO would miss it.

Readings where the paper is silent or garbled:
  * T starts as the number of tokens the scheduled requests hold (the listing initialises it with
    the queue's length, but compares it with a token limit);
  * the request added to the scheduled queue is the candidate R (the listing writes S);
  * n_i counts running requests j != i with G_j > G_i (strictly more left to generate);
  * the current expected latency of a running request is Eq. 3 without a new request
    (dE = 0, W = 0); running requests that already miss their SLO do not veto;
  * an admitted request joins the running ones at once (r = 0) for the candidates after it;
  * equal stringency: the earlier position in the waiting queue goes first.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List, Sequence


@dataclass
class Request:
    input_tokens: int      # W of this request
    slo: float             # latency SLO
    first_token_slo: float  # stringency: how soon the first token is due
    run_time: float = 0.0  # r_i
    g_remaining: int = 0   # G_i
    g_initial: int = 0     # the task's profiled generation length
    delta_e: float = 0.0   # dE if this request is scheduled


def finishes_after(running: Sequence[Request], i: int) -> int:
    """n_i"""
    return sum(1 for j, s in enumerate(running) if j != i and s.g_remaining > running[i].g_remaining)


def expected_latency(running: Sequence[Request], i: int, c: float, new: Request = None) -> float:
    """Eq. 3 (with `new`), or the request's expected latency as things stand (without)."""
    s = running[i]
    d_e = new.delta_e if new is not None else 0.0
    w = new.input_tokens if new is not None else 0
    return d_e + (w + finishes_after(running, i) * s.g_remaining) * c + s.run_time


def schedule(waiting: Sequence[Request], scheduled: Sequence[Request], t_max: int, c: float) -> List[int]:
    """Algorithm 1.  Returns the indices (into `waiting`) of the admitted requests, in admission order."""
    running = [replace(s) for s in scheduled]
    tokens = sum(s.input_tokens for s in running)
    order = sorted(range(len(waiting)), key=lambda i: (waiting[i].first_token_slo, i))
    admitted = []
    for i in order:
        r = waiting[i]
        if r.input_tokens + tokens < t_max:
            ok = True
            for j, s in enumerate(running):
                if expected_latency(running, j, c) < s.slo:           # only requests that meet their SLO now
                    if not expected_latency(running, j, c, r) < s.slo:
                        ok = False
            if ok:
                running.append(replace(r, run_time=0.0))
                tokens += r.input_tokens
                admitted.append(i)
    return admitted


def generation_tick(r: Request, completed: bool, reset_fraction: float = 0.05) -> Request:
    """After one iteration of token generation: G_i is decremented; if it reaches 0 and the request
    has not completed, it is reset to a fraction of its initial value (at least 1)."""
    g = r.g_remaining - 1 if r.g_remaining > 0 else 0
    if g == 0 and not completed:
        g = max(1, int(r.g_initial * reset_fraction))
    return replace(r, g_remaining=g)

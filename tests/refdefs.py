"""Second, independent statements of what the replay computes, used to pin the oracle.

None of these is the oracle's algorithm retyped: the Lindley recursion is replaced by
its max-plus closed form, the slot array by an order statistic of earlier finishes,
and the invariants are checked by a sweep over events.  Pure Python / numpy, small
inputs only.
"""
from __future__ import annotations

import numpy as np


def service_terms(prompt, out, coef):
    """(prefill, per-token decode, decode) in us for one request on a replica with
    coefficients (a, b, c, d); kctx = number of started blocks of 1024 prompt tokens."""
    a, b, c, d = (int(x) for x in coef)
    prompt, out = int(prompt), int(out)
    kctx = -(-prompt // 1024)
    per_tok = c + d * kctx
    return a + b * prompt, per_tok, out * per_tok


def lindley_finish_times(arrival, service, t_on=0):
    """Single-slot FCFS queue, closed form (max-plus unrolling of Lindley's recursion):
    finish_n = max_{k<=n} ( max(arrival_k, t_on) + sum_{i=k..n} service_i )."""
    arrival = np.asarray(arrival, dtype=np.int64)
    service = np.asarray(service, dtype=np.int64)
    n = arrival.shape[0]
    ready = np.maximum(arrival, int(t_on))
    csum = np.concatenate([[0], np.cumsum(service)])
    out = np.empty(n, dtype=np.int64)
    for j in range(n):
        k = np.arange(j + 1)
        out[j] = np.max(ready[k] + (csum[j + 1] - csum[k]))
    return out


def order_statistic_replay(arrival, service, B, t_on=0, t_off=None):
    """B-slot FCFS queue stated without any slot array:
    start_j = max(arrival_j, t_on, F_j), F_j = the B-th largest finish among the
    earlier *served* requests (0 when fewer than B were served).
    Returns (start, finish, rejected) lists; rejected requests have start=finish=None."""
    finishes = []
    start, finish, rejected = [], [], []
    for a, s in zip(arrival, service):
        a, s = int(a), int(s)
        top = sorted(finishes, reverse=True)
        f_b = top[B - 1] if len(top) >= B else 0
        st = max(a, int(t_on), f_b)
        if t_off is not None and st >= int(t_off):
            start.append(None); finish.append(None); rejected.append(True)
            continue
        start.append(st); finish.append(st + s); rejected.append(False)
        finishes.append(st + s)
    return start, finish, rejected


def max_concurrency(start, finish):
    """Largest number of requests in service at one instant; a request occupies
    [start, finish).  Sweep over events, departures before arrivals at equal times."""
    ev = []
    for s, f in zip(start, finish):
        if s is None:
            continue
        ev.append((int(s), 1))
        ev.append((int(f), 0))
    ev.sort()
    cur = best = 0
    for _, kind in ev:
        cur += 1 if kind == 1 else -1
        best = max(best, cur)
    return best

"""CPU oracle for request scheduling with continuous JCT calibration.  TEST INFRASTRUCTURE ONLY.

Plain Python statement of the paper's Algorithm 1 (Section 6.3, "SRJF with continuous JCT
calibration") and of the two policies it is contrasted with (Section 6.2: first-in-first-out,
and shortest-remaining-job-first with the JCT fixed when the request arrives), plus the
single-slot prefix cache of the paper's worked example (the cache holds the state of the last
request that ran).  Shares no code with the library and imports nothing from the product.

Readings: the assignment "score_min <- jct" in the printed algorithm is taken as
"score_min <- score"; n_cached is the length of the common prefix of the request with the
cached tokens, capped at n_input - 1 (one position is always computed); ties go to the request
that was pushed first; the JCT model is either the paper's default proxy n_input - n_cached or
a linear model c0 + c_input * n_input + c_cached * n_cached fitted by least squares.

pick_multi is the same selection when the cache holds several entries (n_cached = the best
any entry offers); with one entry it is pick.

Pinned by tests/test_scheduler.py: the paper's A/B/C/D example (orders and hit counts it
states), brute-force enumeration of the score on small queues (one and several entries), and
numpy's lstsq for the fit.
"""
from __future__ import annotations

import numpy as np


def common_prefix(a, b) -> int:
    n = 0
    for x, y in zip(a, b):
        if x != y:
            break
        n += 1
    return n


def n_cached(tokens, cached) -> int:
    return min(common_prefix(tokens, cached), len(tokens) - 1)


def n_cached_any(tokens, entries) -> int:
    """With a cache of several entries a request reuses the one that spares it most."""
    return max((n_cached(tokens, e) for e in entries), default=0)


def proxy_jct(n_input: int, n_hit: int) -> float:
    """The paper's default JCT proxy: the number of tokens that miss the prefix cache."""
    return float(n_input - n_hit)


def linear_jct(c0: float, c_input: float, c_cached: float):
    return lambda n_input, n_hit: c0 + c_input * n_input + c_cached * n_hit


def fit_linear_jct(n_input, n_hit, jct):
    """Least-squares fit of jct ~ c0 + c_input * n_input + c_cached * n_cached (Section 6.3)."""
    A = np.stack([np.ones(len(n_input)), np.asarray(n_input, dtype=np.float64),
                  np.asarray(n_hit, dtype=np.float64)], axis=1)
    coef, *_ = np.linalg.lstsq(A, np.asarray(jct, dtype=np.float64), rcond=None)
    return tuple(float(c) for c in coef)


def pick(queue, cached, now: float, lam: float, jct=proxy_jct):
    """Algorithm 1.  queue: list of (id, tokens, arrival_time) in push order.
    Returns (index in queue, n_cached of the pick), or (None, 0) for an empty queue."""
    best, best_score, best_hit = None, float("inf"), 0
    for i, (_, tokens, arrival) in enumerate(queue):
        hit = n_cached(tokens, cached)
        score = jct(len(tokens), hit) - lam * (now - arrival)
        if score < best_score:
            best, best_score, best_hit = i, score, hit
    return best, best_hit


def pick_multi(queue, entries, now: float, lam: float, jct=proxy_jct):
    """Algorithm 1 with n_cached taken over a cache of several entries (lists of token ids)."""
    best, best_score, best_hit = None, float("inf"), 0
    for i, (_, tokens, arrival) in enumerate(queue):
        hit = n_cached_any(tokens, entries)
        score = jct(len(tokens), hit) - lam * (now - arrival)
        if score < best_score:
            best, best_score, best_hit = i, score, hit
    return best, best_hit


def run_queue(requests, policy: str, lam: float = 0.0, jct=proxy_jct):
    """All requests are waiting at time 0 and run one after another; the prefix cache holds
    the tokens of the request that ran last (the example's "can only store the state of one
    request").  policy: "fifo" | "srjf" (JCT fixed at arrival, empty cache) | "calibrated".
    requests: list of (id, tokens).  Returns (order of ids, number of requests that hit)."""
    queue = [(rid, tok, 0.0) for rid, tok in requests]
    cached, order, hits = [], [], 0
    while queue:
        if policy == "fifo":
            i = 0
        elif policy == "srjf":
            i = min(range(len(queue)), key=lambda j: (jct(len(queue[j][1]), 0), j))
        elif policy == "calibrated":
            i, _ = pick(queue, cached, 0.0, lam, jct)
        else:
            raise ValueError(policy)
        rid, tok, _ = queue.pop(i)
        hits += 1 if n_cached(tok, cached) > 0 else 0
        cached = list(tok)
        order.append(rid)
    return order, hits

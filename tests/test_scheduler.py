"""Scheduling (Section 6.3, Algorithm 1): the oracle against the paper's worked example and
brute force, the library's host-side scheduler against the oracle.  No GPU."""
import itertools
import os

import numpy as np
import pytest

from oracle import scheduler_oracle as S
from paper_2505_07203_amd import binding as B

HERE = os.path.dirname(os.path.abspath(__file__))


def example_requests():
    """Lengths A < C < B < D; A and D share a prefix, B and C share another one."""
    p1, p2 = list(range(1000, 1800)), list(range(5000, 5800))
    return [("A", p1 + list(range(100))), ("B", p2 + list(range(200, 1100))),
            ("C", p2 + list(range(2000, 2500))), ("D", p1 + list(range(3000, 4200)))]


def golden_example():
    rows = {}
    for line in open(os.path.join(HERE, "golden", "scheduling_example.txt")):
        if line.strip() and not line.startswith("#"):
            policy, order, hits = line.split()
            rows[policy] = (order.split(","), int(hits))
    return rows


def test_oracle_reproduces_the_papers_example():
    reqs = example_requests()
    lens = {k: len(v) for k, v in reqs}
    assert lens["A"] < lens["C"] < lens["B"] < lens["D"]
    for policy, (order, hits) in golden_example().items():
        got_order, got_hits = S.run_queue(reqs, policy)
        assert (got_order, got_hits) == (order, hits), policy


def test_oracle_pick_is_the_argmin_of_the_score():
    """Brute force: enumerate the scores by hand on small random queues."""
    rng = np.random.default_rng(0)
    for _ in range(200):
        cached = rng.integers(0, 3, rng.integers(0, 12)).tolist()
        queue = [(i, rng.integers(0, 3, rng.integers(1, 12)).tolist(), float(rng.uniform(0, 5))) for i in range(rng.integers(1, 6))]
        now, lam = 6.0, float(rng.choice([0.0, 0.5, 500.0]))
        scores = []
        for _, t, arr in queue:
            m = 0
            while m < min(len(t) - 1, len(cached)) and t[m] == cached[m]:
                m += 1
            scores.append((len(t) - m) - lam * (now - arr))
        i, hit = S.pick(queue, cached, now, lam)
        assert scores[i] == min(scores) and i == scores.index(min(scores))
        assert hit == S.n_cached(queue[i][1], cached)
    assert S.pick([], [], 0.0, 1.0) == (None, 0)


def test_starvation_term():
    """A long request that has waited long enough overtakes a short fresh one (lambda > 0 only)."""
    queue = [(0, list(range(5000)), 0.0), (1, list(range(100)), 9.9)]
    assert S.pick(queue, [], 10.0, 0.0)[0] == 1
    assert S.pick(queue, [], 10.0, 500.0)[0] == 0          # 5000 - 500*10 < 100 - 500*0.1


def test_library_scheduler_matches_oracle():
    rng = np.random.default_rng(1)
    for trial in range(30):
        lam = float(rng.choice([0.0, 3.0, 500.0]))
        sch = B.Scheduler(lam)
        linear = trial % 3 == 0
        jct = S.proxy_jct
        if linear:
            c = (float(rng.uniform(0, 5)), float(rng.uniform(0.5, 2)), float(-rng.uniform(0.1, 0.9)))
            sch.po_sched_set_jct_model(*c)
            jct = S.linear_jct(*c)
        queue, cached, now = [], [], 0.0
        for step in range(40):
            if rng.random() < 0.6 or not queue:
                base = cached[:rng.integers(0, len(cached) + 1)] if rng.random() < 0.5 else []
                tok = list(base) + rng.integers(0, 50, rng.integers(1, 30)).tolist()
                rid = 1000 * trial + step
                queue.append((rid, tok, now))
                sch.po_sched_push(rid, tok, now)
            else:
                i, hit = S.pick(queue, cached, now, lam, jct)
                rid, hit_lib = sch.po_sched_pick(cached, now)
                assert (rid, hit_lib) == (queue[i][0], hit)
                cached = queue.pop(i)[1]
            now += float(rng.uniform(0, 0.5))
            assert sch.po_sched_size() == len(queue)
        sch.po_sched_destroy()


def test_oracle_pick_multi_by_brute_force():
    rng = np.random.default_rng(5)
    for _ in range(200):
        entries = [rng.integers(0, 3, rng.integers(0, 12)).tolist() for _ in range(rng.integers(0, 4))]
        queue = [(i, rng.integers(0, 3, rng.integers(1, 12)).tolist(), float(rng.uniform(0, 5))) for i in range(rng.integers(1, 6))]
        now, lam = 6.0, float(rng.choice([0.0, 0.5, 500.0]))
        scores, hits = [], []
        for _, t, arr in queue:
            best = 0
            for e in entries:
                m = 0
                while m < min(len(t) - 1, len(e)) and t[m] == e[m]:
                    m += 1
                best = max(best, m)
            hits.append(best)
            scores.append((len(t) - best) - lam * (now - arr))
        i, hit = S.pick_multi(queue, entries, now, lam)
        assert i == scores.index(min(scores)) and hit == hits[i]
        if len(entries) == 1:
            assert (i, hit) == S.pick(queue, entries[0], now, lam)


def test_library_pick_multi_matches_oracle():
    """A cache of three entries replaced least-recently-used first, as the library's K/V cache does."""
    rng = np.random.default_rng(7)
    for trial in range(20):
        lam = float(rng.choice([0.0, 3.0]))
        sch = B.Scheduler(lam)
        queue, entries, now = [], [], 0.0
        for step in range(50):
            if rng.random() < 0.6 or not queue:
                src = entries[rng.integers(0, len(entries))] if entries and rng.random() < 0.6 else []
                tok = list(src[:rng.integers(0, len(src) + 1)]) + rng.integers(0, 50, rng.integers(1, 30)).tolist()
                rid = 1000 * trial + step
                queue.append((rid, tok, now))
                sch.po_sched_push(rid, tok, now)
            else:
                i, hit = S.pick_multi(queue, entries, now, lam)
                assert sch.po_sched_pick_multi(entries, now) == (queue[i][0], hit)
                entries = (entries + [queue.pop(i)[1]])[-3:]
            now += float(rng.uniform(0, 0.5))
        assert sch.po_sched_size() == len(queue)
        sch.po_sched_destroy()
    sch = B.Scheduler(0.0)
    assert sch.po_sched_pick_multi([], 0.0) == (-1, 0)
    sch.po_sched_push(1, [1, 2, 3], 0.0)
    assert sch.po_sched_pick_multi([], 0.0) == (1, 0)


def test_library_matches_long_prefixes_exactly():
    """Common prefixes longer than the library's 64-token compare blocks, ending at every offset inside a block."""
    rng = np.random.default_rng(11)
    base = rng.integers(0, 1000, 700).tolist()
    for m in (0, 1, 63, 64, 65, 127, 128, 129, 191, 300, 511, 512, 513, 699):
        sch = B.Scheduler(0.0)
        req = base[:m] + [1001] + rng.integers(0, 1000, 40).tolist()         # differs from the cache at position m
        sch.po_sched_push(5, req, 0.0)
        assert sch.po_sched_pick(base, 0.0) == (5, m)
        assert S.n_cached(req, base) == m
        sch.po_sched_push(6, base[:m + 1] if m < 699 else base, 0.0)          # wholly inside the cache: capped at len - 1
        rid, hit = sch.po_sched_pick_multi([base[:10], base], 0.0)
        assert rid == 6 and hit == (m if m < 699 else 699)


def test_library_scheduler_on_the_papers_example():
    want = golden_example()["calibrated"]
    sch = B.Scheduler(0.0)
    for rid, (name, tok) in enumerate(example_requests()):
        sch.po_sched_push(rid, tok, 0.0)
    names = [n for n, _ in example_requests()]
    toks = dict(enumerate(t for _, t in example_requests()))
    cached, order, hits = [], [], 0
    while sch.po_sched_size():
        rid, hit = sch.po_sched_pick(cached, 0.0)
        order.append(names[rid])
        hits += hit > 0
        cached = toks[rid]
    assert (order, hits) == want
    assert sch.po_sched_pick(cached, 0.0) == (-1, 0)


def test_jct_model_fit_matches_lstsq():
    """Section 6.3: a linear model on profiled (n_input, n_cached) pairs at 1000-token granularity."""
    rng = np.random.default_rng(2)
    pairs = [(n, c) for n in range(1000, 33000, 1000) for c in range(0, n, 4000)]
    n_in = np.array([p[0] for p in pairs]); n_c = np.array([p[1] for p in pairs])
    jct = 3.0 + 0.019 * n_in - 0.012 * n_c + rng.normal(0, 0.5, len(pairs))
    want = S.fit_linear_jct(n_in, n_c, jct)
    sch = B.Scheduler(500.0)
    got = sch.po_sched_fit_jct_model(n_in, n_c, jct)
    assert np.allclose(got, want, rtol=1e-9, atol=1e-9)
    # closed form: exact data are recovered exactly
    got2 = sch.po_sched_fit_jct_model(n_in, n_c, 1.0 + 2.0 * n_in - 0.5 * n_c)
    assert np.allclose(got2, (1.0, 2.0, -0.5), rtol=1e-10, atol=1e-8)
    with pytest.raises(B.PoError):
        sch.po_sched_fit_jct_model([1, 2, 3], [2, 4, 6], [1.0, 2.0, 3.0])      # collinear


def test_scheduler_argument_errors():
    sch = B.Scheduler(1.0)
    with pytest.raises(B.PoError):
        sch.po_sched_push(1, [], 0.0)
    with pytest.raises(B.PoError):
        B.Scheduler(-1.0)

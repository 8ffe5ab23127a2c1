"""Pins for oracle/projection.py. The paper prints no worked example for this step
(parity unpinned); the reading is pinned by a hand-worked case, by brute-force
recounts written independently here, and by structural invariants. No GPU."""
import json
import os
from collections import deque
from fractions import Fraction

import numpy as np
import pytest

from oracle import mips, projection as P
from paper_2409_10516_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_worked_example():
    g = json.load(open(os.path.join(GOLD, "projection_hand.json")))
    L = np.array(g["L"])
    pop = P.popularity(L, g["N"])
    assert pop.tolist() == g["pop"]
    assert P.popularity_order(pop).tolist() == g["pi"]
    for key, c in g["cooccurrence"].items():
        a, b = map(int, key.split(","))
        assert P.cooccurrence_of(L, a).get(b, 0) == c
        assert P.cooccurrence_of(L, b).get(a, 0) == c
    for a, want in g["ranked"].items():
        assert P.ranked_candidates(L, int(a), pop) == want
    adj, entry = P.project(L, g["N"], g["deg"])
    assert entry == g["entry"]
    assert adj.tolist() == g["adj"]


def test_equal_jaccard_prefers_larger_count_then_lower_id():
    # key 0 is in two lists; key 1 shares both and is in two more (J = 2/4);
    # keys 2 and 3 share one list each and are nowhere else (J = 1/2): a three-way
    # tie in J, broken by c (key 1 first), then by id (2 before 3).
    L = np.array([[0, 1, 3], [0, 1, 2], [1, 4, 5], [1, 6, 7]])
    pop = P.popularity(L, 8)
    assert P.ranked_candidates(L, 0, pop) == [1, 2, 3]


def _brute_counts(L, N):
    pop = [0] * N
    c = {}
    for row in L:
        for x in row:
            pop[int(x)] += 1
        for i in range(len(row)):
            for j in range(len(row)):
                if i != j:
                    key = (int(row[i]), int(row[j]))
                    c[key] = c.get(key, 0) + 1
    return pop, c


def _check_graph(L, N, deg, adj, entry):
    pop, c = _brute_counts(L, N)
    assert pop == P.popularity(L, N).tolist()
    order = sorted(range(N), key=lambda i: (-pop[i], i))
    assert entry == order[0]
    pos = {k: t for t, k in enumerate(order)}
    for a in range(N):
        row = [int(x) for x in adj[a]]
        valid = [x for x in row if x >= 0]
        assert row[:len(valid)] == valid, "padding must be at the end"
        assert a not in valid and len(set(valid)) == len(valid)
        assert all(0 <= x < N for x in valid)
        kids = [order[t] for t in (2 * pos[a] + 1, 2 * pos[a] + 2) if t < N]
        assert valid[:len(kids)] == kids
        rest = valid[len(kids):]
        cand = [b for (x, b) in c if x == a]
        # independent ranking with exact fractions
        rank = sorted(cand, key=lambda b: (-Fraction(c[(a, b)], pop[a] + pop[b] - c[(a, b)]),
                                           -c[(a, b)], b))
        want = [b for b in rank if b not in kids][:deg - len(kids)]
        assert rest == want
    # reachability: BFS from entry covers every key
    seen = {entry}
    dq = deque([entry])
    while dq:
        u = dq.popleft()
        for v in adj[u]:
            v = int(v)
            if v >= 0 and v not in seen:
                seen.add(v)
                dq.append(v)
    assert len(seen) == N


@pytest.mark.parametrize("seed,N,M,knn,deg", [(0, 40, 12, 5, 6), (1, 64, 30, 6, 8),
                                              (2, 33, 50, 4, 3), (3, 20, 3, 7, 16)])
def test_invariants_and_brute_force_recount(seed, N, M, knn, deg):
    w = synth.make_integer_case(seed, N=N, M=M, d=16, knn=knn, deg=deg)
    L, _ = mips.knn_lists(w.Q_prefill[0, 0].numpy(), w.K[0, 0].numpy(), knn)
    adj, entry = P.project(L, N, deg)
    _check_graph(L, N, deg, adj, entry)


def test_cooccurrence_is_symmetric_and_rows_option():
    r = np.random.default_rng(5)
    L = np.array([r.choice(50, size=6, replace=False) for _ in range(40)])
    for a in range(0, 50, 7):
        for b, c in P.cooccurrence_of(L, a).items():
            assert P.cooccurrence_of(L, b)[a] == c
    full, e1 = P.project(L, 50, 8)
    part, e2 = P.project(L, 50, 8, rows=[3, 11, 49])
    assert e1 == e2
    for a in (3, 11, 49):
        assert part[a].tolist() == full[a].tolist()
    assert (part[0] == -1).all()


def test_degree_two_is_backbone_only_and_deg_below_two_rejected():
    L = np.array([[0, 1, 2], [2, 3, 4]])
    adj, entry = P.project(L, 6, 2)
    assert entry == 2 and adj.shape == (6, 2)
    with pytest.raises(ValueError):
        P.project(L, 6, 1)

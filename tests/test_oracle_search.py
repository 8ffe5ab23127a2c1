"""Pins for oracle/search.py and oracle/decode.py: hand traces, the exhaustive-beam
invariant, structural checks, the decision-gap report, and the opt-in float32 score against
float64. No GPU."""
import json
import os

import numpy as np
import pytest

from oracle import attention as A, decode as D, mips, projection as P, search as S
from paper_2409_10516_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_traced_path_graph():
    g = json.load(open(os.path.join(GOLD, "search_hand.json")))
    adj = np.array(g["adj"])
    q = np.zeros(16); q[0] = 1.0
    for case in g["cases"]:
        K = np.zeros((6, 16)); K[:, 0] = case["scores"]
        ids, st = S.greedy_search(q, K, adj, case["entry"], case["ef"], case["topk"],
                                  case["expand"])
        assert ids.tolist() == case["ids"], case
        for key in ("n_visited", "n_expanded", "n_iters"):
            assert st[key] == case[key], (key, case)


def test_score32_against_float64_and_exact_on_integers():
    r = np.random.default_rng(0)
    q = r.normal(size=128).astype(np.float32)
    K = r.normal(size=(500, 128)).astype(np.float32)
    s = S.score32(q, K)
    ref = K.astype(np.float64) @ q.astype(np.float64)
    bound = 1e-5 * np.linalg.norm(q.astype(np.float64)) * np.linalg.norm(K.astype(np.float64), axis=1)
    assert s.dtype == np.float32 and np.all(np.abs(s - ref) <= bound)
    qi = r.integers(-4, 5, size=128).astype(np.float32)
    Ki = r.integers(-4, 5, size=(300, 128)).astype(np.float32)
    assert np.array_equal(S.score32(qi, Ki).astype(np.float64), Ki.astype(np.float64) @ qi)
    # a dropped chunk or a transposed operand would show here
    e = np.zeros((128, 128), np.float32); np.fill_diagonal(e, 1)
    assert np.array_equal(S.score32(q, e), q)
    with pytest.raises(ValueError):
        S.score32(np.zeros(10), np.zeros((1, 10)))


def test_score32_identical_rows_score_identically():
    r = np.random.default_rng(1)
    q = r.normal(size=128).astype(np.float32)
    k = r.normal(size=128).astype(np.float32)
    s = S.score32(q, np.stack([k] * 5 + [k[::-1]]))
    assert len(set(s[:5].tolist())) == 1


def _graph(seed, N=64, M=24, knn=6, deg=8, d=16):
    w = synth.make_integer_case(seed, N=N, M=M, d=d, knn=knn, deg=deg)
    K = w.K[0, 0].numpy(); V = w.V[0, 0].numpy()
    adj, entry, L = D.build_index(K, w.Q_prefill[0, 0].numpy(), deg, knn)
    return w, K, V, adj, entry


@pytest.mark.parametrize("seed", range(4))
@pytest.mark.parametrize("expand", [1, 3, 8])
def test_exhaustive_beam_returns_bruteforce_topk(seed, expand):
    """With ef >= N nothing is ever dropped and the backbone reaches every key, so
    the result is the exact top-k over the non-static ids."""
    w, K, V, adj, entry = _graph(seed)
    W = A.static_ids(64, 2, 4)
    for q in w.q_decode[:, 0, 0].numpy():
        ids, st = S.greedy_search(q, K, adj, entry, ef=64, topk=7, expand=expand, exclude=W)
        assert ids.tolist() == mips.topk_bruteforce(q, K, 7, exclude=W).tolist()
        assert st["n_visited"] == 64


def test_complete_graph_one_expansion_suffices():
    r = np.random.default_rng(3)
    N = 30
    K = r.integers(-3, 4, size=(N, 16)).astype(np.float32)
    q = r.integers(-3, 4, size=16).astype(np.float32)
    adj = np.array([[j for j in range(N) if j != i] for i in range(N)])
    ids, st = S.greedy_search(q, K, adj, 4, ef=5, topk=5)
    assert ids.tolist() == mips.topk_bruteforce(q, K, 5).tolist()
    assert st["n_visited"] == N


@pytest.mark.parametrize("expand", [1, 2, 5])
def test_structural_invariants(expand):
    w = synth.make_config0(N=512, M=128, T=4, window=16)
    K = w.K[0, 0].numpy()
    adj, entry, _ = D.build_index(K, w.Q_prefill[0, 0].numpy(), 8, 8)
    W = A.static_ids(512, 4, 16)
    for q in w.q_decode[:, 0, 0].numpy():
        ids, st = S.greedy_search(q, K, adj, entry, ef=24, topk=10, expand=expand, exclude=W)
        beam = st["beam"]
        assert len(beam) <= 24 and st["n_visited"] <= 1 + st["n_expanded"] * 8
        keys = [(-s, i) for s, i in beam]
        assert keys == sorted(keys)
        for s, i in beam:
            assert abs(s - float(K[i].astype(np.float64) @ q.astype(np.float64))) <= 1e-12 * abs(s)
        valid = ids[ids >= 0]
        assert not set(valid.tolist()) & set(W.tolist())
        assert valid.tolist() == [i for _, i in beam if i not in set(W.tolist())][:10]
        assert st["n_returned"] == len(valid)


def test_argument_checks_and_padding():
    w, K, V, adj, entry = _graph(0)
    q = w.q_decode[0, 0, 0].numpy()
    with pytest.raises(ValueError):
        S.greedy_search(q, K, adj, entry, ef=3, topk=5)
    ids, st = S.greedy_search(q, K, adj, entry, ef=64, topk=64, exclude=np.arange(60))
    assert st["n_returned"] == 4 and (ids[4:] == -1).all() and (ids[:4] >= 60).all()


@pytest.mark.parametrize("seed", range(3))
def test_decode_with_everything_retrieved_is_full_attention(seed):
    """Sparse + static merge with every non-static token retrieved equals Eq. 1."""
    w, K, V, adj, entry = _graph(seed)
    for q in w.q_decode[:, 0, 0].numpy():
        out, lse, ids, st = D.decode_step(q, K, V, adj, entry, sink=2, window=4,
                                          topk=58, ef=64, expand=2)
        of, lf = A.full_attention(q, K, V)
        assert np.allclose(out, of, rtol=1e-12, atol=1e-13) and np.isclose(lse, lf)
        assert sorted(ids.tolist()) == list(range(2, 60))


def test_decode_equals_attention_over_static_plus_retrieved():
    w, K, V, adj, entry = _graph(1)
    q = w.q_decode[0, 0, 0].numpy()
    out, lse, ids, st = D.decode_step(q, K, V, adj, entry, 2, 4, topk=5, ef=12)
    both = np.concatenate([A.static_ids(64, 2, 4), ids[ids >= 0]])
    o2, l2 = A.partial_attention(q, K, V, both)
    assert np.allclose(out, o2, rtol=1e-12, atol=1e-13) and np.isclose(lse, l2)


def test_config0_planted_duplicates_tie_break_and_recall_band():
    """Config 0: the 8 planted rows of a decode query are bit-identical, so they tie
    exactly and must come out in ascending id order when found."""
    w = synth.make_config0()
    K = w.K[0, 0].numpy()
    adj, entry, L = D.build_index(K, w.Q_prefill[0, 0].numpy(), w.deg, w.knn)
    W = A.static_ids(w.N, w.sink, w.window)
    rec = []
    for t in range(4):
        q = w.q_decode[t, 0, 0].numpy()
        ids, st = S.greedy_search(q, K, adj, entry, w.ef, w.topk, expand=1, exclude=W)
        truth = mips.topk_bruteforce(q, K, w.topk, exclude=W)
        planted = set(w.planted[t].tolist())
        assert planted <= set(truth.tolist())
        found = [i for i in ids.tolist() if i in planted]
        assert found == sorted(found)
        rec.append(mips.recall(ids, truth))
    assert 0.3 < np.mean(rec) <= 1.0


def test_default_scores_are_float64_and_the_float32_order_is_opt_in():
    """On integer-valued inputs every arithmetic is exact, so the two score functions give the
    same walk; on real-valued inputs the default beam carries float64 inner products and the
    opt-in one float32 values."""
    w, K, V, adj, entry = _graph(2)
    q = w.q_decode[0, 0, 0].numpy()
    a = S.greedy_search(q, K, adj, entry, ef=12, topk=5, expand=2)
    b = S.greedy_search(q, K, adj, entry, ef=12, topk=5, expand=2, score_fn=S.score32)
    assert a[0].tolist() == b[0].tolist() and a[1]["beam"] == b[1]["beam"]
    w2 = synth.make_config0(N=256, M=64, T=1, window=8)
    K2 = w2.K[0, 0].numpy(); q2 = w2.q_decode[0, 0, 0].numpy()
    adj2, e2, _ = D.build_index(K2, w2.Q_prefill[0, 0].numpy(), 8, 8)
    _, st64 = S.greedy_search(q2, K2, adj2, e2, ef=16, topk=4)
    _, st32 = S.greedy_search(q2, K2, adj2, e2, ef=16, topk=4, score_fn=S.score32)
    ref = K2.astype(np.float64) @ q2.astype(np.float64)
    assert all(abs(s - ref[i]) <= 1e-12 * abs(s) for s, i in st64["beam"])
    assert all(np.float32(s) == s for s, i in st32["beam"])
    assert any(abs(s - ref[i]) > 1e-9 * abs(s) for s, i in st32["beam"])


def test_min_gap_reports_the_closest_decision():
    """A path graph 0-1-2-3-4-5 walked from node 0 with scores chosen by hand. The decisions:
    ef = 2 drops the worse of three entries after each step, the result orders its two ids."""
    adj = np.array([[1, -1], [0, 2], [1, 3], [2, 4], [3, 5], [4, -1]])
    q = np.zeros(16); q[0] = 1.0
    K = np.zeros((6, 16)); K[:, 0] = [1.0, 2.0, 4.0, 4.0 + 4e-6, 3.0, 0.5]
    ids, st = S.greedy_search(q, K, adj, 0, ef=2, topk=2)
    assert ids.tolist() == [3, 2]
    assert abs(st["min_gap"] - 4e-6 / (4.0 + 4e-6)) < 1e-12        # the order of 3 and 2 in the result
    K[3, 0] = 8.0
    ids, st = S.greedy_search(q, K, adj, 0, ef=2, topk=2)
    # closest decision now: beam {3: 8, 2: 4} against the newcomer 4 (score 3) at the cut: |4 - 3| / 4
    assert ids.tolist() == [3, 2] and abs(st["min_gap"] - 0.25) < 1e-12
    # bit-identical rows tie exactly in any arithmetic: decided by id, not reported as a gap
    K[:, 0] = [1.0, 2.0, 4.0, 4.0, 0.25, 0.125]
    ids, st = S.greedy_search(q, K, adj, 0, ef=3, topk=2)
    assert ids.tolist() == [2, 3] and st["min_gap"] > 0.4


def test_hand_traced_walks_from_a_seed_set():
    g = json.load(open(os.path.join(GOLD, "search_hand.json")))
    adj = np.array(g["adj"])
    q = np.zeros(16); q[0] = 1.0
    for case in g["seed_cases"]:
        K = np.zeros((6, 16)); K[:, 0] = case["scores"]
        ids, st = S.greedy_search(q, K, adj, case["seeds"][0], case["ef"], case["topk"], case["expand"],
                                  seeds=case["seeds"])
        assert ids.tolist() == case["ids"], case
        for key in ("n_visited", "n_expanded", "n_iters"):
            assert st[key] == case[key], (key, case)


def test_backbone_seeds_are_the_most_popular_keys_of_a_projected_graph():
    """For a graph made by projection.py the first two slots of a row are the key's children in the
    heap over (popularity descending, id ascending), so the seeds must be that order's head,
    recomputed here from the KNN lists alone."""
    w = synth.make_config0(N=300, M=200, T=1, window=8)
    K = w.K[0, 0].numpy()
    adj, entry, L = D.build_index(K, w.Q_prefill[0, 0].numpy(), 8, 6)
    pop = np.bincount(L.ravel(), minlength=300)
    order = np.lexsort((np.arange(300), -pop))
    for R in (1, 2, 3, 10, 64, 149, 300):
        assert S.backbone_seeds(adj, entry, R).tolist() == order[:R].tolist(), R
    # a hand-made tree with a missing child and a repeated node: positions 0..6 hold
    # 4, 2, 5, -, 4(again), 1, 0
    adj2 = np.array([[-1, -1], [-1, -1], [-1, 4], [-1, -1], [2, 5], [1, 0]])
    assert S.backbone_seeds(adj2, 4, 7).tolist() == [4, 2, 5, 1, 0]
    assert S.backbone_seeds(adj2, 4, 2).tolist() == [4, 2]
    with pytest.raises(ValueError):
        S.backbone_seeds(adj2, 4, 0)


@pytest.mark.parametrize("seed", range(3))
def test_seeded_walk_invariants(seed):
    """seeds = [entry] is the single-entry walk; with ef >= N any seed set returns the exact
    top-k (every key stays reachable); seeds are counted as visited, not as expanded."""
    w, K, V, adj, entry = _graph(seed)
    W = A.static_ids(64, 2, 4)
    for q in w.q_decode[:, 0, 0].numpy():
        a = S.greedy_search(q, K, adj, entry, ef=12, topk=5, expand=2, exclude=W)
        b = S.greedy_search(q, K, adj, entry, ef=12, topk=5, expand=2, exclude=W, seeds=[entry])
        assert a[0].tolist() == b[0].tolist() and a[1] == b[1]
        sd = S.backbone_seeds(adj, entry, 9)
        ids, st = S.greedy_search(q, K, adj, entry, ef=64, topk=7, expand=3, exclude=W, seeds=sd)
        assert ids.tolist() == mips.topk_bruteforce(q, K, 7, exclude=W).tolist()
        assert st["n_visited"] == 64
        ids, st = S.greedy_search(q, K, adj, entry, ef=4, topk=2, expand=1, seeds=sd)
        assert st["n_visited"] >= 9 and st["n_expanded"] == st["n_iters"] >= 1
        out, lse, ids2, st2 = D.decode_step(q, K, V, adj, entry, 2, 4, topk=5, ef=12, expand=2, n_seeds=9)
        ids3, _ = S.greedy_search(q, K, adj, entry, 12, 5, 2, exclude=W, seeds=sd)
        assert ids2.tolist() == ids3.tolist()
    with pytest.raises(ValueError):
        S.greedy_search(q, K, adj, entry, ef=4, topk=2, seeds=[1, 1])

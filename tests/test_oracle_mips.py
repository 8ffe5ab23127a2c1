"""Pins for oracle/mips.py: library stable sort, brute force, tie-breaks. No GPU."""
import numpy as np
import pytest

from oracle import mips


def _loop_topk(q, K, k, exclude=()):
    """Selection by repeated scan, written independently of mips.py."""
    s = [float(sum(float(a) * float(b) for a, b in zip(q, row))) for row in K]
    left = [i for i in range(len(s)) if i not in set(exclude)]
    out = []
    while left and len(out) < k:
        best = left[0]
        for i in left[1:]:
            if s[i] > s[best] or (s[i] == s[best] and i < best):
                best = i
        out.append(best)
        left.remove(best)
    return out


@pytest.mark.parametrize("seed", range(3))
def test_topk_matches_scan_and_stable_sort(seed):
    r = np.random.default_rng(seed)
    K = r.integers(-3, 4, size=(60, 6)).astype(float)      # many exact ties
    q = r.integers(-3, 4, size=6).astype(float)
    got = mips.topk_bruteforce(q, K, 10, exclude=[0, 5, 59])
    assert got.tolist() == _loop_topk(q, K, 10, exclude=[0, 5, 59])
    s = K @ q
    lib = np.argsort(-s, kind="stable")                    # stable => lower id first
    assert mips.topk_bruteforce(q, K, 60).tolist() == lib.tolist()


def test_duplicate_keys_lower_id_wins():
    K = np.array([[1.0, 0], [2.0, 0], [2.0, 0], [0.5, 0], [2.0, 0]])
    assert mips.topk_bruteforce([1.0, 0], K, 3).tolist() == [1, 2, 4]
    assert mips.topk_bruteforce([1.0, 0], K, 3, exclude=[1]).tolist() == [2, 4, 0]
    assert mips.topk_bruteforce([1.0, 0], K, 9).tolist() == [1, 2, 4, 0, 3]


@pytest.mark.parametrize("seed", range(2))
def test_knn_lists_rows_are_bruteforce(seed):
    r = np.random.default_rng(10 + seed)
    K = r.integers(-2, 3, size=(40, 5)).astype(float)
    Q = r.integers(-2, 3, size=(7, 5)).astype(float)
    L, S = mips.knn_lists(Q, K, 6, chunk=3)
    for j in range(7):
        assert L[j].tolist() == _loop_topk(Q[j], K, 6)
        assert np.array_equal(S[j], (K @ Q[j])[L[j]])
    with pytest.raises(ValueError):
        mips.knn_lists(Q, K, 41)


def test_knn_is_non_causal_and_unscaled():
    # the last key is the best match for the first query: it must be listed
    K = np.eye(4)
    Q = np.array([[0, 0, 0, 5.0], [1.0, 0, 0, 0]])
    L, S = mips.knn_lists(Q, K, 1)
    assert L[:, 0].tolist() == [3, 0] and S[:, 0].tolist() == [5.0, 1.0]


def test_recall():
    assert mips.recall([1, 2, 3, -1], [1, 2, 3, 4]) == 0.75
    assert mips.recall([4, 3, 2, 1], [1, 2, 3, 4]) == 1.0
    assert mips.recall([], [1, 2]) == 0.0
    assert mips.recall([7, 8], [-1, -1]) == 1.0


def test_rerank_is_bruteforce_restricted_to_the_candidates():
    """rerank(q, K, cand, k) must equal the exact top-k over all keys with everything outside
    `cand` excluded; -1 entries are ignored and short lists are padded."""
    rng = np.random.default_rng(11)
    K = rng.standard_normal((400, 32))
    q = rng.standard_normal(32)
    cand = rng.choice(400, size=60, replace=False)
    outside = np.setdiff1d(np.arange(400), cand)
    want = mips.topk_bruteforce(q, K, 10, exclude=outside)
    got = mips.rerank(q, K, np.concatenate([cand[:30], [-1, -1], cand[30:]]), 10)
    assert got.tolist() == want.tolist()
    short = mips.rerank(q, K, [5, -1, 9], 4)
    assert sorted(short[:2].tolist()) == [5, 9] and short[2:].tolist() == [-1, -1]
    assert mips.rerank(q, K, [-1, -1], 3).tolist() == [-1, -1, -1]

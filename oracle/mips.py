"""Maximum-inner-product order, brute-force top-k, exact KNN lists, recall
(test oracle; see package header).

Similarity is the unscaled inner product (Sec. 2.4: a key is critical for a query
when their inner product is large). One total order is used everywhere:
x beats y iff score_x > score_y, or the scores are equal and id_x < id_y.
"""
import numpy as np


def rank_order(scores, ids):
    """Indices that sort (scores, ids) best-first under the total order above."""
    scores = np.asarray(scores)
    ids = np.asarray(ids)
    return np.lexsort((ids, -scores))


def scores_f64(q, K):
    """<q, k_i> for every key, float64."""
    return np.asarray(K, np.float64) @ np.asarray(q, np.float64)


def topk_bruteforce(q, K, k, exclude=None, score_fn=None):
    """Exact top-k by linear scan (the paper's "Flat" baseline, Sec. 4.1), skipping
    the ids in `exclude`. Returns ids best-first (fewer than k if fewer eligible).
    Scores are float64 inner products unless `score_fn(q, K)` is given (used to take the
    decision in the float32 order of oracle/search.py when a device scan is checked)."""
    s = scores_f64(q, K) if score_fn is None else np.asarray(score_fn(q, K))
    ids = np.arange(s.shape[0], dtype=np.int64)
    if exclude is not None and len(exclude):
        keep = np.ones(s.shape[0], bool)
        keep[np.asarray(exclude, np.int64)] = False
        ids, s = ids[keep], s[keep]
    o = rank_order(s, ids)[:k]
    return ids[o]


def knn_lists(Q, K, knn, chunk=2048):
    """Exact KNN of Sec. 3.2 / Fig. 2b: for each prefill query (row of Q) the ids of
    its `knn` best keys over ALL keys (non-causal), best-first. Returns
    (ids int32 [M][knn], scores float64 [M][knn])."""
    Q = np.asarray(Q, np.float64)
    K = np.asarray(K, np.float64)
    M, N = Q.shape[0], K.shape[0]
    if knn > N:
        raise ValueError("knn > N")
    out = np.empty((M, knn), np.int32)
    sc = np.empty((M, knn), np.float64)
    all_ids = np.arange(N)
    for s0 in range(0, M, chunk):
        S = Q[s0:s0 + chunk] @ K.T
        for r in range(S.shape[0]):
            # only rows scoring at least the knn-th largest value can be in the list
            kth = np.partition(S[r], N - knn)[N - knn]
            cand = all_ids[S[r] >= kth]
            o = cand[rank_order(S[r, cand], cand)[:knn]]
            out[s0 + r] = o
            sc[s0 + r] = S[r, o]
    return out, sc


def rerank(q, K, cand, k, score_fn=None):
    """Re-ranking of a candidate list with the keys themselves (what follows a walk over 8-bit
    keys): the best k of the distinct ids in `cand` (-1 entries ignored) under <q, K[id]>, best
    first, padded with -1 to length k. Scores as in topk_bruteforce."""
    cand = np.asarray([c for c in np.asarray(cand).tolist() if c >= 0], np.int64)
    out = np.full(k, -1, np.int32)
    if cand.size == 0:
        return out
    rows = np.asarray(K)[cand]
    s = scores_f64(q, rows) if score_fn is None else np.asarray(score_fn(q, rows))
    order = rank_order(s, cand)[:k]
    out[:order.size] = cand[order]
    return out


def recall(retrieved, truth):
    """Overlap ratio between retrieved ids and the ground-truth top-k (Sec. 2.4)."""
    truth = [int(t) for t in truth if t >= 0]
    got = set(int(r) for r in retrieved if r >= 0)
    if not truth:
        return 1.0
    return len(got.intersection(truth)) / len(truth)

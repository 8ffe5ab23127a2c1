"""Helpers shared by the tests: tensor conversion, oracle graphs, tolerance rules."""
import numpy as np
import torch

from oracle import attention as OA, decode as OD, mips as OM, projection as OP, search as OS


def to_np(t: torch.Tensor) -> np.ndarray:
    """Exact conversion of a float32/bfloat16 tensor to a float32 numpy array."""
    return t.detach().float().cpu().numpy()


def oracle_graphs(w, knn=None, deg=None):
    """Oracle KNN lists and graphs for every (seq, q head) of a workload.
    -> (adj int32 [n_seq*n_q][N][deg], entries int32 [n_seq*n_q], L [n_seq*n_q][M][knn])"""
    knn = knn or w.knn
    deg = deg or w.deg
    n_seq, n_kv, N, d = w.K.shape
    n_q = w.Q_prefill.shape[1]
    grp = n_q // n_kv
    adjs, ents, Ls = [], [], []
    for s in range(n_seq):
        for h in range(n_q):
            K = to_np(w.K[s, h // grp])
            L, _ = OM.knn_lists(to_np(w.Q_prefill[s, h]), K, knn)
            adj, entry = OP.project(L, N, deg)
            adjs.append(adj); ents.append(entry); Ls.append(L)
    return (np.stack(adjs).astype(np.int32), np.array(ents, np.int32), np.stack(Ls))


def out_close(got, ref, tol):
    """Relative bound on an attention output: max |got - ref| <= tol * max |ref|."""
    got = np.asarray(got, np.float64); ref = np.asarray(ref, np.float64)
    return np.max(np.abs(got - ref)) <= tol * max(np.max(np.abs(ref)), 1e-6)


def lse_close(got, ref, tol):
    if np.isneginf(ref):
        return np.isneginf(got)
    return abs(float(got) - float(ref)) <= tol * max(1.0, abs(float(ref)))


def tol_for(dtype):
    """Tolerances of the benchmark spec: bf16 KV with fp32 accumulate 2e-3, fp32 1e-5."""
    return 2e-3 if dtype == torch.bfloat16 else 1e-5


def knn_equivalent(L_gpu, L_ref, Q, K, rel=1e-5):
    """KNN lists may differ from the float64 oracle only where scores are nearly tied:
    row by row the lists are identical, or the float64 scores of the two lists agree
    position by position within `rel` (relative to the largest score of the row) and the
    GPU row holds distinct in-range ids. Returns the number of rows that differed."""
    L_gpu = np.asarray(L_gpu); L_ref = np.asarray(L_ref)
    assert L_gpu.shape == L_ref.shape
    N = K.shape[0]
    differing = 0
    K64 = np.asarray(K, np.float64)
    for j in range(L_gpu.shape[0]):
        if np.array_equal(L_gpu[j], L_ref[j]):
            continue
        differing += 1
        g = L_gpu[j]
        assert len(set(g.tolist())) == len(g) and g.min() >= 0 and g.max() < N, f"row {j}: bad ids"
        s = K64 @ np.asarray(Q[j], np.float64)
        tol = rel * np.max(np.abs(s))
        assert np.all(np.abs(s[g] - s[L_ref[j]]) <= tol), f"row {j}: not a near-tie difference"
    return differing


NEAR_TIE = 1e-5          # relative score gap under which ids may differ from the float64 oracle


def integer_valued(*arrays):
    """True when every value is a small integer: float32 inner products are then exact in any
    summation order and no near-tie allowance applies."""
    return all(np.array_equal(np.asarray(a), np.rint(np.asarray(a))) and np.abs(np.asarray(a)).max() < 64
               for a in arrays)


def topk_equivalent(got, ref, q, K, rel=NEAR_TIE, eligible=None):
    """An exact top-k list taken with float32 scores against the float64 one: identical, or the
    float64 scores agree position by position within `rel` of the larger magnitude and the
    device's list holds distinct eligible ids (padding in the same cells). Returns True when the
    lists were identical."""
    got = np.asarray(got); ref = np.asarray(ref)
    assert got.shape == ref.shape
    if np.array_equal(got, ref):
        return True
    assert np.array_equal(got < 0, ref < 0), "padding differs"
    g, r = got[got >= 0], ref[ref >= 0]
    assert len(set(g.tolist())) == len(g) and g.max() < K.shape[0], "bad ids"
    if eligible is not None:
        assert set(g.tolist()) <= eligible, "ineligible id"
    K64 = np.asarray(K, np.float64); q64 = np.asarray(q, np.float64)
    sg, sr = K64[g] @ q64, K64[r] @ q64
    assert np.all(np.abs(sg - sr) <= rel * np.maximum(np.abs(sg), np.abs(sr))), "not a near-tie difference"
    return False


def walk_equivalent(ids, stats4, r_ids, rst, q, K, W, rel=NEAR_TIE, exact=False):
    """A device walk against the oracle's float64 walk (oracle/search.py): ids and the four
    counters identical, or - the task's allowance for float32 scores - the oracle's walk took a
    decision between two scores closer than `rel` (rst["min_gap"]); the device's ids must then
    still be a valid result: distinct, in range, outside W, best first by float64 score within
    `rel`, padding at the end. `exact` (integer-valued inputs) allows no difference.
    Returns True when everything was identical."""
    ids = np.asarray(ids); r_ids = np.asarray(r_ids)
    want = [rst["n_visited"], rst["n_expanded"], rst["n_iters"], rst["n_returned"]]
    same = ids.tolist() == r_ids.tolist() and (stats4 is None or list(stats4) == want)
    if same:
        return True
    assert not exact, f"differs from the oracle on exact inputs: {ids.tolist()} vs {r_ids.tolist()}"
    assert rst["min_gap"] < rel, (f"differs from the float64 oracle although its closest decision "
                                  f"had a relative gap of {rst['min_gap']:.3g}")
    v = ids[ids >= 0]
    assert (ids[len(v):] == -1).all() and len(set(v.tolist())) == len(v)
    assert v.size == 0 or (v.min() >= 0 and v.max() < K.shape[0])
    assert not set(v.tolist()) & set(int(i) for i in W)
    s = np.asarray(K, np.float64)[v] @ np.asarray(q, np.float64)
    assert np.all(s[1:] <= s[:-1] + rel * np.maximum(np.abs(s[1:]), np.abs(s[:-1])))
    return False


def decode_matches(out, lse, ids, stats4, q, K, V, adj, entry, sink, window, topk, ef, expand, tol,
                   n_index=None, exact=False, score_fn=None, n_seeds=0):
    """One head of a device decode step against the oracle's (float64 scores unless `score_fn`):
    the walk by walk_equivalent, then out / lse against Eq. 2 and Eq. 4-5 over the ids the device
    returned (the oracle's own when they are identical). Returns True when ids and counters were
    identical."""
    N = np.asarray(K).shape[0]
    W = OA.static_ids(N, sink, window, n_index)
    r_out, r_lse, r_ids, rst = OD.decode_step(q, K, V, adj, entry, sink, window, topk, ef, expand,
                                              n_index=n_index, score_fn=score_fn, n_seeds=n_seeds)
    ids = np.asarray(ids)
    same = walk_equivalent(ids, stats4, r_ids, rst, q, K, W, exact=exact or score_fn is not None)
    if not same:
        o_o, l_o = OA.partial_attention(q, K, V, ids[ids >= 0])
        r_out, r_lse = OA.merge(rst["o_w"], rst["lse_w"], o_o, l_o)
    assert out_close(out, r_out, tol), "attention output"
    assert lse_close(lse, r_lse, tol), "lse"
    return same


class Tally:
    """Counts walks that used the near-tie allowance; it must stay the exception."""
    def __init__(self):
        self.n = 0
        self.differing = 0

    def add(self, same):
        self.n += 1
        self.differing += 0 if same else 1

    def check(self, frac=0.05):
        assert self.differing <= max(1, int(frac * self.n)), (self.differing, self.n)

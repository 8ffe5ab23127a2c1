"""Attention math of the paper, in float64 (test oracle; see package header).

z_i = <q, k_i> / sqrt(d)  and  o = sum_i softmax(z)_i v_i            (Eq. 1)
restricted to an index subset with the softmax renormalised over it   (Eq. 2)
and the exact combination of two disjoint subsets' partial results    (Eq. 4-5).
"""
import numpy as np


def static_ids(N, sink, window, n_index=None):
    """Static pattern W of Sec. 3.3: the first `sink` tokens and the last `window`
    tokens of the N-token context (clipped to [0, N); overlapping ranges merge).
    The paper does not say how tokens generated after the index was built are handled;
    this build attends them densely: with `n_index` given, tokens [n_index, N) join W."""
    s = set(range(0, min(max(sink, 0), N))) | set(range(max(N - max(window, 0), 0), N))
    if n_index is not None:
        s |= set(range(n_index, N))
    return np.array(sorted(s), dtype=np.int64)


def logits(q, K, ids):
    """z_i of Eq. 1 for i in ids."""
    q = np.asarray(q, np.float64)
    Ks = np.asarray(K, np.float64)[np.asarray(ids, np.int64)]
    return Ks @ q / np.sqrt(q.shape[0])


def partial_attention(q, K, V, ids):
    """Eq. 2 over the index set `ids`, in the form Appendix A writes o_W / o_Omega:
    m = max z_i, l = sum exp(z_i - m), o = sum exp(z_i - m) v_i / l.
    Returns (o[d], lse) with lse = m + ln l. An empty set gives (0, -inf)."""
    ids = np.asarray(ids, np.int64)
    d = np.asarray(q).shape[0]
    if ids.size == 0:
        return np.zeros(d, np.float64), -np.inf
    z = logits(q, K, ids)
    m = z.max()
    w = np.exp(z - m)
    l = w.sum()
    o = (w[:, None] * np.asarray(V, np.float64)[ids]).sum(axis=0) / l
    return o, m + np.log(l)


def full_attention(q, K, V):
    """Eq. 1 over every token."""
    return partial_attention(q, K, V, np.arange(np.asarray(K).shape[0]))


def gammas(lse_w, lse_o):
    """Re-scaling factors gamma_1, gamma_2 of Eq. 5. With z~ = max(z~_1, z~_2) (the
    paper leaves z~ undefined; it cancels) gamma_1 = exp(lse_W - lse) and
    gamma_2 = exp(lse_Omega - lse), lse = log(exp(lse_W) + exp(lse_Omega))."""
    if np.isneginf(lse_w) and np.isneginf(lse_o):
        raise ValueError("both partial sets are empty")
    top = max(lse_w, lse_o)
    lse = top + np.log(np.exp(lse_w - top) + np.exp(lse_o - top))
    return np.exp(lse_w - lse), np.exp(lse_o - lse), lse


def merge(o_w, lse_w, o_o, lse_o):
    """Eq. 4: o = gamma_1 o_W + gamma_2 o_Omega. Returns (o, lse)."""
    g1, g2, lse = gammas(lse_w, lse_o)
    return g1 * np.asarray(o_w, np.float64) + g2 * np.asarray(o_o, np.float64), lse

"""One decode step of Algorithm 1 for the fixed static pattern, and the index build
it depends on (test oracle; see package header)."""
import numpy as np

from . import attention, mips, projection, search


def build_index(K, Q_prefill, deg, knn):
    """Sec. 3.2: exact KNN from each prefill query to the keys, projected into a
    key-key graph. Returns (adj [N][deg], entry, L [M][knn])."""
    L, _ = mips.knn_lists(Q_prefill, K, knn)
    adj, entry = projection.project(L, np.asarray(K).shape[0], deg)
    return adj, entry, L


def decode_step(q, K, V, adj, entry, sink, window, topk, ef, expand=1, n_index=None, score_fn=None,
                n_seeds=0):
    """Algorithm 1 with PredictActiveTokens fixed to sink + window (Sec. 3.3):
    Omega = VectorSearch(q) minus the static set; o_Omega by Eq. 2 over Omega;
    o_W by Eq. 2 over W; combined by Eq. 4-5.
    Returns (out[d], lse, ids[topk], stats). `n_index` (default: all N keys) is the
    number of keys the graph was built over; later tokens are part of W. `score_fn` is
    passed to the walk (default: float64 inner products). n_seeds > 0 starts the walk from
    search.backbone_seeds(adj, entry, n_seeds) instead of the entry point alone."""
    N = np.asarray(K).shape[0]
    W = attention.static_ids(N, sink, window, n_index)
    seeds = search.backbone_seeds(adj, entry, n_seeds) if n_seeds else None
    ids, stats = search.greedy_search(q, K, adj, entry, ef, topk, expand, exclude=W, score_fn=score_fn,
                                      seeds=seeds)
    omega = ids[ids >= 0]
    o_o, l_o = attention.partial_attention(q, K, V, omega)
    o_w, l_w = attention.partial_attention(q, K, V, W)
    out, lse = attention.merge(o_w, l_w, o_o, l_o)
    stats = dict(stats, o_omega=o_o, lse_omega=l_o, o_w=o_w, lse_w=l_w)
    return out, lse, ids, stats

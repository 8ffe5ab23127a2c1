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

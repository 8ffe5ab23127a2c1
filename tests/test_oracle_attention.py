"""Pins for oracle/attention.py: the paper's closed forms, a hand-worked example,
and a library softmax. No GPU."""
import json
import os

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

from oracle import attention as A

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rand(seed, N=200, d=16):
    r = np.random.default_rng(seed)
    return r.normal(size=d) * 2, r.normal(size=(N, d)), r.normal(size=(N, d))


def test_hand_worked_example():
    g = json.load(open(os.path.join(GOLD, "attention_hand.json")))
    q = np.array(g["q"])
    K = np.zeros((4, 4))
    K[:, 0] = np.log(np.array(g["k0_exp"], float))
    V = np.array(g["V"], float)
    o, lse = A.full_attention(q, K, V)
    assert np.allclose(o, g["full_out"], rtol=0, atol=1e-14)
    assert np.isclose(np.exp(lse), g["full_lse_exp"], rtol=1e-14)
    ow, lw = A.partial_attention(q, K, V, g["W"])
    oo, lo = A.partial_attention(q, K, V, g["Omega"])
    assert np.allclose(ow, g["o_W"], atol=1e-14) and np.isclose(np.exp(lw), g["lse_W_exp"])
    assert np.allclose(oo, g["o_Omega"], atol=1e-14) and np.isclose(np.exp(lo), g["lse_Omega_exp"])
    g1, g2, l = A.gammas(lw, lo)
    assert np.isclose(g1, g["gamma1"], rtol=1e-14) and np.isclose(g2, g["gamma2"], rtol=1e-14)
    om, lm = A.merge(ow, lw, oo, lo)
    assert np.allclose(om, g["full_out"], atol=1e-14) and np.isclose(lm, lse)


@pytest.mark.parametrize("seed", range(4))
def test_library_softmax(seed):
    q, K, V = _rand(seed)
    z = K @ q / np.sqrt(q.shape[0])
    o, lse = A.full_attention(q, K, V)
    assert np.allclose(o, softmax(z) @ V, rtol=1e-12, atol=1e-13)
    assert np.isclose(lse, logsumexp(z), rtol=1e-13)
    ids = np.array([3, 17, 50, 51, 199])
    o, lse = A.partial_attention(q, K, V, ids)
    assert np.allclose(o, softmax(z[ids]) @ V[ids], rtol=1e-12, atol=1e-13)
    assert np.isclose(lse, logsumexp(z[ids]), rtol=1e-13)


def test_scale_is_inverse_sqrt_d():
    # Eq. 1: z = q.k / sqrt(d). With one key of weight e^z against a zero key:
    q = np.array([3.0, 0, 0, 0, 0, 0, 0, 0, 0])          # d = 9 -> sqrt(d) = 3
    K = np.zeros((2, 9)); K[0, 0] = 5.0                   # z = (15/3, 0) = (5, 0)
    V = np.array([[1.0] * 9, [0.0] * 9])
    o, lse = A.full_attention(q, K, V)
    assert np.isclose(o[0], np.exp(5) / (np.exp(5) + 1), rtol=1e-14)
    assert np.isclose(lse, np.log(np.exp(5) + 1), rtol=1e-14)


@pytest.mark.parametrize("seed", range(4))
def test_merge_of_static_and_rest_is_full_attention(seed):
    """Appendix A: the combined output equals attention over W u Omega; with Omega =
    every non-static token that is Eq. 1."""
    q, K, V = _rand(seed, N=300)
    W = A.static_ids(300, 4, 37)
    rest = np.setdiff1d(np.arange(300), W)
    o, lse = A.merge(*A.partial_attention(q, K, V, W), *A.partial_attention(q, K, V, rest))
    of, lf = A.full_attention(q, K, V)
    assert np.allclose(o, of, rtol=1e-12, atol=1e-13) and np.isclose(lse, lf, rtol=1e-13)


@pytest.mark.parametrize("seed", range(3))
def test_merge_any_split_commutes_and_associates(seed):
    q, K, V = _rand(seed, N=120)
    r = np.random.default_rng(100 + seed)
    perm = r.permutation(120)
    a, b, c = perm[:30], perm[30:75], perm[75:]
    pa, pb, pc = (A.partial_attention(q, K, V, s) for s in (a, b, c))
    ab = A.merge(*pa, *pb)
    ba = A.merge(*pb, *pa)
    assert np.allclose(ab[0], ba[0], rtol=1e-13) and np.isclose(ab[1], ba[1])
    left = A.merge(*ab, *pc)
    right = A.merge(*pa, *A.merge(*pb, *pc))
    full = A.full_attention(q, K, V)
    for x in (left, right):
        assert np.allclose(x[0], full[0], rtol=1e-12, atol=1e-13) and np.isclose(x[1], full[1])
    g1, g2, _ = A.gammas(pa[1], pb[1])
    assert np.isclose(g1 + g2, 1.0, rtol=1e-14)


def test_uniform_logits_average_values():
    r = np.random.default_rng(7)
    q = r.normal(size=8)
    K = np.tile(r.normal(size=8), (50, 1))
    V = r.normal(size=(50, 8))
    o, lse = A.full_attention(q, K, V)
    assert np.allclose(o, V.mean(0), rtol=1e-13)
    assert np.isclose(lse, K[0] @ q / np.sqrt(8) + np.log(50))


def test_large_logits_do_not_overflow():
    q = np.array([1000.0, 0, 0, 0])
    K = np.array([[1.0, 0, 0, 0], [0.999, 0, 0, 0]])
    V = np.eye(2, 4)
    o, lse = A.full_attention(q, K, V)
    assert np.all(np.isfinite(o)) and np.isfinite(lse)
    assert np.isclose(o[0] / o[1], np.exp(0.5), rtol=1e-9)


def test_empty_sets():
    q, K, V = _rand(0, N=10)
    o, lse = A.partial_attention(q, K, V, [])
    assert np.all(o == 0) and np.isneginf(lse)
    full = A.full_attention(q, K, V)
    m = A.merge(*full, o, lse)
    assert np.allclose(m[0], full[0], rtol=1e-15) and m[1] == full[1]
    m = A.merge(o, lse, *full)
    assert np.allclose(m[0], full[0], rtol=1e-15) and m[1] == full[1]
    with pytest.raises(ValueError):
        A.merge(o, lse, o, lse)


def test_static_ids():
    assert A.static_ids(10, 2, 3).tolist() == [0, 1, 7, 8, 9]
    assert A.static_ids(10, 0, 0).tolist() == []
    assert A.static_ids(10, 6, 6).tolist() == list(range(10))      # overlap merges
    assert A.static_ids(5, 8, 1).tolist() == list(range(5))        # clipped
    assert A.static_ids(10, 0, 4).tolist() == [6, 7, 8, 9]


def test_static_ids_after_generation():
    # tokens appended after the index was built (n_index) are attended densely
    assert A.static_ids(12, 2, 3, n_index=10).tolist() == [0, 1, 9, 10, 11]
    assert A.static_ids(12, 2, 1, n_index=8).tolist() == [0, 1, 8, 9, 10, 11]
    assert A.static_ids(12, 2, 3, n_index=12).tolist() == A.static_ids(12, 2, 3).tolist()
    assert A.static_ids(6, 0, 0, n_index=2).tolist() == [2, 3, 4, 5]

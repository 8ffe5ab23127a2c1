"""Pins for oracle/quant.py (8-bit keys for the search; Appendix C names the idea, the scheme is
this build's reading, so these pins are mathematical, not values printed by the paper)."""
import numpy as np
import torch

from oracle import mips as OM, quant as OQ, search as OS
from paper_2409_10516_amd import synth
from tests.util import to_np


def _keys(seed=0, N=500, d=128):
    rng = np.random.default_rng(seed)
    K = (rng.standard_normal((N, d)) * rng.lognormal(0, 0.5, d)).astype(np.float32)
    return torch.from_numpy(K).bfloat16().float().numpy()


def test_range_and_reconstruction_bound():
    K = _keys()
    k8, scale = OQ.quantize_keys(K)
    assert k8.dtype == np.int8 and scale.dtype == np.float32
    assert k8.min() >= -127 and k8.max() <= 127
    # every column uses the full range, and the reconstruction is within half a step (plus the
    # float32 rounding of the division, < 1e-6 of the column's largest value)
    assert (np.abs(k8).max(axis=0) == 127).all()
    err = np.abs(K.astype(np.float64) - k8.astype(np.float64) * scale.astype(np.float64))
    assert (err <= 0.5 * scale[None, :] * (1 + 1e-5)).all()


def test_zero_column_and_empty():
    K = _keys(1, N=40)
    K[:, 7] = 0.0
    k8, scale = OQ.quantize_keys(K)
    assert scale[7] == 1.0 and (k8[:, 7] == 0).all()
    k8, scale = OQ.quantize_keys(np.zeros((0, 16), np.float32))
    assert k8.shape == (0, 16) and (scale == 1.0).all()


def test_integer_keys_are_reproduced_exactly():
    rng = np.random.default_rng(2)
    K = rng.integers(-127, 128, size=(300, 128)).astype(np.float32)
    K[0, :] = 127.0                                        # every column reaches 127: scale = 1
    k8, scale = OQ.quantize_keys(K)
    assert (scale == 1.0).all() and (k8.astype(np.float32) == K).all()
    q = rng.integers(-3, 4, size=128).astype(np.float32)
    s = OS.score32(OQ.scaled_query(q, scale), k8.astype(np.float32))
    assert (s.astype(np.float64) == K.astype(np.float64) @ q.astype(np.float64)).all()


def test_round_half_to_even_and_clamp():
    # one column with max 127 so that scale = 1: .5 cases round to the even neighbour
    K = np.array([[127.0], [0.5], [1.5], [2.5], [-0.5], [-1.5], [126.5]], np.float32)
    k8, scale = OQ.quantize_keys(K)
    assert scale[0] == 1.0
    assert k8[:, 0].tolist() == [127, 0, 2, 2, 0, -2, 126]


def test_score_error_bound():
    K = _keys(3)
    rng = np.random.default_rng(4)
    q = torch.from_numpy(rng.standard_normal(128).astype(np.float32)).bfloat16().float().numpy()
    k8, scale = OQ.quantize_keys(K)
    s8 = OS.score32(OQ.scaled_query(q, scale), k8.astype(np.float32)).astype(np.float64)
    s = K.astype(np.float64) @ q.astype(np.float64)
    bound = 0.5 * float(np.abs(q).astype(np.float64) @ scale.astype(np.float64))
    slack = 1e-5 * np.linalg.norm(q) * np.linalg.norm(K, axis=1).max()
    assert (np.abs(s8 - s) <= bound * (1 + 1e-4) + slack).all()
    # and it is an approximation, not the exact score
    assert np.abs(s8 - s).max() > 0


def test_exact_topk_survives_quantisation_on_llama_shaped_keys():
    w = synth.make_llama_layer(5, N=8192, M=8, T=4, n_q=4, n_kv=1)
    K = to_np(w.K[0, 0])
    k8, scale = OQ.quantize_keys(K)
    overlap = []
    for t in range(4):
        for h in range(4):
            q = to_np(w.q_decode[t, 0, h])
            truth = OM.topk_bruteforce(q, K, 100)
            got = OM.topk_bruteforce(OQ.scaled_query(q, scale), k8.astype(np.float32), 100)
            overlap.append(OM.recall(got, truth))
    assert np.mean(overlap) > 0.95, np.mean(overlap)

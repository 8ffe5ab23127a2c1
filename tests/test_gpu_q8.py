"""8-bit keys for the search: the device's quantised bytes and scales, the walk over them, and the
decode step built on it, element by element against the oracle (oracle/quant.py + search.py)."""
import numpy as np
import pytest
import torch

import paper_2409_10516_amd as ra
from oracle import attention as OA, mips as OM, quant as OQ, search as OS
from paper_2409_10516_amd import synth
from tests.util import (Tally, integer_valued, lse_close, oracle_graphs, out_close, to_np, tol_for,
                        topk_equivalent, walk_equivalent)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _cases():
    return {
        "llama_bf16": lambda: synth.make_llama_layer(51, N=1536, M=512, T=2, n_q=8, n_kv=2, ef=64, topk=20,
                                                     window=100),
        "llama_f32_2seq": lambda: synth.make_llama_layer(52, N=700, M=300, T=2, n_seq=2, n_q=4, n_kv=2,
                                                         dtype=torch.float32, ef=48, topk=16, window=37,
                                                         deg=12, knn=9),
        "integer_ties": lambda: synth.make_integer_case(6, N=300, M=64, T=3, d=128, n_q=2, n_kv=1, deg=8,
                                                        knn=6, topk=9, ef=20, sink=3, window=10),
    }


@pytest.mark.parametrize("name", list(_cases()))
def test_quantised_bytes_and_scales_are_the_oracles(name):
    w = _cases()[name]()
    K8, scale = ra.ra_quantize_keys(w.K.to(DEV))
    K8, scale = K8.cpu().numpy(), scale.cpu().numpy()
    n_seq, n_kv = w.K.shape[:2]
    for s in range(n_seq):
        for g in range(n_kv):
            r8, rs = OQ.quantize_keys(to_np(w.K[s, g]))
            assert np.array_equal(scale[s, g].view(np.uint32), rs.view(np.uint32)), (s, g)
            assert np.array_equal(K8[s, g], r8), (s, g)


def test_quantise_zero_column_and_ragged_row_count():
    K = torch.randn(1, 1, 1001, 128).bfloat16()
    K[0, 0, :, 5] = 0
    K8, scale = ra.ra_quantize_keys(K.to(DEV))
    r8, rs = OQ.quantize_keys(to_np(K[0, 0]))
    assert float(scale[0, 0, 5]) == 1.0 and int(K8[0, 0, :, 5].abs().max()) == 0
    assert np.array_equal(K8[0, 0].cpu().numpy(), r8) and np.array_equal(scale[0, 0].cpu().numpy(), rs)


@pytest.mark.parametrize("name", list(_cases()))
@pytest.mark.parametrize("expand", [1, 16])
def test_search_and_decode_over_8bit_keys(name, expand):
    """Ids and counters against the oracle's float64 walk on (q * scale, K8), identical up to decisions
    between scores closer than 1e-5 relative (none for integer-valued keys); the decode output is
    Eq. 2 / Eq. 4-5 over those ids and W with the original K and V, within the usual tolerance."""
    w = _cases()[name]()
    adj, ent, _ = oracle_graphs(w)
    n_seq, n_kv, N, d = w.K.shape
    n_q = w.Q_prefill.shape[1]
    G = n_q // n_kv
    idx = ra.ra_index_import(torch.from_numpy(adj), torch.from_numpy(ent), n_seq, n_q, n_kv)
    Kd, Vd = w.K.to(DEV), w.V.to(DEV)
    k8 = ra.ra_quantize_keys(Kd)
    tol = tol_for(w.K.dtype)
    W = OA.static_ids(N, w.sink, w.window)
    quant = {(s, g): OQ.quantize_keys(to_np(w.K[s, g])) for s in range(n_seq) for g in range(n_kv)}
    exact = integer_valued(to_np(w.K), to_np(w.q_decode))
    tally = Tally()
    for t in range(w.q_decode.shape[0]):
        q = w.q_decode[t].to(DEV)
        ids_s, st_s = ra.ra_search(q, idx, None, w.sink, w.window, w.topk, w.ef, expand, k8=k8)
        out, lse, ids, st = ra.ra_decode_step(q, idx, Kd, Vd, w.sink, w.window, w.topk, w.ef, expand, k8=k8)
        for s in range(n_seq):
            for h in range(n_q):
                g = s * n_q + h
                r8, rs = quant[s, h // G]
                qh = to_np(w.q_decode[t, s, h])
                q8, k8f = OQ.scaled_query(qh, rs), r8.astype(np.float32)
                r_ids, rst = OS.greedy_search(q8, k8f, adj[g], ent[g], w.ef, w.topk, expand, exclude=W)
                assert torch.equal(ids_s[s, h], ids[s, h]) and torch.equal(st_s[s, h], st[s, h])
                got = ids[s, h].cpu().numpy()
                tally.add(walk_equivalent(got, st[s, h].tolist(), r_ids, rst, q8, k8f, W, exact=exact))
                K, V = to_np(w.K[s, h // G]), to_np(w.V[s, h // G])
                o_o, l_o = OA.partial_attention(qh, K, V, got[got >= 0])
                o_w, l_w = OA.partial_attention(qh, K, V, W)
                r_out, r_lse = OA.merge(o_w, l_w, o_o, l_o)
                assert out_close(out[s, h].cpu().numpy(), r_out, tol)
                assert lse_close(lse[s, h].cpu().numpy(), r_lse, tol)
    tally.check()
    idx.free()


def test_8bit_walk_keeps_recall_on_a_32k_layer():
    w = synth.make_llama_layer(53, N=32768, M=32768, T=2, n_q=4, n_kv=1, device=DEV)
    idx = ra.ra_build_index(w.K, w.Q_prefill, w.deg, w.knn)
    k8 = ra.ra_quantize_keys(w.K)
    rec = []
    for t in range(2):
        ids, _ = ra.ra_search(w.q_decode[t], idx, None, w.sink, w.window, w.topk, w.ef, 32, k8=k8)
        truth = ra.ra_flat_topk(w.q_decode[t], w.K, w.sink, w.window, w.topk)
        for h in range(4):
            rec.append(OM.recall(ids[0, h].cpu().numpy(), truth[0, h].cpu().numpy()))
    assert np.mean(rec) > 0.9, np.mean(rec)
    idx.free()


@pytest.mark.parametrize("name", list(_cases()))
def test_rerank_matches_the_oracle(name):
    """ra_rerank on the 8-bit walk's longer list against the oracle's rerank: with float64 scores
    (identical, or position-wise near-ties), and for float32 inputs id for id with the opt-in
    fixed-order float32 scores; lists with -1 padding and out-of-range ids are handled."""
    w = _cases()[name]()
    adj, ent, _ = oracle_graphs(w)
    n_seq, n_kv, N, d = w.K.shape
    n_q = w.Q_prefill.shape[1]
    G = n_q // n_kv
    idx = ra.ra_index_import(torch.from_numpy(adj), torch.from_numpy(ent), n_seq, n_q, n_kv)
    Kd = w.K.to(DEV)
    k8 = ra.ra_quantize_keys(Kd)
    n_cand = min(w.ef, 2 * w.topk)
    q = w.q_decode[0].to(DEV)
    cand, _ = ra.ra_search(q, idx, None, w.sink, w.window, n_cand, w.ef, 8, k8=k8)
    cand[:, :, 1] = -1                                   # a hole, as padding would leave
    ids = ra.ra_rerank(q, Kd, cand, w.topk).cpu().numpy()
    cand = cand.cpu().numpy()
    for s in range(n_seq):
        for h in range(n_q):
            qh, Kh = to_np(w.q_decode[0, s, h]), to_np(w.K[s, h // G])
            want = OM.rerank(qh, Kh, cand[s, h], w.topk)                # float64 scores
            topk_equivalent(ids[s, h], want, qh, Kh, eligible=set(cand[s, h][cand[s, h] >= 0].tolist()))
            if w.K.dtype == torch.float32:                               # the kernel's documented float32 order
                want32 = OM.rerank(qh, Kh, cand[s, h], w.topk, score_fn=OS.score32)
                assert ids[s, h].tolist() == want32.tolist(), (s, h)
    short = torch.full((n_seq, n_q, 4), -1, dtype=torch.int32, device=DEV)
    short[:, :, 2] = 7
    assert ra.ra_rerank(q, Kd, short, 3).cpu().numpy()[0, 0].tolist() == [7, -1, -1]
    idx.free()


def test_rerank_recovers_the_recall_of_the_8bit_walk():
    w = synth.make_llama_layer(53, N=32768, M=32768, T=2, n_q=4, n_kv=1, device=DEV)
    idx = ra.ra_build_index(w.K, w.Q_prefill, w.deg, w.knn)
    k8 = ra.ra_quantize_keys(w.K)
    r_plain, r_q8, r_rr = [], [], []
    for t in range(2):
        q = w.q_decode[t]
        truth = ra.ra_flat_topk(q, w.K, w.sink, w.window, w.topk)
        plain, _ = ra.ra_search(q, idx, w.K, w.sink, w.window, w.topk, w.ef, 32)
        q8, _ = ra.ra_search(q, idx, None, w.sink, w.window, w.topk, w.ef, 32, k8=k8)
        wide, _ = ra.ra_search(q, idx, None, w.sink, w.window, 2 * w.topk, w.ef, 32, k8=k8)
        rr = ra.ra_rerank(q, w.K, wide, w.topk)
        for h in range(4):
            tr = truth[0, h].cpu().numpy()
            r_plain.append(OM.recall(plain[0, h].cpu().numpy(), tr))
            r_q8.append(OM.recall(q8[0, h].cpu().numpy(), tr))
            r_rr.append(OM.recall(rr[0, h].cpu().numpy(), tr))
    assert np.mean(r_rr) >= np.mean(r_q8) and np.mean(r_rr) >= np.mean(r_plain) - 0.01, (
        np.mean(r_plain), np.mean(r_q8), np.mean(r_rr))
    idx.free()

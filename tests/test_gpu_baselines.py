"""Parity of the exact baselines (flat-scan top-k, full attention) with the CPU oracle. GPU only."""
import numpy as np
import pytest
import torch

import paper_2409_10516_amd as ra
from oracle import attention as OA, mips as OM, search as OS
from paper_2409_10516_amd import synth
from tests.util import lse_close, out_close, to_np, tol_for, topk_equivalent

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _cases():
    return {
        "config0_small": (lambda: synth.make_config0(N=3000, M=8, T=3, window=32), 100),
        "llama_bf16": (lambda: synth.make_llama_layer(11, N=5000, M=8, T=2, n_q=8, n_kv=2,
                                                      window=100), 64),
        "llama_f32_2seq": (lambda: synth.make_llama_layer(12, N=701, M=8, T=2, n_seq=2, n_q=4, n_kv=4,
                                                          dtype=torch.float32, window=37), 16),
        "llama_f32_long": (lambda: synth.make_llama_layer(13, N=6000, M=8, T=1, n_q=4, n_kv=2,
                                                          dtype=torch.float32, window=100), 40),
        "integer_ties": (lambda: synth.make_integer_case(5, N=2500, M=8, T=3, d=128, n_q=2, n_kv=1,
                                                         sink=3, window=10), 200),
        "integer_bf16_g8": (lambda: synth.make_integer_case(6, N=300, M=8, T=2, d=128, n_q=8, n_kv=1,
                                                            dtype=torch.bfloat16, lo=-1, hi=1,
                                                            sink=0, window=0), 33),
    }


@pytest.mark.parametrize("name", list(_cases()))
def test_flat_topk_is_exact(name):
    mk, topk = _cases()[name]
    w = mk()
    n_seq, n_kv, N, d = w.K.shape
    n_q = w.q_decode.shape[2]
    Kd = w.K.to(DEV)
    W = OA.static_ids(N, w.sink, w.window)
    eligible = set(range(N)) - set(W.tolist())
    for t in range(w.q_decode.shape[0]):
        ids = ra.ra_flat_topk(w.q_decode[t].to(DEV), Kd, w.sink, w.window, topk).cpu().numpy()
        for s in range(n_seq):
            for h in range(n_q):
                K = to_np(w.K[s, h // (n_q // n_kv)])
                qq = to_np(w.q_decode[t, s, h])
                # the plain definition (float64 scores): identical, or position-wise near-ties
                ref = OM.topk_bruteforce(qq, K, topk, exclude=W)
                topk_equivalent(ids[s, h], np.pad(ref, (0, topk - len(ref)), constant_values=-1), qq, K,
                                eligible=eligible)
                # and, for float32 inputs, id for id in the kernel's documented float32 order
                if w.K.dtype == torch.float32:
                    ref32 = OM.topk_bruteforce(qq, K, topk, exclude=W, score_fn=OS.score32)
                    assert ids[s, h].tolist() == ref32.tolist(), (name, t, s, h)


def test_flat_topk_pads_when_few_keys_are_eligible():
    w = synth.make_integer_case(3, N=90, M=4, T=1, d=128)
    ids = ra.ra_flat_topk(w.q_decode[0].to(DEV), w.K.to(DEV), 40, 45, 12).cpu().numpy()[0, 0]
    ref = OM.topk_bruteforce(to_np(w.q_decode[0, 0, 0]), to_np(w.K[0, 0]), 12,
                             exclude=OA.static_ids(90, 40, 45))
    assert len(ref) == 5 and ids[:5].tolist() == ref.tolist() and (ids[5:] == -1).all()
    ids = ra.ra_flat_topk(w.q_decode[0].to(DEV), w.K.to(DEV), 60, 60, 4).cpu().numpy()[0, 0]
    assert (ids == -1).all()                     # everything is static


@pytest.mark.parametrize("N", [5000, 40000])
def test_flat_topk_all_scores_equal_takes_lowest_ids(N):
    K = torch.ones((1, 1, N, 128), dtype=torch.bfloat16)
    q = torch.ones((1, 1, 128), dtype=torch.bfloat16)
    ids = ra.ra_flat_topk(q.to(DEV), K.to(DEV), 2, 0, 50).cpu().numpy()[0, 0]
    assert ids.tolist() == list(range(2, 52))


def test_flat_topk_long_context_with_few_eligible_keys():
    """40000 keys of which the static set leaves 300: fewer tiles hold an eligible key than topk asks
    for, so no tile maximum can serve as a threshold and the head is scored as a whole."""
    w = synth.make_llama_layer(43, N=40000, M=8, T=1, n_q=4, n_kv=2)
    sink, window = 100, 40000 - 400
    W = OA.static_ids(40000, sink, window)
    for topk in (50, 400):
        ids = ra.ra_flat_topk(w.q_decode[0].to(DEV), w.K.to(DEV), sink, window, topk).cpu().numpy()
        for h in range(4):
            qq, Kh = to_np(w.q_decode[0, 0, h]), to_np(w.K[0, h // 2])
            ref = OM.topk_bruteforce(qq, Kh, topk, exclude=W)
            assert len(ref) == min(topk, 300)
            topk_equivalent(ids[0, h], np.pad(ref, (0, topk - len(ref)), constant_values=-1), qq, Kh,
                            eligible=set(range(40000)) - set(W.tolist()))


@pytest.mark.parametrize("N,dtype", [(300000, torch.bfloat16), (270001, torch.float32)])
def test_flat_topk_beyond_256k_keys(N, dtype):
    """More than 8192 tiles per head: the second pass reads the tile maxima from device memory instead
    of LDS. Real-valued keys against the float64 brute force, and integer-valued keys with thousands
    of ties around the k-th score (a crowd the candidate lists cannot hold: whole-head fallback)."""
    w = synth.make_llama_layer(47, N=N, M=8, T=1, n_q=2, n_kv=1, dtype=dtype, window=640)
    W = OA.static_ids(N, 4, 640)
    for topk in (100, 700):
        ids = ra.ra_flat_topk(w.q_decode[0].to(DEV), w.K.to(DEV), 4, 640, topk).cpu().numpy()
        for h in range(2):
            qq, Kh = to_np(w.q_decode[0, 0, h]), to_np(w.K[0, 0])
            topk_equivalent(ids[0, h], OM.topk_bruteforce(qq, Kh, topk, exclude=W), qq, Kh)
    wi = synth.make_integer_case(9, N=N, M=4, T=1, d=128, lo=-1, hi=1, dtype=dtype)
    ids = ra.ra_flat_topk(wi.q_decode[0].to(DEV), wi.K.to(DEV), 0, 0, 100).cpu().numpy()[0, 0]
    ref = OM.topk_bruteforce(to_np(wi.q_decode[0, 0, 0]), to_np(wi.K[0, 0]), 100)
    assert ids.tolist() == ref.tolist()


@pytest.mark.parametrize("topk", [1, 100, 1024, 2048])
def test_flat_topk_sampled_threshold_path(topk):
    """40000 keys are 1264 tiles: topk 1 and 100 take their threshold from the tile maxima, 1024 and
    2048 (more than half as many as there are tiles) from a strided sample."""
    w = synth.make_llama_layer(41, N=40000, M=8, T=1, n_q=4, n_kv=2, window=640)
    ids = ra.ra_flat_topk(w.q_decode[0].to(DEV), w.K.to(DEV), 4, 640, topk).cpu().numpy()
    W = OA.static_ids(40000, 4, 640)
    for h in range(4):
        qq, Kh = to_np(w.q_decode[0, 0, h]), to_np(w.K[0, h // 2])
        topk_equivalent(ids[0, h], OM.topk_bruteforce(qq, Kh, topk, exclude=W), qq, Kh)
    # integer-valued keys: thousands of exact ties around the k-th score
    wi = synth.make_integer_case(8, N=40000, M=4, T=1, d=128, lo=-1, hi=1)
    ids = ra.ra_flat_topk(wi.q_decode[0].to(DEV), wi.K.to(DEV), 0, 0, topk).cpu().numpy()[0, 0]
    ref = OM.topk_bruteforce(to_np(wi.q_decode[0, 0, 0]), to_np(wi.K[0, 0]), topk)     # exact in any precision
    assert ids.tolist() == ref.tolist()


@pytest.mark.parametrize("name", list(_cases()))
def test_full_attention_matches_eq1(name):
    mk, _ = _cases()[name]
    w = mk()
    n_seq, n_kv, N, d = w.K.shape
    n_q = w.q_decode.shape[2]
    tol = tol_for(w.K.dtype)
    out, lse = ra.ra_full_attention(w.q_decode[0].to(DEV), w.K.to(DEV), w.V.to(DEV))
    out, lse = out.cpu().numpy(), lse.cpu().numpy()
    for s in range(n_seq):
        for h in range(n_q):
            g = h // (n_q // n_kv)
            ro, rl = OA.full_attention(to_np(w.q_decode[0, s, h]), to_np(w.K[s, g]), to_np(w.V[s, g]))
            assert out_close(out[s, h], ro, tol) and lse_close(lse[s, h], rl, tol)


@pytest.mark.parametrize("n_q,n_kv", [(2, 2), (4, 2), (4, 1), (8, 1), (3, 1)])
def test_full_attention_group_sizes_on_a_long_ragged_context(n_q, n_kv):
    """4321 bf16 tokens: several sub-chunks per workgroup and a ragged last chunk. Groups of up to four
    query heads take their logits from the matrix cores, larger and odd ones from the vector units."""
    w = synth.make_llama_layer(23, N=4321, M=8, T=1, n_q=n_q, n_kv=n_kv)
    out, lse = ra.ra_full_attention(w.q_decode[0].to(DEV), w.K.to(DEV), w.V.to(DEV))
    out, lse = out.cpu().numpy(), lse.cpu().numpy()
    for h in range(n_q):
        g = h // (n_q // n_kv)
        ro, rl = OA.full_attention(to_np(w.q_decode[0, 0, h]), to_np(w.K[0, g]), to_np(w.V[0, g]))
        assert out_close(out[0, h], ro, 2e-3) and lse_close(lse[0, h], rl, 2e-3), (n_q, n_kv, h)


def test_full_attention_long_context_uses_few_records():
    """A 40000-token context takes the multi-sub-chunk path of the attention kernel."""
    w = synth.make_llama_layer(21, N=40000, M=8, T=1, n_q=4, n_kv=2)
    out, lse = ra.ra_full_attention(w.q_decode[0].to(DEV), w.K.to(DEV), w.V.to(DEV))
    out, lse = out.cpu().numpy(), lse.cpu().numpy()
    for h in (0, 3):
        ro, rl = OA.full_attention(to_np(w.q_decode[0, 0, h]), to_np(w.K[0, h // 2]), to_np(w.V[0, h // 2]))
        assert out_close(out[0, h], ro, 2e-3) and lse_close(lse[0, h], rl, 2e-3)


def test_graph_recall_can_be_measured_on_device():
    """recall@k of ra_search against ra_flat_topk equals the recall against the CPU brute force."""
    w = synth.make_llama_layer(31, N=4096, M=2048, T=1, n_q=4, n_kv=2, ef=64, topk=32, window=64,
                               device=DEV)
    idx = ra.ra_build_index(w.K, w.Q_prefill, w.deg, w.knn)
    ids, _ = ra.ra_search(w.q_decode[0], idx, w.K, w.sink, w.window, w.topk, w.ef, 8)
    flat = ra.ra_flat_topk(w.q_decode[0], w.K, w.sink, w.window, w.topk)
    W = OA.static_ids(4096, w.sink, w.window)
    for h in range(4):
        qq, Kh = to_np(w.q_decode[0, 0, h]), to_np(w.K[0, h // 2])
        truth = OM.topk_bruteforce(qq, Kh, w.topk, exclude=W)
        topk_equivalent(flat[0, h].cpu().numpy(), truth, qq, Kh)
        # (a near-tie at the cut of the exact list can move one id)
        assert abs(OM.recall(ids[0, h].cpu().numpy(), flat[0, h].cpu().numpy()) -
                   OM.recall(ids[0, h].cpu().numpy(), truth)) <= 1.0 / w.topk


def _fold16(words):
    """xor over 16-byte pieces (4 uint32 x, y, z, w each) of ((x ^ z) << 32) | (y ^ w)."""
    w = words.reshape(-1, 4).astype(np.uint64)
    f = ((w[:, 0] ^ w[:, 2]) << np.uint64(32)) | (w[:, 1] ^ w[:, 3])
    return int(np.bitwise_xor.reduce(f)) if len(f) else 0


@pytest.mark.parametrize("n16", [1, 999, 8 * 256 * 3 + 5, 1 << 16])
def test_read_probe_reads_every_byte_once(n16):
    """The streaming probe's fold is the xor over all 16-byte pieces of the buffer: every piece is
    read exactly once, ragged tails included."""
    rng = np.random.default_rng(n16)
    host = rng.integers(0, 2**32, size=n16 * 4, dtype=np.uint64).astype(np.uint32)
    buf = torch.from_numpy(host.view(np.int32)).to(DEV)
    out = torch.zeros(1, dtype=torch.int64, device=DEV)
    ra.ra_hbm_read_probe(buf, out)
    assert int(out.cpu().numpy().view(np.uint64)[0]) == _fold16(host)


@pytest.mark.parametrize("rows_in_buf,n_rows,seed", [(1, 5, 0), (37, 1000, 3), (4096, 8 * 64 * 2 + 3, 7), (50000, 200000, 1)])
def test_gather_probe_reads_the_hashed_rows(rows_in_buf, n_rows, seed):
    """The gather probe reads row hash(position, seed) mod rows for every position of the sequence,
    whole rows of 256 bytes: its fold is the xor over those rows (with their multiplicity)."""
    rng = np.random.default_rng(rows_in_buf)
    host = rng.integers(0, 2**32, size=rows_in_buf * 64, dtype=np.uint64).astype(np.uint32)
    buf = torch.from_numpy(host.view(np.int32)).to(DEV)
    out = torch.zeros(1, dtype=torch.int64, device=DEV)
    ra.ra_hbm_gather_probe(buf, n_rows, out, seed=seed)
    x = (np.arange(n_rows, dtype=np.uint64) * np.uint64(0x9e3779b9) + np.uint64(seed)) & np.uint64(0xffffffff)
    x ^= x >> np.uint64(16); x = (x * np.uint64(0x7feb352d)) & np.uint64(0xffffffff)
    x ^= x >> np.uint64(15); x = (x * np.uint64(0x846ca68b)) & np.uint64(0xffffffff)
    x ^= x >> np.uint64(16)
    rows = (x % np.uint64(rows_in_buf)).astype(np.int64)
    assert int(out.cpu().numpy().view(np.uint64)[0]) == _fold16(host.reshape(rows_in_buf, 64)[rows])
    with pytest.raises(ra.RaError):
        ra.ra_hbm_gather_probe(buf, 0, out)

"""Parity of the HIP index build (exact KNN on the matrix cores, projection) with the CPU
oracle, through the C ABI. GPU only."""
import json
import os

import numpy as np
import pytest
import torch

import paper_2409_10516_amd as ra
from oracle import attention as OA, decode as OD, mips as OM, projection as OP
from paper_2409_10516_amd import synth
from tests.util import decode_matches, integer_valued, knn_equivalent, lse_close, out_close, to_np, tol_for

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
GOLD = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(params=["reg", "lds"])
def knn_selection(request):
    """Lists of up to 32 bf16 keys have two selections (pending keys in registers, two query sets per
    wavefront / pending runs in LDS); the library picks by the number of keys, the tests force each
    through the test-only setting."""
    from paper_2409_10516_amd import binding as B
    ra.ra_test_configure(B.RA_TEST_KNN_SELECTION,
                         B.RA_TEST_KNN_REG if request.param == "reg" else B.RA_TEST_KNN_LDS)
    yield request.param
    ra.ra_test_configure(B.RA_TEST_KNN_SELECTION, B.RA_TEST_KNN_AUTO)


def _cases():
    return {
        "config0_small": lambda: synth.make_config0(N=1024, M=256, T=2, window=32),
        "llama_bf16": lambda: synth.make_llama_layer(11, N=1536, M=768, T=2, n_q=8, n_kv=2,
                                                     ef=64, topk=20, window=100),
        "llama_f32_ragged": lambda: synth.make_llama_layer(12, N=701, M=299, T=2, n_seq=2, n_q=4,
                                                           n_kv=4, dtype=torch.float32, ef=48,
                                                           topk=16, window=37, deg=12, knn=9),
        "integer_ties": lambda: synth.make_integer_case(5, N=200, M=64, T=2, d=128, n_q=2,
                                                        n_kv=1, deg=8, knn=6, topk=9, ef=20,
                                                        sink=3, window=10),
        "integer_bf16_knn64": lambda: synth.make_integer_case(6, N=333, M=150, T=2, d=128, n_q=1,
                                                              n_kv=1, dtype=torch.bfloat16, deg=64,
                                                              knn=64, topk=9, ef=20),
        "integer_bf16_knn48": lambda: synth.make_integer_case(7, N=777, M=130, T=2, d=128, n_q=2,
                                                              n_kv=1, dtype=torch.bfloat16, deg=48,
                                                              knn=48, topk=9, ef=20),
        "integer_bf16_knn20": lambda: synth.make_integer_case(9, N=900, M=600, T=2, d=128, n_q=2,
                                                              n_kv=1, dtype=torch.bfloat16, deg=16,
                                                              knn=20, topk=9, ef=20),
        "integer_f32_knn40": lambda: synth.make_integer_case(8, N=450, M=70, T=2, d=128, n_q=1,
                                                             n_kv=1, dtype=torch.float32, deg=16,
                                                             knn=40, topk=9, ef=20),
    }


def _heads(w):
    n_seq, n_kv, N, d = w.K.shape
    n_q = w.Q_prefill.shape[1]
    for s in range(n_seq):
        for h in range(n_q):
            yield s, h, s * n_q + h, to_np(w.K[s, h // (n_q // n_kv)]), to_np(w.Q_prefill[s, h])


@pytest.mark.parametrize("name", list(_cases()))
def test_knn_lists(name, knn_selection):
    w = _cases()[name]()
    L = ra.ra_knn(w.K.to(DEV), w.Q_prefill.to(DEV), w.knn).cpu().numpy()
    for s, h, g, K, Q in _heads(w):
        ref, _ = OM.knn_lists(Q, K, w.knn)
        diff = knn_equivalent(L[s, h], ref, Q, K)
        if name.startswith("integer"):
            assert diff == 0          # integer-valued inputs: every score is exact


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("knn", [5, 32, 48, 64])
@pytest.mark.parametrize("rising", [True, False])
def test_knn_monotone_stream(dtype, knn, rising, knn_selection):
    """Scores that rise with the key id make every key of the stream qualify (the selection folds or
    inserts all the time); falling scores make none qualify after the first knn. Key i scores exactly
    +-i for every query (i = 256 * K[i,1] + K[i,0], both exact in bf16), so the lists are known."""
    N, M = 3001, 77
    K = torch.zeros((1, 1, N, 128), dtype=torch.float32)
    i = torch.arange(N)
    K[0, 0, :, 0] = (i % 256).float()
    K[0, 0, :, 1] = (i // 256).float()
    Q = torch.zeros((1, 1, M, 128), dtype=torch.float32)
    Q[0, 0, :, 0] = 1.0 if rising else -1.0
    Q[0, 0, :, 1] = 256.0 if rising else -256.0
    L = ra.ra_knn(K.to(dtype).to(DEV), Q.to(dtype).to(DEV), knn).cpu().numpy()[0, 0]
    want = np.arange(N - 1, N - 1 - knn, -1) if rising else np.arange(knn)
    assert np.array_equal(L, np.broadcast_to(want, (M, knn)))


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("knn", [7, 32, 64])
def test_knn_stream_order_against_a_minority_of_queries(dtype, knn, knn_selection):
    """The keys are streamed by descending inner product with the head's mean query. Here 60 % of
    the queries are -u and 40 % are +u, so the stream is in the best order for the majority and in
    the worst (every key beats the threshold) for the minority; the lists must not depend on it."""
    N, M = 2500, 90
    K = torch.zeros((1, 1, N, 128), dtype=torch.float32)
    i = torch.arange(N)
    K[0, 0, :, 0] = (i % 256).float()
    K[0, 0, :, 1] = (i // 256).float()
    sign = torch.where(torch.arange(M) % 5 < 3, -1.0, 1.0)
    Q = torch.zeros((1, 1, M, 128), dtype=torch.float32)
    Q[0, 0, :, 0] = sign
    Q[0, 0, :, 1] = 256.0 * sign
    L = ra.ra_knn(K.to(dtype).to(DEV), Q.to(dtype).to(DEV), knn).cpu().numpy()[0, 0]
    for j in range(M):
        want = np.arange(N - 1, N - 1 - knn, -1) if sign[j] > 0 else np.arange(knn)
        assert np.array_equal(L[j], want), j


@pytest.mark.parametrize("N,knn", [(1, 1), (3, 3), (5, 2), (33, 33), (64, 48), (65, 64)])
def test_knn_tiny_key_sets(N, knn, knn_selection):
    """Fewer keys than a stage, than a block, than the sort's smallest chunk: all equal scores, so
    the lists are the lowest ids in order."""
    M = 9
    K = torch.ones((1, 1, N, 128), dtype=torch.bfloat16)
    Q = torch.ones((1, 1, M, 128), dtype=torch.bfloat16)
    L = ra.ra_knn(K.to(DEV), Q.to(DEV), knn).cpu().numpy()[0, 0]
    assert np.array_equal(L, np.broadcast_to(np.arange(knn), (M, knn)))


def _sweep_cases():
    rng = np.random.default_rng(1234)
    cases = []
    for it in range(14):
        dtype = torch.bfloat16 if it % 3 else torch.float32
        n_kv = int(rng.choice([1, 2])); G = int(rng.choice([1, 2, 4]))
        N = int(rng.choice([31, 33, 63, 65, 100, 511, 513, 1000, 2047, 4097]))
        M = int(rng.choice([1, 5, 33, 255, 257, 511, 513, 1025]))
        knn = min(int(rng.choice([1, 2, 5, 16, 31, 32, 33, 40, 48, 49, 64])), N)
        cases.append((it, dtype, n_kv, G, N, M, knn))
    return cases


@pytest.mark.parametrize("it,dtype,n_kv,G,N,M,knn", _sweep_cases())
def test_knn_shape_sweep(it, dtype, n_kv, G, N, M, knn, knn_selection):
    """Key and query counts around the kernel's block, stage and workgroup sizes, list lengths on both
    sides of every selection's limit. Small integer inputs with a shared component: every score is
    exact, ties abound, the stream order is not the storage order."""
    g = torch.Generator(); g.manual_seed(1000 + it)
    K = torch.randint(-3, 4, (1, n_kv, N, 128), generator=g).float()
    Q = torch.randint(-3, 4, (1, n_kv * G, M, 128), generator=g).float()
    K[..., 0] += torch.randint(0, 6, (1, n_kv, N), generator=g).float()
    Q[..., 0] += 2
    L = ra.ra_knn(K.to(dtype).to(DEV), Q.to(dtype).to(DEV), knn).cpu().numpy()
    for h in range(n_kv * G):
        ref, _ = OM.knn_lists(Q[0, h].numpy().astype(np.float64), K[0, h // G].numpy().astype(np.float64), knn)
        assert np.array_equal(L[0, h], ref), h


def test_projection_hand_worked_example():
    g = json.load(open(os.path.join(GOLD, "projection_hand.json")))
    L = torch.tensor([g["L"]], dtype=torch.int32, device=DEV)
    adj, entry = ra.ra_project(L, g["N"], g["deg"])
    assert entry.cpu().tolist() == [g["entry"]]
    assert adj[0].cpu().tolist() == g["adj"]


def test_projection_regimes_of_a_large_graph():
    """More populated keys than the row kernel has LDS counters, with the three kinds of key such a
    graph holds: hubs (in half of all lists: counters in device memory, pipelined list walk), keys of
    about 60 lists (LDS hash table, one workgroup per key) and keys of a handful of lists (one
    wavefront per key). Every hub and middle key and a sample of the small ones against the oracle."""
    rng = np.random.default_rng(17)
    N, M, knn, deg = 20000, 3000, 48, 16
    hubs, mids, rest = np.arange(10), np.arange(10, 310), np.arange(310, N)
    L = np.empty((M, knn), np.int32)
    for j in range(M):
        row = np.concatenate([rng.choice(hubs, 5, replace=False), rng.choice(mids, 6, replace=False),
                              rng.choice(rest, knn - 11, replace=False)])
        L[j] = rng.permutation(row)
    adj, entry = ra.ra_project(torch.from_numpy(L[None]).to(DEV), N, deg)
    adj = adj[0].cpu().numpy()
    rows = np.concatenate([hubs, mids, rng.choice(rest, 400, replace=False)])
    radj, rent = OP.project(L, N, deg, rows=rows)
    assert int(entry[0]) == rent
    pop = np.bincount(L.ravel(), minlength=N)
    assert (pop > 0).sum() > 8192 and pop[hubs].min() > 1000 and 21 < pop[mids].min() and pop[mids].max() <= 85
    for a in rows:
        assert np.array_equal(adj[a], radj[a]), (a, adj[a], radj[a])


@pytest.mark.parametrize("name", list(_cases()))
@pytest.mark.parametrize("deg", [None, 2, 5])
def test_projection_bit_exact_on_oracle_lists(name, deg):
    w = _cases()[name]()
    deg = deg or w.deg
    N = w.K.shape[2]
    Ls, refs = [], []
    for s, h, g, K, Q in _heads(w):
        L, _ = OM.knn_lists(Q, K, w.knn)
        Ls.append(L)
        refs.append(OP.project(L, N, deg))
    adj, entry = ra.ra_project(torch.from_numpy(np.stack(Ls)).to(DEV), N, deg)
    adj, entry = adj.cpu().numpy(), entry.cpu().numpy()
    for g, (radj, rent) in enumerate(refs):
        assert entry[g] == rent
        assert np.array_equal(adj[g], radj), np.argwhere(adj[g] != radj)[:5]


def test_projection_skewed_lists():
    """Every list holds the same two hub keys plus a few others (the shape the Llama-like
    generator produces at scale), and some keys are in no list at all."""
    rng = np.random.default_rng(0)
    N, M, knn, deg = 500, 400, 8, 10
    L = np.empty((M, knn), np.int32)
    for j in range(M):
        rest = rng.choice(np.arange(2, 120), size=knn - 2, replace=False)
        L[j] = np.concatenate([[0, 1], rest])[rng.permutation(knn)]
    radj, rent = OP.project(L, N, deg)
    adj, entry = ra.ra_project(torch.from_numpy(L[None]).to(DEV), N, deg)
    assert int(entry[0]) == rent
    assert np.array_equal(adj[0].cpu().numpy(), radj)


@pytest.mark.parametrize("name", list(_cases()))
def test_build_index_then_decode(name):
    """ra_build_index = KNN + projection; its graph must be the oracle's projection of the
    device's own KNN lists (which may differ from the float64 lists only in near-ties), and a
    decode step on it must match the oracle run on the exported graph."""
    w = _cases()[name]()
    Kd, Vd, Qd = w.K.to(DEV), w.V.to(DEV), w.Q_prefill.to(DEV)
    n_seq, n_kv, N, d = w.K.shape
    n_q = w.Q_prefill.shape[1]
    L = ra.ra_knn(Kd, Qd, w.knn).cpu().numpy()
    idx = ra.ra_build_index(Kd, Qd, w.deg, w.knn)
    assert (idx.n_seq, idx.n_q_heads, idx.n_kv_heads, idx.N, idx.deg) == (n_seq, n_q, n_kv, N, w.deg)
    tol = tol_for(w.K.dtype)
    q = w.q_decode[0]
    out, lse, ids, st = ra.ra_decode_step(q.to(DEV), idx, Kd, Vd, w.sink, w.window, w.topk, w.ef, 4)
    out, lse, ids, st = out.cpu().numpy(), lse.cpu().numpy(), ids.cpu().numpy(), st.cpu().numpy()
    exact = integer_valued(to_np(w.K), to_np(w.q_decode))
    for s, h, g, K, Q in _heads(w):
        radj, rent = OP.project(L[s, h], N, w.deg)
        adj, ent = ra.ra_index_export(idx, s, h)
        assert ent == rent and np.array_equal(adj.numpy(), radj)
        V = to_np(w.V[s, h // (n_q // n_kv)])
        decode_matches(out[s, h], lse[s, h], ids[s, h], st[s, h].tolist(), to_np(q[s, h]), K, V, radj, rent,
                       w.sink, w.window, w.topk, w.ef, 4, tol, exact=exact)
    idx.free()


def test_build_argument_errors():
    w = synth.make_integer_case(1, N=64, M=16, d=128)
    Kd, Qd = w.K.to(DEV), w.Q_prefill.to(DEV)
    with pytest.raises(ra.RaError) as e:
        ra.ra_knn(Kd, Qd, 65)                        # knn > N
    assert e.value.status == 1
    with pytest.raises(ra.RaError) as e:
        ra.ra_build_index(Kd, Qd, 1, 4)              # deg < 2
    assert e.value.status == 1
    with pytest.raises(ra.RaError) as e:
        ra.ra_build_index(Kd[..., :64].contiguous(), Qd[..., :64].contiguous(), 8, 4)   # d != 128
    assert e.value.status == 6

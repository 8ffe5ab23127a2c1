"""ra_attend_noalloc (the entry point for callers that cannot allocate device memory) against
ra_attend, through the C ABI: same kernels, partial records in the library's fixed device array
instead of the handle's workspace, so the outputs must be identical. Two calls in a row, the second
on a smaller input (the array keeps the first call's records), then a call whose records do not
fit. GPU only; collected last."""
import numpy as np
import pytest
import torch

import paper_2409_10516_amd as ra
from oracle import attention as OA
from paper_2409_10516_amd import synth
from tests.util import lse_close, oracle_graphs, out_close, to_np, tol_for

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(seed, N, n_seq, n_q, n_kv, topk, window):
    w = synth.make_llama_layer(seed, N=N, M=64, T=1, n_seq=n_seq, n_q=n_q, n_kv=n_kv, topk=topk, window=window,
                               deg=8, knn=8)
    rng = np.random.default_rng(seed)
    W = OA.static_ids(N, w.sink, window)
    rest = np.setdiff1d(np.arange(N), W)
    ids = -np.ones((n_seq, n_q, topk), np.int32)
    for s in range(n_seq):
        for h in range(n_q):
            nv = topk - (s + h) % 4                                   # some rows are padded
            ids[s, h, :nv] = rng.choice(rest, size=nv, replace=False)
    adj = np.full((n_seq * n_q, N, 2), -1, np.int32)                  # ra_attend reads no graph
    idx = ra.ra_index_import(torch.from_numpy(adj), torch.zeros(n_seq * n_q, dtype=torch.int32), n_seq, n_q, n_kv)
    return w, idx, torch.from_numpy(ids).to(DEV), W


def test_noalloc_attend_equals_ra_attend_twice_in_a_row():
    big = _case(71, N=3000, n_seq=3, n_q=8, n_kv=2, topk=100, window=640)
    small = _case(72, N=500, n_seq=1, n_q=4, n_kv=4, topk=20, window=70)
    for w, idx, ids, W in (big, small):
        Kd, Vd, q = w.K.to(DEV), w.V.to(DEV), w.q_decode[0].to(DEV)
        ref = ra.ra_attend(q, idx, Kd, Vd, w.sink, w.window, ids, partials=True)
        out = torch.full_like(ref[0], float("nan"))
        lse = torch.full_like(ref[1], float("nan"))
        torch.cuda.synchronize()
        before = torch.cuda.mem_get_info()[0]            # free device memory: any hipMalloc would lower it
        got = ra.ra_attend(q, idx, Kd, Vd, w.sink, w.window, ids, noalloc=True, out=out, lse=lse)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == before
        assert torch.equal(got[0], ref[0]) and torch.equal(got[1], ref[1])
        gp = ra.ra_attend(q, idx, Kd, Vd, w.sink, w.window, ids, noalloc=True, partials=True)
        for a, b in zip(gp, ref):
            assert torch.equal(a, b)
        # and both are the oracle's Eq. 2 / Eq. 4-5
        tol = tol_for(w.K.dtype)
        n_seq, n_q = q.shape[:2]
        G = n_q // w.K.shape[1]
        o, l, idn = got[0].cpu().numpy(), got[1].cpu().numpy(), ids.cpu().numpy()
        for s in range(n_seq):
            for h in range(0, n_q, 3):
                K, V = to_np(w.K[s, h // G]), to_np(w.V[s, h // G])
                qq = to_np(w.q_decode[0, s, h])
                oo, lo = OA.partial_attention(qq, K, V, idn[s, h][idn[s, h] >= 0])
                ow, lw = OA.partial_attention(qq, K, V, W)
                ro, rl = OA.merge(ow, lw, oo, lo)
                assert out_close(o[s, h], ro, tol) and lse_close(l[s, h], rl, tol)
        idx.free()


def test_noalloc_attend_rejects_what_does_not_fit():
    # 4096 heads x (11 static + 2 gathered records) x 528 B = 28 MB > the 8 MiB the library keeps
    n_seq, n_q, N = 128, 32, 700
    adj = np.full((n_seq * n_q, N, 2), -1, np.int32)
    idx = ra.ra_index_import(torch.from_numpy(adj), torch.zeros(n_seq * n_q, dtype=torch.int32), n_seq, n_q, 8)
    K = torch.zeros((n_seq, 8, N, 128), dtype=torch.bfloat16, device=DEV)
    q = torch.zeros((n_seq, n_q, 128), dtype=torch.bfloat16, device=DEV)
    ids = torch.full((n_seq, n_q, 100), -1, dtype=torch.int32, device=DEV)
    with pytest.raises(ra.RaError) as e:
        ra.ra_attend(q, idx, K, K, 4, 640, ids, noalloc=True)
    assert e.value.status == 6 and "bytes" in str(e.value)
    ra.ra_attend(q, idx, K, K, 4, 640, ids)            # the allocating call takes it
    idx.free()

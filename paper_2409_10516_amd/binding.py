"""Thin ctypes binding over libra.so (the C ABI in include/ra.h).

Argument marshalling only: every function takes torch tensors that already live on the
GPU, checks dtype/contiguity, passes raw pointers and sizes, and returns the tensors the
library filled. No step of the method is computed here, and there is no CPU fallback:
if the library is missing, loading fails with an error.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# RA_LIBRARY names another build of the same library (a tuning build, say); default: the in-tree one
LIB_PATH = os.environ.get("RA_LIBRARY") or os.path.join(_HERE, "libra.so")

RA_F32, RA_BF16 = 0, 1
RA_CFG_HELPERS, RA_CFG_HELPER_SPIN, RA_CFG_SEEDS, RA_CFG_SEED_SHARES = 0, 1, 2, 3
RA_HELPERS_OFF, RA_HELPERS_ON = 0, 1
# test-only settings (ra_test_configure)
RA_TEST_KNN_SELECTION, RA_TEST_HELPERS_SILENT = 100, 101
RA_TEST_KNN_AUTO, RA_TEST_KNN_REG, RA_TEST_KNN_LDS = 0, 1, 2
STATUS = {0: "RA_OK", 1: "RA_EINVAL", 2: "RA_ESHAPE", 3: "RA_EDTYPE", 4: "RA_ENOMEM",
          5: "RA_EHIP", 6: "RA_EUNSUP"}


class RaError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS.get(status, status)}: {message}")
        self.status = status


_lib = None


def lib() -> C.CDLL:
    """Load libra.so (once). Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; "
                           f"g.build()'` (or python paper_2409_10516_amd/build.py) first")
    L = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int, C.c_int64
    L.ra_last_error.restype = C.c_char_p
    L.ra_version.restype = C.c_char_p
    L.ra_knn.argtypes = [vp, vp, i32, i32, i32, i32, i64, i64, i32, i32, vp, vp]
    L.ra_project.argtypes = [vp, i32, i64, i64, i32, i32, vp, vp, vp]
    L.ra_build_index.argtypes = [vp, vp, i32, i32, i32, i32, i64, i64, i32, i32, i32, vp,
                                 C.POINTER(vp)]
    L.ra_search.argtypes = [vp, vp, vp, i32, i64, i32, i32, i32, i32, i32, vp, vp, vp]
    L.ra_quantize_keys.argtypes = [vp, i32, i32, i32, i64, vp, vp, vp]
    L.ra_quantize_keys.restype = i32
    L.ra_search_q8.argtypes = [vp, vp, vp, vp, i32, i64, i32, i32, i32, i32, i32, vp, vp, vp]
    L.ra_search_q8.restype = i32
    L.ra_decode_step_q8.argtypes = [vp, vp, vp, vp, i32, vp, vp, i64, i32, i32, i32, i32, i32, vp, vp, vp,
                                    vp, vp]
    L.ra_decode_step_q8.restype = i32
    L.ra_rerank.argtypes = [vp, vp, i32, i32, i32, i32, i64, i32, vp, i32, i32, vp, vp]
    L.ra_rerank.restype = i32
    L.ra_attend.argtypes = [vp, vp, vp, vp, i32, i64, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    L.ra_attend_noalloc.argtypes = [vp, vp, vp, vp, i32, i64, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    L.ra_decode_step.argtypes = [vp, vp, vp, vp, i32, i64, i32, i32, i32, i32, i32, vp, vp, vp,
                                 vp, vp]
    L.ra_decode_step_grown.argtypes = [vp, vp, vp, vp, i32, i64, i64, i32, i32, i32, i32, i32, vp, vp,
                                       vp, vp, vp]
    L.ra_decode_step_grown.restype = i32
    L.ra_decode_step_budgets.argtypes = [vp, vp, vp, vp, i32, i64, i32, i32, i32, vp, i32, i32, vp, vp,
                                         vp, vp, vp]
    L.ra_decode_step_budgets.restype = i32
    L.ra_index_import.argtypes = [vp, vp, i32, i32, i32, i64, i32, C.POINTER(vp)]
    L.ra_index_export.argtypes = [vp, i32, i32, vp, vp]
    L.ra_index_info.argtypes = [vp, i32]
    L.ra_index_info.restype = i64
    L.ra_index_configure.argtypes = [vp, i32, i64]
    L.ra_index_configure.restype = i32
    L.ra_test_configure.argtypes = [vp, i32, i64]
    L.ra_test_configure.restype = i32
    L.ra_index_adj.argtypes = [vp]
    L.ra_index_adj.restype = vp
    L.ra_index_entry.argtypes = [vp]
    L.ra_index_entry.restype = vp
    L.ra_index_free.argtypes = [vp]
    L.ra_index_free.restype = None
    L.ra_flat_workspace_bytes.argtypes = [i32, i32, i64]
    L.ra_flat_workspace_bytes.restype = C.c_size_t
    L.ra_flat_topk.argtypes = [vp, vp, i32, i32, i32, i32, i64, i32, i32, i32, i32, vp, C.c_size_t, vp, vp]
    L.ra_flat_topk.restype = i32
    L.ra_full_attention_workspace_bytes.argtypes = [i32, i32, i32, i64]
    L.ra_full_attention_workspace_bytes.restype = C.c_size_t
    L.ra_hbm_read_probe.argtypes = [vp, C.c_size_t, vp, vp]
    L.ra_hbm_gather_probe.argtypes = [vp, C.c_size_t, C.c_size_t, C.c_uint32, vp, vp]
    L.ra_full_attention.argtypes = [vp, vp, vp, i32, i32, i32, i32, i64, i32, vp, C.c_size_t, vp, vp, vp]
    L.ra_full_attention.restype = i32
    for name in ("ra_knn", "ra_project", "ra_build_index", "ra_search", "ra_attend",
                 "ra_attend_noalloc", "ra_hbm_read_probe", "ra_hbm_gather_probe", "ra_decode_step", "ra_index_import",
                 "ra_index_export"):
        getattr(L, name).restype = i32
    _lib = L
    return L


def _check(rc: int):
    if rc != 0:
        raise RaError(rc, lib().ra_last_error().decode())


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return RA_F32
    if t.dtype == torch.bfloat16:
        return RA_BF16
    raise TypeError(f"dtype {t.dtype} is not supported (float32 or bfloat16)")


def _dev(*ts):
    for t in ts:
        if t is None:
            continue
        if not t.is_cuda:
            raise ValueError("tensors must live on the GPU")
        if not t.is_contiguous():
            raise ValueError("tensors must be contiguous")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


class Index:
    """Owns an ra_index handle."""

    def __init__(self, handle: int):
        self._h = C.c_void_p(handle)

    @property
    def handle(self):
        if self._h is None:
            raise RuntimeError("index was freed")
        return self._h

    def info(self, what: int) -> int:
        return int(lib().ra_index_info(self.handle, what))

    n_seq = property(lambda s: s.info(0))
    n_q_heads = property(lambda s: s.info(1))
    n_kv_heads = property(lambda s: s.info(2))
    N = property(lambda s: s.info(3))
    deg = property(lambda s: s.info(4))
    device_bytes = property(lambda s: s.info(5))
    helpers_active = property(lambda s: s.info(6) == 1)
    seed_shares_active = property(lambda s: s.info(8) == 1)

    n_seeds = property(lambda s: s.info(7))

    def configure(self, what: int, value: int) -> None:
        """ra_index_configure: RA_CFG_HELPERS / RA_CFG_HELPER_SPIN / RA_CFG_SEEDS / RA_CFG_SEED_SHARES."""
        _check(lib().ra_index_configure(self.handle, what, value))

    def test_configure(self, what: int, value: int) -> None:
        """ra_test_configure on this handle (test-only settings)."""
        _check(lib().ra_test_configure(self.handle, what, value))

    def free(self):
        if self._h is not None:
            lib().ra_index_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def ra_test_configure(what: int, value: int) -> None:
    """ra_test_configure without a handle (process-wide test-only settings)."""
    _check(lib().ra_test_configure(None, what, value))


def ra_knn(K, Q_prefill, knn: int, stream=None) -> torch.Tensor:
    _dev(K, Q_prefill)
    n_seq, n_kv, N, d = K.shape
    _, n_q, M, _ = Q_prefill.shape
    L = torch.empty((n_seq, n_q, M, knn), dtype=torch.int32, device=K.device)
    _check(lib().ra_knn(_ptr(K), _ptr(Q_prefill), _dt(K), n_seq, n_q, n_kv, N, M, d, knn,
                        _stream(stream), _ptr(L)))
    return L


def ra_project(L: torch.Tensor, N: int, deg: int, stream=None):
    """L: int32 [n_graphs][M][knn] on the GPU -> (adj [n_graphs][N][deg], entry [n_graphs])."""
    _dev(L)
    if L.dtype != torch.int32:
        raise TypeError("L must be int32")
    n_graphs, M, knn = L.shape
    adj = torch.empty((n_graphs, N, deg), dtype=torch.int32, device=L.device)
    entry = torch.empty((n_graphs,), dtype=torch.int32, device=L.device)
    _check(lib().ra_project(_ptr(L), n_graphs, N, M, knn, deg, _stream(stream), _ptr(adj),
                            _ptr(entry)))
    return adj, entry


def ra_build_index(K, Q_prefill, deg: int, knn: int, stream=None) -> Index:
    _dev(K, Q_prefill)
    if K.dtype != Q_prefill.dtype:
        raise TypeError("K and Q_prefill must share a dtype")
    n_seq, n_kv, N, d = K.shape
    _, n_q, M, _ = Q_prefill.shape
    h = C.c_void_p()
    _check(lib().ra_build_index(_ptr(K), _ptr(Q_prefill), _dt(K), n_seq, n_q, n_kv, N, M, d, deg,
                                knn, _stream(stream), C.byref(h)))
    return Index(h.value)


def ra_index_import(adj: torch.Tensor, entries: torch.Tensor, n_seq: int, n_q: int,
                    n_kv: int) -> Index:
    """adj: int32 [n_seq*n_q][N][deg] on the HOST; entries: int32 [n_seq*n_q] on the host."""
    adj = adj.to(torch.int32).contiguous().cpu()
    entries = entries.to(torch.int32).contiguous().cpu()
    g, N, deg = adj.shape
    if g != n_seq * n_q or entries.numel() != g:
        raise ValueError("adj/entries do not match n_seq * n_q graphs")
    h = C.c_void_p()
    _check(lib().ra_index_import(_ptr(adj), _ptr(entries), n_seq, n_q, n_kv, N, deg, C.byref(h)))
    return Index(h.value)


def ra_index_export(idx: Index, seq: int, q_head: int):
    adj = torch.empty((idx.N, idx.deg), dtype=torch.int32)
    entry = torch.empty((1,), dtype=torch.int32)
    _check(lib().ra_index_export(idx.handle, seq, q_head, _ptr(adj), _ptr(entry)))
    return adj, int(entry[0])


def _stats_tensor(n_heads, device):
    return torch.zeros((n_heads, 4), dtype=torch.int32, device=device)


def ra_quantize_keys(K, stream=None):
    """8-bit copy of the keys for the search -> (K8 int8 [n_seq][n_kv][N][128], scale float32
    [n_seq][n_kv][128])."""
    _dev(K)
    n_seq, n_kv, N, d = K.shape
    K8 = torch.empty((n_seq, n_kv, N, d), dtype=torch.int8, device=K.device)
    scale = torch.empty((n_seq, n_kv, d), dtype=torch.float32, device=K.device)
    _check(lib().ra_quantize_keys(_ptr(K), _dt(K), n_seq, n_kv, N, _stream(stream), _ptr(K8), _ptr(scale)))
    return K8, scale


def ra_search(q, idx: Index, K, sink: int, window: int, topk: int, ef: int, expand: int = 1,
              stream=None, with_stats: bool = True, k8=None):
    """-> (ids int32 [n_seq][n_q][topk], stats int32 [n_seq][n_q][4] = visited, expanded,
    iters, returned). With k8 = (K8, scale) from ra_quantize_keys the walk reads the 8-bit keys
    (ra_search_q8) and K may be None."""
    n_seq, n_q, d = q.shape
    ids = torch.empty((n_seq, n_q, topk), dtype=torch.int32, device=q.device)
    st = _stats_tensor(n_seq * n_q, q.device) if with_stats else None
    if k8 is None:
        _dev(q, K)
        _check(lib().ra_search(_ptr(q), idx.handle, _ptr(K), _dt(K), K.shape[2], sink, window, topk,
                               ef, expand, _stream(stream), _ptr(ids), _ptr(st)))
    else:
        K8, scale = k8
        _dev(q, K8, scale)
        _check(lib().ra_search_q8(_ptr(q), idx.handle, _ptr(K8), _ptr(scale), _dt(q), K8.shape[2], sink,
                                  window, topk, ef, expand, _stream(stream), _ptr(ids), _ptr(st)))
    return ids, (st.view(n_seq, n_q, 4) if with_stats else None)


def ra_rerank(q, K, cand, topk: int, stream=None):
    """Best topk of the candidate ids [n_seq][n_q][n_cand] under the exact scores <q, K[id]>
    -> ids int32 [n_seq][n_q][topk]."""
    _dev(q, K, cand)
    n_seq, n_q, d = q.shape
    ids = torch.empty((n_seq, n_q, topk), dtype=torch.int32, device=q.device)
    _check(lib().ra_rerank(_ptr(q), _ptr(K), _dt(K), n_seq, n_q, K.shape[1], K.shape[2], d, _ptr(cand),
                           cand.shape[-1], topk, _stream(stream), _ptr(ids)))
    return ids


def ra_attend(q, idx: Index, K, V, sink: int, window: int, ids: torch.Tensor, stream=None,
              partials: bool = False, noalloc: bool = False, out=None, lse=None):
    """-> (out, lse) or, with partials=True, (out, lse, o_omega, lse_omega, o_w, lse_w).
    noalloc=True calls ra_attend_noalloc (pass out and lse in, then nothing is allocated at all)."""
    _dev(q, K, V, ids, out, lse)
    n_seq, n_q, d = q.shape
    topk = ids.shape[-1]
    f = dict(dtype=torch.float32, device=q.device)
    if out is None:
        out = torch.empty((n_seq, n_q, d), **f)
    if lse is None:
        lse = torch.empty((n_seq, n_q), **f)
    extra = [None] * 4
    if partials:
        extra = [torch.empty((n_seq, n_q, d), **f), torch.empty((n_seq, n_q), **f),
                 torch.empty((n_seq, n_q, d), **f), torch.empty((n_seq, n_q), **f)]
    fn = lib().ra_attend_noalloc if noalloc else lib().ra_attend
    _check(fn(_ptr(q), idx.handle, _ptr(K), _ptr(V), _dt(K), K.shape[2], sink, window,
              topk, _ptr(ids), _stream(stream), _ptr(out), _ptr(lse), *[_ptr(t) for t in extra]))
    return (out, lse, *extra) if partials else (out, lse)


def ra_decode_step(q, idx: Index, K, V, sink: int, window: int, topk: int, ef: int,
                   expand: int = 1, stream=None, out=None, lse=None, ids=None, stats=None,
                   n_tokens: Optional[int] = None, k8=None, topk_per_head=None):
    """One layer's decode-step attention. Output tensors may be passed in to avoid
    allocation; -> (out, lse, ids, stats). With n_tokens given, K/V are caches of capacity
    K.shape[2] rows per head holding n_tokens >= idx.N valid tokens (ra_decode_step_grown). With
    k8 = (K8, scale) from ra_quantize_keys the walk reads the 8-bit keys (ra_decode_step_q8). With
    topk_per_head (device int32 [n_seq][n_q]) every head keeps its own number of ids, at most topk
    (ra_decode_step_budgets)."""
    _dev(q, K, V, out, lse, ids, stats, topk_per_head)
    if topk_per_head is not None and (k8 is not None or n_tokens is not None):
        raise ValueError("topk_per_head goes with neither k8 nor n_tokens")
    n_seq, n_q, d = q.shape
    f = dict(dtype=torch.float32, device=q.device)
    if out is None:
        out = torch.empty((n_seq, n_q, d), **f)
    if lse is None:
        lse = torch.empty((n_seq, n_q), **f)
    if ids is None:
        ids = torch.empty((n_seq, n_q, topk), dtype=torch.int32, device=q.device)
    if stats is None:
        stats = _stats_tensor(n_seq * n_q, q.device).view(n_seq, n_q, 4)
    if topk_per_head is not None:
        if topk_per_head.dtype != torch.int32 or tuple(topk_per_head.shape) != (n_seq, n_q) \
                or not topk_per_head.is_contiguous():
            raise ValueError("topk_per_head must be a contiguous int32 tensor [n_seq][n_q]")
        _check(lib().ra_decode_step_budgets(_ptr(q), idx.handle, _ptr(K), _ptr(V), _dt(K), K.shape[2], sink,
                                            window, topk, _ptr(topk_per_head), ef, expand, _stream(stream),
                                            _ptr(out), _ptr(lse), _ptr(ids), _ptr(stats)))
    elif k8 is not None:
        K8, scale = k8
        _dev(K8, scale)
        _check(lib().ra_decode_step_q8(_ptr(q), idx.handle, _ptr(K), _ptr(V), _dt(K), _ptr(K8), _ptr(scale),
                                       K.shape[2], sink, window, topk, ef, expand, _stream(stream),
                                       _ptr(out), _ptr(lse), _ptr(ids), _ptr(stats)))
    elif n_tokens is None:
        _check(lib().ra_decode_step(_ptr(q), idx.handle, _ptr(K), _ptr(V), _dt(K), K.shape[2], sink,
                                    window, topk, ef, expand, _stream(stream), _ptr(out), _ptr(lse),
                                    _ptr(ids), _ptr(stats)))
    else:
        _check(lib().ra_decode_step_grown(_ptr(q), idx.handle, _ptr(K), _ptr(V), _dt(K), n_tokens,
                                          K.shape[2], sink, window, topk, ef, expand, _stream(stream),
                                          _ptr(out), _ptr(lse), _ptr(ids), _ptr(stats)))
    return out, lse, ids, stats


def ra_hbm_read_probe(buf: torch.Tensor, out: torch.Tensor, stream=None) -> None:
    """Stream `buf` (contiguous device tensor) once; xors a fold of it into out (device int64 [1])."""
    _dev(buf, out)
    _check(lib().ra_hbm_read_probe(_ptr(buf), buf.numel() * buf.element_size(), _stream(stream), _ptr(out)))


def ra_hbm_gather_probe(buf: torch.Tensor, n_rows: int, out: torch.Tensor, seed: int = 0, stream=None) -> None:
    """Read n_rows rows of 256 B of `buf` at hashed row numbers; xors a fold into out (device int64 [1])."""
    _dev(buf, out)
    _check(lib().ra_hbm_gather_probe(_ptr(buf), buf.numel() * buf.element_size(), n_rows, seed, _stream(stream),
                                     _ptr(out)))


def ra_flat_topk(q, K, sink: int, window: int, topk: int, stream=None, workspace=None, ids=None):
    """Exact top-k by linear scan for every (sequence, query head) -> ids int32 [n_seq][n_q][topk]."""
    _dev(q, K, workspace, ids)
    n_seq, n_q, d = q.shape
    n_kv, N = K.shape[1], K.shape[2]
    need = lib().ra_flat_workspace_bytes(n_seq, n_q, N)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    if ids is None:
        ids = torch.empty((n_seq, n_q, topk), dtype=torch.int32, device=q.device)
    _check(lib().ra_flat_topk(_ptr(q), _ptr(K), _dt(K), n_seq, n_q, n_kv, N, d, sink, window, topk,
                              _ptr(workspace), workspace.numel(), _stream(stream), _ptr(ids)))
    return ids


def ra_full_attention(q, K, V, stream=None, workspace=None, out=None, lse=None):
    """Eq. 1 over the whole context -> (out float32 [n_seq][n_q][d], lse float32 [n_seq][n_q])."""
    _dev(q, K, V, workspace, out, lse)
    n_seq, n_q, d = q.shape
    n_kv, N = K.shape[1], K.shape[2]
    need = lib().ra_full_attention_workspace_bytes(n_seq, n_q, n_kv, N)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    f = dict(dtype=torch.float32, device=q.device)
    if out is None:
        out = torch.empty((n_seq, n_q, d), **f)
    if lse is None:
        lse = torch.empty((n_seq, n_q), **f)
    _check(lib().ra_full_attention(_ptr(q), _ptr(K), _ptr(V), _dt(K), n_seq, n_q, n_kv, N, d,
                                   _ptr(workspace), workspace.numel(), _stream(stream), _ptr(out),
                                   _ptr(lse)))
    return out, lse

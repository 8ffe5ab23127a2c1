// C ABI of libra (declared in include/ra.h): argument checks, handle management and the
// sequencing of the device stages. No arithmetic of the method lives here.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <new>

#include "common.h"

static thread_local char g_err[512] = "";

void ra_set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

extern "C" const char* ra_last_error(void) { return g_err; }
extern "C" const char* ra_version(void) { return "libra 0.1 (gfx950)"; }

// ---- shared argument checks (run before any HIP call) ----------------------------------
static ra_status check_dtype(ra_dtype dt) {
    if (dt != RA_F32 && dt != RA_BF16) RA_FAIL(RA_EDTYPE, "unknown dtype %d", (int)dt);
    return RA_OK;
}

static ra_status check_heads(int n_seq, int n_q, int n_kv) {
    if (n_seq < 1 || n_q < 1 || n_kv < 1)
        RA_FAIL(RA_EINVAL, "n_seq, n_q_heads, n_kv_heads must be positive (%d, %d, %d)", n_seq, n_q,
                n_kv);
    if (n_q % n_kv) RA_FAIL(RA_EINVAL, "n_q_heads %d is not a multiple of n_kv_heads %d", n_q, n_kv);
    return RA_OK;
}

static ra_status check_dim(int d) {
    if (d < 1) RA_FAIL(RA_EINVAL, "d must be positive");
    if (d != RA_D) RA_FAIL(RA_EUNSUP, "this build supports d = %d only (got %d)", RA_D, d);
    return RA_OK;
}

static ra_status check_decode_args(const ra_index* idx, int64_t N, int sink, int window, int topk) {
    if (!idx) RA_FAIL(RA_EINVAL, "index handle is NULL");
    if (N != idx->N) RA_FAIL(RA_ESHAPE, "N = %lld but the index was built over %lld keys",
                             (long long)N, (long long)idx->N);
    if (sink < 0 || window < 0) RA_FAIL(RA_EINVAL, "sink and window must be non-negative");
    if (topk < 1) RA_FAIL(RA_EINVAL, "topk must be positive");
    if (topk > RA_MAX_TOPK) RA_FAIL(RA_EUNSUP, "topk %d exceeds RA_MAX_TOPK %d", topk, RA_MAX_TOPK);
    return RA_OK;
}

// the start set the walks of this handle use: its seed sets when configured, else its root sets
static const int32_t* start_sets(const ra_index* ix, int* cap) {
    *cap = ix->n_seeds ? ix->seed_cap : ix->root_cap;
    return ix->n_seeds ? ix->seeds : ix->roots;
}

static ra_status check_seeds_fit(const ra_index* ix, int expand) {
    if (ix->n_seeds > expand * ix->deg)
        RA_FAIL(RA_EINVAL, "n_seeds %d exceeds expand x deg = %d (the seeds are scored like one step's "
                "candidates): raise expand or lower RA_CFG_SEEDS", ix->n_seeds, expand * ix->deg);
    return RA_OK;
}

static ra_status check_search_args(int topk, int ef, int expand) {
    if (ef < 1 || expand < 1) RA_FAIL(RA_EINVAL, "ef and expand must be positive");
    if (ef < topk) RA_FAIL(RA_EINVAL, "ef (%d) must be at least topk (%d)", ef, topk);
    if (ef > RA_MAX_EF) RA_FAIL(RA_EUNSUP, "ef %d exceeds RA_MAX_EF %d", ef, RA_MAX_EF);
    if (expand > RA_MAX_EXPAND)
        RA_FAIL(RA_EUNSUP, "expand %d exceeds RA_MAX_EXPAND %d", expand, RA_MAX_EXPAND);
    return RA_OK;
}

static ra_status check_build_args(int64_t N, int64_t M, int deg, int knn, bool need_deg) {
    if (N < 1 || M < 1) RA_FAIL(RA_EINVAL, "N and M must be positive");
    if (N > 0x7fffffff / 2) RA_FAIL(RA_EUNSUP, "N too large for 31-bit ids");
    if (knn < 1) RA_FAIL(RA_EINVAL, "knn must be positive");
    if (knn > N) RA_FAIL(RA_EINVAL, "knn (%d) exceeds N (%lld)", knn, (long long)N);
    if (knn > RA_MAX_KNN) RA_FAIL(RA_EUNSUP, "knn %d exceeds RA_MAX_KNN %d", knn, RA_MAX_KNN);
    if (need_deg) {
        if (deg < 2) RA_FAIL(RA_EINVAL, "deg must be at least 2 (two backbone slots)");
        if (deg > RA_MAX_DEG) RA_FAIL(RA_EUNSUP, "deg %d exceeds RA_MAX_DEG %d", deg, RA_MAX_DEG);
    }
    return RA_OK;
}

#define RA_TRY(expr)                  \
    do {                              \
        ra_status rc_ = (expr);       \
        if (rc_ != RA_OK) return rc_; \
    } while (0)

// ---- workspace -----------------------------------------------------------------------
static ra_status grow(void** p, size_t* have, size_t need) {
    if (need <= *have) return RA_OK;
    if (*p) RA_HIP(hipFree(*p));
    *p = nullptr;
    *have = 0;
    RA_HIP(hipMalloc(p, need));
    *have = need;
    return RA_OK;
}

// records, ready words and the "helpers off" word of the fused decode kernel's hand-over area
static size_t coop_bytes(const ra_index* ix) {
    const size_t heads = (size_t)ix->n_seq * ix->n_q;
    return heads * RA_COOP_REC * sizeof(float) + (heads + 1) * sizeof(uint32_t);
}

static ra_status new_handle(int n_seq, int n_q, int n_kv, int64_t N, int deg, ra_index** out) {
    ra_index* ix = new (std::nothrow) ra_index();
    if (!ix) RA_FAIL(RA_ENOMEM, "host allocation failed");
    memset(ix, 0, sizeof(*ix));
    ix->n_seq = n_seq; ix->n_q = n_q; ix->n_kv = n_kv; ix->N = N; ix->deg = deg;
    const size_t graphs = (size_t)n_seq * n_q;
    ix->graph_bytes = graphs * N * deg * sizeof(int32_t);
    hipError_t e = hipGetDevice(&ix->device);
    if (e == hipSuccess) e = hipMalloc((void**)&ix->adj, ix->graph_bytes);
    if (e == hipSuccess) e = hipMalloc((void**)&ix->entry, graphs * sizeof(int32_t));
    ix->root_cap = 3 + deg + deg * deg;
    if (e == hipSuccess) e = hipMalloc((void**)&ix->roots, graphs * ix->root_cap * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc((void**)&ix->coop, coop_bytes(ix));
    if (e == hipSuccess) e = hipMemset(ix->coop, 0, coop_bytes(ix));
    ix->coop_mode = RA_HELPERS_ON;
    ix->coop_spin = RA_HELPER_SPIN_DEFAULT;
    ix->seed_parts = RA_SEED_PARTS_DEFAULT;
    if (e != hipSuccess) {
        ra_set_error("allocating the graph (%zu B) failed: %s", ix->graph_bytes, hipGetErrorString(e));
        if (ix->adj) (void)hipFree(ix->adj);
        if (ix->entry) (void)hipFree(ix->entry);
        if (ix->coop) (void)hipFree(ix->coop);
        if (ix->roots) (void)hipFree(ix->roots);
        delete ix;
        return e == hipErrorOutOfMemory ? RA_ENOMEM : RA_EHIP;
    }
    *out = ix;
    return RA_OK;
}

extern "C" void ra_index_free(ra_index* ix) {
    if (!ix) return;
    if (ix->adj) (void)hipFree(ix->adj);
    if (ix->entry) (void)hipFree(ix->entry);
    if (ix->partials) (void)hipFree(ix->partials);
    if (ix->ids_ws) (void)hipFree(ix->ids_ws);
    if (ix->bitset) (void)hipFree(ix->bitset);
    if (ix->coop) (void)hipFree(ix->coop);
    if (ix->roots) (void)hipFree(ix->roots);
    if (ix->seeds) (void)hipFree(ix->seeds);
    if (ix->seedx) (void)hipFree(ix->seedx);
    delete ix;
}

extern "C" ra_status ra_index_configure(ra_index* ix, int what, int64_t value) {
    if (!ix) RA_FAIL(RA_EINVAL, "index handle is NULL");
    switch (what) {
        case RA_CFG_HELPERS: {
            if (value != RA_HELPERS_OFF && value != RA_HELPERS_ON)
                RA_FAIL(RA_EINVAL, "helpers mode %lld", (long long)value);
            // also forgets a wait that ran out: ready words and the off word start from zero
            RA_HIP(hipDeviceSynchronize());
            RA_HIP(hipMemset(ix->coop, 0, coop_bytes(ix)));
            if (ix->seedx) RA_HIP(hipMemset(ix->seedx, 0, ix->seedx_bytes));
            ix->coop_mode = (int)value;
            ix->coop_silent = 0;
            return RA_OK;
        }
        case RA_CFG_HELPER_SPIN:
            if (value < 1 || value > (1 << 24)) RA_FAIL(RA_EINVAL, "spin limit %lld", (long long)value);
            ix->coop_spin = (int)value;
            return RA_OK;
        case RA_CFG_SEED_SHARES:
            if (value != 0 && (value < 2 || value > RA_SEED_PARTS_MAX))
                RA_FAIL(RA_EINVAL, "seed shares %lld: 0 or 2 .. %d", (long long)value, RA_SEED_PARTS_MAX);
            RA_HIP(hipDeviceSynchronize());
            if (ix->seedx) RA_HIP(hipMemset(ix->seedx, 0, ix->seedx_bytes));
            ix->seed_parts = (int)value;
            return RA_OK;
        case RA_CFG_SEEDS: {
            if (value < 0 || value > RA_MAX_SEEDS)
                RA_FAIL(RA_EINVAL, "n_seeds %lld outside [0, %d]", (long long)value, RA_MAX_SEEDS);
            RA_HIP(hipDeviceSynchronize());
            const int n = (int)(value > ix->N ? ix->N : value);
            if (n == 0) {
                ix->n_seeds = 0;
                return RA_OK;
            }
            const size_t graphs = (size_t)ix->n_seq * ix->n_q;
            if (n + 2 > ix->seed_cap) {
                if (ix->seeds) RA_HIP(hipFree(ix->seeds));
                ix->seeds = nullptr;
                ix->seed_cap = 0;
                ix->n_seeds = 0;
                RA_HIP(hipMalloc((void**)&ix->seeds, graphs * (size_t)(n + 2) * sizeof(int32_t)));
                ix->seed_cap = n + 2;
                if (ix->seedx) RA_HIP(hipFree(ix->seedx));
                ix->seedx = nullptr;
                ix->seedx_bytes = RA_SEEDX_KEYS_OFF + graphs * (size_t)(n + 2) * sizeof(uint64_t);
                RA_HIP(hipMalloc((void**)&ix->seedx, ix->seedx_bytes));
                RA_HIP(hipMemset(ix->seedx, 0, ix->seedx_bytes));
            }
            RA_TRY(ra_launch_seeds(ix->adj, ix->entry, (int)graphs, ix->N, ix->deg, n, ix->seeds, ix->seed_cap,
                                   nullptr));
            RA_HIP(hipStreamSynchronize(nullptr));
            ix->n_seeds = n;
            return RA_OK;
        }
        default:
            RA_FAIL(RA_EINVAL, "unknown setting %d", what);
    }
}

extern "C" ra_status ra_test_configure(ra_index* ix, int what, int64_t value) {
    switch (what) {
        case RA_TEST_KNN_SELECTION:
            if (value != RA_TEST_KNN_AUTO && value != RA_TEST_KNN_REG && value != RA_TEST_KNN_LDS)
                RA_FAIL(RA_EINVAL, "knn selection %lld", (long long)value);
            ra_knn_set_selection_override((int)value);
            return RA_OK;
        case RA_TEST_HELPERS_SILENT:
            if (!ix) RA_FAIL(RA_EINVAL, "index handle is NULL");
            if (value != 0 && value != 1) RA_FAIL(RA_EINVAL, "silent helpers %lld", (long long)value);
            RA_HIP(hipDeviceSynchronize());
            RA_HIP(hipMemset(ix->coop, 0, coop_bytes(ix)));
            if (ix->seedx) RA_HIP(hipMemset(ix->seedx, 0, ix->seedx_bytes));
            ix->coop_silent = (int)value;
            return RA_OK;
        default:
            RA_FAIL(RA_EINVAL, "unknown test setting %d", what);
    }
}

extern "C" int64_t ra_index_info(const ra_index* ix, int what) {
    if (!ix) return -1;
    switch (what) {
        case 0: return ix->n_seq;
        case 1: return ix->n_q;
        case 2: return ix->n_kv;
        case 3: return ix->N;
        case 4: return ix->deg;
        case 5: return (int64_t)(ix->graph_bytes + (size_t)ix->n_seq * ix->n_q * 4 +
                                 ix->partials_bytes + ix->ids_bytes + ix->bitset_bytes + coop_bytes(ix) +
                                 ix->seedx_bytes +
                                 (size_t)ix->n_seq * ix->n_q * (ix->root_cap + ix->seed_cap) * sizeof(int32_t));
        case 6: {
            if (ix->coop_mode != RA_HELPERS_ON || ix->coop_silent) return 0;
            const int G = ix->n_q / ix->n_kv;
            if (G != 1 && G != 2 && G != 4 && G != 8) return 0;      // see ra_launch_decode
            const size_t heads = (size_t)ix->n_seq * ix->n_q;
            uint32_t off = 1u;
            if (hipDeviceSynchronize() != hipSuccess ||
                hipMemcpy(&off, reinterpret_cast<const char*>(ix->coop) + heads * RA_COOP_REC * sizeof(float) +
                                    heads * sizeof(uint32_t),
                          sizeof(off), hipMemcpyDeviceToHost) != hipSuccess)
                return -1;
            return off == 0u;
        }
        case 7: return ix->n_seeds;
        case 8: {
            // 1 while the seed shares are on and no head's wait for them has run out
            if (!ix->n_seeds || !ix->seedx || ix->seed_parts < 2 || ix->coop_mode != RA_HELPERS_ON || ix->coop_silent)
                return 0;
            uint32_t off = 1u;
            if (hipDeviceSynchronize() != hipSuccess ||
                hipMemcpy(&off, ix->seedx, sizeof(off), hipMemcpyDeviceToHost) != hipSuccess)
                return -1;
            return off == 0u;
        }
        default: return -1;
    }
}

extern "C" const int32_t* ra_index_adj(const ra_index* ix) { return ix ? ix->adj : nullptr; }
extern "C" const int32_t* ra_index_entry(const ra_index* ix) { return ix ? ix->entry : nullptr; }

extern "C" ra_status ra_index_import(const int32_t* adj_host, const int32_t* entries_host, int n_seq,
                                     int n_q, int n_kv, int64_t N, int deg, ra_index** out) {
    if (!adj_host || !entries_host || !out) RA_FAIL(RA_EINVAL, "NULL argument");
    RA_TRY(check_heads(n_seq, n_q, n_kv));
    if (N < 1) RA_FAIL(RA_EINVAL, "N must be positive");
    if (N > 0x7fffffff / 2) RA_FAIL(RA_EUNSUP, "N too large for 31-bit ids");
    if (deg < 1) RA_FAIL(RA_EINVAL, "deg must be positive");
    if (deg > RA_MAX_DEG) RA_FAIL(RA_EUNSUP, "deg %d exceeds RA_MAX_DEG %d", deg, RA_MAX_DEG);
    const size_t graphs = (size_t)n_seq * n_q;
    for (size_t g = 0; g < graphs; ++g)
        if (entries_host[g] < 0 || entries_host[g] >= N)
            RA_FAIL(RA_EINVAL, "entry point %d of graph %zu is outside [0, N)", entries_host[g], g);
    const size_t cells = graphs * (size_t)N * deg;
    for (size_t i = 0; i < cells; ++i)
        if (adj_host[i] < -1 || adj_host[i] >= N)
            RA_FAIL(RA_EINVAL, "adjacency cell %zu holds %d, outside [-1, N)", i, adj_host[i]);
    ra_index* ix = nullptr;
    RA_TRY(new_handle(n_seq, n_q, n_kv, N, deg, &ix));
    hipError_t e = hipMemcpy(ix->adj, adj_host, ix->graph_bytes, hipMemcpyHostToDevice);
    if (e == hipSuccess)
        e = hipMemcpy(ix->entry, entries_host, graphs * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
        ra_set_error("copying the graph to the device failed: %s", hipGetErrorString(e));
        ra_index_free(ix);
        return RA_EHIP;
    }
    ra_status rc = ra_launch_roots(ix->adj, ix->entry, (int)graphs, N, deg, ix->roots, ix->root_cap, nullptr);
    if (rc == RA_OK && hipStreamSynchronize(nullptr) != hipSuccess) {
        ra_set_error("listing the root sets failed: %s", hipGetErrorString(hipGetLastError()));
        rc = RA_EHIP;
    }
    if (rc != RA_OK) {
        ra_index_free(ix);
        return rc;
    }
    *out = ix;
    return RA_OK;
}

extern "C" ra_status ra_index_export(const ra_index* ix, int seq, int q_head, int32_t* adj_host,
                                     int32_t* entry_host) {
    if (!ix || !adj_host || !entry_host) RA_FAIL(RA_EINVAL, "NULL argument");
    if (seq < 0 || seq >= ix->n_seq || q_head < 0 || q_head >= ix->n_q)
        RA_FAIL(RA_EINVAL, "(seq %d, q_head %d) outside the index (%d x %d)", seq, q_head, ix->n_seq,
                ix->n_q);
    const size_t g = (size_t)seq * ix->n_q + q_head;
    const size_t row_bytes = (size_t)ix->N * ix->deg * sizeof(int32_t);
    RA_HIP(hipDeviceSynchronize());
    RA_HIP(hipMemcpy(adj_host, ix->adj + g * (size_t)ix->N * ix->deg, row_bytes, hipMemcpyDeviceToHost));
    RA_HIP(hipMemcpy(entry_host, ix->entry + g, sizeof(int32_t), hipMemcpyDeviceToHost));
    return RA_OK;
}

// ---- index build -----------------------------------------------------------------------
extern "C" ra_status ra_knn(const void* K, const void* Q, ra_dtype dt, int n_seq, int n_q, int n_kv,
                            int64_t N, int64_t M, int d, int knn, void* stream, int32_t* L_out) {
    if (!K || !Q || !L_out) RA_FAIL(RA_EINVAL, "NULL argument");
    RA_TRY(check_dtype(dt));
    RA_TRY(check_heads(n_seq, n_q, n_kv));
    RA_TRY(check_dim(d));
    RA_TRY(check_build_args(N, M, 2, knn, false));
    void* ws = nullptr;                                    // the order the keys are streamed in
    RA_HIP(hipMalloc(&ws, ra_knn_order_bytes(n_seq * n_q, N)));
    ra_status rc = ra_launch_knn(K, Q, dt, n_seq, n_q, n_kv, N, M, knn, ws, (hipStream_t)stream, L_out);
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    (void)hipFree(ws);
    if (rc != RA_OK) return rc;
    RA_HIP(e);
    return RA_OK;
}

extern "C" ra_status ra_project(const int32_t* L, int n_graphs, int64_t N, int64_t M, int knn,
                                int deg, void* stream, int32_t* adj, int32_t* entry) {
    if (!L || !adj || !entry) RA_FAIL(RA_EINVAL, "NULL argument");
    if (n_graphs < 1) RA_FAIL(RA_EINVAL, "n_graphs must be positive");
    RA_TRY(check_build_args(N, M, deg, knn, true));
    const size_t ws_bytes = ra_project_workspace_bytes(n_graphs, N, M, knn);
    void* ws = nullptr;
    RA_HIP(hipMalloc(&ws, ws_bytes));
    ra_status rc = ra_launch_project(L, n_graphs, N, M, knn, deg, ws, (hipStream_t)stream, adj, entry);
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    (void)hipFree(ws);
    if (rc != RA_OK) return rc;
    RA_HIP(e);
    return RA_OK;
}

extern "C" ra_status ra_build_index(const void* K, const void* Q, ra_dtype dt, int n_seq, int n_q,
                                    int n_kv, int64_t N, int64_t M, int d, int deg, int knn,
                                    void* stream, ra_index** out) {
    if (!K || !Q || !out) RA_FAIL(RA_EINVAL, "NULL argument");
    RA_TRY(check_dtype(dt));
    RA_TRY(check_heads(n_seq, n_q, n_kv));
    RA_TRY(check_dim(d));
    RA_TRY(check_build_args(N, M, deg, knn, true));
    const int graphs = n_seq * n_q;
    ra_index* ix = nullptr;
    RA_TRY(new_handle(n_seq, n_q, n_kv, N, deg, &ix));
    int32_t* L = nullptr;
    void* order_ws = nullptr;
    hipError_t e = hipMalloc((void**)&L, (size_t)graphs * M * knn * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc(&order_ws, ra_knn_order_bytes(graphs, N));
    if (e != hipSuccess) {
        ra_set_error("allocating the KNN lists failed: %s", hipGetErrorString(e));
        if (L) (void)hipFree(L);
        ra_index_free(ix);
        return e == hipErrorOutOfMemory ? RA_ENOMEM : RA_EHIP;
    }
    ra_status rc = ra_launch_knn(K, Q, dt, n_seq, n_q, n_kv, N, M, knn, order_ws, (hipStream_t)stream, L);
    if (rc == RA_OK) rc = ra_project(L, graphs, N, M, knn, deg, stream, ix->adj, ix->entry);
    if (rc == RA_OK)
        rc = ra_launch_roots(ix->adj, ix->entry, graphs, N, deg, ix->roots, ix->root_cap, (hipStream_t)stream);
    if (rc == RA_OK && hipStreamSynchronize((hipStream_t)stream) != hipSuccess) {
        ra_set_error("index build failed on the device: %s", hipGetErrorString(hipGetLastError()));
        rc = RA_EHIP;
    }
    (void)hipFree(L);
    (void)hipFree(order_ws);
    if (rc != RA_OK) {
        ra_index_free(ix);
        return rc;
    }
    *out = ix;
    return RA_OK;
}

// ---- decode step -----------------------------------------------------------------------
// `K` holds the keys the walk scores: the cache's own (kscale == NULL) or their 8-bit copy
static ra_status search_common(const void* q, const ra_index* idx, const void* K, const float* kscale,
                               ra_dtype dt, int64_t N, int sink, int window, int topk, int ef, int expand,
                               void* stream, int32_t* ids, ra_stats* stats) {
    if (!q || !K || !ids) RA_FAIL(RA_EINVAL, "NULL argument");
    RA_TRY(check_dtype(dt));
    RA_TRY(check_decode_args(idx, N, sink, window, topk));
    RA_TRY(check_search_args(topk, ef, expand));
    ra_index* ix = const_cast<ra_index*>(idx);
    RA_TRY(check_seeds_fit(ix, expand));
    if (ra_search_needs_global_bitset(N, ix->deg, ef, expand)) {
        const size_t need = (size_t)ix->n_seq * ix->n_q * ((N + 31) >> 5) * 4;
        RA_TRY(grow((void**)&ix->bitset, &ix->bitset_bytes, need));
    }
    int start_cap;
    const int32_t* start = start_sets(ix, &start_cap);
    return ra_launch_search(q, ix->adj, ix->entry, K, dt, ix->n_seq, ix->n_q, ix->n_kv, N, ix->deg,
                            sink, window, topk, ef, expand, ix->bitset, start, start_cap, kscale,
                            (hipStream_t)stream, ids, stats);
}

extern "C" ra_status ra_search(const void* q, const ra_index* idx, const void* K, ra_dtype dt,
                               int64_t N, int sink, int window, int topk, int ef, int expand,
                               void* stream, int32_t* ids, ra_stats* stats) {
    return search_common(q, idx, K, nullptr, dt, N, sink, window, topk, ef, expand, stream, ids, stats);
}

extern "C" ra_status ra_search_q8(const void* q, const ra_index* idx, const int8_t* K8, const float* scale,
                                  ra_dtype dtq, int64_t N, int sink, int window, int topk, int ef,
                                  int expand, void* stream, int32_t* ids, ra_stats* stats) {
    if (!scale) RA_FAIL(RA_EINVAL, "NULL argument");
    return search_common(q, idx, K8, scale, dtq, N, sink, window, topk, ef, expand, stream, ids, stats);
}

extern "C" ra_status ra_quantize_keys(const void* K, ra_dtype dt, int n_seq, int n_kv, int64_t N,
                                      void* stream, int8_t* K8, float* scale) {
    if (!K || !K8 || !scale) RA_FAIL(RA_EINVAL, "NULL argument");
    RA_TRY(check_dtype(dt));
    if (n_seq < 1 || n_kv < 1) RA_FAIL(RA_EINVAL, "n_seq and n_kv_heads must be positive");
    if (N < 1) RA_FAIL(RA_EINVAL, "N must be positive");
    if ((int64_t)n_seq * n_kv > 65535) RA_FAIL(RA_EUNSUP, "more than 65535 (sequence, KV head) pairs");
    return ra_launch_quantize(K, dt, n_seq * n_kv, N, (hipStream_t)stream, K8, scale);
}

extern "C" ra_status ra_attend(const void* q, const ra_index* idx, const void* K, const void* V,
                               ra_dtype dt, int64_t N, int sink, int window, int topk,
                               const int32_t* ids, void* stream, float* out, float* lse,
                               float* o_omega, float* lse_omega, float* o_w, float* lse_w) {
    if (!q || !K || !V || !ids || !out || !lse) RA_FAIL(RA_EINVAL, "NULL argument");
    RA_TRY(check_dtype(dt));
    RA_TRY(check_decode_args(idx, N, sink, window, topk));
    ra_index* ix = const_cast<ra_index*>(idx);
    const size_t need =
        ra_attend_partial_floats(ix->n_seq, ix->n_q, ix->n_kv, N, sink, window, topk) * sizeof(float);
    RA_TRY(grow((void**)&ix->partials, &ix->partials_bytes, need));
    return ra_launch_attend(q, K, V, dt, ix->n_seq, ix->n_q, ix->n_kv, N, sink, window, topk, ids,
                            ix->partials, (hipStream_t)stream, out, lse, o_omega, lse_omega, o_w,
                            lse_w);
}

extern "C" ra_status ra_attend_noalloc(const void* q, const ra_index* idx, const void* K, const void* V,
                                       ra_dtype dt, int64_t N, int sink, int window, int topk,
                                       const int32_t* ids, void* stream, float* out, float* lse,
                                       float* o_omega, float* lse_omega, float* o_w, float* lse_w) {
    if (!q || !K || !V || !ids || !out || !lse) RA_FAIL(RA_EINVAL, "NULL argument");
    RA_TRY(check_dtype(dt));
    RA_TRY(check_decode_args(idx, N, sink, window, topk));
    return ra_launch_attend_noalloc(q, K, V, dt, idx->n_seq, idx->n_q, idx->n_kv, N, sink, window, topk, ids,
                                    (hipStream_t)stream, out, lse, o_omega, lse_omega, o_w, lse_w);
}

// K8 / kscale: the 8-bit copy of the keys the walk scores, or NULL for the keys themselves
static ra_status decode_common(const void* q, const ra_index* idx, const void* K, const void* V,
                               ra_dtype dt, const int8_t* K8, const float* kscale, const int32_t* budgets,
                               int64_t N, int64_t kv_stride, int sink, int window, int topk, int ef,
                               int expand, void* stream, float* out, float* lse, int32_t* ids,
                               ra_stats* stats) {
    if (!q || !K || !V || !out || !lse) RA_FAIL(RA_EINVAL, "NULL argument");
    RA_TRY(check_dtype(dt));
    if (!idx) RA_FAIL(RA_EINVAL, "index handle is NULL");
    if (N < idx->N)
        RA_FAIL(RA_ESHAPE, "N = %lld is below the %lld keys the index was built over", (long long)N,
                (long long)idx->N);
    if (kv_stride < N)
        RA_FAIL(RA_ESHAPE, "kv_stride %lld is below N = %lld", (long long)kv_stride, (long long)N);
    RA_TRY(check_decode_args(idx, idx->N, sink, window, topk));
    RA_TRY(check_search_args(topk, ef, expand));
    ra_index* ix = const_cast<ra_index*>(idx);
    RA_TRY(check_seeds_fit(ix, expand));
    if (!ids) {
        RA_TRY(grow((void**)&ix->ids_ws, &ix->ids_bytes,
                    (size_t)ix->n_seq * ix->n_q * topk * sizeof(int32_t)));
        ids = ix->ids_ws;
    }
    const size_t heads = (size_t)ix->n_seq * ix->n_q;
    if (ra_decode_needs_global_bitset(ix->N, ix->deg, ef, expand, topk))
        RA_TRY(grow((void**)&ix->bitset, &ix->bitset_bytes, heads * ((ix->N + 31) >> 5) * 4));
    int start_cap;
    const int32_t* start = start_sets(ix, &start_cap);
    return ra_launch_decode(q, ix->adj, ix->entry, K, V, dt, ix->n_seq, ix->n_q, ix->n_kv, ix->N, N,
                            kv_stride, ix->deg, sink, window, topk, ef, expand, ix->bitset, ix->coop,
                            ix->coop_silent ? RA_HELPERS_SILENT_ : ix->coop_mode, ix->coop_spin, start, start_cap, K8, kscale,
                            budgets, ix->n_seeds ? ix->seedx : nullptr, ix->seed_parts,
                            (hipStream_t)stream, out, lse, ids, stats);
}

extern "C" ra_status ra_decode_step_grown(const void* q, const ra_index* idx, const void* K,
                                          const void* V, ra_dtype dt, int64_t N, int64_t kv_stride,
                                          int sink, int window, int topk, int ef, int expand,
                                          void* stream, float* out, float* lse, int32_t* ids,
                                          ra_stats* stats) {
    return decode_common(q, idx, K, V, dt, nullptr, nullptr, nullptr, N, kv_stride, sink, window, topk, ef,
                         expand, stream, out, lse, ids, stats);
}

extern "C" ra_status ra_decode_step_q8(const void* q, const ra_index* idx, const void* K, const void* V,
                                       ra_dtype dt, const int8_t* K8, const float* scale, int64_t N,
                                       int sink, int window, int topk, int ef, int expand, void* stream,
                                       float* out, float* lse, int32_t* ids, ra_stats* stats) {
    if (!K8 || !scale) RA_FAIL(RA_EINVAL, "NULL argument");
    if (idx && N != idx->N)
        RA_FAIL(RA_ESHAPE, "N = %lld but the index was built over %lld keys", (long long)N,
                (long long)idx->N);
    return decode_common(q, idx, K, V, dt, K8, scale, nullptr, N, N, sink, window, topk, ef, expand, stream,
                         out, lse, ids, stats);
}

extern "C" ra_status ra_decode_step_budgets(const void* q, const ra_index* idx, const void* K, const void* V,
                                            ra_dtype dt, int64_t N, int sink, int window, int topk,
                                            const int32_t* topk_per_head, int ef, int expand, void* stream,
                                            float* out, float* lse, int32_t* ids, ra_stats* stats) {
    if (!topk_per_head) RA_FAIL(RA_EINVAL, "NULL argument");
    if (idx && N != idx->N)
        RA_FAIL(RA_ESHAPE, "N = %lld but the index was built over %lld keys", (long long)N,
                (long long)idx->N);
    return decode_common(q, idx, K, V, dt, nullptr, nullptr, topk_per_head, N, N, sink, window, topk, ef, expand,
                         stream, out, lse, ids, stats);
}

extern "C" ra_status ra_decode_step(const void* q, const ra_index* idx, const void* K, const void* V,
                                    ra_dtype dt, int64_t N, int sink, int window, int topk, int ef,
                                    int expand, void* stream, float* out, float* lse, int32_t* ids,
                                    ra_stats* stats) {
    if (idx && N != idx->N)
        RA_FAIL(RA_ESHAPE, "N = %lld but the index was built over %lld keys (ra_decode_step_grown "
                "accepts a longer cache)", (long long)N, (long long)idx->N);
    return ra_decode_step_grown(q, idx, K, V, dt, N, N, sink, window, topk, ef, expand, stream, out, lse,
                                ids, stats);
}

extern "C" ra_status ra_rerank(const void* q, const void* K, ra_dtype dt, int n_seq, int n_q, int n_kv,
                               int64_t N, int d, const int32_t* cand, int n_cand, int topk, void* stream,
                               int32_t* ids) {
    if (!q || !K || !cand || !ids) RA_FAIL(RA_EINVAL, "NULL argument");
    RA_TRY(check_dtype(dt));
    RA_TRY(check_heads(n_seq, n_q, n_kv));
    RA_TRY(check_dim(d));
    if (N < 1) RA_FAIL(RA_EINVAL, "N must be positive");
    if (topk < 1 || n_cand < topk) RA_FAIL(RA_EINVAL, "need 1 <= topk <= n_cand (got %d, %d)", topk, n_cand);
    if (n_cand > RA_MAX_TOPK) RA_FAIL(RA_EUNSUP, "n_cand %d exceeds RA_MAX_TOPK %d", n_cand, RA_MAX_TOPK);
    return ra_launch_rerank(q, K, dt, n_seq, n_q, n_kv, N, cand, n_cand, topk, (hipStream_t)stream, ids);
}

// ---- exact baselines (the paper's "Flat" retrieval and full attention) ---------------------
extern "C" size_t ra_flat_workspace_bytes(int n_seq, int n_q_heads, int64_t N) {
    if (n_seq < 1 || n_q_heads < 1 || N < 1) return 0;
    // one order-preserving key per (head, key), then 16 tile maxima per (head, chunk of 512 keys),
    // then the candidate counters of the second pass
    return (size_t)n_seq * n_q_heads * (N + 16 * ((N + 511) / 512) + RA_FLAT_SLICES) * sizeof(uint32_t);
}

extern "C" ra_status ra_flat_topk(const void* q, const void* K, ra_dtype dt, int n_seq, int n_q,
                                  int n_kv, int64_t N, int d, int sink, int window, int topk,
                                  void* workspace, size_t workspace_bytes, void* stream,
                                  int32_t* ids) {
    if (!q || !K || !ids || !workspace) RA_FAIL(RA_EINVAL, "NULL argument");
    RA_TRY(check_dtype(dt));
    RA_TRY(check_heads(n_seq, n_q, n_kv));
    RA_TRY(check_dim(d));
    if (N < 1) RA_FAIL(RA_EINVAL, "N must be positive");
    if (sink < 0 || window < 0) RA_FAIL(RA_EINVAL, "sink and window must be non-negative");
    if (topk < 1) RA_FAIL(RA_EINVAL, "topk must be positive");
    if (topk > RA_MAX_TOPK) RA_FAIL(RA_EUNSUP, "topk %d exceeds RA_MAX_TOPK %d", topk, RA_MAX_TOPK);
    if (workspace_bytes < ra_flat_workspace_bytes(n_seq, n_q, N))
        RA_FAIL(RA_ESHAPE, "workspace of %zu B is smaller than ra_flat_workspace_bytes", workspace_bytes);
    return ra_launch_flat_topk(q, K, dt, n_seq, n_q, n_kv, N, sink, window, topk,
                               (uint32_t*)workspace, (hipStream_t)stream, ids);
}

extern "C" ra_status ra_hbm_read_probe(const void* buf, size_t bytes, void* stream, uint64_t* out) {
    if (!buf || !out) RA_FAIL(RA_EINVAL, "NULL argument");
    if (bytes < 16 || (bytes & 15) || ((uintptr_t)buf & 15))
        RA_FAIL(RA_EINVAL, "the buffer must be 16-byte aligned and a multiple of 16 bytes long");
    return ra_launch_read_probe(buf, bytes, (hipStream_t)stream, reinterpret_cast<unsigned long long*>(out));
}

extern "C" ra_status ra_hbm_gather_probe(const void* buf, size_t bytes, size_t n_rows, uint32_t seed, void* stream,
                                         uint64_t* out) {
    if (!buf || !out) RA_FAIL(RA_EINVAL, "NULL argument");
    if (bytes < 256 || (bytes & 255) || ((uintptr_t)buf & 15))
        RA_FAIL(RA_EINVAL, "the buffer must be 16-byte aligned and a multiple of 256 bytes long");
    if (n_rows < 1) RA_FAIL(RA_EINVAL, "n_rows must be positive");
    return ra_launch_gather_probe(buf, bytes, n_rows, seed, (hipStream_t)stream,
                                  reinterpret_cast<unsigned long long*>(out));
}

extern "C" size_t ra_full_attention_workspace_bytes(int n_seq, int n_q_heads, int n_kv_heads,
                                                     int64_t N) {
    if (n_seq < 1 || n_q_heads < 1 || n_kv_heads < 1 || N < 1) return 0;
    // partial records of a fully static context, preceded by one padded id per head
    return 256 + (size_t)n_seq * n_q_heads * sizeof(int32_t) +
           ra_attend_partial_floats(n_seq, n_q_heads, n_kv_heads, N, (int)(N > 0x7fffffff ? 0x7fffffff : N),
                                    0, 1) * sizeof(float);
}

__global__ void api_fill_i32_kernel(int32_t* p, int n, int32_t v) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

extern "C" ra_status ra_full_attention(const void* q, const void* K, const void* V, ra_dtype dt,
                                       int n_seq, int n_q, int n_kv, int64_t N, int d,
                                       void* workspace, size_t workspace_bytes, void* stream,
                                       float* out, float* lse) {
    if (!q || !K || !V || !out || !lse || !workspace) RA_FAIL(RA_EINVAL, "NULL argument");
    RA_TRY(check_dtype(dt));
    RA_TRY(check_heads(n_seq, n_q, n_kv));
    RA_TRY(check_dim(d));
    if (N < 1) RA_FAIL(RA_EINVAL, "N must be positive");
    if (N > 0x7fffffff / 2) RA_FAIL(RA_EUNSUP, "N too large");
    if (workspace_bytes < ra_full_attention_workspace_bytes(n_seq, n_q, n_kv, N))
        RA_FAIL(RA_ESHAPE, "workspace of %zu B is smaller than ra_full_attention_workspace_bytes",
                workspace_bytes);
    const int heads = n_seq * n_q;
    int32_t* ids = (int32_t*)workspace;                       // one id per head, all -1: Omega is empty
    float* partials = (float*)((char*)workspace + ((heads * sizeof(int32_t) + 255) & ~(size_t)255));
    hipLaunchKernelGGL(api_fill_i32_kernel, dim3((heads + 255) / 256), dim3(256), 0,
                       (hipStream_t)stream, ids, heads, -1);
    // the whole context as the "static" set of Eq. 2: W = [0, N), Omega empty
    return ra_launch_attend(q, K, V, dt, n_seq, n_q, n_kv, N, (int)N, 0, 1, ids, partials,
                            (hipStream_t)stream, out, lse, nullptr, nullptr, nullptr, nullptr);
}

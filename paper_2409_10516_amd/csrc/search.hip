// Stand-alone launch of the graph search (ra_search); the search itself is in search_dev.h.
#include "search_dev.h"

template <int DT, bool GBITS, int T>
__global__ __launch_bounds__(T) void search_kernel(
    const void* __restrict__ q, const int32_t* __restrict__ adj, const int32_t* __restrict__ entry,
    const void* __restrict__ K, int n_q, int n_kv, int64_t N, int deg, int s, int w, int topk,
    int ef, int expand, uint32_t* __restrict__ gbits, int32_t* __restrict__ ids,
    ra_stats* __restrict__ stats) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    run_search<DT, GBITS, T>(lds_raw, xcd_aware_head(blockIdx.x, gridDim.x, n_q / n_kv), q, adj, entry, K, n_q, n_kv, N, N, deg, s, w, topk, ef,
                          expand, gbits, ids, stats, nullptr, NoHook());
}

__global__ void fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x)
        p[i] = v;
}

size_t ra_search_lds_bytes(int64_t N, int deg, int ef, int expand, bool global_bitset) {
    return search_lds_bytes(N, deg, ef, expand, global_bitset);
}

bool ra_search_needs_global_bitset(int64_t N, int deg, int ef, int expand) {
    return (size_t)((N + 31) >> 5) * 4 > SR_BITSET_LDS_MAX ||
           ra_search_lds_bytes(N, deg, ef, expand, false) > SR_LDS_LIMIT;
}

ra_status ra_launch_search(const void* q, const int32_t* adj, const int32_t* entry, const void* K,
                           ra_dtype dt, int n_seq, int n_q, int n_kv, int64_t N, int deg,
                           int sink, int window, int topk, int ef, int expand, uint32_t* bitset,
                           hipStream_t st, int32_t* ids, ra_stats* stats) {
    int64_t ss = sink < 0 ? 0 : sink, ww = window < 0 ? 0 : window;
    if (ss > N) ss = N;
    if (ww > N) ww = N;
    if (ss + ww >= N) { ss = N; ww = 0; }
    const bool gb = ra_search_needs_global_bitset(N, deg, ef, expand);
    const size_t lds = ra_search_lds_bytes(N, deg, ef, expand, gb);
    if (lds > SR_LDS_LIMIT)
        RA_FAIL(RA_EUNSUP, "search state needs %zu B of LDS (limit %d): lower ef or expand", lds,
                SR_LDS_LIMIT);
    const int heads = n_seq * n_q;
    if (gb) {
        if (!bitset) RA_FAIL(RA_EINVAL, "global visited bitset missing");
        const size_t words = (size_t)heads * ((N + 31) >> 5);
        hipLaunchKernelGGL(fill_u32_kernel, dim3(1024), dim3(256), 0, st, bitset, words, 0u);
    }
    const int threads = search_threads(heads, ef);
#define RA_SR_LAUNCH_T(DTV, GB, TV)                                                               \
    do {                                                                                          \
        RA_LDS_OPT_IN((search_kernel<DTV, GB, TV>), lds);                                         \
        hipLaunchKernelGGL((search_kernel<DTV, GB, TV>), dim3(heads), dim3(TV), lds, st, q, adj,  \
                           entry, K, n_q, n_kv, N, deg, (int)ss, (int)ww, topk, ef, expand,       \
                           bitset, ids, stats);                                                   \
    } while (0)
#define RA_SR_LAUNCH(DTV, GB)                                                                     \
    do {                                                                                          \
        if (threads == 1024) RA_SR_LAUNCH_T(DTV, GB, 1024);                                       \
        else if (threads == 512) RA_SR_LAUNCH_T(DTV, GB, 512);                                    \
        else RA_SR_LAUNCH_T(DTV, GB, 256);                                                        \
    } while (0)
    if (dt == RA_BF16) {
        if (gb) RA_SR_LAUNCH(RA_BF16, true); else RA_SR_LAUNCH(RA_BF16, false);
    } else {
        if (gb) RA_SR_LAUNCH(RA_F32, true); else RA_SR_LAUNCH(RA_F32, false);
    }
#undef RA_SR_LAUNCH_T
#undef RA_SR_LAUNCH
    RA_HIP(hipGetLastError());
    return RA_OK;
}

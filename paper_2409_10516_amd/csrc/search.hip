// Stand-alone launch of the graph search (ra_search); the search itself is in search_dev.h.
#include "search_dev.h"

template <int DT, int KT, bool GBITS, int T>
__global__ __launch_bounds__(T) void search_kernel(
    const void* __restrict__ q, const int32_t* __restrict__ adj, const int32_t* __restrict__ entry,
    const void* __restrict__ K, int n_q, int n_kv, int64_t N, int deg, int s, int w, int topk,
    int ef, int expand, uint32_t* __restrict__ gbits, int32_t* __restrict__ ids,
    ra_stats* __restrict__ stats, const int32_t* __restrict__ roots, int root_cap,
    const float* __restrict__ kscale) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    run_search<DT, KT, GBITS, T>(lds_raw, xcd_aware_head(blockIdx.x, gridDim.x, n_q / n_kv), q, adj, entry, K, n_q, n_kv, N, N, deg, s, w, topk, topk, ef,
                          expand, gbits, ids, stats, nullptr, roots, root_cap, kscale, NoHook());
}

__global__ void fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x)
        p[i] = v;
}


// Root sets (see run_search): per head [0] the number of ids, [1] 1 + the number of the entry
// point's neighbours, then the ids: the entry point, its distinct valid neighbours in row order,
// then the distinct valid neighbours of those that are not among the former, in row order.
// One workgroup per head; a build-time step, written for clarity rather than speed.
#define RT_THREADS 256
__global__ __launch_bounds__(RT_THREADS) void roots_kernel(const int32_t* __restrict__ adj,
                                                           const int32_t* __restrict__ entry, int64_t N,
                                                           int deg, int32_t* __restrict__ roots, int cap) {
    __shared__ int l1[RA_MAX_DEG + 1];
    __shared__ int l2[RA_MAX_DEG * RA_MAX_DEG];
    __shared__ unsigned char keep[RA_MAX_DEG * RA_MAX_DEG];
    __shared__ int n1s;
    const int tid = threadIdx.x, head = blockIdx.x;
    const int32_t* adj_h = adj + (size_t)head * N * deg;
    int32_t* out = roots + (size_t)head * cap;
    const int e0 = entry[head];
    if (tid == 0) {
        int n1 = 1;
        l1[0] = e0;
        for (int j = 0; j < deg; ++j) {
            const int nb = adj_h[(size_t)e0 * deg + j];
            bool ok = nb >= 0 && nb < N;
            for (int x = 0; ok && x < n1; ++x) ok = l1[x] != nb;
            if (ok) l1[n1++] = nb;
        }
        n1s = n1;
    }
    __syncthreads();
    const int n1 = n1s, cells = (n1 - 1) * deg;
    for (int x = tid; x < cells; x += RT_THREADS) {
        int nb = adj_h[(size_t)l1[1 + x / deg] * deg + x % deg];
        if (nb < 0 || nb >= N) nb = -1;
        for (int y = 0; nb >= 0 && y < n1; ++y)
            if (l1[y] == nb) nb = -1;
        l2[x] = nb;
    }
    __syncthreads();
    for (int x = tid; x < cells; x += RT_THREADS) {
        const int nb = l2[x];
        bool k = nb >= 0;
        for (int y = 0; k && y < x; ++y) k = l2[y] != nb;
        keep[x] = k;
    }
    __syncthreads();
    if (tid == 0) {
        int n = 0;
        for (int x = 0; x < n1; ++x) out[2 + n++] = l1[x];
        for (int x = 0; x < cells; ++x)
            if (keep[x]) out[2 + n++] = l2[x];
        out[0] = n;
        out[1] = n1;
    }
}

ra_status ra_launch_roots(const int32_t* adj, const int32_t* entry, int heads, int64_t N, int deg,
                          int32_t* roots, int cap, hipStream_t st) {
    if (deg > RA_MAX_DEG || cap < 3 + deg + deg * deg) RA_FAIL(RA_EINVAL, "root set buffer too small");
    hipLaunchKernelGGL(roots_kernel, dim3(heads), dim3(RT_THREADS), 0, st, adj, entry, N, deg, roots, cap);
    RA_HIP(hipGetLastError());
    return RA_OK;
}

// Seed sets: the first n_seeds positions, breadth first, of the binary tree that slots 0 and 1 of
// every adjacency row span from the entry point (position p has its children at 2p + 1 and 2p + 2;
// for a projected graph this is the head of the popularity order). Positions without a node and
// nodes already listed at an earlier position are dropped, the order kept. Layout of a root set
// with [1] = 0: no id enters the beam as expanded. One workgroup per head; a set-up step.
#define SD_THREADS 1024
__global__ __launch_bounds__(SD_THREADS) void seeds_kernel(const int32_t* __restrict__ adj,
                                                           const int32_t* __restrict__ entry, int64_t N,
                                                           int deg, int n_seeds, int32_t* __restrict__ seeds,
                                                           int cap) {
    __shared__ int pos[RA_MAX_SEEDS];
    __shared__ int keep[RA_MAX_SEEDS];
    __shared__ int wsum[SD_THREADS / RA_WAVE];
    const int tid = threadIdx.x, head = blockIdx.x;
    const int32_t* adj_h = adj + (size_t)head * N * deg;
    int32_t* out = seeds + (size_t)head * cap;
    for (int p = tid; p < n_seeds; p += SD_THREADS) {
        // the path from the root to position p: the bits of p + 1 below its leading one, high to low
        int cur = entry[head];
        const unsigned path = (unsigned)p + 1u;
        for (int b = 30 - __clz(path); b >= 0 && cur >= 0; --b) {
            const int slot = (path >> b) & 1u;
            cur = slot < deg ? adj_h[(size_t)cur * deg + slot] : -1;
            if (cur < 0 || cur >= N) cur = -1;
        }
        pos[p] = cur;
    }
    __syncthreads();
    for (int p = tid; p < n_seeds; p += SD_THREADS) {
        const int id = pos[p];
        bool k = id >= 0;
        for (int y = 0; k && y < p; ++y) k = pos[y] != id;
        keep[p] = k;
    }
    __syncthreads();
    // ordered compaction: RA_MAX_SEEDS <= 2 * SD_THREADS, two rounds of a workgroup-wide prefix sum
    int base = 0;
    for (int p0 = 0; p0 < n_seeds; p0 += SD_THREADS) {
        const int p = p0 + tid;
        const bool k = p < n_seeds && keep[p];
        const unsigned long long m = __ballot(k);
        const int lane = tid & (RA_WAVE - 1), wv = tid / RA_WAVE;
        if (lane == 0) wsum[wv] = __popcll(m);
        __syncthreads();
        int before = base, total = base;
        for (int x = 0; x < SD_THREADS / RA_WAVE; ++x) {
            if (x < wv) before += wsum[x];
            total += wsum[x];
        }
        if (k) out[2 + before + __popcll(m & ((1ull << lane) - 1ull))] = pos[p];
        base = total;
        __syncthreads();
    }
    if (tid == 0) {
        out[0] = base;
        out[1] = 0;
    }
}

ra_status ra_launch_seeds(const int32_t* adj, const int32_t* entry, int heads, int64_t N, int deg,
                          int n_seeds, int32_t* seeds, int cap, hipStream_t st) {
    if (n_seeds < 1 || n_seeds > RA_MAX_SEEDS || cap < 2 + n_seeds) RA_FAIL(RA_EINVAL, "seed set buffer too small");
    hipLaunchKernelGGL(seeds_kernel, dim3(heads), dim3(SD_THREADS), 0, st, adj, entry, N, deg, n_seeds, seeds, cap);
    RA_HIP(hipGetLastError());
    return RA_OK;
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
                           const int32_t* roots, int root_cap, const float* kscale, hipStream_t st,
                           int32_t* ids, ra_stats* stats) {
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
#define RA_SR_LAUNCH_T(DTV, KTV, GB, TV)                                                          \
    do {                                                                                          \
        RA_LDS_OPT_IN((search_kernel<DTV, KTV, GB, TV>), lds);                                    \
        hipLaunchKernelGGL((search_kernel<DTV, KTV, GB, TV>), dim3(heads), dim3(TV), lds, st, q,  \
                           adj, entry, K, n_q, n_kv, N, deg, (int)ss, (int)ww, topk, ef, expand,  \
                           bitset, ids, stats, roots, root_cap, kscale);                          \
    } while (0)
#define RA_SR_LAUNCH(DTV, KTV, GB)                                                                \
    do {                                                                                          \
        if (threads == 1024) RA_SR_LAUNCH_T(DTV, KTV, GB, 1024);                                  \
        else if (threads == 512) RA_SR_LAUNCH_T(DTV, KTV, GB, 512);                               \
        else RA_SR_LAUNCH_T(DTV, KTV, GB, 256);                                                   \
    } while (0)
    // K holds 8-bit keys when kscale is given (the query keeps its own type dt)
    if (dt == RA_BF16) {
        if (kscale) { if (gb) RA_SR_LAUNCH(RA_BF16, RA_KEYS_I8, true); else RA_SR_LAUNCH(RA_BF16, RA_KEYS_I8, false); }
        else if (gb) RA_SR_LAUNCH(RA_BF16, RA_BF16, true); else RA_SR_LAUNCH(RA_BF16, RA_BF16, false);
    } else {
        if (kscale) { if (gb) RA_SR_LAUNCH(RA_F32, RA_KEYS_I8, true); else RA_SR_LAUNCH(RA_F32, RA_KEYS_I8, false); }
        else if (gb) RA_SR_LAUNCH(RA_F32, RA_F32, true); else RA_SR_LAUNCH(RA_F32, RA_F32, false);
    }
#undef RA_SR_LAUNCH_T
#undef RA_SR_LAUNCH
    RA_HIP(hipGetLastError());
    return RA_OK;
}

// The order in which the exact KNN of Sec. 3.2 streams a head's keys.
//
// The top-knn selection is exact whatever the order, but its cost is not: a key goes through the
// selection's slow path whenever its score reaches the query's current threshold, and over a
// stream in storage order that happens about knn * ln(N / knn) times per query. Queries of one
// attention head share a large common component (they are out of distribution with respect to
// the keys, Sec. 2.4), so the keys that score high for the head's MEAN query score high for most
// of its queries. Streaming the keys by descending inner product with that mean raises every
// threshold within the first few stages, and the rest of the stream seldom reaches it.
//
// Three steps per head, none of which can change a result:
//   ko_meanq_kernel   sum of a strided sample of the head's prefill queries (fixed order)
//   ko_proxy_kernel   64-bit sort keys [~ordered(<mean, k_i>):32][i:32], all ones beyond N
//   ko_sort_*         bitonic sort, ascending: chunks in LDS, the wider exchanges in memory
// so entry p is the key of p-th largest inner product (lower id first among equals) and the KNN
// kernel reads the id of stream position p as the low word of entry p, ready to use.
#include "common.h"

typedef unsigned long long u64;

#define KO_SAMPLE 4096            // prefill queries summed per head (at most)
#define KO_CHUNK 8192             // sort keys a workgroup holds in LDS (64 KB)
#define KO_THREADS 1024

// grid: x = head. thread = (slice, dimension): slice s sums samples s, s + 8, ... in that order,
// then the 8 slices are added in order.
template <int DT>
__global__ __launch_bounds__(KO_THREADS) void ko_meanq_kernel(const void* __restrict__ Q, int64_t M,
                                                              float* __restrict__ mq) {
    __shared__ float part[KO_THREADS];
    const int graph = blockIdx.x, d = threadIdx.x % RA_D, s = threadIdx.x / RA_D;
    constexpr int SLICES = KO_THREADS / RA_D;
    const int64_t n_s = M < KO_SAMPLE ? M : KO_SAMPLE;
    float acc = 0.f;
    for (int64_t k = s; k < n_s; k += SLICES) {
        const int64_t j = k * M / n_s;
        const size_t at = ((size_t)graph * M + j) * RA_D + d;
        if constexpr (DT == RA_BF16)
            acc += __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(Q)[at] << 16);
        else
            acc += reinterpret_cast<const float*>(Q)[at];
    }
    part[threadIdx.x] = acc;
    __syncthreads();
    if (s == 0) {
        float t = 0.f;
        for (int i = 0; i < SLICES; ++i) t += part[i * RA_D + d];
        mq[(size_t)graph * RA_D + d] = t;
    }
}

// grid: x = block of 64 stream slots (16 lanes per key row), y = head.
template <int DT>
__global__ __launch_bounds__(KO_THREADS) void ko_proxy_kernel(const void* __restrict__ K,
                                                              const float* __restrict__ mq, int n_q,
                                                              int n_kv, int64_t N, int64_t N_pad,
                                                              u64* __restrict__ keys) {
    const int graph = blockIdx.y, seq = graph / n_q, h = graph % n_q, kvh = h / (n_q / n_kv);
    const int l16 = threadIdx.x & 15;
    const int64_t i = (int64_t)blockIdx.x * (KO_THREADS / 16) + threadIdx.x / 16;
    if (i >= N_pad) return;                     // whole 16-lane groups leave together
    const int64_t row = i < N ? i : N - 1;
    const float* m = mq + (size_t)graph * RA_D + 8 * l16;
    const size_t at = (((size_t)seq * n_kv + kvh) * N + row) * RA_D + 8 * l16;
    float k[8];
    if constexpr (DT == RA_BF16) {
        const uint4 u = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(K) + at);
        k[0] = bf16_lo(u.x); k[1] = bf16_hi(u.x); k[2] = bf16_lo(u.y); k[3] = bf16_hi(u.y);
        k[4] = bf16_lo(u.z); k[5] = bf16_hi(u.z); k[6] = bf16_lo(u.w); k[7] = bf16_hi(u.w);
    } else {
        const float4 a = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(K) + at);
        const float4 b = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(K) + at + 4);
        k[0] = a.x; k[1] = a.y; k[2] = a.z; k[3] = a.w; k[4] = b.x; k[5] = b.y; k[6] = b.z; k[7] = b.w;
    }
    float p = 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) p += k[c] * m[c];
    const int lane = threadIdx.x % RA_WAVE;
    p += __uint_as_float(lane_xor32<1>(__float_as_uint(p), lane));
    p += __uint_as_float(lane_xor32<2>(__float_as_uint(p), lane));
    p += __uint_as_float(lane_xor32<4>(__float_as_uint(p), lane));
    p += __uint_as_float(lane_xor32<8>(__float_as_uint(p), lane));
    if (p != p) p = 0.f;                        // an order is all that is wanted: any place will do
    // ids stay below 2^31, so the all-ones entries beyond N sort behind every key
    if (l16 == 0)
        keys[(size_t)graph * N_pad + i] =
            i < N ? ((u64)(~f32_ordered(p)) << 32) | (u64)(uint32_t)i : ~0ull;
}

// One exchange of the bitonic network on a chunk in LDS: element e and e ^ j, ascending overall
// (the run that holds global index g descends when g & k is set).
__device__ __forceinline__ void ko_exchange(u64* s, int e, int j, bool ascending) {
    const u64 a = s[e], b = s[e | j];
    if ((a > b) == ascending) { s[e] = b; s[e | j] = a; }
}

// grid: x = chunk, y = head. k_first == 0: sorts the chunk (all k up to its length); otherwise
// finishes stage k_first of the global network (j from half a chunk down to 1).
__global__ __launch_bounds__(KO_THREADS) void ko_sort_chunk_kernel(u64* __restrict__ keys, int64_t N_pad,
                                                                   int chunk, int64_t k_first) {
    extern __shared__ __align__(16) unsigned char ko_lds[];
    u64* s = reinterpret_cast<u64*>(ko_lds);
    const int64_t base = (int64_t)blockIdx.x * chunk;
    u64* g = keys + (size_t)blockIdx.y * N_pad + base;
    for (int e = threadIdx.x; e < chunk; e += KO_THREADS) s[e] = g[e];
    __syncthreads();
    const int pairs = chunk / 2;
    for (int64_t k = k_first ? k_first : 2; k_first ? k == k_first : k <= chunk; k <<= 1) {
        const int j_top = k > chunk ? chunk / 2 : (int)(k / 2);
        for (int j = j_top; j >= 1; j >>= 1) {
            for (int t = threadIdx.x; t < pairs; t += KO_THREADS) {
                const int e = ((t & ~(j - 1)) << 1) | (t & (j - 1));      // bit j clear
                ko_exchange(s, e, j, ((base + e) & k) == 0);
            }
            __syncthreads();
        }
    }
    for (int e = threadIdx.x; e < chunk; e += KO_THREADS) g[e] = s[e];
}

// grid: x = block of KO_THREADS pairs, y = head: the exchange at distance j >= chunk of stage k.
__global__ __launch_bounds__(KO_THREADS) void ko_sort_far_kernel(u64* __restrict__ keys, int64_t N_pad,
                                                                 int64_t k, int64_t j) {
    const int64_t t = (int64_t)blockIdx.x * KO_THREADS + threadIdx.x;
    if (t >= N_pad / 2) return;
    const int64_t e = ((t & ~(j - 1)) << 1) | (t & (j - 1));
    u64* g = keys + (size_t)blockIdx.y * N_pad;
    const u64 a = g[e], b = g[e | j];
    const bool ascending = (e & k) == 0;
    if ((a > b) == ascending) { g[e] = b; g[e | j] = a; }
}

static int64_t ko_padded(int64_t N) {
    int64_t p = 2;
    while (p < N) p <<= 1;
    return p;
}

// [n_graphs][N_pad] sort keys, then [n_graphs][RA_D] query sums
size_t ra_knn_order_bytes(int n_graphs, int64_t N) {
    return (size_t)n_graphs * ((size_t)ko_padded(N) * sizeof(u64) + RA_D * sizeof(float));
}

int64_t ra_knn_order_stride(int64_t N) { return ko_padded(N); }

// Fills workspace with the stream order of every head: entry p of head g, at
// workspace[g * ra_knn_order_stride(N) + p], holds the id of the key streamed p-th in its low word.
ra_status ra_launch_knn_order(const void* K, const void* Q, ra_dtype dt, int n_seq, int n_q, int n_kv,
                              int64_t N, int64_t M, void* workspace, hipStream_t st) {
    const int graphs = n_seq * n_q;
    if (graphs > 65535) RA_FAIL(RA_EUNSUP, "more than 65535 (sequence, query head) pairs");
    const int64_t N_pad = ko_padded(N);
    u64* keys = reinterpret_cast<u64*>(workspace);
    float* mq = reinterpret_cast<float*>(keys + (size_t)graphs * N_pad);
    const dim3 pgrid((unsigned)((N_pad + KO_THREADS / 16 - 1) / (KO_THREADS / 16)), (unsigned)graphs);
    if (dt == RA_BF16) {
        hipLaunchKernelGGL(ko_meanq_kernel<RA_BF16>, dim3(graphs), dim3(KO_THREADS), 0, st, Q, M, mq);
        hipLaunchKernelGGL(ko_proxy_kernel<RA_BF16>, pgrid, dim3(KO_THREADS), 0, st, K, mq, n_q, n_kv, N,
                           N_pad, keys);
    } else {
        hipLaunchKernelGGL(ko_meanq_kernel<RA_F32>, dim3(graphs), dim3(KO_THREADS), 0, st, Q, M, mq);
        hipLaunchKernelGGL(ko_proxy_kernel<RA_F32>, pgrid, dim3(KO_THREADS), 0, st, K, mq, n_q, n_kv, N,
                           N_pad, keys);
    }
    const int chunk = (int)(N_pad < KO_CHUNK ? N_pad : KO_CHUNK);
    const size_t lds = (size_t)chunk * sizeof(u64);
    const dim3 cgrid((unsigned)(N_pad / chunk), (unsigned)graphs);
    const dim3 fgrid((unsigned)((N_pad / 2 + KO_THREADS - 1) / KO_THREADS), (unsigned)graphs);
    RA_LDS_OPT_IN(ko_sort_chunk_kernel, lds);
    hipLaunchKernelGGL(ko_sort_chunk_kernel, cgrid, dim3(KO_THREADS), lds, st, keys, N_pad, chunk, (int64_t)0);
    for (int64_t k = 2 * (int64_t)chunk; k <= N_pad; k <<= 1) {
        for (int64_t j = k / 2; j >= chunk; j >>= 1)
            hipLaunchKernelGGL(ko_sort_far_kernel, fgrid, dim3(KO_THREADS), 0, st, keys, N_pad, k, j);
        hipLaunchKernelGGL(ko_sort_chunk_kernel, cgrid, dim3(KO_THREADS), lds, st, keys, N_pad, chunk, k);
    }
    RA_HIP(hipGetLastError());
    return RA_OK;
}

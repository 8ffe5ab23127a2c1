// Stand-alone attention launches (ra_attend); the device code is in attend_dev.h.
#include "attend_dev.h"

// grid: x = record slot (nS static chunks, then G x nG gathered chunks), y = KV head, z = seq.
// GQA groups of another size than the kernel is built for run as G = 1 with one grid row per query
// head, kv_div of which share a KV head (kv_div = 1 otherwise).
template <int DT, int G>
__global__ __launch_bounds__(AT_THREADS) void attend_partial_kernel(
    const void* __restrict__ q, const void* __restrict__ K, const void* __restrict__ V,
    const int32_t* __restrict__ ids, float* __restrict__ partials, int n_q, int n_kv, int64_t N,
    int s, int w, int topk, int nS, int nG, int sub, float scale, int kv_div) {
    extern __shared__ float smem[];
    const int kvh = blockIdx.y / kv_div, seq = blockIdx.z, x = blockIdx.x;
    const int P = nS + nG;
    const size_t esz = DT == RA_BF16 ? 2 : 4;
    const char* Kh = reinterpret_cast<const char*>(K) + ((size_t)seq * n_kv + kvh) * N * RA_D * esz;
    const char* Vh = reinterpret_cast<const char*>(V) + ((size_t)seq * n_kv + kvh) * N * RA_D * esz;
    const int h0 = blockIdx.y * G;
    const char* qg = reinterpret_cast<const char*>(q) + ((size_t)seq * n_q + h0) * RA_D * esz;
    float* rec_g = partials + ((size_t)seq * n_q + h0) * P * AT_RS;
    if (x < nS) {
        RowSrc src{nullptr, N, s, w, s + w, 0};
        if constexpr (DT == RA_BF16 && G <= 4) {
            if (sub > 1) {                      // a long dense range (full attention): logits on the matrix cores
                attend_chunk_mfma<G>(threadIdx.x, qg, Kh, Vh, src, x, sub, scale, rec_g + (size_t)x * AT_RS,
                                     (int64_t)P * AT_RS, smem);
                return;
            }
        }
        attend_chunk<DT, G>(threadIdx.x, true, qg, Kh, Vh, src, x, sub, scale, rec_g + (size_t)x * AT_RS,
                            (int64_t)P * AT_RS, smem);
    } else {
        const int t = x - nS, g = t / nG, c = t % nG;
        RowSrc src{ids + ((size_t)seq * n_q + h0 + g) * topk, N, 0, 0, topk, 0};
        attend_chunk<DT, 1>(threadIdx.x, true, qg + (size_t)g * RA_D * esz, Kh, Vh, src, c, 1, scale,
                            rec_g + ((size_t)g * P + nS + c) * AT_RS, 0, smem);
    }
}

// grid: x = query head, y = seq; block = n_slices x 128 threads (one per slice of the records and
// output dimension). A head with more than sixteen records (a long static range: full attention)
// has its batches of sixteen dealt to up to AT_MERGE_SLICES slices that run side by side and are
// folded through LDS, in slice order, by the first.
#define AT_MERGE_SLICES 8
__global__ __launch_bounds__(AT_MERGE_SLICES * RA_D) void attend_merge_kernel(
    const float* __restrict__ partials, int n_q, int nS, int nG, float* __restrict__ out,
    float* __restrict__ lse, float* __restrict__ o_om, float* __restrict__ lse_om,
    float* __restrict__ o_w, float* __restrict__ lse_w) {
    __shared__ float part[AT_MERGE_SLICES][2][3][RA_D];          // [slice][set][M, L, A][dimension]
    const size_t head = (size_t)blockIdx.y * n_q + blockIdx.x;
    const int t = threadIdx.x % RA_D, slice = threadIdx.x / RA_D, n_slices = blockDim.x / RA_D;
    float M[2] = {-INFINITY, -INFINITY}, L[2] = {0.f, 0.f}, A[2] = {0.f, 0.f};
    merge_accumulate<false>(partials + head * (nS + nG) * AT_RS, nS, nG, t, slice, n_slices, M, L, A);
    if (n_slices > 1) {
#pragma unroll
        for (int set = 0; set < 2; ++set) {
            part[slice][set][0][t] = M[set];
            part[slice][set][1][t] = L[set];
            part[slice][set][2][t] = A[set];
        }
        __syncthreads();
        if (slice != 0) return;
        for (int b = 1; b < n_slices; ++b)
#pragma unroll
            for (int set = 0; set < 2; ++set)
                merge_fold(M[set], L[set], A[set], part[b][set][0][t], part[b][set][1][t], part[b][set][2][t]);
    }
    merge_finish(M, L, A, t, head, out, lse, o_om, lse_om, o_w, lse_w);
}

// 64-row sub-chunks per static workgroup: 1 for the decode step's few hundred static rows, more
// when the static range is long (full attention), so that a head has at most AT_MAX_STATIC_RECORDS
// static records to combine. Measured for full attention over 131072 tokens, 8 KV heads (us per
// layer): 32 records 178, 64 records 115, 128 records 123, 256 records 136 (the kernel's 178 vector
// registers allow two workgroups per compute unit: 512 workgroups run side by side from start to end;
// builds held to fewer registers spill and take 150 us and more).
#ifndef AT_MAX_STATIC_RECORDS
#define AT_MAX_STATIC_RECORDS 64
#endif
static int static_sub(int rows) {
    int sub = 1;
    while (sub < 64 && (rows + AT_CH * sub - 1) / (AT_CH * sub) > AT_MAX_STATIC_RECORDS) sub <<= 1;
    return sub;
}

size_t ra_attend_partial_floats(int n_seq, int n_q, int n_kv, int64_t N, int sink, int window,
                                int topk) {
    int s, w;
    static_ranges(N, sink, window, &s, &w);
    const int sub = static_sub(s + w);
    const int nS = (s + w + AT_CH * sub - 1) / (AT_CH * sub), nG = (topk + AT_CH - 1) / AT_CH;
    return (size_t)n_seq * n_q * (nS + nG) * AT_RS;
}

template <int DT>
static ra_status launch_partial(int G, dim3 grid, size_t lds, hipStream_t st, const void* q,
                                const void* K, const void* V, const int32_t* ids, float* partials,
                                int n_q, int n_kv, int64_t N, int s, int w, int topk, int nS, int nG,
                                int sub, float scale) {
#define RA_AT_CASE(GG)                                                                          \
    case GG:                                                                                    \
        hipLaunchKernelGGL((attend_partial_kernel<DT, GG>), grid, dim3(AT_THREADS), lds, st, q, K, \
                           V, ids, partials, n_q, n_kv, N, s, w, topk, nS, nG, sub, scale, 1);  \
        break;
    switch (G) {
        RA_AT_CASE(1)
        RA_AT_CASE(2)
        RA_AT_CASE(4)
        RA_AT_CASE(8)
        default:                 // any other group size: every query head reads its rows itself
            grid.x = nS + nG;
            grid.y = n_q;
            hipLaunchKernelGGL((attend_partial_kernel<DT, 1>), grid, dim3(AT_THREADS), lds, st, q, K, V,
                               ids, partials, n_q, n_kv, N, s, w, topk, nS, nG, sub, scale, G);
    }
#undef RA_AT_CASE
    return RA_OK;
}

ra_status ra_launch_attend(const void* q, const void* K, const void* V, ra_dtype dt, int n_seq,
                           int n_q, int n_kv, int64_t N, int sink, int window, int topk,
                           const int32_t* ids, float* partials, hipStream_t st, float* out,
                           float* lse, float* o_omega, float* lse_omega, float* o_w,
                           float* lse_w) {
    int s, w;
    static_ranges(N, sink, window, &s, &w);
    const int G = n_q / n_kv;
    const int sub = static_sub(s + w);
    const int nS = (s + w + AT_CH * sub - 1) / (AT_CH * sub), nG = (topk + AT_CH - 1) / AT_CH;
    const float scale = 1.0f / sqrtf((float)RA_D);
    dim3 grid(nS + G * nG, n_kv, n_seq);
    const size_t lds = (size_t)AT_TEAM_LDS_FLOATS * sizeof(float);
    ra_status rc = dt == RA_BF16
        ? launch_partial<RA_BF16>(G, grid, lds, st, q, K, V, ids, partials, n_q, n_kv, N, s, w,
                                  topk, nS, nG, sub, scale)
        : launch_partial<RA_F32>(G, grid, lds, st, q, K, V, ids, partials, n_q, n_kv, N, s, w,
                                 topk, nS, nG, sub, scale);
    if (rc != RA_OK) return rc;
    RA_HIP(hipGetLastError());
    int slices = (nS + nG + 15) / 16;                     // one per batch of sixteen records, at most 8
    if (slices > AT_MERGE_SLICES) slices = AT_MERGE_SLICES;
    hipLaunchKernelGGL(attend_merge_kernel, dim3(n_q, n_seq), dim3(slices * RA_D), 0, st, partials, n_q, nS,
                       nG, out, lse, o_omega, lse_omega, o_w, lse_w);
    RA_HIP(hipGetLastError());
    return RA_OK;
}


// ---- ra_attend for callers that cannot allocate ---------------------------------------------------
// The partial records live in a file-scope device array instead of memory the handle allocates on
// first use. Every device the library runs on holds its own copy of the array at its own address;
// host code never passes the array's name to a kernel, only the address hipGetSymbolAddress gives
// for the current device (looked up once per device and kept).
static __device__ __align__(256) unsigned char scratch[RA_ATTEND_NOALLOC_SCRATCH_BYTES];
static void* g_scratch_addr[RA_MAX_DEVICES];

static ra_status scratch_address(void** out) {
    int dev = 0;
    RA_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= RA_MAX_DEVICES) RA_FAIL(RA_EUNSUP, "device %d out of range", dev);
    if (!g_scratch_addr[dev]) {
        void* p = nullptr;
        RA_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) RA_FAIL(RA_EHIP, "the scratch array has no address on device %d", dev);
        g_scratch_addr[dev] = p;
    }
    *out = g_scratch_addr[dev];
    return RA_OK;
}

ra_status ra_launch_attend_noalloc(const void* q, const void* K, const void* V, ra_dtype dt, int n_seq,
                                   int n_q, int n_kv, int64_t N, int sink, int window, int topk,
                                   const int32_t* ids, hipStream_t st, float* out, float* lse,
                                   float* o_omega, float* lse_omega, float* o_w, float* lse_w) {
    const size_t need = ra_attend_partial_floats(n_seq, n_q, n_kv, N, sink, window, topk) * sizeof(float);
    if (need > RA_ATTEND_NOALLOC_SCRATCH_BYTES)
        RA_FAIL(RA_EUNSUP, "the partial records of this call take %zu bytes, above the %u bytes "
                "ra_attend_noalloc keeps (use ra_attend)", need, (unsigned)RA_ATTEND_NOALLOC_SCRATCH_BYTES);
    void* ptr = nullptr;
    ra_status rc = scratch_address(&ptr);
    if (rc != RA_OK) return rc;
    // nothing to clear: every record the merge reads is written by this call's first kernel
    return ra_launch_attend(q, K, V, dt, n_seq, n_q, n_kv, N, sink, window, topk, ids,
                            reinterpret_cast<float*>(ptr), st, out, lse, o_omega, lse_omega, o_w, lse_w);
}

// Sparse attention over the retrieved set Omega (Eq. 2), dense attention over the static
// set W (Sec. 3.3), and their exact combination (Appendix A, Eq. 4-5).
//
// Split-row design for a part with 256 CUs and few heads in flight: the rows of W and of
// Omega are cut into chunks of 64; one workgroup turns one chunk into a partial record
// (un-normalised sum of exp(z - m) v, the local maximum m, the local sum l). W chunks
// are shared by the query heads of a GQA group (K/V rows are read once for all of them,
// Appendix C: one KV copy per group); Omega chunks belong to one query head. A second tiny
// kernel combines all records of a head with the re-scaling of Eq. 5 generalised from two
// sets to P sets, and can also emit the two set-level results (o_W, lse_W), (o_Omega,
// lse_Omega) of Eq. 4.
//
// Row access: 16 lanes read one 128-element row (16 B per lane for bf16, 2 x 16 B for
// fp32), so a wavefront fetches 4 rows per load instruction and a workgroup 16.
#include "common.h"

#define AT_CH 64            // rows per chunk
#define AT_RS 132           // floats per partial record: 128 acc, m, l, 2 pad
#define AT_THREADS 256

struct RowSrc {             // which context rows a chunk covers
    const int32_t* ids;     // gathered: ids of this head (nullptr for static)
    int64_t N;
    int s, w;               // static ranges [0,s) and [N-w,N)
    int count;              // rows available (Wn or topk)
};

__device__ __forceinline__ int64_t chunk_row(const RowSrc& src, int r) {
    if (r >= src.count) return -1;
    if (src.ids) {
        const int64_t id = src.ids[r];
        return id < src.N ? id : -1;          // -1 padding (or a bad id) is skipped
    }
    return r < src.s ? (int64_t)r : src.N - src.w + (r - src.s);
}

template <int DT>
__device__ __forceinline__ void load_row8(const void* base, int64_t row, int lane16, float* o) {
    if (DT == RA_BF16) {
        const uint4 u = *reinterpret_cast<const uint4*>(
            reinterpret_cast<const uint16_t*>(base) + row * RA_D + lane16 * 8);
        o[0] = bf16_lo(u.x); o[1] = bf16_hi(u.x); o[2] = bf16_lo(u.y); o[3] = bf16_hi(u.y);
        o[4] = bf16_lo(u.z); o[5] = bf16_hi(u.z); o[6] = bf16_lo(u.w); o[7] = bf16_hi(u.w);
    } else {
        const float4* p = reinterpret_cast<const float4*>(
            reinterpret_cast<const float*>(base) + row * RA_D + lane16 * 8);
        const float4 a = p[0], b = p[1];
        o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
        o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
    }
}

// One chunk for NH query heads that share the same K/V rows.
template <int DT, int NH>
__device__ void attend_chunk(const void* q0, const void* Kh, const void* Vh, const RowSrc& src,
                             int chunk, float scale, float* rec0, int64_t rec_stride,
                             float* smem) {
    const int tid = threadIdx.x, grp = tid >> 4, lane16 = tid & 15;
    float qv[NH][8], acc[NH][8], m[NH], l[NH];
#pragma unroll
    for (int g = 0; g < NH; ++g) {
        load_row8<DT>(q0, g, lane16, qv[g]);
        m[g] = -INFINITY;
        l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
    }
    constexpr int RPG = AT_CH / 16;    // rows per 16-lane group
    int64_t rid[RPG];
    float kv[RPG][8], vv[RPG][8];
#pragma unroll
    for (int i = 0; i < RPG; ++i) {
        rid[i] = chunk_row(src, chunk * AT_CH + grp + 16 * i);
        if (rid[i] >= 0) {
            load_row8<DT>(Kh, rid[i], lane16, kv[i]);
            load_row8<DT>(Vh, rid[i], lane16, vv[i]);
        }
    }
#pragma unroll
    for (int i = 0; i < RPG; ++i) {
        if (rid[i] < 0) continue;
#pragma unroll
        for (int g = 0; g < NH; ++g) {
            float dot = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) dot = fmaf(qv[g][e], kv[i][e], dot);
            dot += __shfl_xor(dot, 8, 16);
            dot += __shfl_xor(dot, 4, 16);
            dot += __shfl_xor(dot, 2, 16);
            dot += __shfl_xor(dot, 1, 16);
            const float z = dot * scale;
            const float mn = fmaxf(m[g], z);
            const float corr = expf(m[g] - mn);      // exp(-inf) = 0 on the first row
            const float p = expf(z - mn);
            l[g] = l[g] * corr + p;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[g][e] = fmaf(p, vv[i][e], acc[g][e] * corr);
            m[g] = mn;
        }
    }
    // combine the 16 row-groups of the workgroup, one head at a time
    float* sm = smem;                       // [16]
    float* sl = sm + 16;                    // [16]
    float* sa = sl + 16;                    // [16][128]
#pragma unroll
    for (int g = 0; g < NH; ++g) {
        if (g) __syncthreads();
        if (lane16 == 0) {
            sm[grp] = m[g];
            sl[grp] = l[g];
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) sa[grp * RA_D + lane16 * 8 + e] = acc[g][e];
        __syncthreads();
        if (tid < RA_D) {
            float mx = -INFINITY;
#pragma unroll
            for (int j = 0; j < 16; ++j) mx = fmaxf(mx, sm[j]);
            float a = 0.f, ll = 0.f;
            if (mx > -INFINITY) {
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const float wgt = expf(sm[j] - mx);
                    a = fmaf(sa[j * RA_D + tid], wgt, a);
                    ll = fmaf(sl[j], wgt, ll);
                }
            }
            float* rec = rec0 + g * rec_stride;
            rec[tid] = a;
            if (tid == 0) {
                rec[RA_D] = mx;
                rec[RA_D + 1] = ll;
            }
        }
    }
}

// grid: x = record slot (nS static chunks, then G x nG gathered chunks), y = KV head, z = seq
template <int DT, int G>
__global__ __launch_bounds__(AT_THREADS) void attend_partial_kernel(
    const void* __restrict__ q, const void* __restrict__ K, const void* __restrict__ V,
    const int32_t* __restrict__ ids, float* __restrict__ partials, int n_q, int n_kv, int64_t N,
    int s, int w, int topk, int nS, int nG, float scale) {
    extern __shared__ float smem[];
    const int kvh = blockIdx.y, seq = blockIdx.z, x = blockIdx.x;
    const int P = nS + nG;
    const size_t esz = DT == RA_BF16 ? 2 : 4;
    const char* Kh = reinterpret_cast<const char*>(K) + ((size_t)seq * n_kv + kvh) * N * RA_D * esz;
    const char* Vh = reinterpret_cast<const char*>(V) + ((size_t)seq * n_kv + kvh) * N * RA_D * esz;
    const int h0 = kvh * G;
    const char* qg = reinterpret_cast<const char*>(q) + ((size_t)seq * n_q + h0) * RA_D * esz;
    float* rec_g = partials + ((size_t)seq * n_q + h0) * P * AT_RS;
    if (x < nS) {
        RowSrc src{nullptr, N, s, w, s + w};
        attend_chunk<DT, G>(qg, Kh, Vh, src, x, scale, rec_g + (size_t)x * AT_RS,
                            (int64_t)P * AT_RS, smem);
    } else {
        const int t = x - nS, g = t / nG, c = t % nG;
        RowSrc src{ids + ((size_t)seq * n_q + h0 + g) * topk, N, 0, 0, topk};
        attend_chunk<DT, 1>(qg + (size_t)g * RA_D * esz, Kh, Vh, src, c, scale,
                            rec_g + ((size_t)g * P + nS + c) * AT_RS, 0, smem);
    }
}

// Combination of a head's records: Eq. 4-5 with the re-scaling factors written for P sets.
// grid: x = query head, y = seq; block = 128 threads (one per output dimension).
__global__ __launch_bounds__(RA_D) void attend_merge_kernel(
    const float* __restrict__ partials, int n_q, int nS, int nG, float* __restrict__ out,
    float* __restrict__ lse, float* __restrict__ o_om, float* __restrict__ lse_om,
    float* __restrict__ o_w, float* __restrict__ lse_w) {
    const int h = blockIdx.x, seq = blockIdx.y, t = threadIdx.x;
    const int P = nS + nG;
    const size_t head = (size_t)seq * n_q + h;
    const float* rec = partials + head * P * AT_RS;
    float M[2], L[2], A[2];
#pragma unroll
    for (int set = 0; set < 2; ++set) {
        const int lo = set == 0 ? 0 : nS, hi = set == 0 ? nS : P;
        float mx = -INFINITY;
        for (int i = lo; i < hi; ++i) mx = fmaxf(mx, rec[i * AT_RS + RA_D]);
        float a = 0.f, l = 0.f;
        if (mx > -INFINITY) {
            for (int i = lo; i < hi; ++i) {
                const float wgt = expf(rec[i * AT_RS + RA_D] - mx);
                a = fmaf(rec[i * AT_RS + t], wgt, a);
                l = fmaf(rec[i * AT_RS + RA_D + 1], wgt, l);
            }
        }
        M[set] = mx; L[set] = l; A[set] = a;
    }
    // set-level results of Eq. 4: o_W (set 0) and o_Omega (set 1)
    float* o_set[2] = {o_w, o_om};
    float* l_set[2] = {lse_w, lse_om};
#pragma unroll
    for (int set = 0; set < 2; ++set) {
        const bool empty = !(L[set] > 0.f);
        if (o_set[set]) o_set[set][head * RA_D + t] = empty ? 0.f : A[set] / L[set];
        if (l_set[set] && t == 0) l_set[set][head] = empty ? -INFINITY : M[set] + logf(L[set]);
    }
    // Eq. 5: gamma_i = exp(m_i - m) l_i / sum_j exp(m_j - m) l_j with m = max(m_1, m_2)
    const float mx = fmaxf(M[0], M[1]);
    float o = 0.f, ls = -INFINITY;
    if (mx > -INFINITY) {
        const float e0 = L[0] > 0.f ? expf(M[0] - mx) : 0.f;
        const float e1 = L[1] > 0.f ? expf(M[1] - mx) : 0.f;
        const float l = L[0] * e0 + L[1] * e1;
        o = (A[0] * e0 + A[1] * e1) / l;
        ls = mx + logf(l);
    }
    out[head * RA_D + t] = o;
    if (t == 0) lse[head] = ls;
}

static void static_ranges(int64_t N, int sink, int window, int* s, int* w) {
    int64_t ss = sink < 0 ? 0 : sink, ww = window < 0 ? 0 : window;
    if (ss > N) ss = N;
    if (ww > N) ww = N;
    if (ss + ww >= N) { ss = N; ww = 0; }
    *s = (int)ss;
    *w = (int)ww;
}

size_t ra_attend_partial_floats(int n_seq, int n_q, int n_kv, int64_t N, int sink, int window,
                                int topk) {
    int s, w;
    static_ranges(N, sink, window, &s, &w);
    const int nS = (s + w + AT_CH - 1) / AT_CH, nG = (topk + AT_CH - 1) / AT_CH;
    return (size_t)n_seq * n_q * (nS + nG) * AT_RS;
}

template <int DT>
static ra_status launch_partial(int G, dim3 grid, size_t lds, hipStream_t st, const void* q,
                                const void* K, const void* V, const int32_t* ids, float* partials,
                                int n_q, int n_kv, int64_t N, int s, int w, int topk, int nS, int nG,
                                float scale) {
#define RA_AT_CASE(GG)                                                                          \
    case GG:                                                                                    \
        hipLaunchKernelGGL((attend_partial_kernel<DT, GG>), grid, dim3(AT_THREADS), lds, st, q, K, \
                           V, ids, partials, n_q, n_kv, N, s, w, topk, nS, nG, scale);          \
        break;
    switch (G) {
        RA_AT_CASE(1)
        RA_AT_CASE(2)
        RA_AT_CASE(4)
        RA_AT_CASE(8)
        default:
            RA_FAIL(RA_EUNSUP, "query heads per KV head must be 1, 2, 4 or 8 (got %d)", G);
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
    const int nS = (s + w + AT_CH - 1) / AT_CH, nG = (topk + AT_CH - 1) / AT_CH;
    const float scale = 1.0f / sqrtf((float)RA_D);
    dim3 grid(nS + G * nG, n_kv, n_seq);
    const size_t lds = (size_t)(32 + 16 * RA_D) * sizeof(float);
    ra_status rc = dt == RA_BF16
        ? launch_partial<RA_BF16>(G, grid, lds, st, q, K, V, ids, partials, n_q, n_kv, N, s, w,
                                  topk, nS, nG, scale)
        : launch_partial<RA_F32>(G, grid, lds, st, q, K, V, ids, partials, n_q, n_kv, N, s, w,
                                 topk, nS, nG, scale);
    if (rc != RA_OK) return rc;
    RA_HIP(hipGetLastError());
    hipLaunchKernelGGL(attend_merge_kernel, dim3(n_q, n_seq), dim3(RA_D), 0, st, partials, n_q, nS,
                       nG, out, lse, o_omega, lse_omega, o_w, lse_w);
    RA_HIP(hipGetLastError());
    return RA_OK;
}

// Exact KNN from prefill queries to keys (Sec. 3.2, Fig. 2b): S = Q K^T on the matrix cores
// with the per-query top-knn selection fused behind it, so the M x N score matrix is never
// written anywhere.
//
// The product is computed transposed, one 32-key x 32-query block at a time:
//     C[key i][query j] += A[i][k] * B[k][j],  A = key rows, B = query rows,
// with v_mfma_f32_32x32x16_bf16 (bf16 inputs) or v_mfma_f32_32x32x2_f32 (fp32 inputs). In the
// 32x32 accumulator layout a lane holds ONE query column (lane % 32) and 16 key rows, so the
// selection threshold of a query is a single per-lane register: the common case is a
// max-tree over the lane's 16 scores and one compare. Only scores that reach the threshold
// (about knn * ln(N / knn) per query over the whole stream) take the insertion path, where the
// wavefront inserts them one at a time into the query's sorted list in LDS.
//
// A wavefront owns NQ x 32 queries for the whole key stream (their B operands stay in registers,
// and every key operand fetched feeds NQ MFMA chains); a workgroup is 4 wavefronts. Lists hold 64-bit keys
// [ordered(score):32][~id:32], so "larger key" is "(score descending, id ascending)".
// The inner-product summation order is the hardware's; identical key rows still score
// identically for a given query because they go through the same instruction sequence.
#include "common.h"

#define KN_THREADS 256

typedef unsigned long long u64;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ u64 knn_key(float score, int id) {
    return ((u64)f32_ordered(score) << 32) | (u64)(0xffffffffu - (uint32_t)id);
}
__device__ __forceinline__ int knn_key_id(u64 k) { return (int)(0xffffffffu - (uint32_t)k); }

// Insert (score, id) into the sorted list lst[0..knn) (all 64 lanes cooperate).
// Returns the list's new threshold: the score of its last entry, or -inf while not full.
__device__ __forceinline__ float knn_insert(u64* lst, int knn, float score, int id, int lane) {
    const u64 nk = knn_key(score, id);
    const u64 e = lane < knn ? lst[lane] : 0ull;
    const int pos = __popcll(__ballot(lane < knn && e > nk));   // sorted: a prefix beats nk
    if (pos < knn) {
        if (lane >= pos && lane < knn - 1) lst[lane + 1] = e;
        if (lane == pos) lst[pos] = nk;
    }
    const u64 last = lst[knn - 1];
    return last == 0ull ? -INFINITY : f32_from_ordered((uint32_t)(last >> 32));
}

template <int DT> struct Operand;
template <> struct Operand<RA_BF16> { bf16x8 v[8]; };     // 8 k-steps of 16
template <> struct Operand<RA_F32> { float v[64]; };      // 64 k-steps of 2

// The operand of lane (row = lane % 32, half = lane / 32): dimensions [64*half, 64*half+64)
// of the row. The same assignment is used for keys and queries, so any consistent split of
// the 128 dimensions over k-steps gives the same inner product.
template <int DT>
__device__ __forceinline__ void load_operand(const void* base, int64_t row, int half, Operand<DT>& o) {
    if constexpr (DT == RA_BF16) {
        const uint4* p = reinterpret_cast<const uint4*>(
            reinterpret_cast<const uint16_t*>(base) + row * RA_D + 64 * half);
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const uint4 u = p[s];
            o.v[s] = __builtin_bit_cast(bf16x8, u);
        }
    } else {
        const float4* p = reinterpret_cast<const float4*>(
            reinterpret_cast<const float*>(base) + row * RA_D + 64 * half);
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            const float4 f = p[s];
            o.v[4 * s] = f.x; o.v[4 * s + 1] = f.y; o.v[4 * s + 2] = f.z; o.v[4 * s + 3] = f.w;
        }
    }
}

template <int DT>
__device__ __forceinline__ f32x16 block_scores(const Operand<DT>& a, const Operand<DT>& b) {
    f32x16 c = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if constexpr (DT == RA_BF16) {
#pragma unroll
        for (int s = 0; s < 8; ++s)
            c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v[s], b.v[s], c, 0, 0, 0);
    } else {
#pragma unroll
        for (int s = 0; s < 64; ++s)
            c = __builtin_amdgcn_mfma_f32_32x32x2f32(a.v[s], b.v[s], c, 0, 0, 0);
    }
    return c;
}

// grid: x = block of NQ * 128 queries, y = graph (seq * n_q + h). A wavefront owns NQ sets of 32
// queries, so every key operand it loads feeds NQ MFMA chains.
template <int DT, int NQ>
__global__ __launch_bounds__(KN_THREADS) void knn_kernel(
    const void* __restrict__ K, const void* __restrict__ Q, int n_q, int n_kv, int64_t N, int64_t M,
    int knn, int32_t* __restrict__ L_out) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    constexpr int QPW = 32 * NQ, QPB = QPW * (KN_THREADS / RA_WAVE);
    u64* lists = reinterpret_cast<u64*>(lds_raw);           // [QPB][knn]
    const int tid = threadIdx.x, wv = tid / RA_WAVE, lane = tid % RA_WAVE;
    const int col = lane & 31, half = lane >> 5;
    const int graph = blockIdx.y, seq = graph / n_q, h = graph % n_q, kvh = h / (n_q / n_kv);
    const size_t esz = DT == RA_BF16 ? 2 : 4;
    const char* Kh = reinterpret_cast<const char*>(K) + ((size_t)seq * n_kv + kvh) * N * RA_D * esz;
    const char* Qh = reinterpret_cast<const char*>(Q) + (size_t)graph * M * RA_D * esz;
    const int64_t q0 = (int64_t)blockIdx.x * QPB + wv * QPW;   // first query of this wave

    for (int i = tid; i < QPB * knn; i += KN_THREADS) lists[i] = 0ull;
    u64* my_lists = lists + (size_t)wv * QPW * knn;

    Operand<DT> b[NQ];
#pragma unroll
    for (int sidx = 0; sidx < NQ; ++sidx) {
        int64_t qr = q0 + sidx * 32 + col;
        if (qr >= M) qr = M - 1;                   // clamp loads; such columns are never written
        load_operand<DT>(Qh, qr, half, b[sidx]);
    }
    __syncthreads();

    float tau[NQ];
#pragma unroll
    for (int sidx = 0; sidx < NQ; ++sidx) tau[sidx] = -INFINITY;
    const int64_t nblk = (N + 31) / 32;

    auto load_keys = [&](int64_t kb, Operand<DT>& dst) {
        int64_t kr = kb * 32 + col;
        if (kr >= N) kr = N - 1;
        load_operand<DT>(Kh, kr, half, dst);
    };
    // scores of one 32-key block against the wave's NQ query sets, then the selection
    auto process = [&](const Operand<DT>& a, int64_t kb) {
        f32x16 c[NQ];
#pragma unroll
        for (int sidx = 0; sidx < NQ; ++sidx) c[sidx] = block_scores<DT>(a, b[sidx]);
        const int64_t kbase = kb * 32;
#pragma unroll
        for (int sidx = 0; sidx < NQ; ++sidx) {
            f32x16& cs = c[sidx];
            if (kbase + 32 > N) {                  // ragged tail: rows beyond N never qualify
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (kbase + (r / 4) * 8 + half * 4 + (r % 4) >= N) cs[r] = -INFINITY;
            }
            float mx = fmaxf(cs[0], cs[1]);
#pragma unroll
            for (int r = 2; r < 16; ++r) mx = fmaxf(mx, cs[r]);
            if (__ballot(mx >= tau[sidx]) == 0ull) continue;
            // insertion path (rare after the first few blocks)
            u64* set_lists = my_lists + (size_t)sidx * 32 * knn;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                u64 mask = __ballot(cs[r] >= tau[sidx] && cs[r] > -INFINITY);
                while (mask) {
                    const int src = __ffsll((long long)mask) - 1;
                    const float sc = __shfl(cs[r], src);
                    const int id = (int)(kbase + (r / 4) * 8 + (src >> 5) * 4 + (r % 4));
                    const int jq = src & 31;
                    const float nt = knn_insert(set_lists + (size_t)jq * knn, knn, sc, id, lane);
                    if (col == jq) tau[sidx] = nt;
                    mask &= mask - 1;
                    mask &= __ballot(cs[r] >= tau[sidx] && cs[r] > -INFINITY);
                }
            }
        }
    };
    // two key-operand register sets: the next block's rows are requested before the current
    // block's MFMAs are issued, so their latency hides behind a whole block of matrix work
    Operand<DT> a0, a1;
    load_keys(0, a0);
    for (int64_t kb = 0; kb < nblk; kb += 2) {
        if (kb + 1 < nblk) load_keys(kb + 1, a1);
        process(a0, kb);
        if (kb + 1 >= nblk) break;
        if (kb + 2 < nblk) load_keys(kb + 2, a0);
        process(a1, kb + 1);
    }
    // write the ids, best first
    for (int jq = 0; jq < QPW; ++jq) {
        const int64_t qr = q0 + jq;
        if (qr >= M) break;
        if (lane < knn)
            L_out[((size_t)graph * M + qr) * knn + lane] = knn_key_id(my_lists[(size_t)jq * knn + lane]);
    }
}

ra_status ra_launch_knn(const void* K, const void* Q, ra_dtype dt, int n_seq, int n_q, int n_kv,
                        int64_t N, int64_t M, int knn, hipStream_t st, int32_t* L) {
    if (dt == RA_BF16) {
        constexpr int NQ = 2;
        constexpr int QPB = 32 * NQ * (KN_THREADS / RA_WAVE);
        const dim3 grid((unsigned)((M + QPB - 1) / QPB), (unsigned)(n_seq * n_q));
        const size_t lds = (size_t)QPB * knn * sizeof(u64);
        hipLaunchKernelGGL((knn_kernel<RA_BF16, NQ>), grid, dim3(KN_THREADS), lds, st, K, Q, n_q, n_kv,
                           N, M, knn, L);
    } else {
        constexpr int QPB = 32 * (KN_THREADS / RA_WAVE);
        const dim3 grid((unsigned)((M + QPB - 1) / QPB), (unsigned)(n_seq * n_q));
        const size_t lds = (size_t)QPB * knn * sizeof(u64);
        hipLaunchKernelGGL((knn_kernel<RA_F32, 1>), grid, dim3(KN_THREADS), lds, st, K, Q, n_q, n_kv,
                           N, M, knn, L);
    }
    RA_HIP(hipGetLastError());
    return RA_OK;
}

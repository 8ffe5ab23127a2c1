// One launch per layer for the whole decode step of Algorithm 1 (fixed static pattern): one
// workgroup per (sequence, query head) runs the graph search (search_dev.h) and then, without
// leaving the compute unit, Eq. 2 over W u Omega for its head: the retrieved ids are still
// in LDS, the 64 groups of 16 lanes share the rows of both sets round-robin, every group keeps
// an online (max, sum, weighted sum) over its rows, and the groups' partial results are
// combined with the re-scaling factors of Eq. 5 written for many sets (first across the four
// groups of a wavefront by lane exchange, then across the 16 wavefronts through LDS). Carrying
// the running maximum across both sets is the same arithmetic as computing o_W and o_Omega apart
// and combining them by Eq. 4.
//
// Nothing crosses workgroups, on purpose. A variant that computed the static rows once per GQA
// group in separate workgroups of the same launch, and let the last finisher combine, was
// measured: the agent-scope release/acquire it needs (the part has one L2 per XCD, so the
// fences write back and invalidate L2) cost about 18 us per launch, more than the whole
// attention. Here the four query heads of a group each read the 644 static rows themselves; their
// workgroups are placed on one XCD (xcd_aware_head), so the repeats, like the key rows the four
// searches have in common, are served by that XCD's L2 (measured: 12.8 MB of HBM traffic per
// 128K-context layer against 20.9 MB with workgroup id = head).
#include "attend_dev.h"
#include "search_dev.h"


struct Softmax8 {          // a lane's share of an online-softmax state: 8 of the 128 outputs
    float m, l, acc[8];
};

__device__ __forceinline__ void sm_merge(Softmax8& a, float mo, float lo, const float* acco) {
    const float mn = fmaxf(a.m, mo);
    if (mn == -INFINITY) return;                    // both empty
    const float ca = expf(a.m - mn), co = expf(mo - mn);
    a.l = a.l * ca + lo * co;
#pragma unroll
    for (int e = 0; e < 8; ++e) a.acc[e] = a.acc[e] * ca + acco[e] * co;
    a.m = mn;
}

// exp for the softmax weights: the hardware exponential for bf16 data (its error, about 1e-6
// relative for the exponents that matter, is far below the bf16 inputs'), the library one for fp32.
template <int DT>
__device__ __forceinline__ float sm_exp(float x) { return DT == RA_BF16 ? __expf(x) : expf(x); }

// One more row for a lane's online-softmax state: logit z, the lane's 8 values of the value row.
// The running maximum settles after a few rows, so the rescaling of the sums is skipped unless
// some lane of the wavefront sees a larger logit.
template <int DT>
__device__ __forceinline__ void sm_row(Softmax8& st, float z, const float* v) {
    if (__builtin_amdgcn_ballot_w64(z > st.m) != 0ull) {
        const float mn = fmaxf(st.m, z);
        const float corr = sm_exp<DT>(st.m - mn);       // exp(-inf) = 0 on the first row
        st.l *= corr;
#pragma unroll
        for (int e = 0; e < 8; ++e) st.acc[e] *= corr;
        st.m = mn;
    }
    const float p = sm_exp<DT>(z - st.m);
    st.l += p;
#pragma unroll
    for (int e = 0; e < 8; ++e) st.acc[e] = fmaf(p, v[e], st.acc[e]);
}

// The 8 values of a key or value row that a lane owns, as float32.
template <int DT>
__device__ __forceinline__ void row_floats(const RowBits<DT>& r, float* f) {
    if (DT == RA_BF16) {
        f[0] = bf16_lo(r.a.x); f[1] = bf16_hi(r.a.x); f[2] = bf16_lo(r.a.y); f[3] = bf16_hi(r.a.y);
        f[4] = bf16_lo(r.a.z); f[5] = bf16_hi(r.a.z); f[6] = bf16_lo(r.a.w); f[7] = bf16_hi(r.a.w);
    } else {
        f[0] = __uint_as_float(r.a.x); f[1] = __uint_as_float(r.a.y);
        f[2] = __uint_as_float(r.a.z); f[3] = __uint_as_float(r.a.w);
        f[4] = __uint_as_float(r.b.x); f[5] = __uint_as_float(r.b.y);
        f[6] = __uint_as_float(r.b.z); f[7] = __uint_as_float(r.b.w);
    }
}

// A lane's 8 query values in the form the attention logits want them: bf16 pairs stay packed and
// go through the two-element dot instruction (exact products, float32 sums), fp32 uses fma.
// (The search scores are not computed here: they decide ids and keep their own fixed order.)
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
template <int DT> struct LaneQuery;
template <> struct LaneQuery<RA_BF16> {
    uint4 q;
    __device__ __forceinline__ LaneQuery(const void* qrow, int lane16)
        : q(reinterpret_cast<const uint4*>(qrow)[lane16]) {}
    __device__ __forceinline__ float dot(const RowBits<RA_BF16>& k) const {
        float d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q.x), __builtin_bit_cast(bf16x2, k.a.x), 0.f, false);
        d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q.y), __builtin_bit_cast(bf16x2, k.a.y), d, false);
        d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q.z), __builtin_bit_cast(bf16x2, k.a.z), d, false);
        d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q.w), __builtin_bit_cast(bf16x2, k.a.w), d, false);
        return d;
    }
};
template <> struct LaneQuery<RA_F32> {
    float q[8];
    __device__ __forceinline__ LaneQuery(const void* qrow, int lane16) { load_q8<RA_F32>(qrow, lane16, q); }
    __device__ __forceinline__ float dot(const RowBits<RA_F32>& k) const {
        float f[8];
        row_floats<RA_F32>(k, f);
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) d = fmaf(q[e], f[e], d);
        return d;
    }
};

template <int DT, bool GBITS>
__global__ __launch_bounds__(SR_THREADS) void decode_kernel(
    const void* __restrict__ q, const int32_t* __restrict__ adj, const int32_t* __restrict__ entry,
    const void* __restrict__ K, const void* __restrict__ V, int n_q, int n_kv, int64_t Ng, int64_t N,
    int64_t kv_stride, int64_t wstart, int deg, int s, int topk, int ef, int expand,
    uint32_t* __restrict__ gbits,
    int32_t* __restrict__ ids, ra_stats* __restrict__ stats, int ids_off, float scale,
    float* __restrict__ out, float* __restrict__ lse) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int tid = threadIdx.x, grp = tid >> 4, lane16 = tid & 15;
    const int lane = tid & (RA_WAVE - 1), wv = tid / RA_WAVE;
    const int head = xcd_aware_head(blockIdx.x, gridDim.x, n_q / n_kv);
    const int seq = head / n_q, h = head % n_q, kvh = h / (n_q / n_kv);
    const size_t esz = DT == RA_BF16 ? 2 : 4;
    int32_t* lds_ids = reinterpret_cast<int32_t*>(lds_raw + ids_off);
    const char* Kh = reinterpret_cast<const char*>(K) + ((size_t)seq * n_kv + kvh) * kv_stride * RA_D * esz;
    const char* Vh = reinterpret_cast<const char*>(V) + ((size_t)seq * n_kv + kvh) * kv_stride * RA_D * esz;
    // The graph covers the first Ng of the N tokens now in the cache; W = [0, s) u [wstart, N) with
    // wstart <= Ng, so every token appended after the build is attended densely.
    const int cnt = run_search<DT, GBITS>(lds_raw, head, q, adj, entry, K, n_q, n_kv, Ng, kv_stride, deg,
                                          s, (int)(Ng - wstart), topk, ef, expand, gbits, ids, stats,
                                          lds_ids);
#ifdef SR_PHASE_CLOCKS
    const long long t_attn = clock64();
#endif
    // ---- Eq. 2 over Omega (rows [0, cnt): ids in LDS) and W (rows [cnt, cnt + s + N - wstart))
    const LaneQuery<DT> ql(reinterpret_cast<const char*>(q) + (size_t)head * RA_D * esz, lane16);
    constexpr int DC_ROWS = DT == RA_BF16 ? 6 : 3;       // rows in flight per 16-lane group
    const int R = cnt + s + (int)(N - wstart);
    Softmax8 st;
    st.m = -INFINITY;
    st.l = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) st.acc[e] = 0.f;
    for (int r0 = 0; r0 < R; r0 += SR_NG * DC_ROWS) {
        int64_t rid[DC_ROWS];
        RowBits<DT> kb[DC_ROWS], vb[DC_ROWS];
#pragma unroll
        for (int u = 0; u < DC_ROWS; ++u) {
            const int r = r0 + u * SR_NG + grp;
            int64_t id = -1;
            if (r < cnt) id = lds_ids[r];
            else if (r < R) id = r - cnt < s ? (int64_t)(r - cnt) : wstart + (r - cnt - s);
            rid[u] = id;
            const int64_t safe = id >= 0 ? id : 0;      // loads stay unconditional
            kb[u] = load_key<DT>(Kh, safe, lane16);
            vb[u] = load_key<DT>(Vh, safe, lane16);
        }
#pragma unroll
        for (int u = 0; u < DC_ROWS; ++u) {
            if (rid[u] < 0) continue;
            float dot = ql.dot(kb[u]);
            dot += at_dpp<0xB1>(dot);
            dot += at_dpp<0x4E>(dot);
            dot += at_dpp<0x141>(dot);
            dot += at_dpp<0x140>(dot);
            float v[8];
            row_floats<DT>(vb[u], v);
            sm_row<DT>(st, dot * scale, v);
        }
    }
    // ---- combine the four groups of each wavefront by lane exchange
#pragma unroll
    for (int d = 16; d <= 32; d <<= 1) {
        const float mo = __shfl_xor(st.m, d), lo = __shfl_xor(st.l, d);
        float ao[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) ao[e] = __shfl_xor(st.acc[e], d);
        sm_merge(st, mo, lo, ao);
    }
    // ---- then the 16 wavefronts through LDS (the search state is dead; ids sit behind it)
    float* sm = reinterpret_cast<float*>(lds_raw);          // [16]
    float* sl = sm + SR_THREADS / RA_WAVE;                   // [16]
    float* sa = sl + SR_THREADS / RA_WAVE;                   // [16][128]
    if (lane < 16) {
        if (lane == 0) {
            sm[wv] = st.m;
            sl[wv] = st.l;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) sa[wv * RA_D + lane * 8 + e] = st.acc[e];
    }
    __syncthreads();
    if (tid < RA_D) {
        float mx = -INFINITY;
#pragma unroll
        for (int j = 0; j < SR_THREADS / RA_WAVE; ++j) mx = fmaxf(mx, sm[j]);
        float a = 0.f, l = 0.f;
        if (mx > -INFINITY) {
#pragma unroll
            for (int j = 0; j < SR_THREADS / RA_WAVE; ++j) {
                const float wgt = expf(sm[j] - mx);
                a = fmaf(sa[j * RA_D + tid], wgt, a);
                l = fmaf(sl[j], wgt, l);
            }
        }
        const bool empty = !(l > 0.f);
        out[(size_t)head * RA_D + tid] = empty ? 0.f : a / l;
        if (tid == 0) lse[head] = empty ? -INFINITY : mx + logf(l);
    }
#ifdef SR_PHASE_CLOCKS
    if (tid == 0 && blockIdx.x < 64) sr_phase_ticks[blockIdx.x * SR_NITER * SR_NPHASE + 7] += clock64() - t_attn;
#endif
}

#ifdef SR_PHASE_CLOCKS
// Tuning builds only: copy the phase clocks of the fused kernel to `host` (64 x 16 x 8 values: workgroup,
// search step, phase) and clear them.
extern "C" int ra_dbg_phase_ticks(long long* host) {
    if (hipMemcpyFromSymbol(host, HIP_SYMBOL(sr_phase_ticks), sizeof(long long) * 64 * SR_NITER * SR_NPHASE) != hipSuccess)
        return 1;
    static long long zeros[64 * SR_NITER * SR_NPHASE];
    return hipMemcpyToSymbol(HIP_SYMBOL(sr_phase_ticks), zeros, sizeof(zeros)) != hipSuccess;
}
#endif

static size_t decode_lds_bytes(int64_t N, int deg, int ef, int expand, int topk, bool gb, int* ids_off) {
    size_t a = search_lds_bytes(N, deg, ef, expand, gb);
    const size_t b = (size_t)(SR_THREADS / RA_WAVE) * (RA_D + 2) * sizeof(float);
    if (b > a) a = b;
    a = (a + 15) & ~(size_t)15;
    *ids_off = (int)a;
    return a + (size_t)topk * sizeof(int32_t);
}

bool ra_decode_needs_global_bitset(int64_t N, int deg, int ef, int expand, int topk) {
    int off;
    return (size_t)((N + 31) >> 5) * 4 > SR_BITSET_LDS_MAX ||
           decode_lds_bytes(N, deg, ef, expand, topk, false, &off) > SR_LDS_LIMIT;
}

__global__ void dc_fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x)
        p[i] = v;
}

ra_status ra_launch_decode(const void* q, const int32_t* adj, const int32_t* entry, const void* K,
                           const void* V, ra_dtype dt, int n_seq, int n_q, int n_kv, int64_t Ng, int64_t N,
                           int64_t kv_stride, int deg, int sink, int window, int topk, int ef, int expand,
                           uint32_t* bitset, hipStream_t st, float* out, float* lse, int32_t* ids,
                           ra_stats* stats) {
    // W = [0, s) u [wstart, N): the sink, the sliding window, and every token appended after the
    // index was built (wstart <= Ng); overlapping ranges make everything static
    int64_t s = sink < 0 ? 0 : sink, ww = window < 0 ? 0 : window;
    if (s > N) s = N;
    if (ww > N) ww = N;
    int64_t wstart = N - ww < Ng ? N - ww : Ng;
    if (s >= wstart) { s = 0; wstart = 0; }
    if (N - wstart + s > 0x3fffffff) RA_FAIL(RA_EUNSUP, "static set too large");
    const int heads = n_seq * n_q;
    const bool gb = ra_decode_needs_global_bitset(Ng, deg, ef, expand, topk);
    int ids_off;
    const size_t lds = decode_lds_bytes(Ng, deg, ef, expand, topk, gb, &ids_off);
    if (lds > SR_LDS_LIMIT)
        RA_FAIL(RA_EUNSUP, "decode state needs %zu B of LDS (limit %d): lower ef or expand", lds,
                SR_LDS_LIMIT);
    if (gb) {
        if (!bitset) RA_FAIL(RA_EINVAL, "global visited bitset missing");
        const size_t words = (size_t)heads * ((Ng + 31) >> 5);
        hipLaunchKernelGGL(dc_fill_u32_kernel, dim3(1024), dim3(256), 0, st, bitset, words, 0u);
    }
    const float scale = 1.0f / sqrtf((float)RA_D);
#define RA_DC_GO(DTV, GB)                                                                          \
    do {                                                                                           \
        RA_LDS_OPT_IN((decode_kernel<DTV, GB>), lds);                                              \
        hipLaunchKernelGGL((decode_kernel<DTV, GB>), dim3(heads), dim3(SR_THREADS), lds, st, q,    \
                           adj, entry, K, V, n_q, n_kv, Ng, N, kv_stride, wstart, deg, (int)s,     \
                           topk, ef, expand, bitset, ids, stats, ids_off, scale, out, lse);        \
    } while (0)
    if (dt == RA_BF16) {
        if (gb) RA_DC_GO(RA_BF16, true); else RA_DC_GO(RA_BF16, false);
    } else {
        if (gb) RA_DC_GO(RA_F32, true); else RA_DC_GO(RA_F32, false);
    }
#undef RA_DC_GO
    RA_HIP(hipGetLastError());
    return RA_OK;
}

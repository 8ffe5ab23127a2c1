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
// Device functions shared by the stand-alone attention kernels and the fused decode kernel.
//
// Row access: 16 lanes read one 128-element row (16 B per lane for bf16, 2 x 16 B for
// fp32), so a wavefront fetches 4 rows per load instruction and a workgroup 16.
#pragma once
#include "common.h"

#define AT_CH 64            // rows per chunk
#define AT_RS 132           // floats per partial record: 128 acc, m, l, 2 pad
#define AT_THREADS 256

struct RowSrc {             // which context rows a chunk covers
    const int32_t* ids;     // gathered: ids of this head (nullptr for static)
    int64_t N;
    int s, w;               // static ranges [0,s) and [N-w,N)
    int count;              // rows available (Wn or topk)
    int interleave;         // 0: chunk c covers rows [64c, 64c+64). T > 0: T teams share rows
                            // round-robin, chunk c / local row j covers row
                            // (c / T) * 64 T + (c % T) * 16 + j % 16 + 16 T (j / 16)
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

template <int CTRL>
__device__ __forceinline__ float at_dpp(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}

// The 8 values of a row that a lane owns, as loaded (16 bytes of bf16 or 32 bytes of fp32).
template <int DT> struct Row8;
template <> struct Row8<RA_BF16> { uint4 a; };
template <> struct Row8<RA_F32> { float4 a, b; };

template <int DT>
__device__ __forceinline__ Row8<DT> load_row8_raw(const void* base, int64_t row, int lane16) {
    Row8<DT> r;
    if constexpr (DT == RA_BF16) {
        r.a = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(base) + row * RA_D +
                                              lane16 * 8);
    } else {
        const float4* p = reinterpret_cast<const float4*>(reinterpret_cast<const float*>(base) +
                                                          row * RA_D + lane16 * 8);
        r.a = p[0];
        r.b = p[1];
    }
    return r;
}
// the same with non-temporal loads, for long dense ranges that are streamed once
typedef unsigned int at_u32x4 __attribute__((ext_vector_type(4)));
template <int DT>
__device__ __forceinline__ Row8<DT> load_row8_stream(const void* base, int64_t row, int lane16) {
    Row8<DT> r;
    if constexpr (DT == RA_BF16) {
        const at_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const at_u32x4*>(
            reinterpret_cast<const uint16_t*>(base) + row * RA_D + lane16 * 8));
        r.a = make_uint4(v.x, v.y, v.z, v.w);
    } else {
        const at_u32x4* p = reinterpret_cast<const at_u32x4*>(reinterpret_cast<const float*>(base) +
                                                              row * RA_D + lane16 * 8);
        const at_u32x4 a = __builtin_nontemporal_load(p), b = __builtin_nontemporal_load(p + 1);
        r.a = make_float4(__uint_as_float(a.x), __uint_as_float(a.y), __uint_as_float(a.z), __uint_as_float(a.w));
        r.b = make_float4(__uint_as_float(b.x), __uint_as_float(b.y), __uint_as_float(b.z), __uint_as_float(b.w));
    }
    return r;
}
template <int DT>
__device__ __forceinline__ void row8_floats(const Row8<DT>& r, float* o) {
    if constexpr (DT == RA_BF16) {
        o[0] = bf16_lo(r.a.x); o[1] = bf16_hi(r.a.x); o[2] = bf16_lo(r.a.y); o[3] = bf16_hi(r.a.y);
        o[4] = bf16_lo(r.a.z); o[5] = bf16_hi(r.a.z); o[6] = bf16_lo(r.a.w); o[7] = bf16_hi(r.a.w);
    } else {
        o[0] = r.a.x; o[1] = r.a.y; o[2] = r.a.z; o[3] = r.a.w;
        o[4] = r.b.x; o[5] = r.b.y; o[6] = r.b.z; o[7] = r.b.w;
    }
}
// exp for the softmax weights: the hardware exponential for bf16 data (its error is far below the
// inputs'), the library one for fp32
template <int DT>
__device__ __forceinline__ float at_exp(float x) { return DT == RA_BF16 ? __expf(x) : expf(x); }

// The closing step of a chunk: the (max, sum, weighted sum) states of the 16 lane groups of a team,
// each lane holding 8 of the 128 outputs of its group, become one partial record per head.
template <int NH>
__device__ __forceinline__ void chunk_records(int tid, bool active, const float (&m)[NH], const float (&l)[NH],
                                              const float (&acc)[NH][8], float* rec0, int64_t rec_stride,
                                              float* smem) {
    const int grp = tid >> 4, lane16 = tid & 15;
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
        if (tid < RA_D && active) {
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

// One chunk for NH query heads that share the same K/V rows.
// A call covers `n_sub` consecutive sub-chunks of 64 rows (1 for the decode step; more when a
// long dense range is streamed, so that the number of partial records stays small).
// `tid` is the thread's index inside its team of AT_THREADS threads (a workgroup may hold
// several teams, each with its own `smem`; every team must call this the same number of
// times because it contains workgroup barriers). An inactive team computes on an empty row
// source and writes nothing.
template <int DT, int NH>
__device__ void attend_chunk(int tid, bool active, const void* q0, const void* Kh, const void* Vh,
                             const RowSrc& src, int chunk, int n_sub, float scale, float* rec0,
                             int64_t rec_stride, float* smem) {
    const int grp = tid >> 4, lane16 = tid & 15;
    float qv[NH][8], acc[NH][8], m[NH], l[NH];
#pragma unroll
    for (int g = 0; g < NH; ++g) {
        load_row8<DT>(q0, g, lane16, qv[g]);
        m[g] = -INFINITY;
        l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
    }
    constexpr int RPG = AT_CH / 16;    // rows per 16-lane group and sub-chunk
    // The call covers sub-chunks [chunk * n_sub, (chunk + 1) * n_sub) of 64 rows each. The rows of
    // the next sub-chunk are requested (raw, 16 or 32 bytes per lane and row) before the current
    // one is worked through. Loads are never branched around: a row that does not exist reads
    // row 0 and is skipped, a sub-chunk past the end repeats the last one and is not used.
    const int sub_end = (chunk + 1) * n_sub;
    auto rows_of = [&](int sub, int64_t (&rid)[RPG]) {
        if (sub >= sub_end) sub = sub_end - 1;
#pragma unroll
        for (int i = 0; i < RPG; ++i) {
            const int r = src.interleave
                ? (sub / src.interleave) * AT_CH * src.interleave + (sub % src.interleave) * 16 + grp +
                      16 * src.interleave * i
                : sub * AT_CH + grp + 16 * i;
            rid[i] = chunk_row(src, r);
        }
    };
    auto fetch = [&](const int64_t (&rid)[RPG], Row8<DT> (&kr)[RPG], Row8<DT> (&vr)[RPG]) {
#pragma unroll
        for (int i = 0; i < RPG; ++i) {
            const int64_t row = rid[i] >= 0 ? rid[i] : 0;
            if (n_sub > 1) {                    // a long dense range, streamed once
                kr[i] = load_row8_stream<DT>(Kh, row, lane16);
                vr[i] = load_row8_stream<DT>(Vh, row, lane16);
            } else {
                kr[i] = load_row8_raw<DT>(Kh, row, lane16);
                vr[i] = load_row8_raw<DT>(Vh, row, lane16);
            }
        }
    };
    // One sub-chunk: the RPG logits of every head first (independent chains the compiler can
    // interleave), then one move of the running maximum per head and sub-chunk, then the weighted
    // sums. No branch separates the rows: the dependent latencies of one (row, head) hide behind
    // the others' work.
    auto consume = [&](const int64_t (&rid)[RPG], const Row8<DT> (&kr)[RPG], const Row8<DT> (&vr)[RPG]) {
        float z[NH][RPG];
#pragma unroll
        for (int i = 0; i < RPG; ++i) {
            float kv[8];
            row8_floats<DT>(kr[i], kv);
            const bool have = rid[i] >= 0;
#pragma unroll
            for (int g = 0; g < NH; ++g) {
                float dot = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) dot = fmaf(qv[g][e], kv[e], dot);
                dot += at_dpp<0xB1>(dot);      // xor 1
                dot += at_dpp<0x4E>(dot);      // xor 2
                dot += at_dpp<0x141>(dot);     // half-mirror: the other quad pair of the row of 8
                dot += at_dpp<0x140>(dot);     // mirror: the other half of the row of 16
                z[g][i] = have ? dot * scale : -INFINITY;
            }
        }
        float p[NH][RPG];
#pragma unroll
        for (int g = 0; g < NH; ++g) {
            float mn = m[g];
#pragma unroll
            for (int i = 0; i < RPG; ++i) mn = fmaxf(mn, z[g][i]);
            // exp(-inf - finite) = 0 rescales the empty sums of the first rows; nothing to do while
            // every row so far was missing
            const float corr = mn > -INFINITY ? at_exp<DT>(m[g] - mn) : 1.f;
            m[g] = mn;
            float lsum = 0.f;
#pragma unroll
            for (int i = 0; i < RPG; ++i) {
                p[g][i] = z[g][i] > -INFINITY ? at_exp<DT>(z[g][i] - mn) : 0.f;
                lsum += p[g][i];
            }
            l[g] = fmaf(l[g], corr, lsum);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[g][e] *= corr;
        }
#pragma unroll
        for (int i = 0; i < RPG; ++i) {
            float vv[8];
            row8_floats<DT>(vr[i], vv);
#pragma unroll
            for (int g = 0; g < NH; ++g)
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[g][e] = fmaf(p[g][i], vv[e], acc[g][e]);
        }
    };
    {
        int64_t rid_a[RPG], rid_b[RPG];
        Row8<DT> k_a[RPG], v_a[RPG], k_b[RPG], v_b[RPG];
        int sub = chunk * n_sub;
        rows_of(sub, rid_a);
        fetch(rid_a, k_a, v_a);
        if (n_sub == 1) {                     // the decode step's short sets: nothing to run ahead of
            consume(rid_a, k_a, v_a);
            sub = sub_end;
        }
        for (; sub < sub_end; sub += 2) {
            rows_of(sub + 1, rid_b);
            fetch(rid_b, k_b, v_b);
            consume(rid_a, k_a, v_a);
            if (sub + 1 >= sub_end) break;
            rows_of(sub + 2, rid_a);
            fetch(rid_a, k_a, v_a);
            consume(rid_b, k_b, v_b);
        }
    }
    chunk_records<NH>(tid, active, m, l, acc, rec0, rec_stride, smem);
}

// The same chunk for a long dense range of bf16 rows and up to four heads, with the logits on the
// matrix cores: S = Q K^T is a dense contraction, and on the vector units its 16-lane sums and the
// redundant softmax of every lane cost about as much issue time as the K / V streams leave. A
// wavefront owns 16 consecutive rows of each sub-chunk of 64. v_mfma_f32_16x16x32_bf16 takes them
// as its 32 x 16 operand (lane l: row l % 16, the 16 bytes at 64 j + 16 (l / 16) of the row for
// instruction j = 0..3: four lanes read 64 consecutive bytes, four instructions the whole row) and
// the queries as its 16 x 32 operand (row h = head h, the same bytes of the query; rows past the
// last head are zero), so lane n < 16 ends with the logits of row n for every head. Those lanes do
// the softmax bookkeeping once per row (running maximum shared by the wavefront, weights, their
// sum); the weighted sum of V stays on the vector units with 16 lanes per V row as elsewhere, each
// lane fetching the weight of its row from the lane that computed it. The sum over the 128
// dimensions is rounded in the hardware's order (tolerance of Eq. 1 as for the other path).
__device__ __forceinline__ float first_lane_f32(float v) {        // the builtin moves 32 bits, typed as an integer
    return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(v)));
}
typedef __bf16 at_bf16x8 __attribute__((ext_vector_type(8)));
typedef float at_f32x4 __attribute__((ext_vector_type(4)));
template <int NH>
__device__ void attend_chunk_mfma(int tid, const void* q0, const void* Kh, const void* Vh, const RowSrc& src,
                                  int chunk, int n_sub, float scale, float* rec0, int64_t rec_stride,
                                  float* smem) {
    static_assert(NH >= 1 && NH <= 4, "the heads sit in the first four rows of the query operand");
    const int wv = tid >> 6, lane = tid & 63, n = lane & 15, c = lane >> 4, lane16 = n;
    uint4 qa[4];
    {
        const uint4* qrow = reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(q0) +
                                                           (size_t)(n < NH ? n : 0) * RA_D);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint4 v = qrow[4 * j + c];
            qa[j] = n < NH ? v : make_uint4(0u, 0u, 0u, 0u);
        }
    }
    float acc[NH][8], m[NH], lpart[NH];
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        m[h] = -INFINITY;
        lpart[h] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[h][e] = 0.f;
    }
    struct Tile { int64_t rk; uint4 kb[4]; Row8<RA_BF16> vb[4]; };
    const int sub_end = (chunk + 1) * n_sub;
    auto fetch = [&](int sub, Tile& t) {
        if (sub >= sub_end) sub = sub_end - 1;       // past the end: the last one again, unused
        const int rb = sub * AT_CH + 16 * wv;
        t.rk = chunk_row(src, rb + n);
        const char* kp = reinterpret_cast<const char*>(Kh) + (size_t)(t.rk >= 0 ? t.rk : 0) * (RA_D * 2) + 16 * c;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const at_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const at_u32x4*>(kp + 64 * j));
            t.kb[j] = make_uint4(v.x, v.y, v.z, v.w);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t rv = chunk_row(src, rb + 4 * i + c);
            t.vb[i] = load_row8_stream<RA_BF16>(Vh, rv >= 0 ? rv : 0, lane16);    // a missing row's weight is 0
        }
    };
    auto consume = [&](const Tile& t) {
        at_f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j)
            d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(at_bf16x8, qa[j]),
                                                        __builtin_bit_cast(at_bf16x8, t.kb[j]), d, 0, 0, 0);
        float p[NH];
#pragma unroll
        for (int h = 0; h < NH; ++h) {
            // lanes 0..15 hold row n's logit for head h (the other lanes hold the operand's zero rows)
            const float z = t.rk >= 0 ? d[h] * scale : -INFINITY;
            float mx = z;
            mx = fmaxf(mx, at_dpp<0xB1>(mx));
            mx = fmaxf(mx, at_dpp<0x4E>(mx));
            mx = fmaxf(mx, at_dpp<0x141>(mx));
            mx = fmaxf(mx, at_dpp<0x140>(mx));
            const float mrow = first_lane_f32(mx);                       // of lanes 0..15
            // the running maximum (one value for the whole wavefront) settles after a few tiles: the
            // sums are rescaled only when it moves
            if (mrow > m[h]) {
                const float corr = __expf(m[h] - mrow);                  // exp(-inf) = 0 on the first rows
                m[h] = mrow;
                lpart[h] *= corr;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[h][e] *= corr;
            }
            p[h] = z > -INFINITY ? __expf(z - m[h]) : 0.f;
            lpart[h] += p[h];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float vv[8];
            row8_floats<RA_BF16>(t.vb[i], vv);
#pragma unroll
            for (int h = 0; h < NH; ++h) {
                const float pv = __shfl(p[h], 4 * i + c);                // the weight of row 4 i + c
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[h][e] = fmaf(pv, vv[e], acc[h][e]);
            }
        }
    };
    {
        Tile a, b;
        int sub = chunk * n_sub;
        fetch(sub, a);
        for (; sub < sub_end; sub += 2) {
            fetch(sub + 1, b);
            consume(a);
            if (sub + 1 >= sub_end) break;
            fetch(sub + 2, a);
            consume(b);
        }
    }
    // the wavefront's sums of weights sit in lanes 0..15: add them up, hand them to its first lane
    // group (the four groups of a wavefront share its maximum), and close like any chunk
    float l[NH];
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        float v = lpart[h];
        v += at_dpp<0xB1>(v);
        v += at_dpp<0x4E>(v);
        v += at_dpp<0x141>(v);
        v += at_dpp<0x140>(v);
        const float tot = first_lane_f32(v);
        l[h] = c == 0 ? tot : 0.f;
    }
    chunk_records<NH>(tid, true, m, l, acc, rec0, rec_stride, smem);
}

// Combination of one head's P = nS + nG partial records: Eq. 4-5 with the re-scaling factors
// written for P sets. Called by 128 threads (t = output dimension). COHERENT = true reads the
// records past the L1 cache (they were written by other workgroups of the same launch).
template <bool COHERENT>
__device__ __forceinline__ float rec_load(const float* p) {
    if (COHERENT)
        return __int_as_float(__hip_atomic_load(reinterpret_cast<const int*>(p), __ATOMIC_RELAXED,
                                                __HIP_MEMORY_SCOPE_AGENT));
    return *p;
}

// Online (max, sum, weighted sum) of the records of one head, per set (0: the static chunks,
// 1: the gathered chunks), over the batches of sixteen records slice, slice + n_slices, ...
// Sixteen at a time so that their loads are in flight together (one round trip for the usual
// P <= 16).
template <bool COHERENT>
__device__ __forceinline__ void merge_accumulate(const float* rec, int nS, int nG, int t, int slice,
                                                 int n_slices, float (&M)[2], float (&L)[2],
                                                 float (&A)[2]) {
    const int P = nS + nG;
    for (int i0 = slice * 16; i0 < P; i0 += n_slices * 16) {
        float rm[16], rl[16], ra[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int i = i0 + u < P ? i0 + u : P - 1;
            rm[u] = rec_load<COHERENT>(rec + i * AT_RS + RA_D);
            rl[u] = rec_load<COHERENT>(rec + i * AT_RS + RA_D + 1);
            ra[u] = rec_load<COHERENT>(rec + i * AT_RS + t);
        }
#pragma unroll
        for (int set = 0; set < 2; ++set) {
            const int lo = set == 0 ? 0 : nS, hi = set == 0 ? nS : P;
            float cm = M[set];
#pragma unroll
            for (int u = 0; u < 16; ++u)
                if (i0 + u >= lo && i0 + u < hi) cm = fmaxf(cm, rm[u]);
            if (cm > -INFINITY) {
                const float corr = expf(M[set] - cm);      // 0 while the set's max is still -inf
                float a = A[set] * corr, l = L[set] * corr;
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    if (i0 + u >= lo && i0 + u < hi) {
                        const float wgt = expf(rm[u] - cm);
                        a = fmaf(ra[u], wgt, a);
                        l = fmaf(rl[u], wgt, l);
                    }
                }
                M[set] = cm; L[set] = l; A[set] = a;
            }
        }
    }
}

// One more (max, sum, weighted sum) folded into a set's running one.
__device__ __forceinline__ void merge_fold(float& M, float& L, float& A, float m, float l, float a) {
    const float cm = fmaxf(M, m);
    if (cm > -INFINITY) {
        const float c0 = expf(M - cm), c1 = expf(m - cm);
        A = A * c0 + a * c1;
        L = L * c0 + l * c1;
        M = cm;
    }
}

// Eq. 4 per set and Eq. 5 across the two sets, from their (max, sum, weighted sum); t = output dimension.
__device__ __forceinline__ void merge_finish(const float (&M)[2], const float (&L)[2], const float (&A)[2],
                                             int t, size_t head, float* __restrict__ out,
                                             float* __restrict__ lse, float* __restrict__ o_om,
                                             float* __restrict__ lse_om, float* __restrict__ o_w,
                                             float* __restrict__ lse_w) {
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

// static set W of Sec. 3.3 as two id ranges [0, s) and [N - w, N); overlapping ranges merge
static inline void static_ranges(int64_t N, int sink, int window, int* s, int* w) {
    int64_t ss = sink < 0 ? 0 : sink, ww = window < 0 ? 0 : window;
    if (ss > N) ss = N;
    if (ww > N) ww = N;
    if (ss + ww >= N) { ss = N; ww = 0; }
    *s = (int)ss;
    *w = (int)ww;
}

#define AT_TEAM_LDS_FLOATS (32 + 16 * RA_D)      // LDS floats one team of attend_chunk needs

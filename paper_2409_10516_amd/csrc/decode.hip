// One launch per layer for the whole decode step of Algorithm 1 (fixed static pattern). A
// workgroup per (sequence, query head) runs the graph search (search_dev.h) and then, without
// leaving the compute unit, Eq. 2 over the retrieved set Omega for its head: the retrieved ids
// are still in LDS, the groups of 16 lanes share the rows round-robin, every group keeps an
// online (max, sum, weighted sum) over its rows, and the groups' partial results are combined
// with the re-scaling factors of Eq. 5 written for many sets (first across the four groups of a
// wavefront by lane exchange, then across the wavefronts through LDS), together with the
// (max, sum, weighted sum) of the static set W: carrying maxima across sets this way is the same
// arithmetic as computing o_W and o_Omega apart and combining them by Eq. 4.
//
// The attention over the static set W does not depend on the search, so it is taken off the
// head's critical path: the launch has one extra "helper" workgroup per (sequence, KV head) that
// reads the rows of W once for the whole GQA group and leaves (max, sum, weighted sums) per query
// head in a hand-over area; the head's workgroup picks its record up after the search and only
// attends to the retrieved rows itself. Helpers have the lowest workgroup ids, never wait for
// anything, and are finished before the first search is. (A launch with few searches has one
// helper per query head instead: see ra_launch_decode.)
//
// The hand-over uses no fence. A variant with agent-scope release/acquire was measured: the part
// has one L2 per XCD, so those fences write back and invalidate L2, about 18 us per launch, more
// than the whole attention. Instead the few words that cross workgroups are written and read with
// relaxed agent-scope atomics, which go around the non-coherent cache levels on their own: the
// helper stores its records, waits until the stores have completed (s_waitcnt vmcnt(0), barrier),
// then stores the ready word; the head polls the ready word, then loads the record, then clears
// the ready word for the next launch. The wait is bounded: a head that does not see its ready word
// within the limit attends to W itself (the same code that runs when helpers are off) and turns
// the helpers off for later launches, so a ready word that arrives late is never taken for the
// next launch's. Query heads of a GQA group still run on one XCD (xcd_aware_head) so that the key
// rows their searches have in common are served by that XCD's L2.
//
// A walk that starts from a seed set first scores the whole set, and what bounds that is the rate
// at which one compute unit takes in scattered key rows. A launch with few searches leaves most
// compute units idle, so it has "seed" workgroups as well (between the helpers and the heads):
// each scores one share of one head's set (score_seed_share) and stores the 64-bit keys in a
// hand-over area of their own, one slot per position of the set. A key is never zero and is one
// 64-bit store, so the slot itself says whether its key has come: the head's threads poll their
// slots (bounded), take the keys and zero the slots for the next launch. If a key does not come
// in time the head scores its set itself and switches the shares off for later launches. Same
// relaxed agent-scope accesses as above; no ordering between different words is needed at all.
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
    __device__ __forceinline__ void load(const void* qrow, int lane16) {
        q = reinterpret_cast<const uint4*>(qrow)[lane16];
    }
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
    __device__ __forceinline__ void load(const void* qrow, int lane16) { load_q8<RA_F32>(qrow, lane16, q); }
    __device__ __forceinline__ float dot(const RowBits<RA_F32>& k) const {
        float f[8];
        row_floats<RA_F32>(k, f);
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) d = fmaf(q[e], f[e], d);
        return d;
    }
};

// Combine the online-softmax states of the lane groups of a workgroup of T threads into one (max,
// sum, weighted sum for output `tid`), valid in threads tid < 128 (T >= 128): first the four
// groups of each wavefront by lane exchange, then the T/64 wavefronts through LDS (T/64 * 130
// floats at `lds`). Two barriers.
template <int T>
__device__ __forceinline__ void sm_combine(Softmax8 st, float* lds, int tid, float& mx, float& l, float& a) {
    const int lane = tid & (RA_WAVE - 1), wv = tid / RA_WAVE;
#pragma unroll
    for (int d = 16; d <= 32; d <<= 1) {
        const float mo = __shfl_xor(st.m, d), lo = __shfl_xor(st.l, d);
        float ao[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) ao[e] = __shfl_xor(st.acc[e], d);
        sm_merge(st, mo, lo, ao);
    }
    float* sm = lds;                                         // [16]
    float* sl = sm + T / RA_WAVE;                   // [16]
    float* sa = sl + T / RA_WAVE;                   // [16][128]
    __syncthreads();                                         // whatever was in `lds` is dead
    if (lane < 16) {
        if (lane == 0) {
            sm[wv] = st.m;
            sl[wv] = st.l;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) sa[wv * RA_D + lane * 8 + e] = st.acc[e];
    }
    __syncthreads();
    mx = -INFINITY;
    a = 0.f;
    l = 0.f;
    if (tid < RA_D) {
#pragma unroll
        for (int j = 0; j < T / RA_WAVE; ++j) mx = fmaxf(mx, sm[j]);
        if (mx > -INFINITY) {
#pragma unroll
            for (int j = 0; j < T / RA_WAVE; ++j) {
                const float wgt = expf(sm[j] - mx);
                a = fmaf(sa[j * RA_D + tid], wgt, a);
                l = fmaf(sl[j], wgt, l);
            }
        }
    }
}

// Helper workgroup: Eq. 2 over W for NH query heads that share one KV head (heads head0 ..
// head0 + NH - 1), each row of W read once; leaves one record per head and then its ready word.
template <int DT, int NH, int T>
__device__ __forceinline__ void static_helper(unsigned char* lds_raw, const void* q, int head0, const char* Kh,
                                              const char* Vh, int s, int64_t wstart, int64_t N, float scale,
                                              float* rec, uint32_t* ready) {
    const int tid = threadIdx.x, grp = tid >> 4, lane16 = tid & 15;
    const size_t esz = DT == RA_BF16 ? 2 : 4;
    constexpr int ROWS = DT == RA_BF16 ? 4 : 2;              // rows in flight per 16-lane group
    LaneQuery<DT> ql[NH];
    Softmax8 st[NH];
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        ql[h].load(reinterpret_cast<const char*>(q) + (size_t)(head0 + h) * RA_D * esz, lane16);
        st[h].m = -INFINITY;
        st[h].l = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) st[h].acc[e] = 0.f;
    }
    const int R = s + (int)(N - wstart);
    for (int r0 = 0; r0 < R; r0 += (T / 16) * ROWS) {
        bool live[ROWS];
        RowBits<DT> kb[ROWS], vb[ROWS];
#pragma unroll
        for (int u = 0; u < ROWS; ++u) {
            const int r = r0 + u * (T / 16) + grp;
            live[u] = r < R;
            const int64_t id = !live[u] ? 0 : r < s ? (int64_t)r : wstart + (r - s);   // loads stay unconditional
            kb[u] = load_key<DT>(Kh, id, lane16);
            vb[u] = load_key<DT>(Vh, id, lane16);
        }
#pragma unroll
        for (int u = 0; u < ROWS; ++u) {
            if (!live[u]) continue;
            float v[8];
            row_floats<DT>(vb[u], v);
#pragma unroll
            for (int h = 0; h < NH; ++h) {
                float dot = ql[h].dot(kb[u]);
                dot += at_dpp<0xB1>(dot);
                dot += at_dpp<0x4E>(dot);
                dot += at_dpp<0x141>(dot);
                dot += at_dpp<0x140>(dot);
                sm_row<DT>(st[h], dot * scale, v);
            }
        }
    }
#pragma unroll
    for (int h = 0; h < NH; ++h) {
        float mx, l, a;
        sm_combine<T>(st[h], reinterpret_cast<float*>(lds_raw), tid, mx, l, a);
        if (tid < RA_D) {
            float* r = rec + (size_t)(head0 + h) * RA_COOP_REC;
            if (tid == 0) {
                xwg_store(r, mx);
                xwg_store(r + 1, l);
            }
            xwg_store(r + 4 + tid, a);
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0): this wavefront's record stores have completed
    __syncthreads();                          // ... and every other wavefront's
    if (tid < NH) xwg_store(ready + head0 + tid, 1u);
}

// The head's wait for its helper, run while the search writes its result (see NoHook): one thread
// of the second wavefront polls the ready word, a bounded number of times, and leaves in LDS
// whether it came; if it did not, helpers are turned off for later launches.
struct AwaitHelper {
    const uint32_t* ready_word;
    uint32_t* off_word;
    uint32_t* lds_word;
    int spin;
    bool on;
    // this head's keys in the seed hand-over area, the area's "shares off" word, whether the launch
    // has seed workgroups
    u64* seed_keys;
    uint32_t* seed_off;
    bool seed_on;
    static constexpr bool kSeedShare = true;
    __device__ __forceinline__ bool seeds_shared() const { return seed_on; }
    // Keys c0 and c1 of the head's start set (c1 < 0: only c0, and k1 = k0), polled together a bounded
    // number of times, the slots zeroed for the next launch once the keys are taken; a key that did
    // not come reads 0. A poll is a trip to memory (agent-scope loads go around the caches); more
    // than one in flight per slot was measured and is slower.
    __device__ __forceinline__ void take_seed_keys(int c0, int c1, u64& k0, u64& k1) const {
        u64* p0 = seed_keys + c0;
        u64* p1 = seed_keys + (c1 >= 0 ? c1 : c0);
        k0 = 0ull;
        k1 = 0ull;
        for (int i = 0; i < spin; ++i) {
            if (k0 == 0ull) k0 = xwg_load(p0);               // (a slot whose key has come is not read again)
            if (k1 == 0ull) k1 = xwg_load(p1);
            if (k0 != 0ull && k1 != 0ull) break;
            __builtin_amdgcn_s_sleep(6);
        }
        if (k0 != 0ull) xwg_store(p0, 0ull);
        if (c1 >= 0 && k1 != 0ull) xwg_store(p1, 0ull);
    }
    // a key did not come: later launches score in the head again, so that keys that arrive late
    // are never taken for a later launch's
    __device__ __forceinline__ void seeds_missed() const { xwg_store(seed_off, 1u); }
    __device__ __forceinline__ void before_output() const {
        if (!on || threadIdx.x != RA_WAVE) return;
        uint32_t f = 0u;
        for (int i = 0; i < spin; ++i) {
            f = xwg_load(ready_word);
            if (f) break;
            __builtin_amdgcn_s_sleep(32);
        }
        if (!f) xwg_store(off_word, 1u);
        *lds_word = f;
    }
};

// BUDGETS: every head keeps its own number of ids (budgets[head]) instead of topk. A variant of
// its own because the value lives through the whole walk: read in the common kernel, even behind a
// test for a null pointer, it cost 1.5 % of the step.
template <int DT, int KT, bool GBITS, int T, bool BUDGETS>
__global__ __launch_bounds__(T) void decode_kernel(
    const void* __restrict__ q, const int32_t* __restrict__ adj, const int32_t* __restrict__ entry,
    const void* __restrict__ K, const void* __restrict__ V, int n_q, int n_kv, int64_t Ng, int64_t N,
    int64_t kv_stride, int64_t wstart, int deg, int s, int topk, int ef, int expand,
    uint32_t* __restrict__ gbits,
    int32_t* __restrict__ ids, ra_stats* __restrict__ stats, int ids_off, float scale,
    float* __restrict__ out, float* __restrict__ lse, float* coop, int n_helpers, int coop_mode,
    int coop_spin, const int32_t* __restrict__ roots, int root_cap, const void* __restrict__ Ksearch,
    const float* __restrict__ kscale, const int32_t* __restrict__ budgets, uint32_t* seedx, int seed_parts,
    int seed_stride, int helper_heads) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int tid = threadIdx.x, grp = tid >> 4, lane16 = tid & 15;
    const size_t esz = DT == RA_BF16 ? 2 : 4;
    const int G = n_q / n_kv;
    const int n_heads = ((int)gridDim.x - n_helpers) / (1 + seed_parts);
    // hand-over area: records, ready words, "helpers off" word (set by a head whose wait ran out)
    uint32_t* ready = reinterpret_cast<uint32_t*>(coop + (size_t)n_heads * RA_COOP_REC);
    const bool helpers = n_helpers > 0 && xwg_load(ready + n_heads) == 0u;
    if ((int)blockIdx.x < n_helpers) {
        // ---- helper workgroup of (sequence, KV head) blockIdx.x: attention over W for its G heads
        if (!helpers || coop_mode == RA_HELPERS_SILENT_) return;
        // helper_heads of the group's G query heads per helper workgroup (G: one helper per group, W
        // read once; fewer where the launch leaves compute units idle: the helpers of a group then
        // run side by side on one XCD and share the rows in its L2)
        const int n_groups = n_heads / G;
        const int g = (int)blockIdx.x % n_groups, part = (int)blockIdx.x / n_groups;
        const char* Kg = reinterpret_cast<const char*>(K) + (size_t)g * kv_stride * RA_D * esz;
        const char* Vg = reinterpret_cast<const char*>(V) + (size_t)g * kv_stride * RA_D * esz;
        // G is 1, 2, 4 or 8 when helpers are on; 4 heads per pass over W (2 for fp32: registers)
        constexpr int PASS = DT == RA_BF16 ? 4 : 2;
        const int h_end = (part + 1) * helper_heads;
        for (int h0 = part * helper_heads; h0 < h_end; h0 += PASS) {
            const int head0 = g * G + h0;
            if (h_end - h0 >= PASS) static_helper<DT, PASS, T>(lds_raw, q, head0, Kg, Vg, s, wstart, N, scale, coop, ready);
            else if (h_end - h0 == 2) static_helper<DT, 2, T>(lds_raw, q, head0, Kg, Vg, s, wstart, N, scale, coop, ready);
            else static_helper<DT, 1, T>(lds_raw, q, head0, Kg, Vg, s, wstart, N, scale, coop, ready);
        }
        return;
    }
    // seed hand-over area: [0] the "shares off" word, then (from byte RA_SEEDX_KEYS_OFF) seed_stride
    // 64-bit keys per head, zero between launches
    u64* seed_keys_all = reinterpret_cast<u64*>(reinterpret_cast<char*>(seedx) + RA_SEEDX_KEYS_OFF);
    const bool shares = seed_parts > 0 && xwg_load(seedx) == 0u;
    if ((int)blockIdx.x < n_helpers + n_heads * seed_parts) {
        // ---- seed workgroup: one share of one head's start set (on the XCD of the head's workgroup
        //      when the number of heads is a multiple of 8)
        if (!shares || coop_mode == RA_HELPERS_SILENT_) return;
        const int i = (int)blockIdx.x - n_helpers;
        const int part = i / n_heads, hd = xcd_aware_head(i % n_heads, n_heads, G);
        score_seed_share<DT, KT, T>(hd, part, seed_parts, q, Ksearch, n_q, n_kv, kv_stride, roots, root_cap,
                                    root_cap - 2, expand * deg, kscale, seed_keys_all + (size_t)hd * seed_stride);
        return;
    }
    const int head = xcd_aware_head((int)blockIdx.x - n_helpers - n_heads * seed_parts, n_heads, G);
    const int seq = head / n_q, h = head % n_q, kvh = h / G;
    int32_t* lds_ids = reinterpret_cast<int32_t*>(lds_raw + ids_off);
    uint32_t* lds_word = reinterpret_cast<uint32_t*>(lds_ids + topk);
    const char* Kh = reinterpret_cast<const char*>(K) + ((size_t)seq * n_kv + kvh) * kv_stride * RA_D * esz;
    const char* Vh = reinterpret_cast<const char*>(V) + ((size_t)seq * n_kv + kvh) * kv_stride * RA_D * esz;
    // The graph covers the first Ng of the N tokens now in the cache; W = [0, s) u [wstart, N) with
    // wstart <= Ng, so every token appended after the build is attended densely.
    // the walk scores Ksearch: K itself, or its 8-bit copy (with kscale)
    // ids kept for this head: topk, or its own budget clamped into [1, topk]
    int take = topk;
    if constexpr (BUDGETS) {
        const int b = budgets[head];
        take = b < 1 ? 1 : b > topk ? topk : b;
    }
    const int cnt = run_search<DT, KT, GBITS, T>(lds_raw, head, q, adj, entry, Ksearch, n_q, n_kv, Ng, kv_stride, deg,
                                          s, (int)(Ng - wstart), topk, take, ef, expand, gbits, ids, stats,
                                          lds_ids, roots, root_cap, kscale,
                                          AwaitHelper{ready + head, ready + n_heads, lds_word,
                                                      coop_spin, helpers,
                                                      seed_keys_all + (size_t)head * seed_stride, seedx,
                                                      shares});
#ifdef SR_PHASE_CLOCKS
    const long long t_attn = clock64();
#endif
    // ---- the helper's record for this head, if its ready word came (AwaitHelper)
    bool have_w = false;
    float mw = -INFINITY, lw = 0.f, aw = 0.f;
    if (helpers) {
        have_w = *lds_word != 0u;
        if (have_w && tid < RA_D) {
            const float* r = coop + (size_t)head * RA_COOP_REC;
            mw = xwg_load(r);
            lw = xwg_load(r + 1);
            aw = xwg_load(r + 4 + tid);
        }
    }
    // ---- Eq. 2 over Omega (rows [0, cnt): ids in LDS) and, without a record, W (rows
    //      [cnt, cnt + s + N - wstart))
    LaneQuery<DT> ql;
    ql.load(reinterpret_cast<const char*>(q) + (size_t)head * RA_D * esz, lane16);
    constexpr int DC_ROWS = DT == RA_BF16 ? 6 : 3;       // rows in flight per 16-lane group
    const int R = cnt + (have_w ? 0 : s + (int)(N - wstart));
    Softmax8 st;
    st.m = -INFINITY;
    st.l = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) st.acc[e] = 0.f;
    for (int r0 = 0; r0 < R; r0 += (T / 16) * DC_ROWS) {
        int64_t rid[DC_ROWS];
        RowBits<DT> kb[DC_ROWS], vb[DC_ROWS];
#pragma unroll
        for (int u = 0; u < DC_ROWS; ++u) {
            if (r0 + u * (T / 16) >= R) break;          // uniform: no group has a row in this slot
            const int r = r0 + u * (T / 16) + grp;
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
            if (r0 + u * (T / 16) >= R) break;
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
    // ---- Eq. 4-5: the lane groups' partial results and the helper's record, re-scaled to one maximum
    float mx, l, a;
    sm_combine<T>(st, reinterpret_cast<float*>(lds_raw), tid, mx, l, a);
    if (tid < RA_D) {
        const float m2 = fmaxf(mx, mw);
        if (m2 > -INFINITY) {
            const float c1 = expf(mx - m2), c2 = expf(mw - m2);
            a = a * c1 + aw * c2;
            l = l * c1 + lw * c2;
        }
        const bool empty = !(l > 0.f);
        out[(size_t)head * RA_D + tid] = empty ? 0.f : a / l;
        if (tid == 0) {
            lse[head] = empty ? -INFINITY : m2 + logf(l);
            if (have_w) xwg_store(ready + head, 0u);     // taken: the next launch starts from "not ready"
        }
    }
#ifdef SR_PHASE_CLOCKS
    if (tid == 0 && head < 64) sr_phase_ticks[head * SR_NITER * SR_NPHASE + 7] += clock64() - t_attn;
#endif
}

#ifdef SR_PHASE_CLOCKS
// Tuning builds only: copy the phase clocks of the fused kernel to `host` (64 x 16 x 8 values: workgroup,
// search step, phase) and clear them.
#ifdef SR_WAVE_CLOCKS
extern "C" int ra_dbg_wave_ticks(long long* host) {
    return hipMemcpyFromSymbol(host, HIP_SYMBOL(sr_wave_ticks), sizeof(long long) * 64) != hipSuccess;
}
#endif
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
    return a + (size_t)topk * sizeof(int32_t) + 16;        // ids, then a word for the ready flag
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

// helper workgroups in front of the heads' in a decode launch: one per (sequence, KV head), for
// GQA groups of 1, 2, 4 or 8 while the handle has them switched on
static int decode_helper_slots(const float* coop, int coop_mode, int n_seq, int n_q, int n_kv) {
    const int G = n_q / n_kv;
    const bool coop_on = coop && coop_mode != RA_HELPERS_OFF && (G == 1 || G == 2 || G == 4 || G == 8);
    return coop_on ? n_seq * n_kv : 0;
}

// Threads per workgroup of the fused launch. With the start sets scored by seed workgroups and the
// static set by helpers, what a head's workgroup is left with is mostly merges and barriers, which
// 512 threads get through sooner than 1024 (128K layer, 32 searches: 28.4 against 29.6 us; 27.3 against
// 29.6 us for 128 searches of 32K keys, and still 37.5 against 49.1 us when 256 searches and their 64
// helpers outnumber the compute units); a beam of more than 256 entries keeps 1024 threads (its steps
// gather thousands of rows: 215 against 200 us on the 1M-key configuration). From 512 searches on,
// 256 threads as in the stand-alone search (48.3 against 52.8 us).
static int decode_threads(int heads, int ef) {
    if (ef > 256) return search_threads(heads, ef);
    return heads <= 384 ? 512 : 256;
}

// compute units of the current device (asked once per device)
static int decode_compute_units() {
    static int cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) n = 0;
        cached[dev] = n > 0 ? n : -1;
    }
    return cached[dev] > 0 ? cached[dev] : 0;
}

ra_status ra_launch_decode(const void* q, const int32_t* adj, const int32_t* entry, const void* K,
                           const void* V, ra_dtype dt, int n_seq, int n_q, int n_kv, int64_t Ng, int64_t N,
                           int64_t kv_stride, int deg, int sink, int window, int topk, int ef, int expand,
                           uint32_t* bitset, float* coop, int coop_mode, int coop_spin,
                           const int32_t* roots, int root_cap, const void* K8, const float* kscale,
                           const int32_t* budgets, uint32_t* seedx, int seed_parts, hipStream_t st,
                           float* out, float* lse, int32_t* ids, ra_stats* stats) {
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
    // one helper workgroup per (sequence, KV head) in front of the heads' (GQA groups of 1, 2, 4 or 8)
    if (!coop) RA_FAIL(RA_EINVAL, "hand-over area missing");
    int n_helpers = decode_helper_slots(coop, coop_mode, n_seq, n_q, n_kv);
    const int threads = decode_threads(heads, ef);
    // One helper per query head instead of one per KV head where the launch leaves compute units idle
    // (few searches): with 512 threads a helper's pass over W for a whole group ends later than a
    // short walk does (128K layer: 26.5 against 27.25 us). The helpers of a group run side by side on
    // one XCD and find each other's rows in its L2.
    int helper_heads = n_q / n_kv;
    if (n_helpers > 0 && threads >= 512 && 2 * heads <= decode_compute_units()) {
        n_helpers *= helper_heads;
        helper_heads = 1;
    }
    const void* Ksearch = kscale ? K8 : K;
    // a start set scored in shares by workgroups of their own: only where every workgroup of the
    // launch has a compute unit to itself (few searches, 512 or 1024 threads each); fewer shares when
    // the part has too few compute units, none below two
    int parts = 0;
    if (seedx && seed_parts > 0 && roots && threads >= 512 && coop_mode != RA_HELPERS_OFF) {
        const int room = (decode_compute_units() - n_helpers) / heads - 1;
        parts = seed_parts < room ? seed_parts : room;
        if (parts > RA_SEED_PARTS_MAX) parts = RA_SEED_PARTS_MAX;
        if (parts < 2) parts = 0;
    }
    const int seed_stride = root_cap;
    if (kscale && !K8) RA_FAIL(RA_EINVAL, "8-bit keys missing");
#define RA_DC_GO_T(DTV, KTV, GB, TV) RA_DC_GO_TB(DTV, KTV, GB, TV, false)
#define RA_DC_GO_TB(DTV, KTV, GB, TV, BU)                                                          \
    do {                                                                                           \
        RA_LDS_OPT_IN((decode_kernel<DTV, KTV, GB, TV, BU>), lds);                                 \
        hipLaunchKernelGGL((decode_kernel<DTV, KTV, GB, TV, BU>),                                  \
                           dim3(heads * (1 + parts) + n_helpers), dim3(TV),                        \
                           lds, st, q, adj, entry, K, V, n_q, n_kv, Ng, N, kv_stride, wstart, deg, \
                           (int)s, topk, ef, expand, bitset, ids, stats, ids_off, scale, out, lse, \
                           coop, n_helpers, coop_mode, coop_spin, roots, root_cap, Ksearch,        \
                           kscale, budgets, seedx, parts, seed_stride, helper_heads);              \
    } while (0)
#define RA_DC_GO(DTV, KTV, GB)                                                                     \
    do {                                                                                           \
        if (threads == 1024) RA_DC_GO_T(DTV, KTV, GB, 1024);                                       \
        else if (threads == 512) RA_DC_GO_T(DTV, KTV, GB, 512);                                    \
        else RA_DC_GO_T(DTV, KTV, GB, 256);                                                        \
    } while (0)
    if (budgets) {
        // per-head budgets: the walk over the keys as stored, visited bitsets in LDS
        if (kscale || gb)
            RA_FAIL(RA_EUNSUP, "per-head budgets go with neither 8-bit keys nor visited bitsets in device "
                               "memory (context too long for LDS at this ef and expand)");
#define RA_DC_GO_B(DTV)                                                                            \
    do {                                                                                           \
        if (threads == 1024) RA_DC_GO_TB(DTV, DTV, false, 1024, true);                             \
        else if (threads == 512) RA_DC_GO_TB(DTV, DTV, false, 512, true);                          \
        else RA_DC_GO_TB(DTV, DTV, false, 256, true);                                              \
    } while (0)
        if (dt == RA_BF16) RA_DC_GO_B(RA_BF16); else RA_DC_GO_B(RA_F32);
#undef RA_DC_GO_B
    } else if (dt == RA_BF16) {
        if (kscale) { if (gb) RA_DC_GO(RA_BF16, RA_KEYS_I8, true); else RA_DC_GO(RA_BF16, RA_KEYS_I8, false); }
        else if (gb) RA_DC_GO(RA_BF16, RA_BF16, true); else RA_DC_GO(RA_BF16, RA_BF16, false);
    } else {
        if (kscale) { if (gb) RA_DC_GO(RA_F32, RA_KEYS_I8, true); else RA_DC_GO(RA_F32, RA_KEYS_I8, false); }
        else if (gb) RA_DC_GO(RA_F32, RA_F32, true); else RA_DC_GO(RA_F32, RA_F32, false);
    }
#undef RA_DC_GO_T
#undef RA_DC_GO_TB
#undef RA_DC_GO
    RA_HIP(hipGetLastError());
    return RA_OK;
}

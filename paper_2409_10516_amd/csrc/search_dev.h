// VectorSearch(q) of Algorithm 1: bounded best-first walk over one head's key graph
// (Sec. 2.4 describes proximity-graph search as a greedy walk towards the most similar
// vectors). One workgroup per (sequence, query head), of 1024, 512 or 256 threads (search_threads
// below; the fused decode launch chooses for itself); the whole search state lives in LDS:
//   * visited: an exact bitset over the N keys (N/8 bytes; a global-memory bitset is used
//     instead when the context is too long for LDS),
//   * beam: at most ef entries, always sorted, as 64-bit keys
//         [ordered(score) : 32][0x7fffffff - id : 31][not-yet-expanded : 1]
//     so that "larger key" is exactly "(score descending, id ascending)" and one integer
//     compare decides; ids are unique in the beam, so the flag bit never decides.
// Each step expands the `expand` best unexpanded entries at once: their adjacency rows
// are read with one coalesced load per row, unvisited neighbours are claimed with an LDS
// atomic-or (which also removes duplicates), their key rows are gathered by 16-lane
// groups (16 B per lane; four rows per wavefront load), scored, filtered against the
// beam's worst entry, and merged into the beam by rank: a kept candidate's place is the
// number of beam entries above it (binary search) plus the number of candidates above it
// (counted); a beam entry's place is its index plus a prefix sum over the candidates' slots.
// No sort, no serial insertion, and the next step's picks fall out of the same numbers. The
// beam after a step is the top-ef of a set union, so it does not depend on the order in which
// candidates were claimed.
//
// Scores decide integer results, so every kernel that ranks keys (this walk, the flat scan, the
// re-rank) computes them in one and the same way: each of 16 lanes sums its 8 contiguous products,
// then the 16 partial sums are added pairwise over adjacent lanes (xor 1, 2, 4, 8). Identical key
// rows therefore score identically everywhere. fp32 keys and 8-bit keys: product rounded, then
// added, left to right (a CPU reference can reproduce every bit). bf16 keys: four two-element dot
// instructions per lane (exact products, the hardware's own accumulation).
#pragma once
#include "common.h"

#define SR_THREADS 1024          // largest workgroup; the kernels are also built for 512 and 256 threads
#define SR_LDS_LIMIT RA_LDS_LIMIT
#define SR_BITSET_LDS_MAX (128 * 1024) // a longer visited bitset (over 2^20 keys) lives in global memory
#ifndef SR_UNROLL
#define SR_UNROLL 8               // key rows in flight per 16-lane group
#endif
#ifndef SR_ADJ_LOADS
#define SR_ADJ_LOADS 8            // adjacency cells a thread has in flight while it claims neighbours
#endif


enum { C_MISSED = 0, C_NCAND = 1, C_NKEEP = 2, C_NUNEXP = 3, C_LO = 4, C_HI = 5, C_NSURV = 6, C_BIN = 7, C_WTOT = 8,
       C_COUNT = 8 + SR_THREADS / RA_WAVE };
#define SR_PREFILTER_SLACK 64     // a step that keeps more than ef + this many candidates drops the hopeless ones first
#define SR_PREFILTER_REGS 8       // ... when a thread can hold its share of them (nk <= 8 T)

typedef unsigned long long u64;

// Phase clocks for tuning builds (-DSR_PHASE_CLOCKS): thread 0 of the workgroups of the first 64 searches adds the
// ticks spent in each phase to a device array that ra_dbg_phase_ticks copies out. Off otherwise.
#ifdef SR_PHASE_CLOCKS
#define SR_NPHASE 16
#define SR_NITER 16
static __device__ long long sr_phase_ticks[64 * SR_NITER * SR_NPHASE];
#ifdef SR_WAVE_CLOCKS
// (with -DSR_WAVE_CLOCKS: wall-clock stamps of the first head's workgroup, [0..3] search entered,
// state cleared, claims made, start set's keys in LDS, and of the first and last of its seed
// workgroups, [8..11] and [16..19]: entered, header read, first rows scored, first keys stored;
// ra_dbg_wave_ticks copies them out)
static __device__ long long sr_wave_ticks[64];
#endif
// ticks are added up in LDS (a fire-and-forget add) and copied out when the search has ended
#define SR_TICK_INIT                                                                           \
    __shared__ long long tick_lds_[SR_NITER * SR_NPHASE];                                      \
    for (int i_ = threadIdx.x; i_ < SR_NITER * SR_NPHASE; i_ += blockDim.x) tick_lds_[i_] = 0; \
    __syncthreads();                                                                           \
    long long tick_ = clock64(); int tick_it_ = 0
#define SR_TICK_ITER(i) tick_it_ = (i) < SR_NITER ? (i) : SR_NITER - 1
#define SR_TICK(p)                                                                             \
    do {                                                                                       \
        if (threadIdx.x == 0) {                                                                \
            const long long now_ = clock64();                                                  \
            tick_lds_[tick_it_ * SR_NPHASE + (p)] += now_ - tick_;                             \
            tick_ = now_;                                                                      \
        }                                                                                      \
    } while (0)
#define SR_TICK_FLUSH                                                                          \
    do {                                                                                       \
        if (head < 64)                                                                         \
            for (int i_ = threadIdx.x; i_ < SR_NITER * SR_NPHASE; i_ += blockDim.x)            \
                sr_phase_ticks[head * SR_NITER * SR_NPHASE + i_] += tick_lds_[i_];             \
    } while (0)
#else
#define SR_TICK_INIT
#define SR_TICK_ITER(i)
#define SR_TICK(p)
#define SR_TICK_FLUSH
#endif

template <int V> struct sr_int { static constexpr int value = V; };      // a compile-time row count as an argument

__device__ __forceinline__ u64 make_key(float score, int id) {
    return ((u64)f32_ordered(score) << 32) | ((u64)(uint32_t)(0x7fffffff - id) << 1) | 1ull;
}
__device__ __forceinline__ int key_id(u64 k) { return 0x7fffffff - (int)((uint32_t)k >> 1); }

template <int DT>
__device__ __forceinline__ void load_q8(const void* q, int lane16, float* qv) {
    if (DT == RA_BF16) {
        const uint4 u = reinterpret_cast<const uint4*>(q)[lane16];
        qv[0] = bf16_lo(u.x); qv[1] = bf16_hi(u.x); qv[2] = bf16_lo(u.y); qv[3] = bf16_hi(u.y);
        qv[4] = bf16_lo(u.z); qv[5] = bf16_hi(u.z); qv[6] = bf16_lo(u.w); qv[7] = bf16_hi(u.w);
    } else {
        const float4 a = reinterpret_cast<const float4*>(q)[lane16 * 2];
        const float4 b = reinterpret_cast<const float4*>(q)[lane16 * 2 + 1];
        qv[0] = a.x; qv[1] = a.y; qv[2] = a.z; qv[3] = a.w;
        qv[4] = b.x; qv[5] = b.y; qv[6] = b.z; qv[7] = b.w;
    }
}

// A lane's share of the query in the form the score wants it: bf16 pairs stay packed (they go
// through the two-element dot instruction), fp32 queries and queries over 8-bit keys are floats.
template <int KT> struct ScoreQuery { float v[8]; };
template <> struct ScoreQuery<RA_BF16> { uint4 p; };
template <int DT, int KT>
__device__ __forceinline__ void load_score_query(const void* qrow, int lane16, ScoreQuery<KT>& sq) {
    if constexpr (KT == RA_BF16) sq.p = reinterpret_cast<const uint4*>(qrow)[lane16];
    else load_q8<DT>(qrow, lane16, sq.v);
}

// Raw 32 B (fp32) / 16 B (bf16) of a key row owned by this lane.
template <int DT> struct RowBits { uint4 a; uint4 b; };

template <int DT>
__device__ __forceinline__ RowBits<DT> load_key(const void* Kh, int64_t row, int lane16) {
    RowBits<DT> r;
    if (DT == RA_KEYS_I8) {
        // 8 of the row's 128 signed bytes
        const uint2 u = reinterpret_cast<const uint2*>(reinterpret_cast<const int8_t*>(Kh) + row * RA_D)[lane16];
        r.a = make_uint4(u.x, u.y, 0u, 0u);
        r.b = r.a;
    } else if (DT == RA_BF16) {
        r.a = reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(Kh) + row * RA_D)[lane16];
        r.b = r.a;
    } else {
        const uint4* p = reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(Kh) + row * RA_D);
        r.a = p[lane16 * 2];
        r.b = p[lane16 * 2 + 1];
    }
    return r;
}

// The same for a kernel that streams every row once (a scan): non-temporal loads, which leave the
// caches to data that is read again (measured on a plain read of 1 GiB: 7.1 against 6.2 TB/s).
typedef unsigned int ra_u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int ra_u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 load16_stream(const void* p) {
    const ra_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const ra_u32x4*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
template <int DT>
__device__ __forceinline__ RowBits<DT> load_key_stream(const void* Kh, int64_t row, int lane16) {
    RowBits<DT> r;
    if (DT == RA_KEYS_I8) {
        const ra_u32x2 u = __builtin_nontemporal_load(
            reinterpret_cast<const ra_u32x2*>(reinterpret_cast<const int8_t*>(Kh) + row * RA_D) + lane16);
        r.a = make_uint4(u.x, u.y, 0u, 0u);
        r.b = r.a;
    } else if (DT == RA_BF16) {
        r.a = load16_stream(reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(Kh) + row * RA_D) + lane16);
        r.b = r.a;
    } else {
        const uint4* p = reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(Kh) + row * RA_D);
        r.a = load16_stream(p + lane16 * 2);
        r.b = load16_stream(p + lane16 * 2 + 1);
    }
    return r;
}

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}

// The fixed-order inner product described in the file header, in two parts: a lane's share (its 8
// dimensions, summed left to right), then the pairwise tree over the 16 lanes of the group.
typedef __bf16 sr_bf16x2 __attribute__((ext_vector_type(2)));
template <int DT>
__device__ __forceinline__ float score_share(const RowBits<DT>& r, const ScoreQuery<DT>& sq) {
    float acc;
    if constexpr (DT == RA_KEYS_I8) {
        const float* qv = sq.v;
        // qv holds query * scale; the key bytes convert to float32 exactly; product rounded, then added
        acc = __fmul_rn(qv[0], (float)(int8_t)(r.a.x));
        acc = __fadd_rn(acc, __fmul_rn(qv[1], (float)(int8_t)(r.a.x >> 8)));
        acc = __fadd_rn(acc, __fmul_rn(qv[2], (float)(int8_t)(r.a.x >> 16)));
        acc = __fadd_rn(acc, __fmul_rn(qv[3], (float)(int8_t)(r.a.x >> 24)));
        acc = __fadd_rn(acc, __fmul_rn(qv[4], (float)(int8_t)(r.a.y)));
        acc = __fadd_rn(acc, __fmul_rn(qv[5], (float)(int8_t)(r.a.y >> 8)));
        acc = __fadd_rn(acc, __fmul_rn(qv[6], (float)(int8_t)(r.a.y >> 16)));
        acc = __fadd_rn(acc, __fmul_rn(qv[7], (float)(int8_t)(r.a.y >> 24)));
    } else if constexpr (DT == RA_BF16) {
        // four two-element dot instructions (exact products, float32 accumulation in the hardware's
        // own rounding: within an ulp of the running sum per instruction, the same bits for the same
        // operands): 4 vector instructions per row share instead of 8 conversions and 8 fma
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(sr_bf16x2, sq.p.x), __builtin_bit_cast(sr_bf16x2, r.a.x), 0.f, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(sr_bf16x2, sq.p.y), __builtin_bit_cast(sr_bf16x2, r.a.y), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(sr_bf16x2, sq.p.z), __builtin_bit_cast(sr_bf16x2, r.a.z), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(sr_bf16x2, sq.p.w), __builtin_bit_cast(sr_bf16x2, r.a.w), acc, false);
    } else {
        const float* qv = sq.v;
        // product rounded, then added (this file is compiled with contraction off)
        acc = __fmul_rn(qv[0], __uint_as_float(r.a.x));
        acc = __fadd_rn(acc, __fmul_rn(qv[1], __uint_as_float(r.a.y)));
        acc = __fadd_rn(acc, __fmul_rn(qv[2], __uint_as_float(r.a.z)));
        acc = __fadd_rn(acc, __fmul_rn(qv[3], __uint_as_float(r.a.w)));
        acc = __fadd_rn(acc, __fmul_rn(qv[4], __uint_as_float(r.b.x)));
        acc = __fadd_rn(acc, __fmul_rn(qv[5], __uint_as_float(r.b.y)));
        acc = __fadd_rn(acc, __fmul_rn(qv[6], __uint_as_float(r.b.z)));
        acc = __fadd_rn(acc, __fmul_rn(qv[7], __uint_as_float(r.b.w)));
    }
    return acc;
}
// All 16 lanes of the group return the same value.
template <int DT>
__device__ __forceinline__ float score_fixed(const RowBits<DT>& r, const ScoreQuery<DT>& sq) {
    float acc = score_share<DT>(r, sq);
    // pairwise tree over adjacent lanes with DPP lane permutations inside a row of 16:
    // quad_perm [1,0,3,2] and [2,3,0,1] are xor 1 and xor 2; after them the four lanes of a
    // quad hold the same sum, so half-mirror (i -> 7-i) and mirror (i -> 15-i) deliver exactly
    // what xor 4 and xor 8 would, and float addition commutes.
    acc = __fadd_rn(acc, dpp_f32<0xB1>(acc));
    acc = __fadd_rn(acc, dpp_f32<0x4E>(acc));
    acc = __fadd_rn(acc, dpp_f32<0x141>(acc));
    acc = __fadd_rn(acc, dpp_f32<0x140>(acc));
    return acc;
}

// The same tree for R rows at once (R = 1, 2, 4, 8 or 16 shares per lane): at level k a lane and its
// partner (lane ^ 2^k) split the rows they both still hold, each adding the partner's share of the
// rows it keeps, so the work halves per level instead of every lane adding up every row; once one
// row is left the remaining levels add as in score_fixed. Lane l of the group ends with the sum of
// row l & (R - 1): the same operands added in the same pairs as in score_fixed, hence the same bits.
// Partner values: quad_perm for xor 1 and 2, a row rotation by 8 for xor 8, and for xor 4 two
// row shifts by 4, each written to the banks of four lanes it is right for.
template <int K>
__device__ __forceinline__ float lane16_xor(float x) {
    if constexpr (K == 0) return dpp_f32<0xB1>(x);
    else if constexpr (K == 1) return dpp_f32<0x4E>(x);
    else if constexpr (K == 3) return dpp_f32<0x128>(x);
    else {
        const int v = __float_as_int(x);
        int t = __builtin_amdgcn_update_dpp(v, v, 0x104, 0xF, 0x5, false);      // lanes 0-3, 8-11 <- lane + 4
        t = __builtin_amdgcn_update_dpp(t, v, 0x114, 0xF, 0xA, false);          // lanes 4-7, 12-15 <- lane - 4
        return __int_as_float(t);
    }
}
template <int K, int N>
__device__ __forceinline__ void rows_tree_level(float* a, int lane16) {
    if constexpr (N > 1) {
        const bool hi = (lane16 >> K) & 1;
#pragma unroll
        for (int j = 0; j < N / 2; ++j) {
            const float keep = hi ? a[2 * j + 1] : a[2 * j];
            const float send = hi ? a[2 * j] : a[2 * j + 1];
            a[j] = __fadd_rn(keep, lane16_xor<K>(send));
        }
    } else {
        a[0] = __fadd_rn(a[0], lane16_xor<K>(a[0]));
    }
}
template <int R>
__device__ __forceinline__ float rows_tree(float (&a)[R], int lane16) {
    static_assert(R == 1 || R == 2 || R == 4 || R == 8 || R == 16, "a power of two up to the lanes of a group");
    rows_tree_level<0, R>(a, lane16);
    rows_tree_level<1, (R > 1 ? R / 2 : 1)>(a, lane16);
    rows_tree_level<2, (R > 2 ? R / 4 : 1)>(a, lane16);
    rows_tree_level<3, (R > 4 ? R / 8 : 1)>(a, lane16);
    return a[0];
}

// number of entries of the descending array arr[0..n) that beat k (flag bit ignored)
__device__ __forceinline__ int count_better(const u64* arr, int n, u64 k) {
    int lo = 0, hi = n;
    const u64 kk = k | 1ull;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if ((arr[mid] | 1ull) > kk) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// Inclusive prefix sum over the 64 lanes of a wavefront (all lanes active): shifts inside each
// row of 16 lanes, then lane 15 of a row added to the next row, then lane 31 to the upper half.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_or_zero(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xF, false);
}
__device__ __forceinline__ int wave_incl_scan(int v) {
    v += dpp_or_zero<0x111, 0xF>(v);      // row_shr:1
    v += dpp_or_zero<0x112, 0xF>(v);      // row_shr:2
    v += dpp_or_zero<0x114, 0xF>(v);      // row_shr:4
    v += dpp_or_zero<0x118, 0xF>(v);      // row_shr:8
    v += dpp_or_zero<0x142, 0xA>(v);      // row_bcast:15 into rows 1 and 3
    v += dpp_or_zero<0x143, 0xC>(v);      // row_bcast:31 into rows 2 and 3
    return v;
}

// the same, counting only entries whose not-yet-expanded flag is clear
__device__ __forceinline__ int count_above16_expanded(const u64* arr, int n, u64 k) {
    u64 v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) v[u] = arr[u];
    int cnt = 0;
#pragma unroll
    for (int u = 0; u < 16; ++u) cnt += (u < n && v[u] > k && !(v[u] & 1ull)) ? 1 : 0;
    return cnt;
}

// the same when all 16 entries count
__device__ __forceinline__ int count_above16_full(const u64* arr, u64 k) {
    u64 v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) v[u] = arr[u];
    int cnt = 0;
#pragma unroll
    for (int u = 0; u < 16; ++u) cnt += v[u] > k ? 1 : 0;
    return cnt;
}

static_assert(RA_MAX_EF + RA_MAX_EXPAND * RA_MAX_DEG < 65536, "ranks and merge counts are kept in 16 bits");

// number of the first min(n, 16) entries of arr that are larger than k; all 16 are read (the
// caller's buffer has 16 entries of slack) so that the loads go out together.
__device__ __forceinline__ int count_above16(const u64* arr, int n, u64 k) {
    u64 v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) v[u] = arr[u];
    int cnt = 0;
#pragma unroll
    for (int u = 0; u < 16; ++u) cnt += (u < n && v[u] > k) ? 1 : 0;
    return cnt;
}

// Workgroup -> (sequence, query head). Consecutive workgroup ids are dealt round-robin to the 8
// XCDs, each with its own L2. The query heads of a GQA group read the same key and value rows, so
// they are given workgroup ids that are congruent modulo 8 (group + n_groups * member) and share
// one L2, whenever the number of groups is a multiple of 8; otherwise the identity map is used.
__device__ __forceinline__ int xcd_aware_head(int block, int heads, int G) {
    const int n_groups = heads / G;
    if (G == 1 || (n_groups & 7)) return block;
    return (block % n_groups) * G + block / n_groups;
}

// The whole search of one (sequence, query head) by one workgroup of T threads.
// N is the number of keys the graph covers; the key rows of a (sequence, KV head) start every
// kv_stride rows (kv_stride >= N: the cache may hold tokens appended after the index was built).
// `lds_raw` is the workgroup's dynamic LDS (ra_search_lds_bytes of it). Writes ids/stats of
// `head`; when `lds_ids` is not null the ids are also left there (LDS) for a fused consumer.
// Returns the number of valid ids. Ends with the whole workgroup past a barrier.
// A caller's hook into run_search: before_output() is called by every thread when the walk has
// ended, ahead of the phase in which the first wavefront writes the result (the others idle until
// the closing barrier, which also publishes whatever the hook left in LDS).
// Its kSeedShare says whether the start set of a seeded walk may be scored by other workgroups of
// the launch (score_seed_share below): then seeds_shared() says whether it is in this launch,
// take_seed_keys(c0, c1, k0, k1) waits (bounded) for keys c0 and c1 of the set (c1 < 0: only c0; k1 is
// then k0 again) and leaves 0 for one that did not come, and seeds_missed() is called by one thread
// when some key did not.
struct NoHook {
    static constexpr bool kSeedShare = false;
    __device__ __forceinline__ void before_output() const {}
};

// Words that cross workgroups inside one launch: relaxed agent-scope atomics, which go around the
// cache levels that are not coherent across the part's XCDs.
__device__ __forceinline__ void xwg_store(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void xwg_store(uint32_t* p, uint32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void xwg_store(u64* p, u64 v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float xwg_load(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t xwg_load(const uint32_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ u64 xwg_load(const u64* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// One of `parts` shares of a head's seed set, scored by a workgroup of its own (T threads) while the
// head's workgroup clears its state and claims the set's ids: what bounds the scoring of a start set
// is the rate at which one compute unit takes in scattered rows, and a launch with few searches
// leaves most compute units idle. The keys (the same bits the head would have made: same share
// sums, same tree) go to keys[c] for the share's positions c of the set. A key is never zero and
// is written by one 64-bit store, so the slot itself tells the head that its key has come; the head
// zeroes it again when it has taken the key. n_cfg is the size the sets were listed for (a head's
// set may have fewer ids): shares are cut by it, so the ids can be requested together with the set's
// header. A set that is no seed set, or does not fit the candidate array of the walk (maxc), is
// left to the head, which applies the same test and does not wait then.
template <int DT, int KT, int T>
__device__ __forceinline__ void score_seed_share(int head, int part, int parts, const void* __restrict__ q,
                                                 const void* __restrict__ K, int n_q, int n_kv, int64_t kv_stride,
                                                 const int32_t* __restrict__ roots, int root_cap, int n_cfg,
                                                 int maxc, const float* __restrict__ kscale, u64* keys) {
    const int tid = threadIdx.x, grp = tid >> 4, lane16 = tid & 15;
    const int seq = head / n_q, h = head % n_q, kvh = h / (n_q / n_kv);
    const size_t esz = DT == RA_BF16 ? 2 : 4;
    const size_t ksz = KT == RA_KEYS_I8 ? 1 : KT == RA_BF16 ? 2 : 4;
    const int32_t* root = roots + (size_t)head * root_cap;
    const int per = (n_cfg + parts - 1) / parts;
    const int c_beg = part * per;
    // (twice the rows in flight per lane group where the workgroup is small: the walk's own registers
    // are not live here, and a share is then one trip to memory again)
    constexpr int R = (T <= 512 && KT != RA_F32) ? 2 * SR_UNROLL : SR_UNROLL, PER = T / 16;
    const char* Kh = reinterpret_cast<const char*>(K) + ((size_t)seq * n_kv + kvh) * kv_stride * RA_D * ksz;
    ScoreQuery<KT> qv;
    load_score_query<DT, KT>(reinterpret_cast<const char*>(q) + (size_t)head * RA_D * esz, lane16, qv);
    if constexpr (KT == RA_KEYS_I8) {
        const float* sc = kscale + ((size_t)seq * n_kv + kvh) * RA_D + lane16 * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) qv.v[e] = __fmul_rn(qv.v[e], sc[e]);
    }
    const int n_root = root[0], n_first = root[1];
#ifdef SR_WAVE_CLOCKS
    const int wslot_ = head == 0 && tid == 0 ? (part == 0 ? 8 : part == parts - 1 ? 16 : -1) : -1;
    if (wslot_ >= 0) sr_wave_ticks[wslot_] = wall_clock64();
    if (wslot_ >= 0 && n_root >= 0) sr_wave_ticks[wslot_ + 1] = wall_clock64();
#endif
    for (int c0 = c_beg; c0 < c_beg + per; c0 += R * PER) {
        // ids first, wherever the set ends (slots up to root_cap - 3 exist), then the header decides
        const int cw = c0 + (lane16 & (R - 1)) * PER + grp;      // the key this lane will write
        int idw = root[2 + min(cw, root_cap - 3)];
        int idv[R];
#pragma unroll
        for (int u = 0; u < R; ++u) idv[u] = root[2 + min(c0 + u * PER + grp, root_cap - 3)];
        if (n_first != 0 || n_root < 1 || n_root > maxc) return;
        const int c_end = min(n_root, c_beg + per);
        if (c0 >= c_end) return;
        const int id0 = root[2];
        RowBits<KT> rows[R];
#pragma unroll
        for (int u = 0; u < R; ++u)                           // past the end: the set's first row again
            rows[u] = load_key<KT>(Kh, c0 + u * PER + grp < c_end ? idv[u] : id0, lane16);
        float sh[R];
#pragma unroll
        for (int u = 0; u < R; ++u) sh[u] = score_share<KT>(rows[u], qv);
        const float sc = rows_tree<R>(sh, lane16);
#ifdef SR_WAVE_CLOCKS
        if (wslot_ >= 0 && sc == sc) sr_wave_ticks[wslot_ + 2] = wall_clock64();
#endif
        if (lane16 < R && cw < c_end) xwg_store(keys + cw, make_key(sc, idw));
#ifdef SR_WAVE_CLOCKS
        __builtin_amdgcn_s_waitcnt(0x0F70);
        if (wslot_ >= 0) sr_wave_ticks[wslot_ + 3] = wall_clock64();
        if (head == 0 && (tid & 63) == 0 && tid < 512) sr_wave_ticks[32 + part * 8 + tid / 64] = wall_clock64();
#endif
    }
}

template <int DT, int KT, bool GBITS, int T, typename Hook>
__device__ __forceinline__ int run_search(
    unsigned char* lds_raw, int head, const void* __restrict__ q, const int32_t* __restrict__ adj,
    const int32_t* __restrict__ entry, const void* __restrict__ K, int n_q, int n_kv, int64_t N,
    int64_t kv_stride, int deg, int s, int w, int topk, int take, int ef, int expand,
    uint32_t* __restrict__ gbits, int32_t* __restrict__ ids, ra_stats* __restrict__ stats, int32_t* lds_ids,
    const int32_t* __restrict__ roots, int root_cap, const float* __restrict__ kscale, const Hook& hook) {
    const int tid = threadIdx.x, grp = tid >> 4, lane16 = tid & 15;
    const int lane = tid & (RA_WAVE - 1), wv = tid / RA_WAVE;
    const int seq = head / n_q, h = head % n_q, kvh = h / (n_q / n_kv);
    const size_t esz = DT == RA_BF16 ? 2 : 4;                                   // of the query
    const size_t ksz = KT == RA_KEYS_I8 ? 1 : KT == RA_BF16 ? 2 : 4;            // of the keys the walk scores
    const char* Kh = reinterpret_cast<const char*>(K) + ((size_t)seq * n_kv + kvh) * kv_stride * RA_D * ksz;
    const int32_t* adj_h = adj + (size_t)head * N * deg;
    const int maxc = expand * deg;
    const int nwords = (int)((N + 31) >> 5);

    SR_TICK_INIT;
#ifdef SR_WAVE_CLOCKS
    if (head == 0 && tid == 0) sr_wave_ticks[0] = wall_clock64();      // search entered
#endif
    u64* cur = reinterpret_cast<u64*>(lds_raw);
    u64* nxt = cur + ef;
    u64* ckey = nxt + ef;            // [maxc + 16] candidates that passed the beam threshold
    int* cid = reinterpret_cast<int*>(ckey + maxc + 16);  // [maxc] claimed neighbour ids
    int* cnt = cid + maxc;           // [maxc] merge counters of the candidates, zero between steps
    int* hist = cnt + maxc;          // [ef + 1] candidates per beam slot, zero between steps
    int* hist_nxt = hist + ef + 1;   // [ef + 1] the one the next step fills
    int* picks = hist_nxt + ef + 1;  // [RA_MAX_EXPAND]
    int* ctr = picks + RA_MAX_EXPAND;
    int* wtot = ctr + C_WTOT;
    // urank[i], i in [0, bn]: unexpanded entries among the first i of the beam, as of the last pick
    // but before its picks were marked expanded (two buffers, swapped with the beam's)
    uint16_t* urank = reinterpret_cast<uint16_t*>(ctr + C_COUNT);    // [ef + 1]
    uint16_t* urank_nxt = urank + ef + 1;                            // [ef + 1]
    uint32_t* bits = GBITS ? gbits + (size_t)head * nwords
                           : reinterpret_cast<uint32_t*>(urank_nxt + ef + 1);

    ScoreQuery<KT> qv;
    load_score_query<DT, KT>(reinterpret_cast<const char*>(q) + (size_t)head * RA_D * esz, lane16, qv);
    if constexpr (KT == RA_KEYS_I8) {
        // 8-bit keys: k ~ k8 * scale per dimension, so the walk scores <q * scale, k8>
        const float* sc = kscale + ((size_t)seq * n_kv + kvh) * RA_D + lane16 * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) qv.v[e] = __fmul_rn(qv.v[e], sc[e]);
    }
    const int e0 = entry[head];
    // The first two steps of a walk do not depend on the query: the entry point is expanded, then
    // all its neighbours are (when `expand` and ef are at least their number). What they visit,
    // the entry point's root set, is listed with the index (ra_launch_roots): [0] its size,
    // [1] 1 + the number of the entry point's neighbours, then the ids, those first. With it the
    // two steps become one: every key of the set is scored in one gather and the beam is the
    // top ef of them, the entry point and its neighbours marked expanded. Same beam, same visited
    // set, same counters as the two steps taken one after the other.
    const int32_t* root = roots ? roots + (size_t)head * root_cap : nullptr;
    int n_root = 0, n_first = 0, my_root = -1;
    if (root) {
        n_root = root[0];
        n_first = root[1];
        my_root = root[2 + (tid < root_cap - 2 ? tid : 0)];      // unconditional: same trip as the header
    }
    // (the loads above are in flight while the LDS state is cleared)
    if (!GBITS)
        for (int i = tid; i < nwords; i += T) bits[i] = 0u;
    for (int i = tid; i < maxc + 2 * ef + 2; i += T) cnt[i] = 0;      // cnt, hist, hist_nxt
    // A seed set (ra_launch_seeds) has the same layout with [1] = 0: the walk starts from all of its
    // keys at once, scored in one gather, the best ef of them in the beam and none of them expanded.
    // That is a start of its own, not a shortcut for steps of the single-entry walk: no step is
    // counted for it. (The host checks that a seed set fits the candidate arrays.)
    const bool seeded = root && n_first == 0;
    const bool fill = root && n_root <= maxc &&
                      (seeded ? n_root >= 1 : n_first > 1 && expand >= n_first - 1 && ef >= n_first);
    __syncthreads();                                             // the LDS state is cleared
    SR_TICK(12);
#ifdef SR_WAVE_CLOCKS
    if (head == 0 && tid == 0) sr_wave_ticks[1] = wall_clock64();
#endif
    int bn, n_visited, n_expanded, n_iters;
    bool first = fill;               // the coming step is that doubled first step
    if (fill) {
        for (int c = tid; c < n_root; c += T) {
            const int id = c == tid ? my_root : root[2 + c];
            cid[c] = id;
            atomicOr(&bits[id >> 5], 1u << (id & 31));
        }
        if (tid == 0) {
            urank[0] = 0;
            ctr[C_NCAND] = n_root;
            ctr[C_NKEEP] = n_root;           // every key of a start set is kept (scored below)
            ctr[C_NUNEXP] = 0;
            ctr[C_LO] = -1;
            ctr[C_HI] = 0;
            ctr[C_NSURV] = 0;
            ctr[C_MISSED] = 0;
        }
        bn = 0; n_visited = 0; n_expanded = 0; n_iters = 0;
    } else {
        if (grp == 0) {
            const RowBits<KT> r = load_key<KT>(Kh, e0, lane16);
            const float sc = score_fixed<KT>(r, qv);
            if (tid == 0) {
                // the beam is the entry point alone, and the first step can only pick it: leave the
                // state a merge would leave (pick in place, flag cleared, counts of unexpanded entries)
                cur[0] = make_key(sc, e0) & ~1ull;
                picks[0] = e0;
                urank[0] = 0;
                ctr[C_NCAND] = 0;
                ctr[C_NKEEP] = 0;
                ctr[C_NUNEXP] = 1;
                atomicOr(&bits[e0 >> 5], 1u << (e0 & 31));
            }
        }
        bn = 1; n_visited = 1; n_expanded = 0; n_iters = 0;
    }
    bool picked = true;              // the merge of the last step already chose this step's picks
    // Adjacency rows likely to be expanded soon are touched ahead of time (one word of the row's
    // first line), so that the row is in this XCD's L2 when its step reads it: the rows of the
    // candidates a step keeps, touched while they are merged, and the rows of the beam entries that
    // are next in line after the coming step's picks. The words land in early_a / early_b and only
    // feed a test that never holds; they are consumed one phase later, when they have long arrived.
    uint32_t early_a = 0u, early_b = 0u, early_acc = 0u;
    __syncthreads();
    SR_TICK(13);
#ifdef SR_WAVE_CLOCKS
    if (head == 0 && tid == 0) sr_wave_ticks[2] = wall_clock64();      // claims made
#endif
    if (fill) {
        // ---- the start set is scored here, ahead of the loop, where few registers are live: twice
        //      the rows in flight of a step's gather (a seed set of a thousand keys is one trip to
        //      memory for 1024 threads). The beam is empty, so every key is kept; the first
        //      n_first of a root set enter as expanded.
        constexpr int SEED_ROWS = KT == RA_F32 ? SR_UNROLL : 2 * SR_UNROLL;
        uint32_t lo = 0xffffffffu, hi = 0u;                  // of the ordered score bits (see the pre-filter)
        // R rows per 16-lane group with no branch between them: the ids leave LDS in one batch, the
        // rows are all requested before the first is scored, and each is scored as it arrives
        auto score_rows = [&](auto rows_c, int c0) __attribute__((always_inline)) {
            constexpr int R = decltype(rows_c)::value;
            RowBits<KT> rows[R];
            int idv[R];
#pragma unroll
            for (int u = 0; u < R; ++u) {
                const int c = c0 + u * (T / 16) + grp;
                idv[u] = c < n_root ? cid[c] : -1;           // (only the last call of a set is ragged)
            }
#pragma unroll
            for (int u = 0; u < R; ++u) rows[u] = load_key<KT>(Kh, idv[u] >= 0 ? idv[u] : e0, lane16);
            float part[R];
#pragma unroll
            for (int u = 0; u < R; ++u) part[u] = score_share<KT>(rows[u], qv);
            const float sc = rows_tree<R>(part, lane16);     // of row lane16 (R = 16), lane16 & (R - 1) in general
            const int c = c0 + (lane16 & (R - 1)) * (T / 16) + grp;
            if (lane16 < R && c < n_root) {
                u64 key = make_key(sc, cid[c]);
                if (c < n_first) key &= ~1ull;
                ckey[c] = key;                               // all are kept: no counter needed
                const uint32_t so = (uint32_t)(key >> 32);
                lo = so < lo ? so : lo;
                hi = so > hi ? so : hi;
            }
        };
        bool shared = false;
        if constexpr (Hook::kSeedShare) {
            if (seeded && hook.seeds_shared()) {
                // the keys come from other workgroups of the launch: every thread takes those of its
                // positions as they arrive; if one does not, the set is scored here after all
                bool came = true;
                for (int c = tid; c < n_root; c += 2 * T) {
                    const bool two = c + T < n_root;
                    u64 k0, k1;
                    hook.take_seed_keys(c, two ? c + T : -1, k0, k1);
                    came = came && k0 != 0ull && k1 != 0ull;
#ifdef SR_WAVE_CLOCKS
                    if (head == 0 && (c & 127) == 0 && c < 1024) sr_wave_ticks[24 + c / 128] = wall_clock64();
#endif
                    ckey[c] = k0;
                    if (two) ckey[c + T] = k1;
                    const uint32_t s0 = (uint32_t)(k0 >> 32), s1 = (uint32_t)(k1 >> 32);
                    lo = min(lo, min(s0, s1));
                    hi = max(hi, max(s0, s1));
                }
                if (!came) ctr[C_MISSED] = 1;
                __syncthreads();
                shared = ctr[C_MISSED] == 0;
                if (!shared) {
                    if (tid == 0) hook.seeds_missed();
                    lo = 0xffffffffu;
                    hi = 0u;
                }
            }
        }
        if (!shared) {
            constexpr int PER = T / 16;                      // rows one call takes per row in flight
            int c0 = 0;
            for (; n_root - c0 >= SEED_ROWS * PER; c0 += SEED_ROWS * PER) score_rows(sr_int<SEED_ROWS>{}, c0);
            if constexpr (SEED_ROWS > 8)
                if (n_root - c0 >= 8 * PER) { score_rows(sr_int<8>{}, c0); c0 += 8 * PER; }
            if (n_root - c0 >= 4 * PER) { score_rows(sr_int<4>{}, c0); c0 += 4 * PER; }
            if (n_root - c0 >= 2 * PER) { score_rows(sr_int<2>{}, c0); c0 += 2 * PER; }
            if (n_root - c0 >= PER) { score_rows(sr_int<1>{}, c0); c0 += PER; }
            if (n_root - c0 > 0) score_rows(sr_int<1>{}, c0);
        }
        // every lane may hold extremes of its keys: fold the wavefront
#pragma unroll
        for (int d = 1; d < RA_WAVE; d <<= 1) {
            lo = min(lo, (uint32_t)__shfl_xor((int)lo, d));
            hi = max(hi, (uint32_t)__shfl_xor((int)hi, d));
        }
        if (lane == 0) {
            atomicMin(reinterpret_cast<unsigned int*>(&ctr[C_LO]), lo);
            atomicMax(reinterpret_cast<unsigned int*>(&ctr[C_HI]), hi);
        }
    }
#ifdef SR_WAVE_CLOCKS
    if (head == 0 && tid == 0) sr_wave_ticks[3] = wall_clock64();      // start set's keys in LDS
#endif
    SR_TICK(5);

    for (;;) {
        SR_TICK_ITER(n_iters);
        int np;
        if (first) {
            np = 0;                  // nothing of the (empty) beam is expanded: see the set-up
        } else if (!picked) {
            // ---- pick the `expand` best unexpanded entries: the beam is sorted, so the picks are
            //      the first `expand` set flags in beam order. T entries per round, one per
            //      thread: ballot prefix inside a wavefront, wavefront totals through LDS, the
            //      rounds before it carried in `total`. The round loop also covers index bn, one
            //      past the end, whose rank is the number of unexpanded entries in all.
            int total = 0;
            for (int e0 = 0; e0 <= bn; e0 += T) {
                const int e = e0 + tid;
                const u64 mykey = e < bn ? cur[e] : 0ull;
                const bool un = (mykey & 1ull) != 0;
                const u64 unmask = __ballot(un);
                if (lane == 0) wtot[wv] = __popcll(unmask);
                if (tid == 0) {
                    ctr[C_NCAND] = 0;
                    ctr[C_NKEEP] = 0;
                    ctr[C_NUNEXP] = 0;
                }
                __syncthreads();
                int before = total;
                for (int x = 0; x < T / RA_WAVE; ++x) {
                    const int c = wtot[x];
                    if (x < wv) before += c;
                    total += c;
                }
                const int rank = before + __popcll(unmask & ((1ull << lane) - 1ull));
                if (e <= bn) urank[e] = (uint16_t)rank;
                if (un && rank < expand) {
                    picks[rank] = key_id(mykey);
                    cur[e] = mykey & ~1ull;
                }
                __syncthreads();
            }
            np = total < expand ? total : expand;
            if (np == 0) break;
        } else {
            // the merge left the picks in place and counted the unexpanded entries
            const int total = ctr[C_NUNEXP];
            np = total < expand ? total : expand;
            if (np == 0) break;
            if (tid == 0) urank[bn] = (uint16_t)total;
        }
        SR_TICK(0);
        if (first) {
            if (!seeded) {
                n_iters = 2;         // the entry point's step and its neighbours' step
                n_expanded = n_first;
            }
        } else {
            ++n_iters;
            n_expanded += np;
        }

        // ---- read the picked adjacency rows (all loads issued before any is consumed),
        //      claim unvisited neighbours (the doubled first step has its candidates already)
        if (!first) {
            const int cells = np * deg;
            // cell x is slot x % deg of pick x / deg; the quotient by a multiplication (exact while
            // x * deg < 2^32: there are at most RA_MAX_EXPAND * deg cells), because a division per
            // cell costs more than everything else in this loop
            const uint32_t deg_m = 0xffffffffu / (uint32_t)deg + 1u;
            // L cells per thread and pass, all L loads issued before the first claim: 8 for a wide
            // step (8192 cells), fewer for a narrow one, where the loads past the last cell are waste
            auto claim_cells = [&](auto loads_c) __attribute__((always_inline)) {
                constexpr int L = decltype(loads_c)::value;
                for (int x0 = 0; x0 < cells; x0 += T * L) {
                    int nbv[L];
#pragma unroll
                    for (int u = 0; u < L; ++u) {
                        // out-of-range slots re-read the last cell: loads without a branch around
                        // them can all be issued before the first one is consumed
                        const int x = x0 + u * T + tid;
                        const int xc = x < cells ? x : cells - 1;
                        const int xr = (int)__umulhi((uint32_t)xc, deg_m);       // xc / deg
                        const int v = adj_h[(size_t)picks[xr] * deg + (xc - xr * deg)];
                        nbv[u] = x < cells ? v : -1;
                    }
#pragma unroll
                    for (int u = 0; u < L; ++u) {
                        const int nb = nbv[u];
                        if (nb >= 0 && nb < N) {
                            const uint32_t bit = 1u << (nb & 31);
                            const uint32_t old = atomicOr(&bits[nb >> 5], bit);
                            if (!(old & bit)) cid[atomicAdd(&ctr[C_NCAND], 1)] = nb;
                        }
                    }
                }
            };
            if (cells > 4 * T) claim_cells(sr_int<SR_ADJ_LOADS>{});
            else claim_cells(sr_int<2>{});
        }
        __syncthreads();
        const int nc = ctr[C_NCAND];
        n_visited += nc;
        SR_TICK(1);
        if (tid == 0) {
            ctr[C_NUNEXP] = 0;               // everyone read it before the barrier above
            if (!first) {                    // (a start set's extremes were collected while it was scored)
                ctr[C_LO] = -1;              // as unsigned: the largest value; see the pre-filter below
                ctr[C_HI] = 0;
                ctr[C_NSURV] = 0;
            }
        }
        early_acc ^= early_a ^ early_b;      // issued a phase or more ago
        early_a = early_b = 0u;

        // ---- gather and score the new candidates; keep those that can enter the beam
        const u64 worst = bn == ef ? (cur[bn - 1] >> 1) : 0ull;
        // (R rows per 16-lane group with no branch between them, as for a start set)
        auto gather_rows = [&](auto rows_c, int c0) __attribute__((always_inline)) {
            constexpr int R = decltype(rows_c)::value;
            RowBits<KT> rows[R];
            int cidv[R];
#pragma unroll
            for (int u = 0; u < R; ++u) {
                const int c = c0 + u * (T / 16) + grp;
                cidv[u] = c < nc ? cid[c] : -1;
            }
            // groups without a candidate re-read the entry row instead of branching
#pragma unroll
            for (int u = 0; u < R; ++u) rows[u] = load_key<KT>(Kh, cidv[u] >= 0 ? cidv[u] : e0, lane16);
            float part[R];
#pragma unroll
            for (int u = 0; u < R; ++u) part[u] = score_share<KT>(rows[u], qv);
            const float sc = rows_tree<R>(part, lane16);     // of row lane16 & (R - 1)
            const int c = c0 + (lane16 & (R - 1)) * (T / 16) + grp;
            if (lane16 < R && c < nc) {
                const u64 key = make_key(sc, cid[c]);
                if ((key >> 1) > worst) ckey[atomicAdd(&ctr[C_NKEEP], 1)] = key;
            }
        };
        if (!first) {                                        // (a start set is scored already)
            constexpr int PER = T / 16;
            int c0 = 0;
            for (; nc - c0 >= SR_UNROLL * PER; c0 += SR_UNROLL * PER) gather_rows(sr_int<SR_UNROLL>{}, c0);
            if constexpr (SR_UNROLL > 4)
                if (nc - c0 >= 4 * PER) { gather_rows(sr_int<4>{}, c0); c0 += 4 * PER; }
            if (nc - c0 >= 2 * PER) { gather_rows(sr_int<2>{}, c0); c0 += 2 * PER; }
            if (nc - c0 >= PER) { gather_rows(sr_int<1>{}, c0); c0 += PER; }
            if (nc - c0 > 0) gather_rows(sr_int<1>{}, c0);
        }
        __syncthreads();
        int nk = ctr[C_NKEEP];
        SR_TICK(2);
        if (nk == 0) {               // uniform: nothing enters the beam
            picked = false;
            continue;
        }
        // ---- pre-filter. At most ef of the kept candidates can enter the beam, and the merge below
        //      ranks them against each other at a cost quadratic in their number. A step that keeps
        //      many more than ef (a seed set scored at once) first drops those that cannot be among
        //      its best ef: the scores are cut into 256 equal-width bins between the smallest and
        //      the largest, a histogram finds the highest bin b such that the bins
        //      from b up hold at least ef candidates, and only those survive, compacted in place.
        //      Everything dropped is below at least ef survivors; which survive does not depend on
        //      the order of the candidates. The claimed ids (cid) are dead by now: their first 256
        //      words are the histogram.
        // A seed set (empty beam, nothing expanded, every key kept) goes one step further: the same
        // bins also order the survivors. A survivor's place among the kept keys is the number of
        // keys in higher bins (a suffix sum over the histogram) plus its rank inside its own bin,
        // found by comparing it with the few keys that share the bin: the survivors are dealt into
        // buckets by bin (ckey is free: every thread holds its keys in registers), and each one
        // then counts the larger keys of its bucket. That replaces the merge below, whose counting
        // is quadratic in the survivors (about ef of them), for the one step where it is large;
        // beam, picks and counters come out as the merge would leave them (all entries unexpanded:
        // the unexpanded entries above a key are its position).
        bool bucketed = false;
        if (nk > ef + SR_PREFILTER_SLACK && nk <= SR_PREFILTER_REGS * T && maxc >= 256) {
            const bool buckets = first && seeded && maxc >= 768;
            u64 mine[SR_PREFILTER_REGS];
            uint32_t lo = 0xffffffffu, hi = 0u;
#pragma unroll
            for (int r = 0; r < SR_PREFILTER_REGS; ++r) {
                const int c = r * T + tid;
                mine[r] = c < nk ? ckey[c] : 0ull;
                if (c < nk) {
                    const uint32_t sc = (uint32_t)(mine[r] >> 32);
                    lo = sc < lo ? sc : lo;
                    hi = sc > hi ? sc : hi;
                }
            }
            if (!first) {                    // (a start set's extremes are known already)
#pragma unroll
                for (int d = 1; d < RA_WAVE; d <<= 1) {
                    const uint32_t ol = __shfl_xor(lo, d), oh = __shfl_xor(hi, d);
                    lo = ol < lo ? ol : lo;
                    hi = oh > hi ? oh : hi;
                }
                if (lane == 0) {
                    atomicMin(reinterpret_cast<unsigned int*>(&ctr[C_LO]), lo);
                    atomicMax(reinterpret_cast<unsigned int*>(&ctr[C_HI]), hi);
                }
            }
            if (tid < 256) { cid[tid] = 0; if (buckets) cid[512 + tid] = 0; }    // counts; bucket fill
            __syncthreads();
            // bin = (score - lowest) * 255 / (highest - lowest), truncated: every operation is
            // monotone in the score, so a larger score never lands in a lower bin. Non-finite
            // scores (from non-finite inputs) leave the factor at zero: one bin, everything survives.
            const float lo_f = f32_from_ordered((uint32_t)ctr[C_LO]);
            const float width = f32_from_ordered((uint32_t)ctr[C_HI]) - lo_f;
            const float to_bin = width > 0.f && width < INFINITY ? 255.0f / width : 0.f;
            int bin[SR_PREFILTER_REGS];
#pragma unroll
            for (int r = 0; r < SR_PREFILTER_REGS; ++r) {
                const float b = (f32_from_ordered((uint32_t)(mine[r] >> 32)) - lo_f) * to_bin;
                bin[r] = b >= 255.f ? 255 : b > 0.f ? (int)b : 0;
                if (r * T + tid < nk) atomicAdd(&cid[bin[r]], 1);
            }
            __syncthreads();
            if (wv == 0) {
                // lane l owns bins 4l .. 4l + 3; candidates in the bins from b up = total - (those below b)
                const int b0 = cid[4 * lane], b1 = cid[4 * lane + 1], b2 = cid[4 * lane + 2], b3 = cid[4 * lane + 3];
                const int incl = wave_incl_scan(b0 + b1 + b2 + b3);
                const int total = __builtin_amdgcn_readlane(incl, RA_WAVE - 1);
                const int from3 = total - incl + b3, from2 = from3 + b2, from1 = from2 + b1, from0 = from1 + b0;
                const int best = from3 >= ef ? 3 : from2 >= ef ? 2 : from1 >= ef ? 1 : from0 >= ef ? 0 : -1;
                const u64 has = __ballot(best >= 0);          // never empty: bin 0 and up hold all nk > ef
                if (lane == 63 - __clzll(has)) {
                    ctr[C_BIN] = 4 * lane + best;
                    if (buckets) ctr[C_NSURV] = best == 3 ? from3 : best == 2 ? from2 : best == 1 ? from1 : from0;
                }
                if (buckets) {                               // keys in the bins above each bin
                    cid[256 + 4 * lane + 3] = from3 - b3;
                    cid[256 + 4 * lane + 2] = from2 - b2;
                    cid[256 + 4 * lane + 1] = from1 - b1;
                    cid[256 + 4 * lane] = from0 - b0;
                }
            }
            __syncthreads();
            const int bstar = ctr[C_BIN];
            if (buckets) {
                const int nsurv = ctr[C_NSURV];              // >= ef
#pragma unroll
                for (int r = 0; r < SR_PREFILTER_REGS; ++r)
                    if (r * T + tid < nk && bin[r] >= bstar)
                        ckey[cid[256 + bin[r]] + atomicAdd(&cid[512 + bin[r]], 1)] = mine[r];
                __syncthreads();
                for (int p = tid; p < nsurv; p += T) {
                    u64 k = ckey[p];
                    const float b = (f32_from_ordered((uint32_t)(k >> 32)) - lo_f) * to_bin;
                    const int kb = b >= 255.f ? 255 : b > 0.f ? (int)b : 0;
                    const int bs = cid[256 + kb], be = bs + cid[kb];
                    int pos = bs;
                    for (int j = bs; j < be; ++j) pos += ckey[j] > k ? 1 : 0;
                    if (pos < ef) {
                        if (pos < expand) {                  // this step's picks: the first `expand` entries
                            picks[pos] = key_id(k);
#ifndef SR_NO_EARLY_TOUCH
                            early_a = *reinterpret_cast<const uint32_t*>(adj_h + (size_t)key_id(k) * deg);
#endif
                            k &= ~1ull;
                        }
                        nxt[pos] = k;
                        urank_nxt[pos] = (uint16_t)pos;
                    }
                }
                if (tid == 0) {
                    ctr[C_NUNEXP] = ef;                      // every entry of the new beam (nsurv >= ef)
                    ctr[C_NCAND] = 0;
                    ctr[C_NKEEP] = 0;
                }
                nk = nsurv;
                bucketed = true;
            }
            if (!bucketed) {
#pragma unroll
            for (int r = 0; r < SR_PREFILTER_REGS; ++r)
                if (r * T + tid < nk && bin[r] >= bstar) ckey[atomicAdd(&ctr[C_NSURV], 1)] = mine[r];
            __syncthreads();
            nk = ctr[C_NSURV];
            }
        }
        SR_TICK(11);

        // ---- merge by rank into the other beam buffer, truncating at ef. The final position of
        //      an element of (beam u kept candidates) is the number of elements that beat it.
        //      A candidate: the beam entries above it (binary search in the sorted beam: its slot)
        //      plus the candidates above it (counted, 16 comparisons per task, tasks spread over
        //      the workgroup). A beam entry: its index plus the candidates whose slot is at or
        //      before it, a prefix sum over the histogram of slots. The same numbers give the
        //      count of *unexpanded* elements above each element (every candidate is unexpanded;
        //      for the beam's part urank has it), so the next step's picks, the elements with
        //      fewer than `expand` unexpanded ones above them, fall out of the merge.
        if (!bucketed) {
            const int E = bn + nk;
            const int nch = (nk + 15) >> 4;
            const int items = nk * nch;
#ifndef SR_NO_EARLY_TOUCH
            if (tid < nk)
                early_a = *reinterpret_cast<const uint32_t*>(adj_h + (size_t)key_id(ckey[tid]) * deg);
#endif
            for (int c = tid; c < nk; c += T) {
                const int b = count_better(cur, bn, ckey[c]);
                if (b) atomicAdd(&cnt[c], b << 16);           // high half: beam entries above it
                atomicAdd(&hist[b], 1);
            }
            SR_TICK(8);
            const float inv_nk = 1.0f / (float)nk;
            // (tasks are dealt from the last thread down: the first threads, busy with the binary
            // searches above, get the fewest)
            for (int a = T - 1 - tid; a < items; a += T) {
                // a = ch * nk + c without an integer division: the float quotient is off by at most one
                int ch = (int)((float)a * inv_nk), c = a - ch * nk;
                if (c < 0) { --ch; c += nk; }
                if (c >= nk) { ++ch; c -= nk; }
                const int above = ch + 1 < nch ? count_above16_full(ckey + ch * 16, ckey[c])
                                               : count_above16(ckey + ch * 16, nk - ch * 16, ckey[c]);
                if (above) atomicAdd(&cnt[c], above);
                if (first && n_first > 0) {
                    // the doubled first step has expanded candidates too: how many of those beat
                    // this one goes into the counter's high half (the beam is empty, so it is free)
                    const int exp_above = count_above16_expanded(ckey + ch * 16, nk - ch * 16, ckey[c]);
                    if (exp_above) atomicAdd(&cnt[c], exp_above << 16);
                }
            }
            SR_TICK(9);
            __syncthreads();
            SR_TICK(3);
            if (tid == 0) {
                ctr[C_NCAND] = 0;
                ctr[C_NKEEP] = 0;
            }
            for (int i = tid; i <= ef; i += T) hist_nxt[i] = 0;
            SR_TICK(10);
            for (int e0 = 0; e0 < E; e0 += T) {                   // T elements per round
                const int e = e0 + tid;
                // candidates above beam entry e: inclusive prefix sum of hist, by wavefront, each
                // adding up the part of hist before its own 64 entries itself (no second barrier)
                int cbeam = 0;
                if (e0 + wv * RA_WAVE < bn) {                     // this wavefront has beam entries
                    int before = 0;
                    for (int x = 0; x < e0 / RA_WAVE + wv; ++x) before += hist[x * RA_WAVE + lane];
                    before = __builtin_amdgcn_readlane(wave_incl_scan(before), RA_WAVE - 1);
                    cbeam = before + wave_incl_scan(e < bn ? hist[e] : 0);
                }
                bool un = false;
                if (e < E) {
                    const bool beam = e < bn;
                    u64 k;
                    int c, b;                                     // candidates / beam entries above
                    if (beam) {
                        k = cur[e];
                        c = cbeam;
                        b = e;
                    } else {
                        const int both = cnt[e - bn];
                        cnt[e - bn] = 0;
                        k = ckey[e - bn];
                        c = both & 0xffff;
                        b = both >> 16;
                    }
                    int pos, ur;                                  // ur: unexpanded elements above this one
                    if (first) {                                  // empty beam; b counts expanded candidates above
                        pos = c;
                        ur = c - b;
                        b = 0;
                    } else {
                        pos = b + c;
                        const int ub = (int)urank[b] - np;        // this step's picks are expanded now
                        ur = c + (ub > 0 ? ub : 0);
                    }
                    un = pos < ef && (k & 1ull);
                    if (un && ur < expand) {
                        picks[ur] = key_id(k);
                        k &= ~1ull;
                    }
#ifndef SR_NO_EARLY_TOUCH
                    else if (beam && un && ur < 2 * expand) {     // next in line after those picks
                        early_b = *reinterpret_cast<const uint32_t*>(adj_h + (size_t)key_id(k) * deg);
                    }
#endif
                    if (pos < ef) {
                        nxt[pos] = k;
                        urank_nxt[pos] = (uint16_t)ur;
                    }
                }
                const u64 um = __ballot(un);
                if (lane == 0 && um) atomicAdd(&ctr[C_NUNEXP], __popcll(um));
            }
        }
        __syncthreads();
        SR_TICK(4);
        bn = bn + nk < ef ? bn + nk : ef;
        u64* t = cur; cur = nxt; nxt = t;
        uint16_t* tu = urank; urank = urank_nxt; urank_nxt = tu;
        int* th = hist; hist = hist_nxt; hist_nxt = th;
        picked = true;
        first = false;
    }

    hook.before_output();
    early_acc ^= early_a ^ early_b;
    if (early_acc == 0x9e3779b9u && N < 0) ids[(size_t)head * topk] = -1;    // never: keeps the early touches alive
    // ---- result: best-first beam entries outside the static set W = [0,s) u [N-w,N)
    if (tid < RA_WAVE) {
        int32_t* out = ids + (size_t)head * topk;
        int cnt = 0;
        // (a row of ids has topk cells; this head returns at most `take` <= topk of them)
        for (int base = 0; base < bn && cnt < take; base += RA_WAVE) {
            const int i = base + tid;
            const int id = i < bn ? key_id(cur[i]) : -1;
            const bool ok = i < bn && id >= s && id < N - w;
            const u64 mask = __ballot(ok);
            const int pos = cnt + __popcll(mask & ((1ull << tid) - 1ull));
            if (ok && pos < take) {
                out[pos] = id;
                if (lds_ids) lds_ids[pos] = id;
            }
            cnt += __popcll(mask);
        }
        if (cnt > take) cnt = take;
        for (int i = cnt + tid; i < topk; i += RA_WAVE) {
            out[i] = -1;
            if (lds_ids) lds_ids[i] = -1;
        }
        if (tid == 0) ctr[C_NKEEP] = cnt;
        if (stats && tid == 0) {
            ra_stats st;
            st.n_visited = n_visited;
            st.n_expanded = n_expanded;
            st.n_iters = n_iters;
            st.n_returned = cnt;
            stats[head] = st;
        }
    }
    __syncthreads();
    SR_TICK(6);
    SR_TICK_FLUSH;
    return ctr[C_NKEEP];
}


// Threads per search. One search per compute unit or fewer (the latency-bound case): the largest
// workgroup finishes a search soonest. More searches than compute units: smaller workgroups, so
// that several searches share a compute unit and one's trips to HBM hide behind another's work
// (measured at 512 searches of 32K keys: 111 us per launch with 1024 threads, 74 with 512, 68 with 256).
static inline int search_threads(int heads, int ef) {
    if (heads <= 256 || ef > 512) return 1024;
    return ef > 256 ? 512 : 256;
}

// LDS bytes run_search needs.
static inline size_t search_lds_bytes(int64_t N, int deg, int ef, int expand, bool global_bitset) {
    const int maxc = expand * deg;
    size_t b = (size_t)2 * ef * 8 + (size_t)(maxc + 16) * 8 + (size_t)maxc * 4 + (size_t)(maxc + 2 * ef + 2) * 4 +
               (RA_MAX_EXPAND + C_COUNT) * 4 + (size_t)(ef + 1) * 4;
    if (!global_bitset) b += (size_t)((N + 31) >> 5) * 4;
    return b;
}

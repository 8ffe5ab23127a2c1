// The paper's exact baselines on the same harness: "Flat" retrieval (exact top-k by scanning
// every key, Sec. 4.1 and Table 5) and full attention over the whole context (Eq. 1). On a part
// with 8 TB/s of HBM these set the honest reference for the graph search: one layer's keys at
// 128K context are 268 MB, i.e. tens of microseconds of streaming.
//
// Flat top-k, two kernels:
//   1. flat_scores_kernel: streams K once per KV head and scores every key against the query
//      heads of its GQA group (16 lanes per key row, the same fixed-order float32 inner product
//      as the graph search, so both rank keys identically); writes one order-preserving uint32
//      per (head, key), 0 for keys of the static set W, which retrieval must not return, and
//      the largest of them per tile: the FL_TILE keys that one 16-lane group scores in a chunk
//      of FL_CHUNK (FL_ROWS consecutive keys out of every 16 x FL_ROWS), so a tile maximum
//      stays in registers until it is written.
//   2. flat_select_kernel: one workgroup per head. The topk-th largest tile maximum is a
//      threshold that at least topk keys reach, so every key of the answer (and every tie of
//      its last one) lies at or above it, in a tile whose maximum does: only those tiles (about
//      topk of them) are read again, their keys at or above the threshold are collected and
//      sorted by (score descending, id ascending) with a bitonic network in LDS. With too few
//      tiles for that, a threshold placed from a strided sample and one pass over all keys do
//      the same; when neither can place a safe threshold, an exact radix select over all keys
//      (four 8-bit histogram passes) finds the k-th largest key, and the keys above it plus the
//      lowest ids among its ties are taken.
#include "search_dev.h"

#define FL_THREADS 256
#define FL_CHUNK 512               // keys per workgroup of the scoring kernel
#define FL_SEL_T 1024
#define FL_ROWS 8                  // key rows in flight per 16-lane group
#define FL_TILE (FL_CHUNK / 16)     // keys per tile maximum: chunk base + 128 (j / 8) + 8 group + j % 8, j < FL_TILE
#define FL_TILES_MAX 8192          // tiles per head whose maxima (and list) fit LDS: 256K keys; four times as many from memory

// grid: x = chunk of FL_CHUNK keys, y = KV head, z = seq. GQA groups of another size than the
// kernel is built for run as G = 1 with one grid row per query head, kv_div of which share a KV head.
// STORE = false: only the tile maxima are written (the keys of the few tiles that matter are scored
// again by flat_rescore_kernel).
template <int DT, int G, bool STORE>
__global__ __launch_bounds__(FL_THREADS) void flat_scores_kernel(
    const void* __restrict__ q, const void* __restrict__ K, int n_q, int n_kv, int64_t N, int s, int w,
    uint32_t* __restrict__ keys, uint32_t* __restrict__ tile_max, int64_t n_tiles, int kv_div) {
    const int tid = threadIdx.x, grp = tid >> 4, lane16 = tid & 15;
    const int kvh = blockIdx.y / kv_div, seq = blockIdx.z, h0 = seq * n_q + blockIdx.y * G;
    const size_t esz = DT == RA_BF16 ? 2 : 4;
    const char* Kh = reinterpret_cast<const char*>(K) + ((size_t)seq * n_kv + kvh) * N * RA_D * esz;
    ScoreQuery<DT> qv[G];
#pragma unroll
    for (int g = 0; g < G; ++g)
        load_score_query<DT, DT>(reinterpret_cast<const char*>(q) + (size_t)(h0 + g) * RA_D * esz, lane16, qv[g]);
    const int64_t base = (int64_t)blockIdx.x * FL_CHUNK;
    uint32_t best[G];
#pragma unroll
    for (int g = 0; g < G; ++g) best[g] = 0u;
    // A 16-lane group takes FL_ROWS consecutive rows per round (a wavefront 4 x FL_ROWS rows, whole
    // cache lines either way). Lane u ends with the score of row u, so the FL_ROWS keys of a group
    // and head leave in one store, 32 consecutive keys (128 bytes) per wavefront, with no branch
    // around the scoring.
    // (the rows of the next round are requested before the current round is scored)
    RowBits<DT> nxt[FL_ROWS];
    auto request = [&](int r0) {
        const int64_t id0 = base + r0 + grp * FL_ROWS;
#pragma unroll
        for (int u = 0; u < FL_ROWS; ++u)
            nxt[u] = load_key_stream<DT>(Kh, id0 + u < N ? id0 + u : N - 1, lane16);   // loads stay unconditional
    };
    request(0);
#pragma unroll
    for (int r0 = 0; r0 < FL_CHUNK; r0 += 16 * FL_ROWS) {
        RowBits<DT> rows[FL_ROWS];
#pragma unroll
        for (int u = 0; u < FL_ROWS; ++u) rows[u] = nxt[u];
        if (r0 + 16 * FL_ROWS < FL_CHUNK) request(r0 + 16 * FL_ROWS);
        const int64_t id0 = base + r0 + grp * FL_ROWS;
        // the 16-lane sums of the FL_ROWS rows as one halving tree (rows_tree): lane u ends with row u's
        uint32_t mine[G];
        {
            const int64_t id = id0 + (lane16 & (FL_ROWS - 1));
            const bool counts = id < N && id >= s && id < N - w;      // keys of W (and past the end) read as 0
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float part[FL_ROWS];
#pragma unroll
                for (int u = 0; u < FL_ROWS; ++u) part[u] = score_share<DT>(rows[u], qv[g]);
                const float sc = rows_tree<FL_ROWS>(part, lane16);
                mine[g] = counts ? f32_ordered(sc) : 0u;
            }
        }
        const int64_t my_id = id0 + lane16;
        if (lane16 < FL_ROWS && my_id < N) {
#pragma unroll
            for (int g = 0; g < G; ++g) {
                if (STORE) keys[(size_t)(h0 + g) * N + my_id] = mine[g];
                best[g] = mine[g] > best[g] ? mine[g] : best[g];
            }
        }
    }
    // the tile maximum: over the lanes of the group that kept keys
#pragma unroll
    for (int g = 0; g < G; ++g) {
        uint32_t m = best[g], o;
        o = lane_xor32<1>(m, tid); m = o > m ? o : m;
        o = lane_xor32<2>(m, tid); m = o > m ? o : m;
        o = lane_xor32<4>(m, tid); m = o > m ? o : m;
        o = lane_xor32<8>(m, tid); m = o > m ? o : m;
        best[g] = m;
    }
    if (lane16 == 0) {
        const int64_t tile = (int64_t)blockIdx.x * 16 + grp;
#pragma unroll
        for (int g = 0; g < G; ++g) tile_max[(size_t)(h0 + g) * n_tiles + tile] = best[g];
    }
}

// Radix select over keys kh[0], kh[stride], ... (n of them): the `want`-th largest key, found
// exactly by four 8-bit histogram passes, most significant digit first. Returns it in *T, the
// number of entries wanted among the keys equal to it in *need_eq and their total in *eq_total.
__device__ __forceinline__ void radix_select(const uint32_t* __restrict__ kh, int64_t n, int64_t stride,
                                             unsigned want, unsigned* hist, unsigned* wsum,
                                             unsigned* s_prefix, unsigned* s_need,
                                             unsigned* s_eq_total) {
    const int tid = threadIdx.x;
    if (tid == 0) { *s_prefix = 0u; *s_need = want; }
    __syncthreads();
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256) hist[tid] = 0u;
        __syncthreads();
        const unsigned prefix = *s_prefix, need = *s_need;     // both stable until the barrier below
        const unsigned himask = shift == 24 ? 0u : (0xffffffffu << (shift + 8));
        for (int64_t i0 = tid; i0 < n; i0 += FL_SEL_T * 4) {
            uint32_t kv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t i = i0 + (int64_t)u * FL_SEL_T;
                kv[u] = kh[(i < n ? i : n - 1) * stride];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (i0 + (int64_t)u * FL_SEL_T < n && (kv[u] & himask) == prefix)
                    atomicAdd(&hist[(kv[u] >> shift) & 255u], 1u);
        }
        __syncthreads();
        // the digit where the count, accumulated from the largest digit down, reaches `need`:
        // thread t < 256 owns digit 255 - t; inclusive scan over t, one thread matches
        unsigned v = 0u, inc = 0u;
        if (tid < 256) {
            v = hist[255 - tid];
            inc = v;
#pragma unroll
            for (int d = 1; d < RA_WAVE; d <<= 1) {
                const unsigned o = __shfl_up(inc, d);
                if ((tid & (RA_WAVE - 1)) >= d) inc += o;
            }
            if ((tid & (RA_WAVE - 1)) == RA_WAVE - 1) wsum[tid / RA_WAVE] = inc;
        }
        __syncthreads();
        if (tid < 256) {
            for (int x = 0; x < tid / RA_WAVE; ++x) inc += wsum[x];
            const unsigned excl = inc - v;
            if (excl < need && (inc >= need || tid == 255)) {
                const unsigned bin = 255u - (unsigned)tid;
                *s_prefix = prefix | (bin << shift);
                *s_need = need - excl;           // how many are wanted from this digit's keys
                if (shift == 0) *s_eq_total = v;
            }
        }
        __syncthreads();
    }
}

#define FL_CAND 4096               // candidate capacity of the fast path
#define FL_SLICES RA_FLAT_SLICES    // workgroups per head that score the listed tiles again
#define FL_SLICE_CAND 1024         // candidates one of them can hold

// Second pass of the scan that stores no keys. Every workgroup of a head finds T0, a tile maximum
// that at least topk tile maxima reach (so at least topk keys reach it, and the answer and all ties
// of its last key lie in tiles whose maximum does), lists those tiles, and scores its share of them
// again - the same rows through the same instructions as the first pass, hence the same bits -
// appending every key at or above T0 to its own list: pairs (key, id) in the slice's eighth of the
// head's key area, their number in cand_count[head][slice]. A head with T0 = 0 (fewer than topk
// tiles hold an eligible key) or a slice with more candidates than it can hold (a crowd of ties)
// sets the top bit of the count instead: the select kernel then scores the whole head itself.
// grid: x = slice, y = head; a wavefront takes one tile at a time (a 16-lane group one run of 8 rows).
// BIG: more tiles than fit LDS (over 256K keys): the maxima are read where they are, in device memory
// (a few passes over at most 128 KB that the cache holds), and only the list of tiles is in LDS.
template <int DT, bool BIG>
__global__ __launch_bounds__(FL_SEL_T) void flat_rescore_kernel(
    const void* __restrict__ q, const void* __restrict__ K, int n_q, int n_kv, int64_t N, int s, int w,
    const uint32_t* __restrict__ tile_max, int64_t n_tiles, int topk, uint32_t* __restrict__ keys,
    uint32_t* __restrict__ cand_count, int cand_cap) {
    __shared__ unsigned hist[256];
    __shared__ unsigned s_ntl, s_prefix, s_cnt, s_lo, s_hi, s_t0;
    __shared__ uint32_t tm_lds[BIG ? 1 : FL_TILES_MAX];
    __shared__ unsigned short s_tl[FL_TILES_MAX];
    __shared__ unsigned long long mine[FL_SLICE_CAND];        // this workgroup's candidates: (key, id)
    const int tid = threadIdx.x, lane = tid & (RA_WAVE - 1), wv = tid / RA_WAVE, g4 = lane >> 4, lane16 = tid & 15;
    const int head = blockIdx.y, slice = blockIdx.x;
    const int seq = head / n_q, kvh = (head % n_q) / (n_q / n_kv);
    const size_t esz = DT == RA_BF16 ? 2 : 4;
    const char* Kh = reinterpret_cast<const char*>(K) + ((size_t)seq * n_kv + kvh) * N * RA_D * esz;
    ScoreQuery<DT> qv;
    load_score_query<DT, DT>(reinterpret_cast<const char*>(q) + (size_t)head * RA_D * esz, lane16, qv);
    const uint32_t* tm_mem = tile_max + (size_t)head * n_tiles;
    if constexpr (!BIG)
        for (int64_t t = tid; t < n_tiles; t += FL_SEL_T) tm_lds[t] = tm_mem[t];
    auto tm = [&](int64_t t) -> uint32_t { if constexpr (BIG) return tm_mem[t]; else return tm_lds[t]; };
    if (tid == 0) { s_ntl = 0u; s_cnt = 0u; s_lo = 0xffffffffu; s_hi = 0u; s_t0 = 0xffffffffu; }
    if (tid < 256) hist[tid] = 0u;
    __syncthreads();
    // A threshold that at least topk tile maxima reach, without an exact selection: the maxima are
    // cut into 255 equal-width bins between the smallest and the largest (bin 0 is for tiles with no
    // eligible key, whose maximum is 0), b is the highest bin such that the bins from b up hold at
    // least topk maxima, and T0 is the smallest maximum in those bins. It is at or below the
    // topk-th largest maximum, so nothing of the answer is lost, and a tile whose maximum reaches
    // T0 lies in those bins (the binning is monotone), so "maximum >= T0" lists exactly them.
    {
        uint32_t lo = 0xffffffffu, hi = 0u;
        for (int64_t t = tid; t < n_tiles; t += FL_SEL_T) {
            const uint32_t v = tm(t);
            if (v) { lo = v < lo ? v : lo; hi = v > hi ? v : hi; }
        }
#pragma unroll
        for (int d = 1; d < RA_WAVE; d <<= 1) {
            const uint32_t ol = __shfl_xor(lo, d), oh = __shfl_xor(hi, d);
            lo = ol < lo ? ol : lo;
            hi = oh > hi ? oh : hi;
        }
        if (lane == 0) { atomicMin(&s_lo, lo); atomicMax(&s_hi, hi); }
    }
    __syncthreads();
    const float lo_f = f32_from_ordered(s_lo);
    const float width = s_hi ? f32_from_ordered(s_hi) - lo_f : 0.f;
    const float to_bin = width > 0.f && width < INFINITY ? 254.0f / width : 0.f;
    auto bin_of = [&](uint32_t v) {
        if (!v) return 0;
        const float b = (f32_from_ordered(v) - lo_f) * to_bin;
        return 1 + (b >= 254.f ? 254 : b > 0.f ? (int)b : 0);
    };
    for (int64_t t = tid; t < n_tiles; t += FL_SEL_T) atomicAdd(&hist[bin_of(tm(t))], 1u);
    __syncthreads();
    if (wv == 0) {
        // lane l owns bins 4l .. 4l + 3; maxima in the bins from b up = total - (those below b)
        const int b0 = (int)hist[4 * lane], b1 = (int)hist[4 * lane + 1], b2 = (int)hist[4 * lane + 2],
                  b3 = (int)hist[4 * lane + 3];
        const int incl = wave_incl_scan(b0 + b1 + b2 + b3);
        const int total = __builtin_amdgcn_readlane(incl, RA_WAVE - 1);
        const int from3 = total - incl + b3, from2 = from3 + b2, from1 = from2 + b1, from0 = from1 + b0;
        const int best = from3 >= topk ? 3 : from2 >= topk ? 2 : from1 >= topk ? 1 : from0 >= topk ? 0 : -1;
        const unsigned long long has = __ballot(best >= 0);     // never empty: n_tiles >= 2 topk
        if (lane == 63 - __clzll(has)) s_prefix = (unsigned)(4 * lane + best);
    }
    __syncthreads();
    const int bstar = (int)s_prefix;
    if (bstar > 0) {
        uint32_t m = 0xffffffffu;
        for (int64_t t = tid; t < n_tiles; t += FL_SEL_T) {
            const uint32_t v = tm(t);
            if (bin_of(v) >= bstar) m = v < m ? v : m;
        }
#pragma unroll
        for (int d = 1; d < RA_WAVE; d <<= 1) {
            const uint32_t o = __shfl_xor(m, d);
            m = o < m ? o : m;
        }
        if (lane == 0) atomicMin(&s_t0, m);
    }
    __syncthreads();
    const uint32_t T0 = bstar > 0 ? s_t0 : 0u;
    if (T0 == 0u) {
        if (tid == 0) cand_count[head * FL_SLICES + slice] = 0x80000000u;
        return;
    }
    // this workgroup's share: the listed tiles whose number is congruent to its slice (the order of
    // a list differs from workgroup to workgroup, the tile numbers do not)
    for (int64_t t = tid; t < n_tiles; t += FL_SEL_T)
        if ((int)(t % FL_SLICES) == slice && tm(t) >= T0) {
            const unsigned at = atomicAdd(&s_ntl, 1u);
            if (at < FL_TILES_MAX) s_tl[at] = (unsigned short)t;
        }
    __syncthreads();
    if (s_ntl > FL_TILES_MAX) {              // (only with more tiles than the list holds: a crowd of ties)
        if (tid == 0) cand_count[head * FL_SLICES + slice] = 0x80000000u;
        return;
    }
    const int ntl = (int)s_ntl;
    for (int l = wv; l < ntl; l += FL_SEL_T / RA_WAVE) {
        const int64_t tl = s_tl[l];
        const int64_t id0 = (tl / 16) * FL_CHUNK + g4 * (16 * FL_ROWS) + (tl % 16) * FL_ROWS;
        RowBits<DT> rows[FL_ROWS];
#pragma unroll
        for (int u = 0; u < FL_ROWS; ++u) rows[u] = load_key<DT>(Kh, id0 + u < N ? id0 + u : N - 1, lane16);
        float part[FL_ROWS];
#pragma unroll
        for (int u = 0; u < FL_ROWS; ++u) part[u] = score_share<DT>(rows[u], qv);
        const float sc = rows_tree<FL_ROWS>(part, lane16);
        const int64_t id = id0 + (lane16 & (FL_ROWS - 1));
        const bool counts = id < N && id >= s && id < N - w;
        const uint32_t key = counts ? f32_ordered(sc) : 0u;
        if (lane16 < FL_ROWS && key >= T0) {
            const unsigned at = atomicAdd(&s_cnt, 1u);
            if (at < FL_SLICE_CAND) mine[at] = ((unsigned long long)key << 32) | (uint32_t)id;
        }
    }
    __syncthreads();
    const unsigned cnt = s_cnt;
    const bool fits = cnt <= (unsigned)cand_cap;
    if (tid == 0) cand_count[head * FL_SLICES + slice] = fits ? cnt : 0x80000000u;
    if (!fits) return;
    uint32_t* region = keys + (size_t)head * N + (size_t)slice * (N / FL_SLICES);
    for (unsigned i = tid; i < cnt; i += FL_SEL_T) {
        region[2 * (size_t)i] = (uint32_t)(mine[i] >> 32);
        region[2 * (size_t)i + 1] = (uint32_t)mine[i];
    }
}

// Every key of one head scored by one workgroup into kh[0..N) (0 for the static set W): what the
// select kernel falls back on when the second pass could not place a threshold.
template <int DT>
__device__ __forceinline__ void flat_score_head(const void* q, const void* K, int head, int n_q, int n_kv,
                                                int64_t N, int s, int w, uint32_t* kh) {
    const int tid = threadIdx.x, grp = tid >> 4, lane16 = tid & 15;
    const int seq = head / n_q, kvh = (head % n_q) / (n_q / n_kv);
    const size_t esz = DT == RA_BF16 ? 2 : 4;
    const char* Kh = reinterpret_cast<const char*>(K) + ((size_t)seq * n_kv + kvh) * N * RA_D * esz;
    ScoreQuery<DT> qv;
    load_score_query<DT, DT>(reinterpret_cast<const char*>(q) + (size_t)head * RA_D * esz, lane16, qv);
    for (int64_t b = 0; b < N; b += (FL_SEL_T / 16) * FL_ROWS) {
        const int64_t id0 = b + grp * FL_ROWS;
        RowBits<DT> rows[FL_ROWS];
#pragma unroll
        for (int u = 0; u < FL_ROWS; ++u) rows[u] = load_key<DT>(Kh, id0 + u < N ? id0 + u : N - 1, lane16);
        float part[FL_ROWS];
#pragma unroll
        for (int u = 0; u < FL_ROWS; ++u) part[u] = score_share<DT>(rows[u], qv);
        const float sc = rows_tree<FL_ROWS>(part, lane16);
        const int64_t id = id0 + (lane16 & (FL_ROWS - 1));
        if (lane16 < FL_ROWS && id < N) kh[id] = id >= s && id < N - w ? f32_ordered(sc) : 0u;
    }
}

#define FL_SAMPLE 4096             // keys sampled to place the threshold

// grid: x = head; block = FL_SEL_T threads. ids_out [heads][topk], padded with -1.
// Fast path: a threshold is placed from a strided sample so that about four times topk keys
// lie above it (the rank-r key of a 1-in-`stride` sample sits near rank r * stride of the
// whole); one pass collects every key at or above it; if at least topk and at most FL_CAND were
// collected, sorting them gives the exact answer (all ties of the k-th key are in the set).
// Otherwise (tiny or adversarial inputs) the exact radix select over all keys decides.
// two_pass: the keys were not stored; the candidates come from flat_rescore_kernel (q, K, n_q, n_kv,
// s, w are for the head that has to score itself after all, see there).
template <int DT>
__global__ __launch_bounds__(FL_SEL_T) void flat_select_kernel(uint32_t* __restrict__ keys,
                                                               const uint32_t* __restrict__ tile_max,
                                                               int64_t n_tiles, int64_t N, int topk,
                                                               int32_t* __restrict__ ids_out, bool two_pass,
                                                               const uint32_t* __restrict__ cand_count,
                                                               const void* __restrict__ q,
                                                               const void* __restrict__ K, int n_q, int n_kv,
                                                               int s, int w) {
    __shared__ unsigned hist[256], wsum4[4];
    __shared__ unsigned s_ntl;
    __shared__ unsigned short s_tl[FL_TILES_MAX];
    __shared__ unsigned s_prefix, s_need, s_cnt, s_eq_total, s_run;
    __shared__ unsigned long long sel[FL_CAND];
    __shared__ int wtot[FL_SEL_T / RA_WAVE];
    const int tid = threadIdx.x, lane = tid & (RA_WAVE - 1), wv = tid / RA_WAVE;
    uint32_t* kh = keys + (size_t)blockIdx.x * N;
    int32_t* out = ids_out + (size_t)blockIdx.x * topk;
    int n = -1;                                  // number of selected entries once known
    if (two_pass) {
        unsigned c = 0u, bad = 0u, start[FL_SLICES + 1];
#pragma unroll
        for (int j = 0; j < FL_SLICES; ++j) {
            const unsigned cj = cand_count[blockIdx.x * FL_SLICES + j];
            bad |= cj & 0x80000000u;
            start[j] = c;
            c += cj & 0x7fffffffu;
        }
        start[FL_SLICES] = c;
        if (!bad && c >= (unsigned)topk && c <= FL_CAND) {
            // entry i of the eight lists laid end to end (all loads in one trip)
            for (unsigned i = tid; i < c; i += FL_SEL_T) {
                int j = 0;
#pragma unroll
                for (int x = 1; x < FL_SLICES; ++x) j += i >= start[x] ? 1 : 0;
                unsigned first = 0u;
#pragma unroll
                for (int x = 1; x < FL_SLICES; ++x) first = j == x ? start[x] : first;
                const uint32_t* e = kh + (size_t)j * (N / FL_SLICES) + 2 * (size_t)(i - first);
                sel[i] = ((unsigned long long)e[0] << 32) | (0xffffffffu - e[1]);
            }
            n = (int)c;
        } else {
            __syncthreads();                     // (every thread has read the counts)
            flat_score_head<DT>(q, K, (int)blockIdx.x, n_q, n_kv, N, s, w, kh);
        }
        __syncthreads();
    }
    if (!two_pass && n_tiles >= 2 * (int64_t)topk && n_tiles <= FL_TILES_MAX) {
        // ---- tile path: T0 = the topk-th largest tile maximum (exact), then only the tiles at or above it
        // the head's tile maxima, copied into LDS (the candidate array is not in use yet)
        uint32_t* tm = reinterpret_cast<uint32_t*>(sel);
        for (int64_t t = tid; t < n_tiles; t += FL_SEL_T) tm[t] = tile_max[(size_t)blockIdx.x * n_tiles + t];
        __syncthreads();
        radix_select(tm, n_tiles, 1, (unsigned)topk, hist, wsum4, &s_prefix, &s_need, &s_eq_total);
        const uint32_t T0 = s_prefix;
        if (tid == 0) { s_cnt = 0u; s_ntl = 0u; }
        __syncthreads();
        if (T0 != 0u) {
            for (int64_t t = tid; t < n_tiles; t += FL_SEL_T)
                if (tm[t] >= T0) s_tl[atomicAdd(&s_ntl, 1u)] = (unsigned short)t;
            __syncthreads();
            const int ntl = (int)s_ntl;
            // thread = (tile of the list, key of the tile); four tiles of the list per thread in flight
            constexpr int TPI = FL_SEL_T / FL_TILE;              // list entries per pass of the workgroup
            const int sub = tid / FL_TILE, kk = tid % FL_TILE;
            for (int l0 = 0; l0 < ntl; l0 += 4 * TPI) {
                uint32_t kv[4];
                int64_t ki[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {                 // loads first, all in flight
                    const int l = l0 + u * TPI + sub;
                    const int64_t tl = s_tl[l < ntl ? l : ntl - 1];
                    ki[u] = (tl / 16) * FL_CHUNK + (kk / FL_ROWS) * (16 * FL_ROWS) + (tl % 16) * FL_ROWS + kk % FL_ROWS;
                    kv[u] = kh[ki[u] < N ? ki[u] : N - 1];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (l0 + u * TPI + sub < ntl && ki[u] < N && kv[u] >= T0) {
                        const unsigned at = atomicAdd(&s_cnt, 1u);
                        if (at < FL_CAND)
                            sel[at] = ((unsigned long long)kv[u] << 32) | (0xffffffffu - (uint32_t)ki[u]);
                    }
                }
            }
        }
        __syncthreads();
        const unsigned c = s_cnt;
        if (T0 != 0u && c >= (unsigned)topk && c <= FL_CAND) n = (int)c;
        __syncthreads();
    }
    const int64_t stride = N / FL_SAMPLE;
    if (n < 0 && stride >= 8 && (int64_t)topk * 4 <= N / 4) {
        const unsigned want = (unsigned)((4 * (int64_t)topk + stride - 1) / stride) + 2u;
        radix_select(kh, N / stride, stride, want, hist, wsum4, &s_prefix, &s_need, &s_eq_total);
        const uint32_t T0 = s_prefix;
        if (tid == 0) s_cnt = 0u;
        __syncthreads();
        if (T0 != 0u) {
            for (int64_t i0 = tid; i0 < N; i0 += FL_SEL_T * 8) {
                uint32_t kv[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {                 // loads first, all in flight
                    const int64_t i = i0 + (int64_t)u * FL_SEL_T;
                    kv[u] = kh[i < N ? i : N - 1];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int64_t i = i0 + (int64_t)u * FL_SEL_T;
                    if (i < N && kv[u] >= T0) {
                        const unsigned at = atomicAdd(&s_cnt, 1u);
                        if (at < FL_CAND)
                            sel[at] = ((unsigned long long)kv[u] << 32) | (0xffffffffu - (uint32_t)i);
                    }
                }
            }
        }
        __syncthreads();
        const unsigned c = s_cnt;
        if (T0 != 0u && c >= (unsigned)topk && c <= FL_CAND) n = (int)c;
        __syncthreads();
    }
    if (n < 0) {
        // ---- exact radix select over all keys (keys of W are 0 and sort last)
        radix_select(kh, N, 1, (unsigned)topk, hist, wsum4, &s_prefix, &s_need, &s_eq_total);
        const uint32_t T = s_prefix;             // the topk-th largest key
        const unsigned need_eq = s_need;         // entries wanted among the keys equal to T
        const unsigned eq_total = s_eq_total;
        if (tid == 0) { s_cnt = 0u; s_run = 0u; }
        __syncthreads();
        // collect every key above T; among the ties, the lowest ids
        const bool ordered = eq_total > need_eq; // more ties than wanted: take them in id order
        for (int64_t i0 = 0; i0 < N; i0 += FL_SEL_T) {
            const int64_t i = i0 + tid;
            const uint32_t k = i < N ? kh[i] : 0u;
            if (i < N && k > T)
                sel[atomicAdd(&s_cnt, 1u)] = ((unsigned long long)k << 32) | (0xffffffffu - (uint32_t)i);
            const bool tie = i < N && k == T && T != 0u;
            if (!ordered) {
                if (tie) sel[atomicAdd(&s_cnt, 1u)] = ((unsigned long long)k << 32) | (0xffffffffu - (uint32_t)i);
            } else {
                // stable: a tie is taken iff fewer than need_eq ties precede it
                const unsigned long long m = __ballot(tie);
                if (lane == 0) wtot[wv] = __popcll(m);
                __syncthreads();
                unsigned before = s_run;
                for (int x = 0; x < wv; ++x) before += wtot[x];
                const unsigned rank = before + __popcll(m & ((1ull << lane) - 1ull));
                if (tie && rank < need_eq)
                    sel[atomicAdd(&s_cnt, 1u)] = ((unsigned long long)k << 32) | (0xffffffffu - (uint32_t)i);
                __syncthreads();
                if (tid == 0) {
                    unsigned tot = 0;
                    for (int x = 0; x < FL_SEL_T / RA_WAVE; ++x) tot += wtot[x];
                    s_run += tot;
                }
                __syncthreads();
            }
        }
        __syncthreads();
        n = (int)s_cnt;                          // <= topk (fewer when W leaves fewer eligible keys)
    }
    // ---- order by (score descending, id ascending) = 64-bit key descending
    if (n <= FL_SEL_T) {
        // few candidates (the usual case): a thread's candidate goes where the count of larger keys says
        const unsigned long long mine = tid < n ? sel[tid] : 0ull;
        int rank = 0;
        for (int x = 0; x < n; ++x) rank += sel[x] > mine ? 1 : 0;
        if (tid < n && rank < topk) out[rank] = (int32_t)(0xffffffffu - (uint32_t)mine);
        for (int i = n + tid; i < topk; i += FL_SEL_T) out[i] = -1;
        return;
    }
    int n2 = 1;
    while (n2 < n) n2 <<= 1;
    for (int i = n + tid; i < n2; i += FL_SEL_T) sel[i] = 0ull;
    __syncthreads();
    for (int k = 2; k <= n2; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = tid; i < n2; i += FL_SEL_T) {
                const int ixj = i ^ j;
                if (ixj > i) {
                    const unsigned long long a = sel[i], b = sel[ixj];
                    const bool desc = (i & k) == 0;
                    if (desc ? (a < b) : (a > b)) { sel[i] = b; sel[ixj] = a; }
                }
            }
            __syncthreads();
        }
    }
    for (int i = tid; i < topk; i += FL_SEL_T)
        out[i] = i < n ? (int32_t)(0xffffffffu - (uint32_t)sel[i]) : -1;
}

// Re-ranking of a candidate list with the keys themselves (what follows a walk over 8-bit keys):
// one workgroup per (sequence, query head) scores its candidates with the search's fixed-order
// inner product (16 lanes per key row), ranks them by counting, and writes the best topk.
#define RR_THREADS 256
#define RR_ROWS 4                  // key rows in flight per 16-lane group
template <int DT>
__global__ __launch_bounds__(RR_THREADS) void rerank_kernel(const void* __restrict__ q,
                                                            const void* __restrict__ K, int n_q, int n_kv,
                                                            int64_t N, const int32_t* __restrict__ cand,
                                                            int n_cand, int topk, int32_t* __restrict__ ids) {
    __shared__ unsigned long long keys[RA_MAX_TOPK];
    __shared__ int n_valid;
    const int tid = threadIdx.x, grp = tid >> 4, lane16 = tid & 15;
    const int head = blockIdx.x, seq = head / n_q, kvh = (head % n_q) / (n_q / n_kv);
    const size_t esz = DT == RA_BF16 ? 2 : 4;
    const char* Kh = reinterpret_cast<const char*>(K) + ((size_t)seq * n_kv + kvh) * N * RA_D * esz;
    const int32_t* ch = cand + (size_t)head * n_cand;
    int32_t* out = ids + (size_t)head * topk;
    ScoreQuery<DT> qv;
    load_score_query<DT, DT>(reinterpret_cast<const char*>(q) + (size_t)head * RA_D * esz, lane16, qv);
    if (tid == 0) n_valid = 0;
    __syncthreads();
    for (int c0 = 0; c0 < n_cand; c0 += 16 * RR_ROWS) {
        RowBits<DT> rows[RR_ROWS];
        int id[RR_ROWS];
#pragma unroll
        for (int u = 0; u < RR_ROWS; ++u) {
            const int c = c0 + u * 16 + grp;
            id[u] = c < n_cand ? ch[c] : -1;
            if (id[u] >= N) id[u] = -1;
            rows[u] = load_key<DT>(Kh, id[u] >= 0 ? id[u] : 0, lane16);       // loads stay unconditional
        }
#pragma unroll
        for (int u = 0; u < RR_ROWS; ++u) {
            const int c = c0 + u * 16 + grp;
            const float sc = score_fixed<DT>(rows[u], qv);
            if (lane16 == 0 && c < n_cand) {
                // [ordered(score)][~id]: larger key = (score descending, id ascending); 0 = no candidate
                keys[c] = id[u] < 0 ? 0ull
                                    : ((unsigned long long)f32_ordered(sc) << 32) | (0xffffffffu - (uint32_t)id[u]);
                if (id[u] >= 0) atomicAdd(&n_valid, 1);
            }
        }
    }
    __syncthreads();
    const int nv = n_valid;
    for (int c = tid; c < n_cand; c += RR_THREADS) {
        const unsigned long long k = keys[c];
        if (k == 0ull) continue;
        int rank = 0;
        for (int x = 0; x < n_cand; ++x) rank += keys[x] > k ? 1 : 0;
        if (rank < topk) out[rank] = (int32_t)(0xffffffffu - (uint32_t)k);
    }
    for (int i = (nv < topk ? nv : topk) + tid; i < topk; i += RR_THREADS) out[i] = -1;
}

ra_status ra_launch_rerank(const void* q, const void* K, ra_dtype dt, int n_seq, int n_q, int n_kv, int64_t N,
                           const int32_t* cand, int n_cand, int topk, hipStream_t st, int32_t* ids) {
    if (dt == RA_BF16)
        hipLaunchKernelGGL(rerank_kernel<RA_BF16>, dim3(n_seq * n_q), dim3(RR_THREADS), 0, st, q, K, n_q, n_kv,
                           N, cand, n_cand, topk, ids);
    else
        hipLaunchKernelGGL(rerank_kernel<RA_F32>, dim3(n_seq * n_q), dim3(RR_THREADS), 0, st, q, K, n_q, n_kv,
                           N, cand, n_cand, topk, ids);
    RA_HIP(hipGetLastError());
    return RA_OK;
}

ra_status ra_launch_flat_topk(const void* q, const void* K, ra_dtype dt, int n_seq, int n_q, int n_kv,
                              int64_t N, int sink, int window, int topk, uint32_t* keys_ws,
                              hipStream_t st, int32_t* ids) {
    const int64_t n_tiles = 16 * ((N + FL_CHUNK - 1) / FL_CHUNK);
    uint32_t* tile_max = keys_ws + (size_t)n_seq * n_q * N;      // [heads][n_tiles], after the keys
    int64_t ss = sink < 0 ? 0 : sink, ww = window < 0 ? 0 : window;
    if (ss > N) ss = N;
    if (ww > N) ww = N;
    if (ss + ww >= N) { ss = N; ww = 0; }
    const int G = n_q / n_kv;
    const int heads = n_seq * n_q;
    uint32_t* cand_count = tile_max + (size_t)heads * n_tiles;   // [heads][FL_SLICES], after the tile maxima
    // Two passes without stored keys whenever the tile maxima can place the threshold: writing the
    // 16.8 MB of keys of a 128K layer costs the scan a fifth of its time, and all but a few thousand
    // of them are never read again. Candidate pairs (key, id) live in the head's key area.
    // (pairs a slice can hold: its eighth of the key area, and what its workgroup keeps in LDS)
    const int cand_cap = (int)(N / FL_SLICES / 2 < FL_SLICE_CAND ? N / FL_SLICES / 2 : FL_SLICE_CAND);
    const bool two_pass = n_tiles >= 2 * (int64_t)topk && n_tiles <= 4 * FL_TILES_MAX && cand_cap >= 64;
    const bool big = n_tiles > FL_TILES_MAX;                     // (tile numbers stay below 2^16 in the lists)
    const dim3 grid((unsigned)((N + FL_CHUNK - 1) / FL_CHUNK), n_kv, n_seq);
    // any other group size than 1, 2, 4, 8: one grid row per query head, every head scans its keys itself
    const dim3 grid1(grid.x, n_q, n_seq);
#define RA_FL_GO(DTV, GG, GRID, DIV)                                                                          \
    do {                                                                                                      \
        if (two_pass)                                                                                         \
            hipLaunchKernelGGL((flat_scores_kernel<DTV, GG, false>), GRID, dim3(FL_THREADS), 0, st, q, K, n_q,  \
                               n_kv, N, (int)ss, (int)ww, keys_ws, tile_max, n_tiles, DIV);                   \
        else                                                                                                  \
            hipLaunchKernelGGL((flat_scores_kernel<DTV, GG, true>), GRID, dim3(FL_THREADS), 0, st, q, K, n_q,   \
                               n_kv, N, (int)ss, (int)ww, keys_ws, tile_max, n_tiles, DIV);                   \
    } while (0)
#define RA_FL_DT(DTV)                                                                                         \
    do {                                                                                                      \
        switch (G) {                                                                                          \
            case 1: RA_FL_GO(DTV, 1, grid, 1); break;                                                         \
            case 2: RA_FL_GO(DTV, 2, grid, 1); break;                                                         \
            case 4: RA_FL_GO(DTV, 4, grid, 1); break;                                                         \
            case 8: RA_FL_GO(DTV, 8, grid, 1); break;                                                         \
            default: RA_FL_GO(DTV, 1, grid1, G);                                                              \
        }                                                                                                     \
        RA_HIP(hipGetLastError());                                                                            \
        if (two_pass && big) {                                                                                \
            hipLaunchKernelGGL((flat_rescore_kernel<DTV, true>), dim3(FL_SLICES, heads), dim3(FL_SEL_T), 0, st, \
                               q, K, n_q, n_kv, N, (int)ss, (int)ww, tile_max, n_tiles, topk, keys_ws,        \
                               cand_count, cand_cap);                                                         \
        } else if (two_pass) {                                                                                \
            hipLaunchKernelGGL((flat_rescore_kernel<DTV, false>), dim3(FL_SLICES, heads), dim3(FL_SEL_T), 0, st, \
                               q, K, n_q, n_kv, N, (int)ss, (int)ww, tile_max, n_tiles, topk, keys_ws,        \
                               cand_count, cand_cap);                                                         \
            RA_HIP(hipGetLastError());                                                                        \
        }                                                                                                     \
        hipLaunchKernelGGL((flat_select_kernel<DTV>), dim3(heads), dim3(FL_SEL_T), 0, st, keys_ws, tile_max,    \
                           n_tiles, N, topk, ids, two_pass, cand_count, q, K, n_q, n_kv, (int)ss, (int)ww);   \
    } while (0)
    if (dt == RA_BF16) RA_FL_DT(RA_BF16); else RA_FL_DT(RA_F32);
#undef RA_FL_DT
#undef RA_FL_GO
    RA_HIP(hipGetLastError());
    return RA_OK;
}


// ---- streaming-read probe ---------------------------------------------------------------------
// Reads a buffer once, start to end, and folds it into one word: what a read-only streaming kernel
// sustains on the device, the yardstick the scan kernels above are compared with. The shape is the
// best of those measured on a 1 GiB buffer: every workgroup owns one contiguous span, 256 threads,
// 16 bytes per lane and load, 8 non-temporal loads in flight, 16 workgroups per compute unit
// (7.1 TB/s; 6.2 with ordinary loads; 4.8 to 6.4 when the grid walks the buffer in strides).
#define PR_THREADS 256
#define PR_LOADS 8
__global__ __launch_bounds__(PR_THREADS) void read_probe_kernel(const uint4* __restrict__ p, size_t n16,
                                                                unsigned long long* __restrict__ out) {
    const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t b0 = (size_t)blockIdx.x * per, b1 = b0 + per < n16 ? b0 + per : n16;
    uint4 acc = make_uint4(0u, 0u, 0u, 0u);
    for (size_t i = b0 + threadIdx.x; i < b1; i += (size_t)PR_THREADS * PR_LOADS) {
        uint4 v[PR_LOADS];
#pragma unroll
        for (int u = 0; u < PR_LOADS; ++u) {
            const size_t j = i + (size_t)u * PR_THREADS;
            v[u] = load16_stream(p + (j < b1 ? j : i));      // loads stay unconditional
        }
#pragma unroll
        for (int u = 0; u < PR_LOADS; ++u)
            if (i + (size_t)u * PR_THREADS < b1) { acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w; }
    }
    unsigned long long w = ((unsigned long long)(acc.x ^ acc.z) << 32) | (acc.y ^ acc.w);
#pragma unroll
    for (int d = 1; d < RA_WAVE; d <<= 1) w ^= __shfl_xor(w, d);
    if ((threadIdx.x & (RA_WAVE - 1)) == 0 && w) atomicXor(out, w);
}

// The same for rows of 256 bytes at scattered places, the access pattern of the walk's gathers: every
// group of 16 lanes asks for 8 rows at a time, 16 bytes per lane, at row numbers drawn by a
// counter-based hash of the row's index in the sequence (so a run is reproducible and rows repeat
// only by chance); the grid walks the sequence of n_rows indices.
#define PG_THREADS 1024
#define PG_ROWS 8
__device__ __forceinline__ uint32_t pg_hash(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}
__global__ __launch_bounds__(PG_THREADS) void gather_probe_kernel(const uint4* __restrict__ p, uint32_t rows_in_buf,
                                                                  size_t n_rows, uint32_t seed,
                                                                  unsigned long long* __restrict__ out) {
    const int lane16 = threadIdx.x & 15;
    const size_t groups = (size_t)gridDim.x * (PG_THREADS / 16);
    const size_t g = (size_t)blockIdx.x * (PG_THREADS / 16) + (threadIdx.x >> 4);
    uint4 acc = make_uint4(0u, 0u, 0u, 0u);
    for (size_t i = g * PG_ROWS; i < n_rows; i += groups * PG_ROWS) {
        uint4 v[PG_ROWS];
#pragma unroll
        for (int u = 0; u < PG_ROWS; ++u) {
            const size_t j = i + u < n_rows ? i + u : i;         // loads stay unconditional
            const uint32_t row = pg_hash((uint32_t)j * 0x9e3779b9u + seed) % rows_in_buf;
            v[u] = load16_stream(p + (size_t)row * 16 + lane16);
        }
#pragma unroll
        for (int u = 0; u < PG_ROWS; ++u)
            if (i + u < n_rows) { acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w; }
    }
    unsigned long long w = ((unsigned long long)(acc.x ^ acc.z) << 32) | (acc.y ^ acc.w);
#pragma unroll
    for (int d = 1; d < RA_WAVE; d <<= 1) w ^= __shfl_xor(w, d);
    if ((threadIdx.x & (RA_WAVE - 1)) == 0 && w) atomicXor(out, w);
}

ra_status ra_launch_gather_probe(const void* buf, size_t bytes, size_t n_rows, uint32_t seed, hipStream_t st,
                                 unsigned long long* out) {
    const size_t rows_in_buf = bytes / 256;
    if (rows_in_buf < 1 || rows_in_buf > 0xffffffffull) RA_FAIL(RA_EINVAL, "buffer of %zu B: 1 .. 2^32 - 1 rows of 256 B", bytes);
    size_t blocks = (n_rows + (size_t)(PG_THREADS / 16) * PG_ROWS - 1) / ((size_t)(PG_THREADS / 16) * PG_ROWS);
    if (blocks > 512) blocks = 512;                          // two workgroups per compute unit
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(gather_probe_kernel, dim3((unsigned)blocks), dim3(PG_THREADS), 0, st,
                       reinterpret_cast<const uint4*>(buf), (uint32_t)rows_in_buf, n_rows, seed, out);
    RA_HIP(hipGetLastError());
    return RA_OK;
}

ra_status ra_launch_read_probe(const void* buf, size_t bytes, hipStream_t st, unsigned long long* out) {
    const size_t n16 = bytes / 16;
    size_t blocks = (n16 + (size_t)PR_THREADS * PR_LOADS - 1) / ((size_t)PR_THREADS * PR_LOADS);
    if (blocks > 256 * 16) blocks = 256 * 16;                // 16 workgroups per compute unit
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(read_probe_kernel, dim3((unsigned)blocks), dim3(PR_THREADS), 0, st,
                       reinterpret_cast<const uint4*>(buf), n16, out);
    RA_HIP(hipGetLastError());
    return RA_OK;
}

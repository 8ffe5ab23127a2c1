// VectorSearch(q) of Algorithm 1: bounded best-first walk over one head's key graph
// (Sec. 2.4 describes proximity-graph search as a greedy walk towards the most similar
// vectors). One workgroup of 256 threads per (sequence, query head); the whole search state
// lives in LDS:
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
// beam's worst entry, sorted, and merged into the beam by rank (two binary searches per
// element, no serial insertion). The beam after a step is the top-ef of a set union, so
// it does not depend on the order in which candidates were claimed.
//
// Scores decide integer results, so they are computed in one fixed float32 order: each
// of 16 lanes sums its 8 contiguous products left to right, then the 16 partial sums are
// added pairwise over adjacent lanes (xor 1, 2, 4, 8). Identical key rows therefore score
// identically, and a CPU reference can reproduce every bit.
#include "common.h"

#define SR_THREADS 256
#define SR_LDS_LIMIT (64 * 1024)

enum { C_NPICK = 0, C_NCAND = 1, C_NKEEP = 2, C_COUNT = 8 };

typedef unsigned long long u64;

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

// Raw 32 B (fp32) / 16 B (bf16) of a key row owned by this lane.
template <int DT> struct RowBits { uint4 a; uint4 b; };

template <int DT>
__device__ __forceinline__ RowBits<DT> load_key(const void* Kh, int64_t row, int lane16) {
    RowBits<DT> r;
    if (DT == RA_BF16) {
        r.a = reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(Kh) + row * RA_D)[lane16];
        r.b = r.a;
    } else {
        const uint4* p = reinterpret_cast<const uint4*>(reinterpret_cast<const float*>(Kh) + row * RA_D);
        r.a = p[lane16 * 2];
        r.b = p[lane16 * 2 + 1];
    }
    return r;
}

// The fixed-order inner product described in the file header. All 16 lanes of the group
// return the same value.
template <int DT>
__device__ __forceinline__ float score_fixed(const RowBits<DT>& r, const float* qv) {
    float acc;
    if (DT == RA_BF16) {
        // bf16 x bf16 products are exact in float32, so fma == multiply-then-add here
        acc = qv[0] * bf16_lo(r.a.x);
        acc = fmaf(qv[1], bf16_hi(r.a.x), acc);
        acc = fmaf(qv[2], bf16_lo(r.a.y), acc);
        acc = fmaf(qv[3], bf16_hi(r.a.y), acc);
        acc = fmaf(qv[4], bf16_lo(r.a.z), acc);
        acc = fmaf(qv[5], bf16_hi(r.a.z), acc);
        acc = fmaf(qv[6], bf16_lo(r.a.w), acc);
        acc = fmaf(qv[7], bf16_hi(r.a.w), acc);
    } else {
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
    acc = __fadd_rn(acc, __shfl_xor(acc, 1, 16));
    acc = __fadd_rn(acc, __shfl_xor(acc, 2, 16));
    acc = __fadd_rn(acc, __shfl_xor(acc, 4, 16));
    acc = __fadd_rn(acc, __shfl_xor(acc, 8, 16));
    return acc;
}

// number of entries of the descending array arr[0..n) that beat k (flag bit ignored)
__device__ __forceinline__ int count_better(const u64* arr, int n, u64 k) {
    int lo = 0, hi = n;
    const u64 kk = k >> 1;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if ((arr[mid] >> 1) > kk) lo = mid + 1; else hi = mid;
    }
    return lo;
}

static __host__ __device__ inline int next_pow2(int x) {
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}

template <int DT, bool GBITS>
__global__ __launch_bounds__(SR_THREADS) void search_kernel(
    const void* __restrict__ q, const int32_t* __restrict__ adj, const int32_t* __restrict__ entry,
    const void* __restrict__ K, int n_q, int n_kv, int64_t N, int deg, int s, int w, int topk,
    int ef, int expand, uint32_t* __restrict__ gbits, int32_t* __restrict__ ids,
    ra_stats* __restrict__ stats) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int tid = threadIdx.x, grp = tid >> 4, lane16 = tid & 15;
    const int head = blockIdx.x, seq = head / n_q, h = head % n_q, kvh = h / (n_q / n_kv);
    const size_t esz = DT == RA_BF16 ? 2 : 4;
    const char* Kh = reinterpret_cast<const char*>(K) + ((size_t)seq * n_kv + kvh) * N * RA_D * esz;
    const int32_t* adj_h = adj + (size_t)head * N * deg;
    const int maxc = expand * deg, maxc2 = next_pow2(maxc);
    const int nwords = (int)((N + 31) >> 5);

    u64* cur = reinterpret_cast<u64*>(lds_raw);
    u64* nxt = cur + ef;
    u64* ckey = nxt + ef;            // [maxc2] candidates that passed the beam threshold
    u64* skey = ckey + maxc2;        // [maxc2] the same, sorted
    int* cid = reinterpret_cast<int*>(skey + maxc2);   // [maxc] claimed neighbour ids
    int* picks = cid + maxc;         // [RA_MAX_EXPAND]
    int* ctr = picks + RA_MAX_EXPAND;
    uint32_t* bits = GBITS ? gbits + (size_t)head * nwords
                           : reinterpret_cast<uint32_t*>(ctr + C_COUNT);

    if (!GBITS)
        for (int i = tid; i < nwords; i += SR_THREADS) bits[i] = 0u;
    float qv[8];
    load_q8<DT>(reinterpret_cast<const char*>(q) + (size_t)head * RA_D * esz, lane16, qv);
    const int e0 = entry[head];
    __syncthreads();
    if (grp == 0) {
        const RowBits<DT> r = load_key<DT>(Kh, e0, lane16);
        const float sc = score_fixed<DT>(r, qv);
        if (tid == 0) {
            cur[0] = make_key(sc, e0);
            atomicOr(&bits[e0 >> 5], 1u << (e0 & 31));
        }
    }
    int bn = 1, n_visited = 1, n_expanded = 0, n_iters = 0;
    __syncthreads();

    for (;;) {
        // ---- pick the `expand` best unexpanded entries (wavefront 0 scans the sorted beam)
        if (tid < RA_WAVE) {
            int np = 0;
            for (int base = 0; base < bn && np < expand; base += RA_WAVE) {
                const int i = base + tid;
                const u64 k = i < bn ? cur[i] : 0ull;
                const bool un = (k & 1ull) != 0;
                const u64 mask = __ballot(un);
                const int before = __popcll(mask & ((1ull << tid) - 1ull));
                if (un && np + before < expand) {
                    picks[np + before] = key_id(k);
                    cur[i] = k & ~1ull;
                }
                np += __popcll(mask);
            }
            if (tid == 0) {
                ctr[C_NPICK] = np < expand ? np : expand;
                ctr[C_NCAND] = 0;
                ctr[C_NKEEP] = 0;
            }
        }
        __syncthreads();
        const int np = ctr[C_NPICK];
        if (np == 0) break;
        ++n_iters;
        n_expanded += np;

        // ---- read the picked adjacency rows, claim unvisited neighbours
        for (int x = tid; x < np * deg; x += SR_THREADS) {
            const int node = picks[x / deg];
            const int nb = adj_h[(size_t)node * deg + (x % deg)];
            if (nb >= 0 && nb < N) {
                const uint32_t bit = 1u << (nb & 31);
                const uint32_t old = atomicOr(&bits[nb >> 5], bit);
                if (!(old & bit)) cid[atomicAdd(&ctr[C_NCAND], 1)] = nb;
            }
        }
        __syncthreads();
        const int nc = ctr[C_NCAND];
        n_visited += nc;

        // ---- gather and score the new candidates; keep those that can enter the beam
        const u64 worst = bn == ef ? (cur[bn - 1] >> 1) : 0ull;
        for (int c0 = 0; c0 < nc; c0 += 64) {
            RowBits<DT> rows[4];
            int cidv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = c0 + u * 16 + grp;
                cidv[u] = c < nc ? cid[c] : -1;
                if (cidv[u] >= 0) rows[u] = load_key<DT>(Kh, cidv[u], lane16);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (cidv[u] < 0) continue;
                const float sc = score_fixed<DT>(rows[u], qv);
                if (lane16 == 0) {
                    const u64 key = make_key(sc, cidv[u]);
                    if ((key >> 1) > worst) ckey[atomicAdd(&ctr[C_NKEEP], 1)] = key;
                }
            }
        }
        __syncthreads();
        const int nk = ctr[C_NKEEP];
        if (nk == 0) continue;       // uniform: nothing enters the beam

        // ---- sort the kept candidates (best first)
        const u64* sorted;
        if (nk <= SR_THREADS) {
            if (tid < nk) {
                const u64 mine = ckey[tid];
                int r = 0;
                for (int j = 0; j < nk; ++j) r += (ckey[j] > mine) ? 1 : 0;
                skey[r] = mine;
            }
            sorted = skey;
        } else {
            const int n2 = next_pow2(nk);
            for (int i = nk + tid; i < n2; i += SR_THREADS) ckey[i] = 0ull;
            __syncthreads();
            for (int k = 2; k <= n2; k <<= 1) {
                for (int j = k >> 1; j > 0; j >>= 1) {
                    for (int i = tid; i < n2; i += SR_THREADS) {
                        const int ixj = i ^ j;
                        if (ixj > i) {
                            const u64 a = ckey[i], b = ckey[ixj];
                            const bool desc = (i & k) == 0;
                            if (desc ? (a < b) : (a > b)) {
                                ckey[i] = b;
                                ckey[ixj] = a;
                            }
                        }
                    }
                    __syncthreads();
                }
            }
            sorted = ckey;
        }
        __syncthreads();

        // ---- merge by rank into the other beam buffer, truncating at ef
        for (int i = tid; i < bn; i += SR_THREADS) {
            const u64 k = cur[i];
            const int pos = i + count_better(sorted, nk, k);
            if (pos < ef) nxt[pos] = k;
        }
        for (int j = tid; j < nk; j += SR_THREADS) {
            const u64 k = sorted[j];
            const int pos = j + count_better(cur, bn, k);
            if (pos < ef) nxt[pos] = k;
        }
        __syncthreads();
        bn = bn + nk < ef ? bn + nk : ef;
        u64* t = cur; cur = nxt; nxt = t;
    }

    // ---- result: best-first beam entries outside the static set W = [0,s) u [N-w,N)
    if (tid < RA_WAVE) {
        int32_t* out = ids + (size_t)head * topk;
        int cnt = 0;
        for (int base = 0; base < bn && cnt < topk; base += RA_WAVE) {
            const int i = base + tid;
            const int id = i < bn ? key_id(cur[i]) : -1;
            const bool ok = i < bn && id >= s && id < N - w;
            const u64 mask = __ballot(ok);
            const int pos = cnt + __popcll(mask & ((1ull << tid) - 1ull));
            if (ok && pos < topk) out[pos] = id;
            cnt += __popcll(mask);
        }
        if (cnt > topk) cnt = topk;
        for (int i = cnt + tid; i < topk; i += RA_WAVE) out[i] = -1;
        if (stats && tid == 0) {
            ra_stats st;
            st.n_visited = n_visited;
            st.n_expanded = n_expanded;
            st.n_iters = n_iters;
            st.n_returned = cnt;
            stats[head] = st;
        }
    }
}

__global__ void fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x)
        p[i] = v;
}

size_t ra_search_lds_bytes(int64_t N, int deg, int ef, int expand, bool global_bitset) {
    const int maxc = expand * deg, maxc2 = next_pow2(maxc);
    size_t b = (size_t)2 * ef * 8 + (size_t)2 * maxc2 * 8 + (size_t)maxc * 4 +
               (RA_MAX_EXPAND + C_COUNT) * 4;
    if (!global_bitset) b += (size_t)((N + 31) >> 5) * 4;
    return b;
}

bool ra_search_needs_global_bitset(int64_t N, int deg, int ef, int expand) {
    return ra_search_lds_bytes(N, deg, ef, expand, false) > SR_LDS_LIMIT;
}

ra_status ra_launch_search(const void* q, const int32_t* adj, const int32_t* entry, const void* K,
                           ra_dtype dt, int n_seq, int n_q, int n_kv, int64_t N, int deg,
                           int sink, int window, int topk, int ef, int expand, uint32_t* bitset,
                           hipStream_t st, int32_t* ids, ra_stats* stats) {
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
#define RA_SR_LAUNCH(DTV, GB)                                                                     \
    hipLaunchKernelGGL((search_kernel<DTV, GB>), dim3(heads), dim3(SR_THREADS), lds, st, q, adj,  \
                       entry, K, n_q, n_kv, N, deg, (int)ss, (int)ww, topk, ef, expand, bitset,   \
                       ids, stats)
    if (dt == RA_BF16) {
        if (gb) RA_SR_LAUNCH(RA_BF16, true); else RA_SR_LAUNCH(RA_BF16, false);
    } else {
        if (gb) RA_SR_LAUNCH(RA_F32, true); else RA_SR_LAUNCH(RA_F32, false);
    }
#undef RA_SR_LAUNCH
    RA_HIP(hipGetLastError());
    return RA_OK;
}

// Projection of the query->key KNN lists into a key-key graph (Sec. 3.2: keys connected to
// the same query vectors are linked and the query vectors are dropped). Integer arithmetic
// only, so identical lists give bit-identical graphs.
//
// Reading implemented (the paper states the step in one sentence):
//   pop(i)  = number of lists holding key i;   c(a,b) = number of lists holding both;
//   pi      = keys by (pop descending, id ascending); entry = pi[0];
//   row(a)  = [pi[2t+1], pi[2t+2]] for a = pi[t] (a binary heap over popularity: every key is
//             reachable from the entry) followed by a's co-listed keys ranked by the Jaccard
//             overlap c / (pop(a) + pop(b) - c), ties by larger c, then lower id, until deg.
//
// Device plan, all stream-ordered, no host round trip:
//   1. pop by atomic histogram over the list cells, through a per-workgroup LDS table so that a
//      hub costs one atomic per workgroup instead of one per list.
//   2. one workgroup per graph: prefix sums over the keys (CSR offsets of the inverted lists,
//      compaction of the keys with pop > 0), a stable 4-bit LSD radix sort of those keys by
//      descending pop, and from it pi, its inverse pos, pop by position, and the entry point.
//   3. inverted lists (key -> the lists that hold it) filled through per-key cursors (ranges
//      reserved per workgroup through the same kind of LDS table), and a copy of the lists with
//      every key replaced by its position in pi.
//   4. backbone children and -1 padding for every row (fully coalesced).
//   5. rows of the populated keys, in pi order (largest first). For key a: stream the lists that
//      hold a (whole rows of the translated lists, coalesced), count each co-listed key, collect
//      the candidates with (count, popularity, id), and select the best 64 in rank order: 64
//      candidates at a time go through a bitonic network across the lanes of a wavefront
//      (fractions compared by 64-bit cross-multiplication) and are merged into its running best
//      64; chunks that cannot beat the 64th are skipped. Three regimes by the number of lists:
//        - few (lists x knn <= 1024): one key per wavefront, counts in an LDS hash table, no
//          workgroup barrier (pj_rows_small_kernel);
//        - the rest: one key per workgroup (pj_rows_kernel), counts in an LDS table indexed by
//          position when the graph has at most 8192 populated keys, else in an LDS hash table
//          (moderate keys) or in the workgroup's scratch in device memory (hubs); the four
//          wavefronts share the candidates and the first one merges their results;
//        - hubs (thousands of lists) run their lists through a three-deep load pipeline.
// No global sort of the M*knn*(knn-1) co-occurrence pairs is needed: the skewed keys that sit
// in nearly every list are simply the longest-running work items and are scheduled first.
#include <type_traits>

#include "common.h"

#define PJ_T 1024                 // threads of the ordering kernel
#define PJ_ROW_T 256              // threads of the row kernel
#define PJ_MAX_WG 2048

typedef unsigned long long u64;

struct ProjWs {                   // per-graph device arrays, carved from one workspace
    int32_t* pop;                 // [N]
    int32_t* pos;                 // [N]   position of key in pi
    int32_t* pi;                  // [N]
    int32_t* off;                 // [N+1] CSR offsets of inverted lists
    int32_t* cur;                 // [N]   fill cursors
    int32_t* inv;                 // [M*knn]
    int32_t* lp;                  // [M*knn] the lists with every key replaced by its position in pi (-1: none)
    int32_t* hk[2];               // [cap] radix ping-pong: keys
    int32_t* hi[2];               // [cap] radix ping-pong: ids
    int32_t* H;                   // [1]   number of populated keys
};

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct ProjLayout {
    size_t per_graph, o_pop, o_pos, o_pi, o_off, o_cur, o_inv, o_lp, o_hk0, o_hk1, o_hi0, o_hi1, o_H;
    size_t scratch_per_wg, o_scratch;
    int n_wg;
    int64_t cap;
};

static ProjLayout proj_layout(int n_graphs, int64_t N, int64_t M, int knn) {
    ProjLayout l;
    const int64_t cells = M * knn;
    l.cap = N < cells ? N : cells;
    size_t o = 0;
    l.o_pop = o; o += align256((size_t)N * 4);
    l.o_pos = o; o += align256((size_t)N * 4);
    l.o_pi = o; o += align256((size_t)N * 4);
    l.o_off = o; o += align256((size_t)(N + 1) * 4);
    l.o_cur = o; o += align256((size_t)N * 4);
    l.o_inv = o; o += align256((size_t)cells * 4);
    l.o_lp = o; o += align256((size_t)cells * 4);
    l.o_hk0 = o; o += align256((size_t)l.cap * 4);
    l.o_hk1 = o; o += align256((size_t)l.cap * 4);
    l.o_hi0 = o; o += align256((size_t)l.cap * 4);
    l.o_hi1 = o; o += align256((size_t)l.cap * 4);
    l.o_H = o; o += 256;
    l.per_graph = o;
    // row kernel scratch: per workgroup four int arrays of `cap` entries
    l.scratch_per_wg = align256((size_t)l.cap * 4) * 4;     // counters, candidates, two tuple columns
    int per_graph_wg = 128;
    while (per_graph_wg > 1 &&
           ((size_t)per_graph_wg * n_graphs > PJ_MAX_WG ||
            (size_t)per_graph_wg * n_graphs * l.scratch_per_wg > ((size_t)8 << 30)))
        per_graph_wg >>= 1;
    l.n_wg = per_graph_wg;
    l.o_scratch = l.per_graph * n_graphs;
    return l;
}

size_t ra_project_workspace_bytes(int n_graphs, int64_t N, int64_t M, int knn) {
    const ProjLayout l = proj_layout(n_graphs, N, M, knn);
    return l.o_scratch + (size_t)l.n_wg * n_graphs * l.scratch_per_wg;
}

__device__ __forceinline__ ProjWs carve(char* ws, const ProjLayout& l, int g) {
    char* b = ws + (size_t)g * l.per_graph;
    ProjWs w;
    w.pop = (int32_t*)(b + l.o_pop); w.pos = (int32_t*)(b + l.o_pos); w.pi = (int32_t*)(b + l.o_pi);
    w.off = (int32_t*)(b + l.o_off); w.cur = (int32_t*)(b + l.o_cur); w.inv = (int32_t*)(b + l.o_inv);
    w.lp = (int32_t*)(b + l.o_lp);
    w.hk[0] = (int32_t*)(b + l.o_hk0); w.hk[1] = (int32_t*)(b + l.o_hk1);
    w.hi[0] = (int32_t*)(b + l.o_hi0); w.hi[1] = (int32_t*)(b + l.o_hi1);
    w.H = (int32_t*)(b + l.o_H);
    return w;
}

// ---- 0. clear --------------------------------------------------------------------------
__global__ void pj_zero_kernel(char* ws, ProjLayout l, int64_t N, int n_graphs) {
    const int g = blockIdx.y;
    ProjWs w = carve(ws, l, g);
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < N;
         i += (int64_t)gridDim.x * blockDim.x) {
        w.pop[i] = 0;
        w.cur[i] = 0;
    }
    // counter tables of the row kernel must start at zero
    uint32_t* sc = (uint32_t*)(ws + l.o_scratch);
    const size_t words = (size_t)l.n_wg * n_graphs * l.scratch_per_wg / 4;
    const size_t stride = (size_t)gridDim.x * gridDim.y * blockDim.x;
    for (size_t i = ((size_t)blockIdx.y * gridDim.x + blockIdx.x) * blockDim.x + threadIdx.x;
         i < words; i += stride)
        sc[i] = 0u;
}

// ---- 1. pop ----------------------------------------------------------------------------
// The queries share their favourite keys (a hub is in nearly every list), so plain atomic adds
// would queue up on a handful of addresses. Each workgroup counts in a small direct-mapped table
// in LDS first (slot = key mod PJ_HOT, owned by the first key that claims it; other keys that
// map there go straight to memory) and adds every owned slot to memory once at the end.
#define PJ_HOT 2048
__global__ __launch_bounds__(256) void pj_pop_kernel(const int32_t* __restrict__ L, char* ws,
                                                     ProjLayout l, int64_t cells, int64_t N) {
    __shared__ int s_tag[PJ_HOT];
    __shared__ int s_num[PJ_HOT];
    const int g = blockIdx.y;
    ProjWs w = carve(ws, l, g);
    const int32_t* Lg = L + (size_t)g * cells;
    for (int x = threadIdx.x; x < PJ_HOT; x += blockDim.x) { s_tag[x] = -1; s_num[x] = 0; }
    __syncthreads();
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < cells;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int32_t k = Lg[i];
        if (k >= 0 && k < N) {
            const int x = k & (PJ_HOT - 1);
            const int owner = atomicCAS(&s_tag[x], -1, k);
            if (owner == -1 || owner == k) atomicAdd(&s_num[x], 1);
            else atomicAdd(&w.pop[k], 1);
        }
    }
    __syncthreads();
    for (int x = threadIdx.x; x < PJ_HOT; x += blockDim.x)
        if (s_tag[x] >= 0) atomicAdd(&w.pop[s_tag[x]], s_num[x]);
}

// ---- 2. ordering -----------------------------------------------------------------------
// exclusive scan of one int per thread over the workgroup; *total receives the sum
__device__ __forceinline__ int block_exscan(int v, int* wsum, int* total) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, nw = blockDim.x >> 6;
    int inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int n = __shfl_up(inc, d);
        if (lane >= d) inc += n;
    }
    if (lane == 63) wsum[wv] = inc;
    __syncthreads();
    int base = 0, tot = 0;
    for (int i = 0; i < nw; ++i) {
        const int s = wsum[i];
        if (i < wv) base += s;
        tot += s;
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

__global__ __launch_bounds__(PJ_T) void pj_order_kernel(char* ws, ProjLayout l, int64_t N, int64_t M,
                                                        int32_t* __restrict__ entry) {
    __shared__ int wsum[PJ_T / 64];
    __shared__ int wtot[PJ_T / 64][16];
    __shared__ int base[16];
    const int g = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    ProjWs w = carve(ws, l, g);

    // A. compaction of populated keys (ascending id), CSR offsets, zero-pop ranks
    int hot_run = 0, off_run = 0;
    for (int64_t b0 = 0; b0 < N; b0 += PJ_T) {
        const int64_t i = b0 + tid;
        const int p = i < N ? w.pop[i] : 0;
        const int hot = p > 0 ? 1 : 0;
        int th, tp;
        const int eh = block_exscan(hot, wsum, &th);
        const int ep = block_exscan(p, wsum, &tp);
        if (i < N) {
            w.off[i] = off_run + ep;
            const int hr = hot_run + eh;
            if (hot) {
                w.hi[0][hr] = (int)i;
                w.hk[0][hr] = (int)(M - p);          // ascending key = descending pop
            } else {
                w.pos[i] = (int)i - hr;              // rank among zero-pop keys (H added below)
            }
        }
        hot_run += th;
        off_run += tp;
    }
    const int H = hot_run;
    if (tid == 0) {
        w.off[N] = off_run;
        *w.H = H;
    }
    __syncthreads();

    // B. stable LSD radix sort of (key, id) by key, 4 bits per pass
    int bits = 1;
    while (((int64_t)1 << bits) < M) ++bits;
    int src = 0;
    for (int shift = 0; shift < bits; shift += 4) {
        if (tid < 16) base[tid] = 0;
        __syncthreads();
        for (int b0 = 0; b0 < H; b0 += PJ_T) {
            const int i = b0 + tid;
            if (i < H) atomicAdd(&base[(w.hk[src][i] >> shift) & 15], 1);
        }
        __syncthreads();
        if (tid == 0) {
            int run = 0;
            for (int v = 0; v < 16; ++v) {
                const int c = base[v];
                base[v] = run;
                run += c;
            }
        }
        __syncthreads();
        for (int b0 = 0; b0 < H; b0 += PJ_T) {
            const int i = b0 + tid;
            const bool valid = i < H;
            const int key = valid ? w.hk[src][i] : 0, id = valid ? w.hi[src][i] : 0;
            const int dg = (key >> shift) & 15;
            int wrank = 0;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const u64 mask = __ballot(valid && dg == v);
                if (dg == v) wrank = __popcll(mask & ((1ull << lane) - 1ull));
                if (lane == 0) wtot[wv][v] = __popcll(mask);
            }
            __syncthreads();
            if (valid) {
                int before = 0;
                for (int x = 0; x < wv; ++x) before += wtot[x][dg];
                const int dst = base[dg] + before + wrank;
                w.hk[src ^ 1][dst] = key;
                w.hi[src ^ 1][dst] = id;
            }
            __syncthreads();
            if (tid < 16) {
                int add = 0;
                for (int x = 0; x < PJ_T / 64; ++x) add += wtot[x][tid];
                base[tid] += add;
            }
            __syncthreads();
        }
        src ^= 1;
    }
    __syncthreads();

    // C. pi, pos, entry
    for (int t = tid; t < H; t += PJ_T) {
        const int id = w.hi[src][t];
        w.pi[t] = id;
        w.pos[id] = t;
        w.hk[0][t] = w.pop[id];        // from here on hk[0] is the popularity by position
    }
    for (int64_t i = tid; i < N; i += PJ_T) {
        if (w.pop[i] == 0) {
            const int p = H + w.pos[i];
            w.pos[i] = p;
            w.pi[p] = (int)i;
        }
    }
    if (tid == 0) entry[g] = H > 0 ? w.hi[src][0] : 0;
}

// ---- 3. inverted lists -----------------------------------------------------------------
// Same trick for the fill cursors: a workgroup first counts its cells per hot key in LDS, takes
// one range of every such key's inverted list with a single atomic add, and hands out the places
// inside its ranges with LDS atomics in a second pass over the same cells. The order of the
// entries inside an inverted list is immaterial (only co-occurrence counts come out of them).
__global__ __launch_bounds__(256) void pj_inv_kernel(const int32_t* __restrict__ L, char* ws,
                                                     ProjLayout l, int64_t cells, int knn, int64_t N) {
    __shared__ int s_tag[PJ_HOT];
    __shared__ int s_num[PJ_HOT];
    __shared__ int s_base[PJ_HOT];
    const int g = blockIdx.y;
    ProjWs w = carve(ws, l, g);
    const int32_t* Lg = L + (size_t)g * cells;
    for (int x = threadIdx.x; x < PJ_HOT; x += blockDim.x) { s_tag[x] = -1; s_num[x] = 0; }
    __syncthreads();
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < cells;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int32_t k = Lg[i];
        if (k >= 0 && k < N) {
            const int x = k & (PJ_HOT - 1);
            const int owner = atomicCAS(&s_tag[x], -1, k);
            if (owner == -1 || owner == k) atomicAdd(&s_num[x], 1);
        }
    }
    __syncthreads();
    for (int x = threadIdx.x; x < PJ_HOT; x += blockDim.x) {
        if (s_tag[x] >= 0) s_base[x] = atomicAdd(&w.cur[s_tag[x]], s_num[x]);
        s_num[x] = 0;                                  // now the cursor inside the range
    }
    __syncthreads();
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < cells;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int32_t k = Lg[i];
        int32_t p = -1;
        if (k >= 0 && k < N) {
            const int x = k & (PJ_HOT - 1);
            const int slot = s_tag[x] == k ? s_base[x] + atomicAdd(&s_num[x], 1)
                                           : atomicAdd(&w.cur[k], 1);
            w.inv[w.off[k] + slot] = (int32_t)(i / knn);
            p = w.pos[k];
        }
        w.lp[i] = p;
    }
}

// ---- 4. backbone + padding for every row -----------------------------------------------
__global__ void pj_backbone_kernel(char* ws, ProjLayout l, int64_t N, int deg,
                                   int32_t* __restrict__ adj) {
    const int g = blockIdx.y;
    ProjWs w = carve(ws, l, g);
    int32_t* adj_g = adj + (size_t)g * N * deg;
    const int64_t cells = N * deg;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < cells;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t a = i / deg;
        const int slot = (int)(i % deg);
        int32_t v = -1;
        if (slot < 2) {
            const int64_t ch = 2 * (int64_t)w.pos[a] + 1 + slot;
            if (ch < N) v = w.pi[ch];
        }
        adj_g[i] = v;
    }
}

// ---- 5. rows of populated keys ---------------------------------------------------------
struct Cand { uint32_t c, pb; int32_t b; };

// is x ranked before y for a key of popularity pa?  (Jaccard desc, count desc, id asc)
__device__ __forceinline__ bool cand_before(const Cand& x, const Cand& y, uint32_t pa) {
    const u64 lhs = (u64)x.c * (u64)(pa + y.pb - y.c);
    const u64 rhs = (u64)y.c * (u64)(pa + x.pb - x.c);
    if (lhs != rhs) return lhs > rhs;
    if (x.c != y.c) return x.c > y.c;
    return x.b < y.b;
}

// "no candidate": count 0 ranks after every real candidate (whose count is at least 1)
__device__ __forceinline__ Cand cand_none() {
    Cand x; x.c = 0u; x.pb = 0u; x.b = 0x7fffffff;
    return x;
}
__device__ __forceinline__ Cand cand_lane(const Cand& x, int src) {
    Cand y;
    y.c = (uint32_t)__builtin_amdgcn_readlane((int)x.c, src);
    y.pb = (uint32_t)__builtin_amdgcn_readlane((int)x.pb, src);
    y.b = __builtin_amdgcn_readlane(x.b, src);
    return y;
}
// one compare-exchange step of a bitonic network over the 64 lanes: partner lane ^ J; the lane
// keeps the better of the two when keep_best, else the worse
template <int J>
__device__ __forceinline__ Cand cand_exchange(const Cand& v, bool keep_best, uint32_t pa, int lane) {
    Cand o;
    o.c = lane_xor32<J>(v.c, lane);
    o.pb = lane_xor32<J>(v.pb, lane);
    o.b = (int32_t)lane_xor32<J>((uint32_t)v.b, lane);
    return (cand_before(o, v, pa) == keep_best) ? o : v;
}
// 64 candidates, one per lane, into rank order (DESC: lane 0 the best; else lane 63 the best)
template <bool DESC>
__device__ __forceinline__ Cand cand_sort64(Cand v, uint32_t pa, int lane) {
#define PJ_STEP(K_, J_) v = cand_exchange<J_>(v, (((lane & J_) == 0) == ((lane & K_) == 0)) == DESC, pa, lane);
    PJ_STEP(2, 1)
    PJ_STEP(4, 2) PJ_STEP(4, 1)
    PJ_STEP(8, 4) PJ_STEP(8, 2) PJ_STEP(8, 1)
    PJ_STEP(16, 8) PJ_STEP(16, 4) PJ_STEP(16, 2) PJ_STEP(16, 1)
    PJ_STEP(32, 16) PJ_STEP(32, 8) PJ_STEP(32, 4) PJ_STEP(32, 2) PJ_STEP(32, 1)
    PJ_STEP(64, 32) PJ_STEP(64, 16) PJ_STEP(64, 8) PJ_STEP(64, 4) PJ_STEP(64, 2) PJ_STEP(64, 1)
#undef PJ_STEP
    return v;
}
// a bitonic sequence of 64 into descending rank order
__device__ __forceinline__ Cand cand_merge64(Cand v, uint32_t pa, int lane) {
    v = cand_exchange<32>(v, (lane & 32) == 0, pa, lane);
    v = cand_exchange<16>(v, (lane & 16) == 0, pa, lane);
    v = cand_exchange<8>(v, (lane & 8) == 0, pa, lane);
    v = cand_exchange<4>(v, (lane & 4) == 0, pa, lane);
    v = cand_exchange<2>(v, (lane & 2) == 0, pa, lane);
    v = cand_exchange<1>(v, (lane & 1) == 0, pa, lane);
    return v;
}

// Row of the key at position t: its backbone children pi[2t+1], pi[2t+2], then the ranked
// candidates (lane l of `best` holds the l-th best, `want` of them count) that are not among
// the children, until deg entries; -1 beyond. One wavefront.
__device__ __forceinline__ void write_row(int32_t* row, const Cand& best, int want, int t,
                                          const int32_t* pi, int64_t N, int deg, int lane) {
    int32_t kids[2] = {-1, -1};
    int nk = 0;
    for (int s = 0; s < 2 && nk < deg; ++s) {
        const int64_t ch = 2 * (int64_t)t + 1 + s;
        if (ch < N) kids[nk++] = pi[ch];
    }
    const bool keep = best.c > 0u && lane < want && best.b != kids[0] && best.b != kids[1];
    const unsigned long long km = __ballot(keep);
    const int at = nk + __popcll(km & ((1ull << lane) - 1ull));
    const int total = nk + __popcll(km);
    if (lane < nk) row[lane] = kids[lane];
    if (keep && at < deg) row[at] = best.b;
    if (lane >= total && lane < deg) row[lane] = -1;
}

// Keys with few lists are handled one per wavefront (pj_rows_small_kernel), the others one per
// workgroup: the first position in pi (popularity descending) whose key has at most `limit` lists.
#define PJ_SMALL_TOUCH 2048       // list cells (lists x knn) of a key the wavefront kernel takes
#define PJ_SMALL_SLOTS 4096       // its hash table: at most half full
#define PJ_SMALL_WAVES 4
__device__ __forceinline__ int small_limit(int knn) {
    const int lim = PJ_SMALL_TOUCH / knn;
    return lim < 127 ? lim : 127;                 // a count must fit the 7 bits of a table entry
}
__device__ __forceinline__ int first_small(const int32_t* pop_by_pos, int H, int knn) {
    if (H >= (1 << 24)) return H;                 // a position must fit the other 25 bits
    const int limit = small_limit(knn);
    int lo = 0, hi = H;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (pop_by_pos[mid] > limit) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// One more co-occurrence of the key at position `key - 1` in an open-addressing table of `slots`
// (a power of two) LDS words, entry = key << 7 | count; the table is never more than half full.
__device__ __forceinline__ void lds_table_bump(uint32_t* tab, int slots, uint32_t key) {
    const uint32_t mask = (uint32_t)slots - 1u;
    uint32_t h = ((key * 2654435761u) >> 12) & mask;
    for (int probe = 0; probe < slots; ++probe) {
        uint32_t v = __hip_atomic_load(&tab[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (v == 0u) {
            v = atomicCAS(&tab[h], 0u, (key << 7) | 1u);
            if (v == 0u) return;                      // claimed, count 1
        }
        if ((v >> 7) == key) { atomicAdd(&tab[h], 1u); return; }
        h = (h + 1u) & mask;
    }
}

#define PJ_LDS_CNT 8192           // co-occurrence counters kept in LDS when the populated set fits
#define PJ_LDS_TUP 2048           // candidate tuples kept in LDS when the candidate list fits

// Rows of the populated keys of one graph. LDSCNT: the counter table (indexed by pi-position,
// < H) lives in LDS instead of the workgroup's global scratch; LDS atomics are an order of
// magnitude cheaper than L2 atomics and the table is small whenever the queries share their
// favourite keys (H is a few thousand at 128K context).
template <bool LDSCNT>
__device__ __forceinline__ void rows_for_graph(const int32_t* __restrict__ Lg, const ProjWs& w,
                                               uint32_t* cnt, int32_t* cand, uint32_t* tc_g,
                                               uint32_t* tp_g, uint32_t* tc_l, uint32_t* tp_l,
                                               int32_t* tb_l, int64_t N, int knn, int deg, int H,
                                               int32_t* __restrict__ adj_g, int* s_ncand,
                                               Cand (*s_best)[64], uint32_t* lds_tab) {
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int kp = knn <= 32 ? 32 : 64;
    const int t_end = first_small(w.hk[0], H, knn);       // the rest is pj_rows_small_kernel's
    for (int t = blockIdx.x; t < t_end; t += gridDim.x) {
        const int a = w.pi[t];
        const uint32_t pa = (uint32_t)w.pop[a];
        const int o0 = w.off[a];
        // With more populated keys than LDS counters, a key of moderate size still counts in LDS:
        // the counter array serves as an open-addressing table (entry = (position + 1) << 7 |
        // count, at most half full); only the hubs of such a graph count in device memory.
        const bool hashed = !LDSCNT && pa <= 127u && (int)pa * knn <= PJ_LDS_CNT / 2 && H < (1 << 24);
        if (tid == 0) *s_ncand = 0;
        __syncthreads();
        // count co-listed keys; the first touch of a counter appends the key (its position in pi)
        // to the candidates. A run of kp lanes (kp = 32 or 64 >= knn) reads one list, lane e its
        // e-th entry (one coalesced row of the position-translated lists, so no lookup per
        // entry is left).
        {
            const int e = tid & (kp - 1), r0 = tid / kp, rstep = PJ_ROW_T / kp;
            auto count_lists = [&](auto unroll_tag, int li_begin, int li_end) {
                constexpr int U = decltype(unroll_tag)::value;
                for (int li0 = li_begin + r0; li0 < li_end; li0 += U * rstep) {
                    int pp[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int li = li0 + u * rstep;
                        const int j = w.inv[o0 + (li < li_end ? li : li_end - 1)];
                        pp[u] = (li < li_end && e < knn) ? w.lp[(size_t)j * knn + (e < knn ? e : 0)] : -1;
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        if (pp[u] < 0 || pp[u] == t) continue;
                        if (hashed) {
                            lds_table_bump(lds_tab, PJ_LDS_CNT, (uint32_t)pp[u] + 1u);
                        } else if (atomicAdd(&cnt[pp[u]], 1u) == 0u) {
                            cand[atomicAdd(s_ncand, 1)] = pp[u];
                        }
                    }
                }
            };
            // A hub sits in tens of thousands of lists and one workgroup walks them all. Its lists
            // go through a three-deep pipeline, sixteen per lane and stage: the list numbers of
            // pass i + 2 and the rows of pass i + 1 are in flight while pass i bumps its counters
            // (a pass that ran list number -> row -> counters in sequence would be two memory
            // latencies long). Indices past the end are clamped, never branched around.
            constexpr int UB = 16;
            const int per_pass = UB * rstep;
            const int n_pass = (int)pa >= 8 * per_pass ? (int)pa / per_pass : 0;
            if (n_pass) {
                int j0[UB], j1[UB], j2[UB], p0[UB], p1[UB];
                auto load_inv = [&](int pass, int (&jj)[UB]) {
                    if (pass >= n_pass) pass = n_pass - 1;
#pragma unroll
                    for (int u = 0; u < UB; ++u) jj[u] = w.inv[o0 + pass * per_pass + r0 + u * rstep];
                };
                auto load_rows = [&](const int (&jj)[UB], int (&pp)[UB]) {
#pragma unroll
                    for (int u = 0; u < UB; ++u) pp[u] = w.lp[(size_t)jj[u] * knn + (e < knn ? e : 0)];
                };
                load_inv(0, j0);
                load_inv(1, j1);
                load_rows(j0, p0);
                for (int pass = 0; pass < n_pass; ++pass) {
                    load_inv(pass + 2, j2);
                    load_rows(j1, p1);
#pragma unroll
                    for (int u = 0; u < UB; ++u) {
                        if (e < knn && p0[u] >= 0 && p0[u] != t && atomicAdd(&cnt[p0[u]], 1u) == 0u)
                            cand[atomicAdd(s_ncand, 1)] = p0[u];
                    }
#pragma unroll
                    for (int u = 0; u < UB; ++u) { p0[u] = p1[u]; j1[u] = j2[u]; }
                }
            }
            count_lists(std::integral_constant<int, 4>{}, n_pass * per_pass, (int)pa);
        }
        __syncthreads();
        if (hashed) {                    // empty the table into the candidate list (entries as they are)
            for (int q = tid; q < PJ_LDS_CNT; q += PJ_ROW_T) {
                const uint32_t v = lds_tab[q];
                if (v != 0u) {
                    lds_tab[q] = 0u;
                    cand[atomicAdd(s_ncand, 1)] = (int32_t)v;
                }
            }
            __syncthreads();
        }
        const int nc = *s_ncand;
        const int want = nc < deg ? nc : deg;
        // gather (count, popularity, id) of every candidate once; reset its counter on the way
        const bool tl = nc <= PJ_LDS_TUP;
        uint32_t* tc = tl ? tc_l : tc_g;
        uint32_t* tp = tl ? tp_l : tp_g;
        int32_t* tb = tl ? tb_l : cand;
        for (int x = tid; x < nc; x += PJ_ROW_T) {
            int pb = cand[x];
            if (hashed) {
                tc[x] = (uint32_t)pb & 127u;
                pb = (int)((uint32_t)pb >> 7) - 1;
            } else {
                tc[x] = cnt[pb];
                cnt[pb] = 0u;
            }
            tp[x] = (uint32_t)w.hk[0][pb];
            tb[x] = w.pi[pb];            // the candidate list itself, when the tuples stay in global memory
        }
        __syncthreads();
        // best 64 of this wavefront's chunks, sorted: lane l holds its l-th best
        Cand best = cand_none();
        for (int x0 = wv * 64; x0 < nc; x0 += PJ_ROW_T) {
            Cand cd = cand_none();
            if (x0 + lane < nc) { cd.b = tb[x0 + lane]; cd.c = tc[x0 + lane]; cd.pb = tp[x0 + lane]; }
            const Cand last = cand_lane(best, 63);
            if (__ballot(cand_before(cd, last, pa)) == 0ull) continue;     // nothing here makes the 64
            cd = cand_sort64<false>(cd, pa, lane);                          // ascending: lane l = (63-l)-th best
            if (cand_before(cd, best, pa)) best = cd;                      // bitonic: the best 64 of the 128
            best = cand_merge64(best, pa, lane);
        }
        if (wv > 0) {
            s_best[wv - 1][lane] = best;
        }
        __syncthreads();
        // row = backbone children, then ranked candidates not already present
        if (wv == 0) {
            for (int o = 0; o < PJ_ROW_T / 64 - 1; ++o) {
                Cand cd = s_best[o][63 - lane];                             // descending list, reversed
                if (cand_before(cd, best, pa)) best = cd;
                best = cand_merge64(best, pa, lane);
            }
            write_row(adj_g + (size_t)a * deg, best, want, t, w.pi, N, deg, lane);
        }
        __syncthreads();
    }
}

__global__ __launch_bounds__(PJ_ROW_T) void pj_rows_kernel(const int32_t* __restrict__ L, char* ws,
                                                           ProjLayout l, int64_t N, int64_t M,
                                                           int knn, int deg,
                                                           int32_t* __restrict__ adj) {
    __shared__ int s_ncand;
    __shared__ Cand s_best[PJ_ROW_T / 64 - 1][64];
    __shared__ uint32_t s_cnt[PJ_LDS_CNT];
    __shared__ uint32_t s_tc[PJ_LDS_TUP], s_tp[PJ_LDS_TUP];
    __shared__ int32_t s_tb[PJ_LDS_TUP];
    const int g = blockIdx.y;
    ProjWs w = carve(ws, l, g);
    const int32_t* Lg = L + (size_t)g * M * knn;
    int32_t* adj_g = adj + (size_t)g * N * deg;
    char* sc = ws + l.o_scratch + ((size_t)g * gridDim.x + blockIdx.x) * l.scratch_per_wg;
    const size_t quarter = l.scratch_per_wg / 4;
    uint32_t* cnt_g = (uint32_t*)sc;                               // [cap] indexed by pos, zero at rest
    int32_t* cand = (int32_t*)(sc + quarter);                      // [cap]
    uint32_t* tc_g = (uint32_t*)(sc + 2 * quarter);                // [cap]
    uint32_t* tp_g = (uint32_t*)(sc + 3 * quarter);                // [cap]
    const int H = *w.H;
    if (H <= PJ_LDS_CNT) {
        for (int i = threadIdx.x; i < H; i += PJ_ROW_T) s_cnt[i] = 0u;
        __syncthreads();
        rows_for_graph<true>(Lg, w, s_cnt, cand, tc_g, tp_g, s_tc, s_tp, s_tb, N, knn, deg, H, adj_g,
                             &s_ncand, s_best, s_cnt);
    } else {
        for (int i = threadIdx.x; i < PJ_LDS_CNT; i += PJ_ROW_T) s_cnt[i] = 0u;
        __syncthreads();
        rows_for_graph<false>(Lg, w, cnt_g, cand, tc_g, tp_g, s_tc, s_tp, s_tb, N, knn, deg, H, adj_g,
                              &s_ncand, s_best, s_cnt);
    }
}

// Rows of the keys with few lists, one key per wavefront, no workgroup barrier. Co-occurrence
// counts go into an open-addressing table in LDS (entry = (position + 1) << 7 | count, sized to
// twice the key's list cells), which is then packed in place into the candidate list; the same
// bitonic selection as above ranks the candidates, whose popularity and id are fetched by position
// one chunk ahead.
__global__ __launch_bounds__(PJ_SMALL_WAVES * 64) void pj_rows_small_kernel(
    char* ws, ProjLayout l, int64_t N, int knn, int deg, int32_t* __restrict__ adj) {
    __shared__ uint32_t s_slot[PJ_SMALL_WAVES][PJ_SMALL_SLOTS];
    const int g = blockIdx.y;
    ProjWs w = carve(ws, l, g);
    int32_t* adj_g = adj + (size_t)g * N * deg;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    uint32_t* slot = s_slot[wv];
    const int H = *w.H;
    const int32_t* ppop = w.hk[0];
    const int kp = knn <= 32 ? 32 : 64, e = lane & (kp - 1), lpp = 64 / kp;     // lists per pass
    for (int x = lane; x < PJ_SMALL_SLOTS; x += 64) slot[x] = 0u;
    const int t_small = first_small(ppop, H, knn);
    for (int t = t_small + blockIdx.x * PJ_SMALL_WAVES + wv; t < H; t += gridDim.x * PJ_SMALL_WAVES) {
        const int a = w.pi[t];
        const int pa = ppop[t];
        const int o0 = w.off[a];
        int slots = 128;
        while (slots < 2 * pa * knn) slots <<= 1;           // <= PJ_SMALL_SLOTS by small_limit()
        // count
        for (int li0 = lane / kp; li0 < pa; li0 += 4 * lpp) {
            int pp[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int li = li0 + u * lpp;
                const int j = w.inv[o0 + (li < pa ? li : pa - 1)];
                pp[u] = (li < pa && e < knn) ? w.lp[(size_t)j * knn + (e < knn ? e : 0)] : -1;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (pp[u] < 0 || pp[u] == t) continue;
                lds_table_bump(slot, slots, (uint32_t)pp[u] + 1u);
            }
        }
        __builtin_amdgcn_wave_barrier();
        // pack the table in place: entry q moves to the number of entries before it
        int nc = 0;
        for (int q0 = 0; q0 < slots; q0 += 64) {
            const uint32_t v = slot[q0 + lane];
            slot[q0 + lane] = 0u;
            const unsigned long long m = __ballot(v != 0u);
            if (v != 0u) slot[nc + __popcll(m & ((1ull << lane) - 1ull))] = v;
            nc += __popcll(m);
        }
        __builtin_amdgcn_wave_barrier();
        // rank the candidates 64 at a time; a chunk's popularity and id are fetched (by position)
        // while the chunk before it is sorted and merged
        auto fetch = [&](int x0, Cand& cd) {
            cd = cand_none();
            const int x = x0 + lane < nc ? x0 + lane : (nc > 0 ? nc - 1 : 0);
            const uint32_t v = nc > 0 ? slot[x] : 0u;
            const int pb = v ? (int)(v >> 7) - 1 : 0;
            const uint32_t pbv = (uint32_t)ppop[pb];
            const int32_t bv = w.pi[pb];
            if (x0 + lane < nc) { cd.c = v & 127u; cd.pb = pbv; cd.b = bv; }
        };
        Cand best = cand_none(), cur, nxt;
        fetch(0, cur);
        for (int x0 = 0; x0 < nc; x0 += 64) {
            fetch(x0 + 64, nxt);
            const Cand last = cand_lane(best, 63);
            if (__ballot(cand_before(cur, last, (uint32_t)pa)) != 0ull) {
                cur = cand_sort64<false>(cur, (uint32_t)pa, lane);
                if (cand_before(cur, best, (uint32_t)pa)) best = cur;
                best = cand_merge64(best, (uint32_t)pa, lane);
            }
            cur = nxt;
        }
        __builtin_amdgcn_wave_barrier();
        for (int x = lane; x < nc; x += 64) slot[x] = 0u;       // the table is empty again
        write_row(adj_g + (size_t)a * deg, best, nc < deg ? nc : deg, t, w.pi, N, deg, lane);
    }
}

ra_status ra_launch_project(const int32_t* L, int n_graphs, int64_t N, int64_t M, int knn, int deg,
                            void* workspace, hipStream_t st, int32_t* adj, int32_t* entry) {
    if (M * (int64_t)knn >= ((int64_t)1 << 31))
        RA_FAIL(RA_EUNSUP, "M * knn must stay below 2^31 list cells");
    const ProjLayout l = proj_layout(n_graphs, N, M, knn);
    char* ws = (char*)workspace;
    const int64_t cells = M * knn;
    const unsigned gx = 256;
    hipLaunchKernelGGL(pj_zero_kernel, dim3(gx, n_graphs), dim3(256), 0, st, ws, l, N, n_graphs);
    hipLaunchKernelGGL(pj_pop_kernel, dim3(gx, n_graphs), dim3(256), 0, st, L, ws, l, cells, N);
    hipLaunchKernelGGL(pj_order_kernel, dim3(n_graphs), dim3(PJ_T), 0, st, ws, l, N, M, entry);
    hipLaunchKernelGGL(pj_inv_kernel, dim3(gx, n_graphs), dim3(256), 0, st, L, ws, l, cells, knn, N);
    hipLaunchKernelGGL(pj_backbone_kernel, dim3(gx, n_graphs), dim3(256), 0, st, ws, l, N, deg, adj);
    hipLaunchKernelGGL(pj_rows_kernel, dim3(l.n_wg, n_graphs), dim3(PJ_ROW_T), 0, st, L, ws, l, N, M,
                       knn, deg, adj);
    const unsigned small_wg = n_graphs >= 512 ? 1u : (unsigned)(512 / n_graphs);   // 2 per compute unit
    hipLaunchKernelGGL(pj_rows_small_kernel, dim3(small_wg, n_graphs), dim3(PJ_SMALL_WAVES * 64), 0, st,
                       ws, l, N, knn, deg, adj);
    RA_HIP(hipGetLastError());
    return RA_OK;
}

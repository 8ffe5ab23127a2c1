// Exact KNN from prefill queries to keys (Sec. 3.2, Fig. 2b): S = Q K^T on the matrix cores
// with the per-query top-knn selection fused behind it, so the M x N score matrix is never
// written anywhere.
//
// The product is computed transposed, one 32-key x 32-query block at a time:
//     C[key i][query j] += A[i][k] * B[k][j],  A = key rows, B = query rows,
// with v_mfma_f32_32x32x16_bf16 (bf16 inputs) or v_mfma_f32_32x32x2_f32 (fp32 inputs). In the
// 32x32 accumulator layout a lane holds ONE query column (lane % 32) and 16 key rows, so the
// selection threshold of a query is a single per-lane register: the common case is a
// max-tree over the lane's 16 scores and one compare. Only scores that reach the threshold go
// further (about knn * ln(N / knn) per query over a stream in storage order, a third of that in
// the order the keys are streamed in here: see knn_order.hip). Three ways to keep them:
//   KN_SEL_LDS (knn <= KN_BUFFERED_KNN): a query owns KN_CAP list slots in LDS, its best knn keys
//     so far, then two runs of pending slots, one per lane that scores for it. A lane appends a
//     key to its own run with a single LDS write (its fill count is a register); when a run cannot
//     take what a lane is about to append (keys come four at a time) the wavefront sorts the 64
//     slots of that query across its lanes (bitonic network), keeps the best knn and raises the
//     threshold.
//   KN_SEL_REG (knn <= KN_REG_KNN, bf16): a lane keeps its pending keys (KN_REG_PEND per query
//     set) in registers and a query's list takes 32 slots, so LDS holds the lists of twice as many
//     queries and a wavefront owns two sets of 32: every key operand read from LDS feeds two
//     independent MFMA chains. Merging a query's few pending keys into its sorted list takes no
//     sort (knn_fold_reg).
//   KN_SEL_INSERT (longer lists): sorted insertion, one key at a time, by the whole wavefront.
// Between two merges a threshold is stale but valid (never above the true one), so nothing is
// lost.
//
// A wavefront owns NQ x 32 queries for the whole key stream (their B operands stay in registers,
// and every key operand fetched feeds NQ MFMA chains); a workgroup is WAVES wavefronts. Lists hold
// 64-bit keys [ordered(score):32][~id:32], so "larger key" is "(score descending, id ascending)".
// The inner-product summation order is the hardware's; identical key rows still score
// identically for a given query because they go through the same instruction sequence.
//
// Key rows reach the matrix cores through LDS. In the operand layout a lane holds 16 bytes of
// its own row per step, so a load straight from memory touches 64 cache lines per instruction
// and the vector cache's line rate, not the matrix cores, sets the pace. Instead the workgroup
// copies the key stream in 16 KB stages with fully coalesced loads (16 lanes per 256-byte row,
// each stage fetched once for all its wavefronts and two stages ahead of its use), stores
// them with the 16-byte chunks of a row XOR-swizzled by the row number, and every wavefront
// reads its operands from there with conflict-free 16-byte LDS reads. Two stage buffers
// alternate; one barrier per stage.

#include "common.h"

#define KN_CAP 64                 // list slots of a query in the buffered selection (one per lane)
#define KN_BUFFERED_KNN 48        // longest list that leaves room for pending slots
#define KN_REG_KNN 32             // longest list of the selection that keeps pending keys in registers
#define KN_REG_MIN_KEYS 49152     // fewest keys for which that selection is the faster one (see ra_launch_knn)
#ifndef KN_REG_PEND
#define KN_REG_PEND 4             // pending keys a lane holds there (at least 4: a group of scores)
#endif
// how the top-knn selection keeps keys that reached a threshold until they are merged into a list
#define KN_SEL_INSERT 0           // not at all: sorted insertion, one key at a time
#define KN_SEL_LDS 1              // in pending runs behind the list in LDS (KN_CAP slots per query)
#define KN_SEL_REG 2              // in registers of the lane that scored them (32 slots per query in LDS)

typedef unsigned long long u64;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

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

// 64 keys, one per lane, sorted descending across the wavefront (bitonic network). Keys are
// distinct or zero, so "the other one is larger" decides every exchange.
__device__ __forceinline__ u64 wave_sort_desc(u64 v, int lane) {
#define KN_EXCHANGE(K_, J_)                                                                   \
    {                                                                                         \
        const u64 o = ((u64)lane_xor32<J_>((uint32_t)(v >> 32), lane) << 32) |                \
                      (u64)lane_xor32<J_>((uint32_t)v, lane);                                 \
        const bool keep_max = ((lane & J_) == 0) == ((lane & K_) == 0);                       \
        v = ((o > v) == keep_max) ? o : v;                                                    \
    }
    KN_EXCHANGE(2, 1)
    KN_EXCHANGE(4, 2) KN_EXCHANGE(4, 1)
    KN_EXCHANGE(8, 4) KN_EXCHANGE(8, 2) KN_EXCHANGE(8, 1)
    KN_EXCHANGE(16, 8) KN_EXCHANGE(16, 4) KN_EXCHANGE(16, 2) KN_EXCHANGE(16, 1)
    KN_EXCHANGE(32, 16) KN_EXCHANGE(32, 8) KN_EXCHANGE(32, 4) KN_EXCHANGE(32, 2) KN_EXCHANGE(32, 1)
    KN_EXCHANGE(64, 32) KN_EXCHANGE(64, 16) KN_EXCHANGE(64, 8) KN_EXCHANGE(64, 4) KN_EXCHANGE(64, 2)
    KN_EXCHANGE(64, 1)
#undef KN_EXCHANGE
    return v;
}

__device__ __forceinline__ u64 readlane64(u64 x, int l) {
    return ((u64)(uint32_t)__builtin_amdgcn_readlane((int)(x >> 32), l) << 32) |
           (u64)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, l);
}

// Fold the pending keys of one query into its list: afterwards slots [0, knn) hold its best knn
// keys in descending order and the pending slots are empty (all 64 lanes cooperate).
// Returns the new threshold: the score of slot knn - 1, or -inf while the list is not full.
__device__ __forceinline__ float knn_fold(u64* lst, int knn, int lane) {
    const u64 v = wave_sort_desc(lst[lane], lane);
    lst[lane] = lane < knn ? v : 0ull;
    const u64 last = readlane64(v, knn - 1);
    return last == 0ull ? -INFINITY : f32_from_ordered((uint32_t)(last >> 32));
}

// The same for a query (number jq of its set) whose pending keys sit in registers: p[] and fill
// are every lane's own, the query's are those of lanes jq and jq + 32. With a few keys to merge
// into a sorted list of 32 a sort is not needed: the list goes to the lower half-wave, the pending
// keys (zero where a lane holds fewer than it could) to lanes 32.. and, one by one as scalars, to
// everyone; a list entry moves down by the number of pending keys above it, a pending key lands at
// the number of keys above it, and every slot below 32 is written exactly once (keys are distinct
// or zero; a zero pending key writes nothing). The caller resets the fill counts of the query's lanes.
__device__ __forceinline__ float knn_fold_reg(u64* lst, int knn, int lane, int jq,
                                              const u64 (&p)[KN_REG_PEND], int fill) {
    constexpr int P = KN_REG_PEND;
    u64 v = lane < 32 ? lst[lane & 31] : 0ull;
    const int f_lo = __builtin_amdgcn_readlane(fill, jq), f_hi = __builtin_amdgcn_readlane(fill, jq + 32);
    u64 x[2 * P];
#pragma unroll
    for (int k = 0; k < P; ++k) {
        x[k] = readlane64(p[k], jq);
        x[P + k] = readlane64(p[k], jq + 32);
    }
#pragma unroll
    for (int k = 0; k < 2 * P; ++k) {
        if (!(k < P ? k < f_lo : k - P < f_hi)) x[k] = 0ull;
        if (lane == 32 + k) v = x[k];
    }
    int pos = lane;
#pragma unroll
    for (int k = 0; k < 2 * P; ++k) {
        const int above = __popcll(__ballot(v > x[k]));      // keys that beat pending key k
        if (lane < 32) pos += v < x[k] ? 1 : 0;
        if (lane == 32 + k) pos = above;
    }
    const bool writes = lane < 32 || (lane < 32 + 2 * P && v != 0ull);
    if (writes && pos < 32) lst[pos] = pos < knn ? v : 0ull;
    const u64 at_end = __ballot(writes && pos == knn - 1);
    const int src = at_end ? __ffsll((long long)at_end) - 1 : 0;
    const u64 last = readlane64(v, src);
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

// A use of every register of an operand (an empty asm statement that only reads them): its loads
// are complete here and cannot sink below later ones. The key stream's waits count loads in
// flight, and an operand load still counted there would turn every one of them into a wait for
// the newest load.
template <int DT>
__device__ __forceinline__ void settle_operand(const Operand<DT>& o) {
    if constexpr (DT == RA_BF16) {
        asm volatile("; operand loaded" ::"v"(o.v[0]), "v"(o.v[1]), "v"(o.v[2]), "v"(o.v[3]), "v"(o.v[4]),
                     "v"(o.v[5]), "v"(o.v[6]), "v"(o.v[7]));
    } else {
#pragma unroll
        for (int s = 0; s < 64; s += 16)
            asm volatile("; operand loaded" ::"v"(o.v[s]), "v"(o.v[s + 1]), "v"(o.v[s + 2]), "v"(o.v[s + 3]),
                         "v"(o.v[s + 4]), "v"(o.v[s + 5]), "v"(o.v[s + 6]), "v"(o.v[s + 7]), "v"(o.v[s + 8]),
                         "v"(o.v[s + 9]), "v"(o.v[s + 10]), "v"(o.v[s + 11]), "v"(o.v[s + 12]),
                         "v"(o.v[s + 13]), "v"(o.v[s + 14]), "v"(o.v[s + 15]));
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

// A staged key row keeps its 16-byte chunks at (chunk ^ (row & 15)): the 16 lanes that write one
// row, and the 16 lanes that read the same chunk of 16 consecutive rows, both cover all 64 banks.
// A lane reads the same chunks of the same row (lane % 32, or 32 rows on: same swizzle) in every
// stage, so the byte offsets are computed once (operand_offsets) and a read is one instruction
// with the stage buffer and the block as a constant displacement.
template <int DT> struct OperandAt { int at[DT == RA_BF16 ? 8 : 16]; };
template <int DT>
__device__ __forceinline__ void operand_offsets(int base, int row, int half, OperandAt<DT>& o) {
    constexpr int ROWB = DT == RA_BF16 ? 256 : 512, CPH = ROWB / 32;   // chunks per half row
    const int sw = row & 15;
#pragma unroll
    for (int s = 0; s < CPH; ++s) o.at[s] = base + row * ROWB + (((half * CPH + s) ^ sw) << 4);
}
template <int DT>
__device__ __forceinline__ void read_operand(const unsigned char* lds, const OperandAt<DT>& at, int disp,
                                             Operand<DT>& o) {
    if constexpr (DT == RA_BF16) {
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const uint4 u = *reinterpret_cast<const uint4*>(lds + at.at[s] + disp);
            o.v[s] = __builtin_bit_cast(bf16x8, u);
        }
    } else {
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            const float4 f = *reinterpret_cast<const float4*>(lds + at.at[s] + disp);
            o.v[4 * s] = f.x; o.v[4 * s + 1] = f.y; o.v[4 * s + 2] = f.z; o.v[4 * s + 3] = f.w;
        }
    }
}

// Stage copy: chunk x of a stage is 16 bytes of the stage's row x / (chunks per row); consecutive
// threads take consecutive chunks, thread tid the chunks tid + i * THREADS, so a thread copies the
// same 16-byte column of one row in every THREADS / (chunks per row) rows. The caller passes the
// key id of the row (stream positions beyond N repeat the last one; their scores are masked
// later). One chunk per call so that the values in flight stay in named registers.
template <int DT>
__device__ __forceinline__ u32x4 fetch_chunk(const char* Kh, int key_id, int column) {
    constexpr int ROWB = DT == RA_BF16 ? 256 : 512;
    return *reinterpret_cast<const u32x4*>(Kh + (size_t)key_id * ROWB + (size_t)column * 16);
}
template <int DT, int THREADS>
__device__ __forceinline__ void store_chunk(unsigned char* buf, int tid, int i, const u32x4& v) {
    constexpr int ROWB = DT == RA_BF16 ? 256 : 512, CPR = ROWB / 16;
    const int x = tid + i * THREADS;
    const int row = x / CPR, c = x % CPR;
    *reinterpret_cast<u32x4*>(buf + row * ROWB + ((c ^ (row & 15)) << 4)) = v;
}

// grid: x = block of NQ * 32 * WAVES queries, y = graph (seq * n_q + h). A wavefront owns NQ sets
// of 32 queries, so every key operand it reads feeds NQ MFMA chains.
// LDS: [NQ * 32 * WAVES][list slots] lists, then two stage buffers of STAGE bytes.
// SEL (KN_SEL_*) selects how keys wait for their list: KN_SEL_REG (knn <= KN_REG_KNN) leaves LDS for
// the lists of twice as many queries, so NQ = 2 and every operand read from LDS feeds two MFMAs;
// KN_SEL_LDS (knn <= KN_BUFFERED_KNN) and sorted insertion run with NQ = 1.
template <int DT, int NQ, int WAVES, int SEL, int STAGE>
__global__ __launch_bounds__(WAVES * RA_WAVE) void knn_kernel(
    const void* __restrict__ K, const void* __restrict__ Q, const u64* __restrict__ order,
    int64_t order_stride, int n_q, int n_kv, int64_t N, int64_t M, int knn,
    int32_t* __restrict__ L_out) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    constexpr int KN_THREADS = WAVES * RA_WAVE;
    constexpr int QPW = 32 * NQ, QPB = QPW * WAVES;
    constexpr int ROWB = DT == RA_BF16 ? 256 : 512;          // bytes of a key row
    constexpr int CPR = ROWB / 16;                            // 16-byte chunks per row
    constexpr int SROWS = STAGE / ROWB;              // key rows per stage
    constexpr int SBLK = SROWS / 32;                          // 32-key blocks per stage
    constexpr int CPT = STAGE / 16 / KN_THREADS;     // chunks a thread copies per stage
    static_assert(SBLK == 1 || SBLK == 2, "a stage holds one or two key blocks");
    static_assert(CPT * KN_THREADS * 16 == STAGE, "threads must tile a stage");
    static_assert(KN_THREADS % CPR == 0, "a thread keeps its 16-byte column");
    constexpr bool BUF = SEL != KN_SEL_INSERT, REGP = SEL == KN_SEL_REG;
    const int lstride = REGP ? KN_REG_KNN : BUF ? KN_CAP : knn;           // list slots per query
    const int pend = REGP ? KN_REG_PEND : (KN_CAP - knn) / 2;             // pending keys a lane can hold (BUF)
    u64* lists = reinterpret_cast<u64*>(lds_raw);           // [QPB][lstride]
    unsigned char* stage_buf = lds_raw + (size_t)QPB * lstride * sizeof(u64);   // 16-byte aligned: QPB is even
    const int tid = threadIdx.x, wv = tid / RA_WAVE, lane = tid % RA_WAVE;
    const int col = lane & 31, half = lane >> 5;
    const int graph = blockIdx.y, seq = graph / n_q, h = graph % n_q, kvh = h / (n_q / n_kv);
    const size_t esz = DT == RA_BF16 ? 2 : 4;
    const char* Kh = reinterpret_cast<const char*>(K) + ((size_t)seq * n_kv + kvh) * N * RA_D * esz;
    const char* Qh = reinterpret_cast<const char*>(Q) + (size_t)graph * M * RA_D * esz;
    const int64_t q0 = (int64_t)blockIdx.x * QPB + wv * QPW;   // first query of this wave
    // the key streamed p-th: the low word of the head's p-th order entry (used as loaded: arithmetic
    // on it would sit right behind the load and wait for it)
    const int* ord = reinterpret_cast<const int*>(order + (size_t)graph * order_stride);
    const int last_pos = (int)N - 1;               // ids and stream positions fit 31 bits
    auto stream_id = [&](int p) __attribute__((always_inline)) { return ord[2 * (size_t)(unsigned)(p < last_pos ? p : last_pos)]; };

    for (int i = tid; i < QPB * lstride; i += KN_THREADS) lists[i] = 0ull;
    u64* my_lists = lists + (size_t)wv * QPW * lstride;

    Operand<DT> b[NQ];
#pragma unroll
    for (int sidx = 0; sidx < NQ; ++sidx) {
        int64_t qr = q0 + sidx * 32 + col;
        if (qr >= M) qr = M - 1;                   // clamp loads; such columns are never written
        load_operand<DT>(Qh, qr, half, b[sidx]);
    }
#pragma unroll
    for (int sidx = 0; sidx < NQ; ++sidx) settle_operand<DT>(b[sidx]);
    __syncthreads();

    float tau[NQ];
    int fill[NQ];                                  // BUF: keys in this lane's pending run
    u64 pr[NQ][KN_REG_PEND];                       // REGP: the run itself
#pragma unroll
    for (int sidx = 0; sidx < NQ; ++sidx) {
        tau[sidx] = -INFINITY;
        fill[sidx] = 0;
#pragma unroll
        for (int k = 0; k < KN_REG_PEND; ++k) pr[sidx][k] = 0ull;
    }

    static_assert(CPT == 2 || CPT == 4, "two or four chunks per thread and stage");
    const int64_t nstage = (N + SROWS - 1) / SROWS;
    struct Held { u32x4 c0, c1, c2, c3; };         // a thread's share of one stage, in registers
    struct Rows { int r0, r1, r2, r3; };           // key ids of the rows that share comes from
    constexpr int RSTEP = KN_THREADS / CPR;        // rows between two chunks of a thread
    auto load_rows = [&](Rows& r, int64_t st) __attribute__((always_inline)) {
        if (st >= nstage) st = nstage - 1;          // past the end: the last stage again, unused
        const int p = (int)st * SROWS + tid / CPR;
        r.r0 = stream_id(p);
        r.r1 = stream_id(p + RSTEP);
        if constexpr (CPT == 4) {
            r.r2 = stream_id(p + 2 * RSTEP);
            r.r3 = stream_id(p + 3 * RSTEP);
        }
    };
    // lane l of every wavefront: the key id of row l of the stage (row l % 32 when a stage has 32)
    auto stage_ids = [&](int64_t st) __attribute__((always_inline)) {
        if (st >= nstage) st = nstage - 1;
        return stream_id((int)st * SROWS + lane % SROWS);
    };
    auto fetch_stage = [&](Held& h, const Rows& r) __attribute__((always_inline)) {
        h.c0 = fetch_chunk<DT>(Kh, r.r0, tid % CPR);
        h.c1 = fetch_chunk<DT>(Kh, r.r1, tid % CPR);
        if constexpr (CPT == 4) {
            h.c2 = fetch_chunk<DT>(Kh, r.r2, tid % CPR);
            h.c3 = fetch_chunk<DT>(Kh, r.r3, tid % CPR);
        }
    };
    auto store_stage = [&](const Held& h, unsigned char* buf) __attribute__((always_inline)) {
        store_chunk<DT, KN_THREADS>(buf, tid, 0, h.c0);
        store_chunk<DT, KN_THREADS>(buf, tid, 1, h.c1);
        if constexpr (CPT == 4) {
            store_chunk<DT, KN_THREADS>(buf, tid, 2, h.c2);
            store_chunk<DT, KN_THREADS>(buf, tid, 3, h.c3);
        }
    };
    // scores of one 32-key block against the wave's NQ query sets, then the selection
    // (kb: the block's place in the stream; ids: stage_ids of its stage; first: its first row there)
    auto process = [&](const Operand<DT>& a, int64_t kb, int ids, int first) __attribute__((always_inline)) {
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
            if constexpr (BUF) {
                float gm[4];
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    gm[g] = fmaxf(fmaxf(cs[4 * g], cs[4 * g + 1]), fmaxf(cs[4 * g + 2], cs[4 * g + 3]));
                const float mx = fmaxf(fmaxf(gm[0], gm[1]), fmaxf(gm[2], gm[3]));
                if (__ballot(mx >= tau[sidx]) == 0ull) continue;
                u64* set_lists = my_lists + (size_t)sidx * 32 * lstride;
                u64* mine = set_lists + (size_t)col * KN_CAP + knn + half * pend;    // KN_SEL_LDS
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    if (__ballot(gm[g] >= tau[sidx]) == 0ull) continue;
                    // a lane needs room for the keys of this group that reach its threshold: fold the
                    // queries short of it (the count can only fall when a fold raises the threshold)
                    int n4 = 0;
#pragma unroll
                    for (int r = 4 * g; r < 4 * g + 4; ++r) n4 += cs[r] >= tau[sidx] ? 1 : 0;
                    u64 need = __ballot(fill[sidx] + n4 > pend);
                    while (need) {
                        const int jq = (__ffsll((long long)need) - 1) & 31;
                        float nt;
                        if constexpr (REGP)
                            nt = knn_fold_reg(set_lists + (size_t)jq * KN_REG_KNN, knn, lane, jq, pr[sidx], fill[sidx]);
                        else
                            nt = knn_fold(set_lists + (size_t)jq * KN_CAP, knn, lane);
                        if (col == jq) { tau[sidx] = nt; fill[sidx] = 0; }
                        need &= need - 1;
                        need &= ~(1ull << (jq + 32)) & ~(1ull << jq);
                    }
#pragma unroll
                    for (int r = 4 * g; r < 4 * g + 4; ++r) {
                        if (cs[r] >= tau[sidx] && cs[r] > -INFINITY) {
                            // the row's id sits in lane `row` of ids (lower half-wave) or four lanes
                            // on (upper): both are read as scalars, then chosen without a branch
                            const int row = first + (r / 4) * 8 + (r % 4);
                            const int lo = __builtin_amdgcn_readlane(ids, row);
                            const int hi = __builtin_amdgcn_readlane(ids, row + 4);
                            const u64 nk = knn_key(cs[r], lo ^ ((lo ^ hi) & -half));
                            if constexpr (REGP) {
#pragma unroll
                                for (int k = 0; k < KN_REG_PEND; ++k)
                                    pr[sidx][k] = fill[sidx] == k ? nk : pr[sidx][k];
                                fill[sidx]++;
                            } else if (fill[sidx] < pend) {      // always, for scores that are numbers
                                mine[fill[sidx]++] = nk;
                            }
                        }
                    }
                }
            } else {
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
                    const int id =
                        __builtin_amdgcn_readlane(ids, first + (r / 4) * 8 + (src >> 5) * 4 + (r % 4));
                    const int jq = src & 31;
                    const float nt = knn_insert(set_lists + (size_t)jq * knn, knn, sc, id, lane);
                    if (col == jq) tau[sidx] = nt;
                    mask &= mask - 1;
                    mask &= __ballot(cs[r] >= tau[sidx] && cs[r] > -INFINITY);
                }
            }
            }
        }
    };
    // one stage of keys against the wave's queries
    OperandAt<DT> a_at;                            // where this lane's key operand sits in a stage buffer
    operand_offsets<DT>((int)(stage_buf - lds_raw), col, half, a_at);
    auto multiply_stage = [&](int cur, int64_t st, int ids) __attribute__((always_inline)) {      // cur: byte offset of the stage buffer
        Operand<DT> a0;
        read_operand<DT>(lds_raw, a_at, cur, a0);
        if constexpr (SBLK == 2) {
            Operand<DT> a1;
            read_operand<DT>(lds_raw, a_at, cur + 32 * ROWB, a1);
            process(a0, st * 2, ids, 0);
            process(a1, st * 2 + 1, ids, 32);   // a block at or beyond N is all masked
        } else {
            process(a0, st, ids, 0);
        }
    };
    // Every thread runs every stage (the barrier needs all of them). Key rows are requested two
    // stages before they are multiplied: a stage sits in registers for one stage time, then in
    // its LDS buffer for the next; the key ids of the rows to request are read two requests
    // ahead, the ids a wavefront needs for the keys it keeps two stages ahead. Loads are never
    // branched around (a conditional load makes every later wait conservative); past the end the
    // last stage is fetched again and dropped. The lead-in ends with a use of everything it
    // loaded (an empty asm statement that only reads the registers), so all its loads are complete
    // there: the compiler orders the lead-in's loads as it likes, and any of them still in flight
    // at the loop's entry would make the loop's waits count for that order.
    Held ha, hb;
    Rows ra, rb;
    int ida, idb;
    {
        Rows r1, r2;
        load_rows(ra, 0);
        load_rows(r1, 1);
        load_rows(r2, 2);
        fetch_stage(ha, ra);
        store_stage(ha, stage_buf);
        ida = stage_ids(0);
        fetch_stage(ha, r1);
        load_rows(ra, 3);
        idb = stage_ids(1);
        fetch_stage(hb, r2);
        load_rows(rb, 4);
        if constexpr (CPT == 4)
            asm volatile("; lead-in loads complete" ::"v"(ha.c0), "v"(ha.c1), "v"(ha.c2), "v"(ha.c3),
                         "v"(hb.c0), "v"(hb.c1), "v"(hb.c2), "v"(hb.c3), "v"(ra.r0), "v"(ra.r1), "v"(ra.r2),
                         "v"(ra.r3), "v"(rb.r0), "v"(rb.r1), "v"(rb.r2), "v"(rb.r3), "v"(ida), "v"(idb));
        else
            asm volatile("; lead-in loads complete" ::"v"(ha.c0), "v"(ha.c1), "v"(hb.c0), "v"(hb.c1),
                         "v"(ra.r0), "v"(ra.r1), "v"(rb.r0), "v"(rb.r1), "v"(ida), "v"(idb));
    }
    __syncthreads();
    for (int64_t st = 0; st < nstage; st += 2) {
        multiply_stage(0, st, ida);
        store_stage(ha, stage_buf + STAGE);             // stage st + 1
        __syncthreads();
        ida = stage_ids(st + 2);
        fetch_stage(ha, ra);                            // stage st + 3
        load_rows(ra, st + 5);
        if (st + 1 >= nstage) break;
        multiply_stage(STAGE, st + 1, idb);
        store_stage(hb, stage_buf);                     // stage st + 2
        __syncthreads();
        idb = stage_ids(st + 3);
        fetch_stage(hb, rb);                            // stage st + 4
        load_rows(rb, st + 6);
    }
    // write the ids, best first
#pragma unroll
    for (int sidx = 0; sidx < NQ; ++sidx) {
        for (int j = 0; j < 32; ++j) {
            const int jq = sidx * 32 + j;
            const int64_t qr = q0 + jq;
            if (qr >= M) break;
            u64* lst = my_lists + (size_t)jq * lstride;
            if constexpr (REGP)
                knn_fold_reg(lst, knn, lane, j, pr[sidx], fill[sidx]);
            else if constexpr (BUF)
                knn_fold(lst, knn, lane);
            if (lane < knn) L_out[((size_t)graph * M + qr) * knn + lane] = knn_key_id(lst[lane]);
        }
    }
}

template <int DT, int NQ, int WAVES, int SEL, int STAGE>
static ra_status knn_launch_as(const void* K, const void* Q, const void* order, int n_seq, int n_q, int n_kv,
                               int64_t N, int64_t M, int knn, hipStream_t st, int32_t* L) {
    constexpr int QPB = 32 * NQ * WAVES;
    const int slots = SEL == KN_SEL_REG ? KN_REG_KNN : SEL == KN_SEL_LDS ? KN_CAP : knn;
    const size_t lds = (size_t)QPB * slots * sizeof(u64) + 2 * STAGE;
    if (lds > RA_LDS_LIMIT)
        RA_FAIL(RA_EUNSUP, "knn %d needs %zu bytes of LDS (limit %d)", knn, lds, RA_LDS_LIMIT);
    RA_LDS_OPT_IN((knn_kernel<DT, NQ, WAVES, SEL, STAGE>), lds);
    const dim3 grid((unsigned)((M + QPB - 1) / QPB), (unsigned)(n_seq * n_q));
    hipLaunchKernelGGL((knn_kernel<DT, NQ, WAVES, SEL, STAGE>), grid, dim3(WAVES * RA_WAVE), lds, st, K, Q,
                       reinterpret_cast<const u64*>(order), ra_knn_order_stride(N), n_q, n_kv, N, M, knn, L);
    RA_HIP(hipGetLastError());
    return RA_OK;
}

// RA_TEST_KNN_SELECTION (ra_test_configure): which top-knn selection bf16 lists of up to 32 keys use
static int g_knn_selection_override = RA_TEST_KNN_AUTO;
void ra_knn_set_selection_override(int v) { g_knn_selection_override = v; }

// bf16: 8 wavefronts per workgroup (one workgroup per compute unit, two wavefronts per SIMD). Lists of
// up to 32 keys: two sets of 32 queries per wavefront, 512 queries x 32 slots x 8 bytes of lists
// beside the stage buffers, pending keys in registers. Up to 48 keys: one set per wavefront, 256
// queries x 64 slots. fp32 operands take twice the registers: 4 wavefronts, one set each.
ra_status ra_launch_knn(const void* K, const void* Q, ra_dtype dt, int n_seq, int n_q, int n_kv,
                        int64_t N, int64_t M, int knn, void* workspace, hipStream_t st, int32_t* L) {
    // the order the keys are streamed in (knn_order.hip), at the start of the workspace
    ra_status rc = ra_launch_knn_order(K, Q, dt, n_seq, n_q, n_kv, N, M, workspace, st);
    if (rc != RA_OK) return rc;
    const bool buf = knn <= KN_BUFFERED_KNN;
    // Pending keys in registers: a fold takes 8 keys at most instead of 32, so the start of the stream,
    // where nearly every key reaches the thresholds, costs more (about 14 ms instead of 6 ms for
    // 32 heads x 131072 queries), and every later key less (0.80 us instead of 0.95 us): it pays
    // from about 50 K keys on. The test-only setting RA_TEST_KNN_SELECTION overrides the choice (the
    // tests run both on small inputs).
    bool reg = knn <= KN_REG_KNN && N >= KN_REG_MIN_KEYS;
    if (g_knn_selection_override == RA_TEST_KNN_REG) reg = knn <= KN_REG_KNN;
    else if (g_knn_selection_override == RA_TEST_KNN_LDS) reg = false;
    if (dt == RA_BF16) {
        if (reg)
            return knn_launch_as<RA_BF16, 2, 8, KN_SEL_REG, 16384>(K, Q, workspace, n_seq, n_q, n_kv, N, M, knn, st, L);
        if (buf)
            return knn_launch_as<RA_BF16, 1, 8, KN_SEL_LDS, 16384>(K, Q, workspace, n_seq, n_q, n_kv, N, M, knn, st, L);
        return knn_launch_as<RA_BF16, 1, 8, KN_SEL_INSERT, 16384>(K, Q, workspace, n_seq, n_q, n_kv, N, M, knn, st, L);
    }
    if (buf)
        return knn_launch_as<RA_F32, 1, 4, KN_SEL_LDS, 16384>(K, Q, workspace, n_seq, n_q, n_kv, N, M, knn, st, L);
    return knn_launch_as<RA_F32, 1, 4, KN_SEL_INSERT, 16384>(K, Q, workspace, n_seq, n_q, n_kv, N, M, knn, st, L);
}

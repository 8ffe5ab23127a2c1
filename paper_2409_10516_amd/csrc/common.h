// Shared host/device declarations of libra (internal; the public ABI is include/ra.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ra.h"

#define RA_D 128            // head dimension this build supports
#define RA_WAVE 64

// ---- error plumbing (host) ---------------------------------------------------------
void ra_set_error(const char* fmt, ...);

#define RA_FAIL(code, ...)            \
    do {                              \
        ra_set_error(__VA_ARGS__);    \
        return (code);                \
    } while (0)

#define RA_HIP(call)                                                              \
    do {                                                                          \
        hipError_t e_ = (call);                                                   \
        if (e_ != hipSuccess) {                                                   \
            ra_set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(e_),   \
                         __FILE__, __LINE__);                                     \
            return e_ == hipErrorOutOfMemory ? RA_ENOMEM : RA_EHIP;               \
        }                                                                         \
    } while (0)

// ---- LDS above 64 KB ------------------------------------------------------------------
#ifndef RA_LDS_LIMIT
#define RA_LDS_LIMIT (160 * 1024)     // LDS a workgroup can have on this part (above 64 KB: opt-in)
#endif
#define RA_MAX_DEVICES 64
// A kernel that wants more than 64 KB of dynamic LDS has to say so once per device (host side).
#define RA_LDS_OPT_IN(KERNEL, BYTES)                                                               \
    do {                                                                                           \
        static size_t granted_[RA_MAX_DEVICES];                                                    \
        int dev_ = 0;                                                                              \
        RA_HIP(hipGetDevice(&dev_));                                                               \
        if (dev_ < 0 || dev_ >= RA_MAX_DEVICES) RA_FAIL(RA_EUNSUP, "device %d out of range", dev_); \
        if ((size_t)(BYTES) > 64 * 1024 && granted_[dev_] < (size_t)(BYTES)) {                      \
            RA_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&KERNEL),                     \
                                       hipFuncAttributeMaxDynamicSharedMemorySize, RA_LDS_LIMIT)); \
            granted_[dev_] = RA_LDS_LIMIT;                                                         \
        }                                                                                          \
    } while (0)

// ---- handle --------------------------------------------------------------------------
struct ra_index {
    int n_seq, n_q, n_kv, deg;
    int64_t N;
    int device;
    int32_t* adj;       // [n_seq*n_q][N][deg]
    int32_t* entry;     // [n_seq*n_q]
    // decode workspace, grown on demand (never shrinks)
    float* partials;    // attention partial records
    size_t partials_bytes;
    int32_t* ids_ws;    // [n_seq*n_q][topk] when the caller passes ids == NULL
    size_t ids_bytes;
    uint32_t* bitset;   // global visited bitsets for contexts too long for LDS
    size_t bitset_bytes;
    // hand-over area of the fused decode kernel: per head a record (RA_COOP_REC floats: max, sum,
    // 2 unused, 128 weighted sums) that a helper workgroup fills with the attention over the
    // static set, then per head a ready word, then one "helpers off" word
    float* coop;
    int coop_mode;      // RA_HELPERS_*
    int coop_spin;      // polls of the ready word before a head gives up on its helper
    int coop_silent;    // test-only (RA_TEST_HELPERS_SILENT): helpers are launched but write nothing
    // seed sets (RA_CFG_SEEDS): [n_seq*n_q][seed_cap] in the layout of the root sets, or null
    int32_t* seeds;
    int n_seeds, seed_cap;
    // seed hand-over area of the fused decode kernel (allocated with the seed sets): one "shares
    // off" word, then from byte RA_SEEDX_KEYS_OFF seed_cap 64-bit keys per head, zero between launches
    uint32_t* seedx;
    size_t seedx_bytes;
    int seed_parts;     // shares a head's start set is scored in by workgroups of their own (0: by the head)
    // root sets: what the first two steps of every walk of a head visit ([n_seq*n_q][root_cap])
    int32_t* roots;
    int root_cap;
    size_t graph_bytes;
};

#define RA_COOP_REC 132
#define RA_SEED_PARTS_MAX 8    /* most shares a head's start set is scored in */
#ifndef RA_SEED_PARTS_DEFAULT
#define RA_SEED_PARTS_DEFAULT 6
#endif
#define RA_SEEDX_KEYS_OFF 256  /* bytes in front of the keys of the seed hand-over area */
#define RA_FLAT_SLICES 8       /* workgroups per head in the second pass of ra_flat_topk (one counter each) */
#define RA_HELPERS_SILENT_ 2   /* launch-time helper mode behind RA_TEST_HELPERS_SILENT */
#define RA_KEYS_I8 2          /* key type of a search over 8-bit keys (beside RA_F32, RA_BF16) */

// ---- launchers implemented in the .hip files (all enqueue on `st`, no sync) ----------
ra_status ra_launch_search(const void* q, const int32_t* adj, const int32_t* entry, const void* K,
                           ra_dtype dt, int n_seq, int n_q, int n_kv, int64_t N, int deg,
                           int sink, int window, int topk, int ef, int expand, uint32_t* bitset,
                           const int32_t* roots, int root_cap, const float* kscale, hipStream_t st,
                           int32_t* ids, ra_stats* stats);
ra_status ra_launch_quantize(const void* K, ra_dtype dt, int n_groups, int64_t N, hipStream_t st,
                             int8_t* K8, float* scale);
ra_status ra_launch_roots(const int32_t* adj, const int32_t* entry, int heads, int64_t N, int deg,
                          int32_t* roots, int cap, hipStream_t st);
// seed sets: per head [0] the number of ids, [1] 0, then the ids (cap >= 2 + n_seeds ints per head)
ra_status ra_launch_seeds(const int32_t* adj, const int32_t* entry, int heads, int64_t N, int deg,
                          int n_seeds, int32_t* seeds, int cap, hipStream_t st);
size_t ra_search_lds_bytes(int64_t N, int deg, int ef, int expand, bool global_bitset);
bool ra_search_needs_global_bitset(int64_t N, int deg, int ef, int expand);

size_t ra_attend_partial_floats(int n_seq, int n_q, int n_kv, int64_t N, int sink, int window,
                                int topk);
ra_status ra_launch_attend(const void* q, const void* K, const void* V, ra_dtype dt, int n_seq,
                           int n_q, int n_kv, int64_t N, int sink, int window, int topk,
                           const int32_t* ids, float* partials, hipStream_t st, float* out,
                           float* lse, float* o_omega, float* lse_omega, float* o_w,
                           float* lse_w);

ra_status ra_launch_attend_noalloc(const void* q, const void* K, const void* V, ra_dtype dt, int n_seq,
                                   int n_q, int n_kv, int64_t N, int sink, int window, int topk,
                                   const int32_t* ids, hipStream_t st, float* out, float* lse,
                                   float* o_omega, float* lse_omega, float* o_w, float* lse_w);

bool ra_decode_needs_global_bitset(int64_t N, int deg, int ef, int expand, int topk);
ra_status ra_launch_decode(const void* q, const int32_t* adj, const int32_t* entry, const void* K,
                           const void* V, ra_dtype dt, int n_seq, int n_q, int n_kv, int64_t Ng, int64_t N,
                           int64_t kv_stride, int deg, int sink, int window, int topk, int ef, int expand,
                           uint32_t* bitset, float* coop, int coop_mode, int coop_spin,
                           const int32_t* roots, int root_cap, const void* K8, const float* kscale,
                           const int32_t* budgets, uint32_t* seedx, int seed_parts, hipStream_t st,
                           float* out, float* lse, int32_t* ids, ra_stats* stats);

ra_status ra_launch_rerank(const void* q, const void* K, ra_dtype dt, int n_seq, int n_q, int n_kv, int64_t N,
                           const int32_t* cand, int n_cand, int topk, hipStream_t st, int32_t* ids);
ra_status ra_launch_read_probe(const void* buf, size_t bytes, hipStream_t st, unsigned long long* out);
ra_status ra_launch_gather_probe(const void* buf, size_t bytes, size_t n_rows, uint32_t seed, hipStream_t st,
                                 unsigned long long* out);
ra_status ra_launch_flat_topk(const void* q, const void* K, ra_dtype dt, int n_seq, int n_q, int n_kv,
                              int64_t N, int sink, int window, int topk, uint32_t* keys_ws,
                              hipStream_t st, int32_t* ids);

// `workspace`: ra_knn_order_bytes(n_seq * n_q, N) bytes of device memory, free again once the
// stream has run the launch
ra_status ra_launch_knn(const void* K, const void* Q, ra_dtype dt, int n_seq, int n_q, int n_kv,
                        int64_t N, int64_t M, int knn, void* workspace, hipStream_t st, int32_t* L);
void ra_knn_set_selection_override(int v);      // RA_TEST_KNN_AUTO / _REG / _LDS
size_t ra_knn_order_bytes(int n_graphs, int64_t N);
int64_t ra_knn_order_stride(int64_t N);
ra_status ra_launch_knn_order(const void* K, const void* Q, ra_dtype dt, int n_seq, int n_q, int n_kv,
                              int64_t N, int64_t M, void* workspace, hipStream_t st);

size_t ra_project_workspace_bytes(int n_graphs, int64_t N, int64_t M, int knn);
ra_status ra_launch_project(const int32_t* L, int n_graphs, int64_t N, int64_t M, int knn, int deg,
                            void* workspace, hipStream_t st, int32_t* adj, int32_t* entry);

// ---- device helpers ------------------------------------------------------------------
#ifdef __HIPCC__
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Monotone map float -> uint32 (larger float -> larger uint). -0 is folded into +0 first
// so that equal floats map to equal integers.
__device__ __forceinline__ uint32_t f32_ordered(float f) {
    f = f + 0.0f;
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float f32_from_ordered(uint32_t o) {
    uint32_t u = (o & 0x80000000u) ? (o & 0x7fffffffu) : ~o;
    return __uint_as_float(u);
}

// The value lane (lane ^ J) holds. Distances below 16 stay inside a row of 16 lanes and use DPP
// moves (quad permutes for 1 and 2, a pair of masked row shifts for 4, a row rotation for 8);
// 16 and 32 use the row and half-wave swap instructions: swapping x with itself leaves one result
// with the even rows (lower half) duplicated and the other with the odd rows (upper half), and
// each lane picks the one that came from its partner.
template <int J>
__device__ __forceinline__ uint32_t lane_xor32(uint32_t x, int lane) {
    if constexpr (J == 1) return (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, 0xB1, 0xF, 0xF, false);
    else if constexpr (J == 2) return (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, 0x4E, 0xF, 0xF, false);
    else if constexpr (J == 4) {
        // lanes 0-3 and 8-11 of a row read four lanes up (row_shl:4), the others four lanes down (row_shr:4)
        const int t = __builtin_amdgcn_update_dpp((int)x, (int)x, 0x104, 0xF, 0x5, false);
        return (uint32_t)__builtin_amdgcn_update_dpp(t, (int)x, 0x114, 0xF, 0xA, false);
    } else if constexpr (J == 8) return (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, 0x128, 0xF, 0xF, false);
    else if constexpr (J == 16) {
        const auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
        return (lane & 16) ? r[0] : r[1];
    } else {
        static_assert(J == 32, "lane distances are powers of two below 64");
        const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
        return (lane & 32) ? r[0] : r[1];
    }
}

#endif

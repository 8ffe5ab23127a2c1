/*
 * libra — RetrievalAttention decode hot path and index build for AMD MI355X (gfx950).
 *
 * C ABI. Every tensor argument is a DEVICE pointer to contiguous row-major memory
 * owned by the caller unless the comment says "host". The library never frees or
 * retains caller tensors; an ra_index owns only its graph and its private workspace.
 * All device work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 * default stream). Decode-path calls return without synchronising. Argument checks
 * run before any HIP call and return a status; nothing aborts or throws across the ABI.
 *
 * Notation (paper, arXiv 2409.10516): N keys per KV head, M prefill queries per query
 * head, d head dimension, W the static token set of Sec. 3.3 (first `sink` and last
 * `window` tokens), Omega the retrieved set, topk = |Omega| requested, ef the search
 * beam width, deg the graph degree bound, knn the length of the exact KNN lists.
 *
 * Shapes: K, V        [n_seq][n_kv_heads][N][d]
 *         Q_prefill   [n_seq][n_q_heads][M][d]
 *         q           [n_seq][n_q_heads][d]
 *         out         [n_seq][n_q_heads][d]   float32
 *         lse         [n_seq][n_q_heads]      float32 (natural log, logits scaled by 1/sqrt(d))
 *         ids         [n_seq][n_q_heads][topk] int32, best first, padded with -1
 * Query head h reads KV head h / (n_q_heads / n_kv_heads): one index per query head,
 * one KV copy per group (Appendix C, "Implementation").
 * Supported: d = 128; dtype float32 or bfloat16 (q, K, V, Q_prefill share the dtype); any number
 * of query heads per KV head (groups of 1, 2, 4 and 8 share each key row among the group's heads
 * in the attention and scan kernels; other group sizes read it once per query head).
 */
#ifndef RA_H
#define RA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ra_index ra_index;   /* opaque; create with ra_build_index / ra_index_import */

typedef enum {
    RA_OK = 0,
    RA_EINVAL = 1,   /* null pointer, non-positive size, ef < topk, knn > N, ...          */
    RA_ESHAPE = 2,   /* sizes inconsistent with each other or with the index             */
    RA_EDTYPE = 3,   /* unknown dtype                                                    */
    RA_ENOMEM = 4,   /* device allocation failed                                         */
    RA_EHIP = 5,     /* a HIP call failed; see ra_last_error()                           */
    RA_EUNSUP = 6    /* valid but not supported by this build (d != 128, deg > 64, ...)  */
} ra_status;

typedef enum { RA_F32 = 0, RA_BF16 = 1 } ra_dtype;

/* Per (sequence, query head) search counters, written by the device. */
typedef struct {
    int32_t n_visited;    /* keys scored (entry included)                                */
    int32_t n_expanded;   /* adjacency rows read                                         */
    int32_t n_iters;      /* dependent search steps                                      */
    int32_t n_returned;   /* valid ids written (<= topk)                                 */
} ra_stats;

/* Limits of this build (checked, RA_EUNSUP beyond them). */
#define RA_MAX_DEG 64
#define RA_MAX_KNN 64
#define RA_MAX_EF 2048
#define RA_MAX_EXPAND 256
#define RA_MAX_SEEDS 2048
#define RA_MAX_TOPK 2048

/* ---- index build (Sec. 3.2) -------------------------------------------------------- */

/* Exact KNN of Sec. 3.2 / Fig. 2b: for every prefill query the ids of its `knn` keys of
 * largest inner product over ALL N keys of its KV head (non-causal, unscaled), ordered
 * best first; ties go to the lower id.  L_out: device int32 [n_seq][n_q_heads][M][knn].
 * Allocates scratch memory (8 bytes per key and query head, rounded up to a power of two of
 * keys) and synchronises `stream` before returning to free it. */
ra_status ra_knn(const void* K, const void* Q_prefill, ra_dtype dt,
                 int n_seq, int n_q_heads, int n_kv_heads, int64_t N, int64_t M, int d,
                 int knn, void* stream, int32_t* L_out);

/* Projection of Sec. 3.2 (keys that share query vectors are linked; queries are dropped).
 * L: device int32 [n_graphs][M][knn] with distinct ids per row. Writes, per graph, the
 * adjacency adj [n_graphs][N][deg] (padded with -1) and the entry point entry [n_graphs]
 * (both device). Integer arithmetic only: identical lists give identical graphs.
 * Reading: candidates of key a are the keys sharing a list with it, ranked by the Jaccard
 * overlap of their list memberships (ties: larger co-occurrence count, then lower id); two
 * slots per row hold the children of a in a binary heap laid over the keys sorted by
 * (membership count descending, id ascending), whose root is the entry point. */
ra_status ra_project(const int32_t* L, int n_graphs, int64_t N, int64_t M, int knn, int deg,
                     void* stream, int32_t* adj, int32_t* entry);

/* ra_knn followed by ra_project for every (sequence, query head); returns a handle that
 * owns the graphs. Synchronises `stream` before returning. */
ra_status ra_build_index(const void* K, const void* Q_prefill, ra_dtype dt,
                         int n_seq, int n_q_heads, int n_kv_heads, int64_t N, int64_t M, int d,
                         int deg, int knn, void* stream, ra_index** out);

/* ---- decode step (Algorithm 1 with the fixed static pattern of Sec. 3.3) ----------- */

/* VectorSearch(q): bounded best-first walk over each head's graph from its entry point.
 * Each step expands the `expand` best unexpanded beam entries (1 = textbook greedy),
 * scores their unvisited neighbours and keeps the best `ef`. Scores are float32 inner
 * products summed in a fixed order; order is (score descending, id ascending). ids
 * receives the best `topk` beam entries outside W. stats may be NULL.
 * Requires 1 <= topk <= ef <= RA_MAX_EF, 1 <= expand <= RA_MAX_EXPAND. */
ra_status ra_search(const void* q, const ra_index* idx, const void* K, ra_dtype dt,
                    int64_t N, int sink, int window, int topk, int ef, int expand,
                    void* stream, int32_t* ids, ra_stats* stats);

/* Eq. 2 over Omega = valid entries of ids (each head its own row of ids) and over W,
 * each as (o, lse), and their combination by Eq. 4-5 into out/lse. The four partial
 * outputs (o_omega [n_seq][n_q][d], lse_omega [n_seq][n_q], o_w, lse_w) may each be NULL.
 * ids must not contain members of W (ra_search guarantees it). A head with an empty
 * Omega gets out = o_W; with W empty too, out = 0 and lse = -inf. */
ra_status ra_attend(const void* q, const ra_index* idx, const void* K, const void* V,
                    ra_dtype dt, int64_t N, int sink, int window, int topk,
                    const int32_t* ids, void* stream, float* out, float* lse,
                    float* o_omega, float* lse_omega, float* o_w, float* lse_w);

/* ra_attend for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc. Same arguments, same kernels, same results as
 * ra_attend; the partial records go to a fixed array of RA_ATTEND_NOALLOC_SCRATCH_BYTES bytes that
 * the library holds on every device it runs on until the process ends, instead of memory the
 * handle allocates on first use. No allocation and no free, ever (the first call on a device looks
 * the array's address up, once). RA_EUNSUP, with the sizes in the message, when the records of the
 * call do not fit: n_seq * n_q_heads * (ceil((sink + window) / 64) + ceil(topk / 64)) * 528 bytes
 * for the decode step's static sets (a few thousand heads of the 128K configuration). All calls on
 * one device share the array: calls that overlap in time on one device race; calls in stream
 * order do not, and nothing has to be cleared between them. */
#define RA_ATTEND_NOALLOC_SCRATCH_BYTES (8u << 20)
ra_status ra_attend_noalloc(const void* q, const ra_index* idx, const void* K, const void* V,
                            ra_dtype dt, int64_t N, int sink, int window, int topk,
                            const int32_t* ids, void* stream, float* out, float* lse,
                            float* o_omega, float* lse_omega, float* o_w, float* lse_w);

/* One layer's decode-step attention for all sequences and query heads: the results of
 * ra_search followed by ra_attend, computed by a single fused launch (search, Eq. 2 over
 * Omega and W, Eq. 4-5). ids and stats may be NULL (ids then live in the index workspace).
 * Calls on one handle share its workspace: calls that overlap in time on one handle race. */
ra_status ra_decode_step(const void* q, const ra_index* idx, const void* K, const void* V,
                         ra_dtype dt, int64_t N, int sink, int window, int topk, int ef,
                         int expand, void* stream, float* out, float* lse, int32_t* ids,
                         ra_stats* stats);

/* The decode step after generation has appended tokens to the KV cache: the index still covers
 * the first N_index keys (the N it was built with), the cache now holds N >= N_index tokens per
 * (sequence, KV head), and consecutive heads start every kv_stride >= N rows
 * (K, V: [n_seq][n_kv_heads][kv_stride][d], rows [0, N) valid). The paper does not say how new
 * tokens enter the index; here they join the static set until the index is rebuilt:
 * W = [0, sink) u [min(N - window, N_index), N), Omega comes from the graph over [0, N_index).
 * With N = N_index and kv_stride = N this is ra_decode_step. */
ra_status ra_decode_step_grown(const void* q, const ra_index* idx, const void* K, const void* V,
                               ra_dtype dt, int64_t N, int64_t kv_stride, int sink, int window,
                               int topk, int ef, int expand, void* stream, float* out, float* lse,
                               int32_t* ids, ra_stats* stats);

/* ra_decode_step with a retrieval budget per (sequence, query head) instead of one for all: the
 * paper's appendix on dynamic retrieval budget allocation varies the number of retrieved tokens
 * over the layers (a different topk per call does that); this call varies it over the heads of
 * one layer as well. topk_per_head: device int32 [n_seq][n_q_heads]; head h keeps the best
 * min(max(topk_per_head[h], 1), topk) ids of its beam outside W and attends to those. The walk
 * itself (ef, expand) is the same for every head. A row of ids still has topk cells (the rest
 * are -1) and stats.n_returned counts the ids kept. RA_EUNSUP where the visited bitsets do not
 * fit LDS (a context too long for this ef and expand). */
ra_status ra_decode_step_budgets(const void* q, const ra_index* idx, const void* K, const void* V,
                                 ra_dtype dt, int64_t N, int sink, int window, int topk,
                                 const int32_t* topk_per_head, int ef, int expand, void* stream,
                                 float* out, float* lse, int32_t* ids, ra_stats* stats);

/* ---- exact baselines on the same harness ------------------------------------------- */

/* The paper's "Flat" retrieval (exact KNN by linear scan, Sec. 4.1 and Table 5): the topk keys of
 * largest inner product outside W for every (sequence, query head), best first, ties to the lower
 * id, padded with -1. Scores are the same fixed-order float32 inner products ra_search uses, so
 * the two rank keys identically and recall of the graph search can be measured on the device.
 * The scan stores no per-key scores when the context is long enough for it (at least 64 x topk keys,
 * at most 1M): it keeps the largest score of every 32 keys, derives a threshold that at least topk
 * of those maxima reach, and scores the few tiles at or above it a second time.
 * workspace: device memory of at least ra_flat_workspace_bytes(n_seq, n_q_heads, N) bytes. */
size_t ra_flat_workspace_bytes(int n_seq, int n_q_heads, int64_t N);
ra_status ra_flat_topk(const void* q, const void* K, ra_dtype dt, int n_seq, int n_q_heads,
                       int n_kv_heads, int64_t N, int d, int sink, int window, int topk,
                       void* workspace, size_t workspace_bytes, void* stream, int32_t* ids);

/* Eq. 1: softmax attention over all N tokens (what the method approximates), as (out, lse).
 * float32 accumulation throughout; for bf16 inputs and GQA groups of up to four query heads the
 * logits of a long context come from the matrix cores (sums of exact bf16 products in the
 * hardware's order), otherwise from the vector units. Same tolerance either way.
 * workspace: device memory of at least ra_full_attention_workspace_bytes(...) bytes. */
size_t ra_full_attention_workspace_bytes(int n_seq, int n_q_heads, int n_kv_heads, int64_t N);
ra_status ra_full_attention(const void* q, const void* K, const void* V, ra_dtype dt, int n_seq,
                            int n_q_heads, int n_kv_heads, int64_t N, int d, void* workspace,
                            size_t workspace_bytes, void* stream, float* out, float* lse);

/* Measurement aid: reads the `bytes` bytes at `buf` (device, 16-byte aligned, a multiple of 16)
 * once with a plain streaming kernel and xors a 64-bit fold of them into *out (device). Timed by
 * the benchmark, it gives the read bandwidth a streaming kernel sustains on the device, which the
 * scan kernels above (Sec. 4.1's exact baselines) are compared with. */
ra_status ra_hbm_read_probe(const void* buf, size_t bytes, void* stream, uint64_t* out);

/* Measurement aid for the gathers of the walk (Sec. 2.4: a search touches scattered key vectors):
 * reads n_rows rows of 256 bytes (a bf16 key of d = 128) of the `bytes` bytes at `buf` (device,
 * 16-byte aligned, a multiple of 256; at most 2^32 - 1 rows), at row numbers drawn by a counter-based
 * hash of (position in the sequence, seed), each row by 16 lanes as the search kernels read it, 8
 * rows in flight per lane group, and xors a 64-bit fold into *out (device). Timed by the benchmark,
 * it gives the bandwidth the device sustains for scattered rows, the bound of a launch whose bytes
 * are mostly start sets. RA_EINVAL for a NULL or misaligned buffer or n_rows = 0. */
ra_status ra_hbm_gather_probe(const void* buf, size_t bytes, size_t n_rows, uint32_t seed, void* stream,
                              uint64_t* out);

/* ---- handle management ------------------------------------------------------------- */

/* Build a handle from HOST arrays adj [n_seq*n_q_heads][N][deg], entries [n_seq*n_q_heads]
 * (copied to the device). Used for persistence and to run device stages on a given graph. */
ra_status ra_index_import(const int32_t* adj_host, const int32_t* entries_host, int n_seq,
                          int n_q_heads, int n_kv_heads, int64_t N, int deg, ra_index** out);

/* Copy one graph back to HOST arrays adj_host [N][deg] and *entry_host. Synchronises. */
ra_status ra_index_export(const ra_index* idx, int seq, int q_head, int32_t* adj_host,
                          int32_t* entry_host);

/* 8-bit keys for the search. Appendix C names 8-bit scalar quantisation of the KV vectors as the
 * paper's next step and gives no scheme; here the keys get an 8-bit copy that only the graph walk
 * reads (half the bytes per scored key), attention keeps using K and V as they are:
 *     scale[d] = max_i |K[i][d]| / 127 (1 for an all-zero column), per (sequence, KV head),
 *     K8[i][d] = clamp(round_half_even(K[i][d] / scale[d]), -127, 127),
 * float32 arithmetic, each division rounded once. The walk scores <q * scale, K8> in the same
 * fixed summation order as ra_search, so its ids and counters are reproducible bit for bit.
 *
 * ra_quantize_keys: K [n_seq][n_kv_heads][N][128] (dt) -> K8 [n_seq][n_kv_heads][N][128] int8,
 * scale [n_seq][n_kv_heads][128] float32; device pointers, caller-owned; enqueued on `stream`.
 * ra_search_q8 / ra_decode_step_q8: ra_search / ra_decode_step with the walk reading K8 and scale
 * (`dtq` is the type of q); N must equal the number of keys the index was built over. The ids are
 * the best topk of the beam under the 8-bit scores; out / lse are Eq. 2 and Eq. 4-5 over those
 * ids and W with the original K and V. Errors as for ra_search / ra_decode_step. */
ra_status ra_quantize_keys(const void* K, ra_dtype dt, int n_seq, int n_kv_heads, int64_t N, void* stream,
                           int8_t* K8, float* scale);
ra_status ra_search_q8(const void* q, const ra_index* idx, const int8_t* K8, const float* scale,
                       ra_dtype dtq, int64_t N, int sink, int window, int topk, int ef, int expand,
                       void* stream, int32_t* ids, ra_stats* stats);
/* Re-ranking with the keys themselves, for a candidate list that came from the 8-bit walk (call
 * ra_search_q8 with a topk of n_cand, then this, then ra_attend): of the distinct ids in cand
 * [n_seq][n_q_heads][n_cand] (-1 and ids >= N are skipped) the best topk under <q, K[id]>, the
 * fixed-order float32 score of ra_search, score descending then id ascending -> ids
 * [n_seq][n_q_heads][topk], padded with -1. 1 <= topk <= n_cand <= RA_MAX_TOPK. */
ra_status ra_rerank(const void* q, const void* K, ra_dtype dt, int n_seq, int n_q_heads, int n_kv_heads,
                    int64_t N, int d, const int32_t* cand, int n_cand, int topk, void* stream, int32_t* ids);
ra_status ra_decode_step_q8(const void* q, const ra_index* idx, const void* K, const void* V, ra_dtype dt,
                            const int8_t* K8, const float* scale, int64_t N, int sink, int window,
                            int topk, int ef, int expand, void* stream, float* out, float* lse,
                            int32_t* ids, ra_stats* stats);

/* what: 0 n_seq, 1 n_q_heads, 2 n_kv_heads, 3 N, 4 deg, 5 bytes of device memory owned,
 * 6 whether ra_decode_step will use helper workgroups (1 / 0; synchronises the device),
 * 7 the seed-set size in use (RA_CFG_SEEDS; 0: single entry point),
 * 8 whether ra_decode_step may score the seed sets in workgroups of their own (RA_CFG_SEED_SHARES;
 *   1 / 0: off, no seed sets, helpers off, or a head's wait for its keys ran out; synchronises the
 *   device). */
int64_t ra_index_info(const ra_index* idx, int what);

/* Settings of the handle's decode path (host side; synchronises the device).
 *
 * ra_decode_step computes the attention over the static set W (Sec. 3.3: o_W of Eq. 4, which
 * does not depend on the retrieval) in extra "helper" workgroups of the same launch, one per
 * (sequence, KV head) - one per query head where the launch leaves compute units idle - while the
 * query heads' workgroups search; each head takes over its
 * helper's result through device memory the handle owns. The wait for that result is bounded:
 * a head that does not get it within RA_CFG_HELPER_SPIN polls computes o_W itself, and the
 * handle stops using helpers until RA_CFG_HELPERS is set again. Results do not depend on the
 * setting beyond the summation order of Eq. 2/4 (same tolerance).
 *   RA_CFG_HELPERS      RA_HELPERS_ON (default), RA_HELPERS_OFF (each head attends to W itself).
 *                       Setting it also clears a wait that ran out.
 *   RA_CFG_HELPER_SPIN  polls before a head gives up, 1 .. 2^24 (default RA_HELPER_SPIN_DEFAULT,
 *                       tens of milliseconds).
 * Helpers are used only for GQA groups of 1, 2, 4 or 8 query heads per KV head; with any other
 * group size every head attends to W itself.
 * The hand-over is ordered without fences: the words that cross workgroups are relaxed
 * agent-scope atomic accesses (on gfx950 these bypass the per-XCD L2), the helper waits for its
 * record stores to complete (s_waitcnt vmcnt(0), workgroup barrier) before it stores the ready
 * word, and the head reads the record only after it has seen the ready word. That ordering is a
 * property of this part's memory system, not of the HIP memory model; the bounded wait and the
 * fall-back keep a launch correct if a ready word never arrives.
 * Two ra_decode_step calls on one handle must not overlap in time (they share this memory,
 * like the handle's other workspaces). Returns RA_EINVAL for an unknown setting or value.
 *
 *   RA_CFG_SEEDS        0 (default): every walk of the handle starts from its head's entry point.
 *                       n in 1 .. RA_MAX_SEEDS: it starts from a seed set instead - the paper does
 *                       not say where a walk starts (Sec. 2.4) - namely the first n positions,
 *                       breadth first, of the binary tree that slots 0 and 1 of the adjacency rows
 *                       span from the entry point (position p has its children at 2p + 1, 2p + 2;
 *                       positions without a node and repeated nodes are dropped). For a graph from
 *                       ra_project these are the n keys that appear in the most KNN lists of the
 *                       prefill queries. All seeds are scored at once, the best ef of them form the
 *                       beam, none is expanded yet; they count as visited, no step is counted for
 *                       them. n = 1 is the single-entry walk. Applies to ra_search, ra_decode_step
 *                       and their variants, which then need n <= expand x deg (RA_EINVAL
 *                       otherwise). Lists the sets on the device and synchronises it.
 *   RA_CFG_SEED_SHARES  into how many shares ra_decode_step cuts a head's seed set, each scored by a
 *                       workgroup of its own in the same launch while the head's workgroup sets up
 *                       (what bounds the scoring of a start set is the rate at which one compute
 *                       unit takes in scattered key rows): 0 (the head scores its set itself) or
 *                       2 .. 8; default 6. Used only where every workgroup of the launch has a compute
 *                       unit to itself (the searches, their shares and the helpers together number at
 *                       most the device's compute units; fewer shares are used to make that so, none
 *                       below two) and a walk has a workgroup of 512 threads or more; RA_HELPERS_OFF
 *                       switches the shares off as well. The keys are the same
 *                       bits whoever computes them, so ids, counters and outputs do not depend on the
 *                       setting. They cross workgroups through device memory the handle owns, one
 *                       64-bit slot per seed that the head polls and zeroes again, with the same
 *                       relaxed agent-scope accesses, the same bounded wait (RA_CFG_HELPER_SPIN
 *                       polls per slot) and the same fall-back as the helpers' records: a head whose
 *                       keys do not arrive scores its set itself and the handle stops using shares
 *                       until RA_CFG_HELPERS or RA_CFG_SEED_SHARES is set again. */
#define RA_CFG_HELPERS 0
#define RA_CFG_HELPER_SPIN 1
#define RA_CFG_SEEDS 2
#define RA_CFG_SEED_SHARES 3
#define RA_HELPERS_OFF 0
#define RA_HELPERS_ON 1
#define RA_HELPER_SPIN_DEFAULT 20000
ra_status ra_index_configure(ra_index* idx, int what, int64_t value);

/* ---- TEST-ONLY settings -------------------------------------------------------------
 * Not for callers of the library: they exist so that the test-suite can reach code paths that
 * inputs alone cannot select. Results never depend on them beyond what is stated.
 *   RA_TEST_KNN_SELECTION   (idx = NULL; process-wide) which of the two top-knn selections
 *                           ra_knn uses for bf16 lists of up to 32 keys: RA_TEST_KNN_AUTO
 *                           (default: chosen by N), RA_TEST_KNN_REG, RA_TEST_KNN_LDS. Same lists
 *                           either way.
 *   RA_TEST_HELPERS_SILENT  (per handle) 1: the helper and seed workgroups of ra_decode_step are
 *                           launched but write nothing, so every head's bounded wait runs out and
 *                           the fall-back is taken; 0: normal. Synchronises the device and clears
 *                           the hand-over areas like RA_CFG_HELPERS. */
#define RA_TEST_KNN_SELECTION 100
#define RA_TEST_HELPERS_SILENT 101
#define RA_TEST_KNN_AUTO 0
#define RA_TEST_KNN_REG 1
#define RA_TEST_KNN_LDS 2
ra_status ra_test_configure(ra_index* idx, int what, int64_t value);

/* Device pointers to the handle's graphs (adj [n_graphs][N][deg], entry [n_graphs]). */
const int32_t* ra_index_adj(const ra_index* idx);
const int32_t* ra_index_entry(const ra_index* idx);

void ra_index_free(ra_index* idx);

/* Message for the calling thread's most recent non-OK status ("" if none). */
const char* ra_last_error(void);

/* Library version string. */
const char* ra_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RA_H */

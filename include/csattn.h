/*
 * csattn.h - C ABI of the CSAttention online-decode library for AMD MI355X (gfx950).
 *
 * The library implements, as hand-written HIP kernels, the per-token decode step of
 * Centroid-Scoring Attention (arXiv 2604.08584, Sec. 3.3 and App. A "All-GPU"), the offline
 * construction of its lookup tables (Sec. 3.2) and the append of new keys/values (Sec. 3.3 (5),
 * first sentence).  Geometry (Sec. 3.1 (i)): the head dimension is cut uniformly into
 * S = n_subspaces subspaces, each with its own C centroids and C table rows; a query probes the
 * tau = n_probe best centroids of every subspace (Sec. 3.3 (1) for tau = 1, the centroid back-off
 * of Sec. 4.4 for tau > 1), M = S * tau rows in all.  S = 8, tau = 1 is the paper's default;
 * S = 1 is a single subspace spanning the whole head dimension.  Table row r of a KV head belongs
 * to subspace r / C and centroid r % C.
 *
 * Conventions
 *   - Every pointer named *_dev is DEVICE memory owned by the caller; the library never
 *     allocates or frees device memory.  Pointers without that suffix are HOST memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue
 *     work on it and return without synchronising unless stated otherwise.
 *   - All calls return CSA_OK (0) or a negative csa_status; nothing aborts or throws.
 *   - B = batch, Hq = n_q_heads, Hkv = n_kv_heads, G = Hq/Hkv, d = head_dim (128),
 *     S = n_subspaces, C = n_centroids, L = list_len, tau = n_probe, M = S * tau, k = budget_k.
 *     Query head h belongs to KV head h / G.  All sequences of the batch share n_pre and n.
 *   - bf16 = the upper 16 bits of an IEEE fp32.  Inputs must be finite.
 *   - A ctx is not thread-safe; calls on one ctx must be issued from one thread at a time and
 *     on streams that are ordered with respect to each other.
 *   - csa_decode_step, csa_decode_step_static and csa_decode_step_reuse only launch kernels on
 *     `stream` (no allocation, no synchronisation, no memset or copy nodes), so they may be captured
 *     into a HIP graph and replayed while the context length stays as captured; csa_append_kv and
 *     csa_decode_step_append bake the position into their launches and are not replayable -
 *     csa_decode_step_append_replayable is the form of a whole iteration that is.
 */
#ifndef CSATTN_H
#define CSATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct csa_ctx csa_ctx; /* opaque host object */

typedef enum {
    CSA_OK = 0,
    CSA_ERR_ARG = -1,       /* NULL / out-of-range argument or unsupported configuration */
    CSA_ERR_STATE = -2,     /* call out of order (e.g. decode before tables exist) */
    CSA_ERR_CAPACITY = -3,  /* append beyond max_ctx */
    CSA_ERR_WORKSPACE = -4, /* bound buffer smaller than csa_workspace_bytes reports */
    CSA_ERR_HIP = -5,       /* a HIP runtime call failed (see csa_last_hip_error) */
    CSA_ERR_RANGE = -6      /* a table score does not fit the score grid (see score_frac_bits) */
} csa_status;

typedef struct {
    int32_t batch;       /* B  >= 1 */
    int32_t n_q_heads;   /* Hq, multiple of n_kv_heads, G = Hq/Hkv <= 16 */
    int32_t n_kv_heads;  /* Hkv >= 1 */
    int32_t head_dim;    /* d, must be 128 */
    int32_t n_centroids; /* C >= 1: query-centric centroids per KV head and subspace (Sec. 3.2 (1)) */
    int32_t list_len;    /* L in [1, 8192]: Top-L capacity per centroid (Sec. 3.1 (iii)) */
    int32_t n_probe;     /* tau in [1, C], S * tau <= 63: centroids probed per subspace
                            (Sec. 3.3 (1), 4.4) */
    int32_t budget_k;    /* k >= 0: keys kept by Top-K (Sec. 3.3 (4)) */
    int32_t n_subspaces; /* S in {1, 2, 4, 8, 16}: uniform split, 128 / S dimensions each */
    int32_t max_ctx;     /* capacity (rows) of the caller's K/V storage per sequence;
                            multiple of page_size when paged; <= 2^24 */
    int32_t page_size;   /* 0: contiguous K/V [B][Hkv][max_ctx][d];
                            16: paged pools [n_pages][Hkv][16][d] + block table */
    int32_t score_frac_bits; /* F >= 0: table scores live on the grid 2^-F;
                                < 0: csa_build_tables picks the finest safe grid */
    int32_t partition_keys;  /* 0 = automatic; else a power of two in [1024, 16384]: size of
                                the key-index ranges the score accumulation is split into */
    int32_t stream_window;   /* 0: appended keys never enter the tables and are all attended;
                                R > 0: streaming updates (Sec. 3.3 (5)) - csa_append_kv try-inserts
                                each new key into the Top-L lists and only the last R positions
                                (the recent window of Sec. 3.3 (4)) are attended unconditionally */
} csa_config;

/*
 * Score grid (decides which keys are kept, so it is part of the interface): a table score s is
 * stored as the integer q = round-half-even(s * 2^F); the accumulated score of a key
 * (Sec. 3.3 (3), w_b = 1) is the exact integer sum of its q over the probed rows.  The library
 * requires M * max|q| < 2^24, so the same sums are also exact in fp32 in any order, and
 * max|q| < 2^18 (a table entry is kept in 32 bits on the device: 19 bits of q, 13 index bits).
 */

/* Validates `cfg` and creates the host object.  No device work, no device allocation. */
int csa_create(const csa_config *cfg, csa_ctx **out);
void csa_destroy(csa_ctx *ctx);

/*
 * Sizes (bytes) of the two device buffers the caller must provide to csa_bind:
 *   tables  - centroids + lookup tables in the library's private layout (persistent state)
 *   scratch - per-step temporaries (contents need not survive between calls, with one exception:
 *             the index set of the last searching step when it was called with NULL sel pointers,
 *             see csa_decode_step_reuse)
 */
int csa_workspace_bytes(const csa_ctx *ctx, size_t *tables_bytes, size_t *scratch_bytes);

/*
 * Attaches the caller's device buffers.  All must be 256-byte aligned and stay valid until
 * csa_destroy or the next csa_bind.
 *   k_cache_dev, v_cache_dev: bf16.  page_size = 0: [B][Hkv][max_ctx][d].
 *                             page_size = 16: pools [n_pages][Hkv][16][d].
 *   block_table_dev: int32 [B][max_ctx/16], logical page -> pool page (paged only, else NULL).
 * Re-binding keeps the table state only if tables_dev is unchanged.
 */
int csa_bind(csa_ctx *ctx, void *tables_dev, size_t tables_bytes, void *scratch_dev,
             size_t scratch_bytes, void *k_cache_dev, void *v_cache_dev,
             const int32_t *block_table_dev);

/*
 * Offline table construction, Sec. 3.2 (2): for every KV head, subspace b and centroid j,
 * s_j(i) = c_j^(b) . k_i^(b) over the prefill keys i < n_pre (raw key sub-vectors), rounded to the
 * score grid, and the L best (score desc, index asc) kept.  Scores are computed in fp32 as one
 * fused-multiply-add chain over the subspace's dimensions in ascending order starting from +0,
 * bf16 inputs widened.
 *   centroids_dev: bf16 [B][Hkv][S][C][d/S], unit norm (Sec. 3.2 (1); clustering is the caller's).
 * K is read from the bound cache, rows [0, n_pre), 1 <= n_pre <= max_ctx (CSA_ERR_ARG otherwise).
 * Sets the context length to n_pre.  May be called again on the same context (a new sequence in
 * the same buffers): tables, context length, key ranges and an automatic score grid start over.
 * SYNCHRONISES `stream` before returning (it reads back an overflow flag); returns
 * CSA_ERR_RANGE if some |q| * M >= 2^24 or |q| >= 2^18 (tables are then unusable).
 */
int csa_build_tables(csa_ctx *ctx, const void *centroids_dev, int32_t n_pre, void *stream);

/*
 * Query-centric centroids, Sec. 3.2 (1): for every KV head and subspace, cosine k-means over the
 * l2-normalised prefill query sub-vectors of the G query heads of the group ("per KV-head group",
 * Sec. 4.4), k-means++ seeding, `iters` Lloyd steps.  Centroids are unit vectors held in bf16
 * between the steps: each step assigns its points to the centroid of largest inner product (bf16
 * operands on the matrix cores, fp32 accumulation; ties to the lower centroid) and replaces a
 * centroid by the re-normalised sum of its normalised members, rounded to bf16 (a cluster without a
 * member keeps its centroid).
 * csa_cluster_queries: every step runs over all G * n_pre points (full batch).
 * csa_cluster_queries_minibatch: the paper names mini-batch k-means without a batch size; here the
 *   pooled points are dealt into n_batches classes (point i belongs to class i % n_batches), the
 *   seeding runs over class 0, step t over class t % n_batches, and a centroid is the re-normalised
 *   sum of every point assigned to it in any step so far (the per-centre running mean of mini-batch
 *   k-means; the starting centroid carries no weight).  n_batches = 1 is the full batch.
 * All problems of a sequence run side by side.  The member sums are fp32: with few short centroids
 * (C * (d/S + 1) <= 8192) they are added with atomics in an order that is not fixed; otherwise each
 * centroid's members are listed (in an order that depends on an atomic cursor) and summed by one
 * wave - either way the last bit of a centroid may differ between runs.
 *   q_pre_dev          bf16 [B][Hq][n_pre][d]: the prefill queries.
 *   u_seed_dev         fp32 [B][Hkv][S][C], uniforms in [0, 1) that drive the seeding: point
 *                      floor(u_0 * n) first, then each next seed is the first point whose running
 *                      sum of squared distances to the nearest seed so far exceeds u_j * total
 *                      (n and the points: those of class 0).  NULL if init_centroids_dev is given.
 *   init_centroids_dev bf16 [B][Hkv][S][C][d/S] starting centroids instead of the seeding, or NULL.
 *   centroids_out_dev  bf16 [B][Hkv][S][C][d/S]: the input csa_build_tables expects.
 *   mean_cos_dev       fp32 [B][Hkv][S][max(iters,1)]: mean cosine of a step's points to their
 *                      assigned centroid (full batch: non-decreasing up to rounding); or NULL.
 *   assign_dev         int32 [B][Hkv][S][G*n_pre]: assignments of the last step (mini-batches: -1
 *                      for the points outside the last step's class); or NULL.
 *   work_dev           scratch of csa_cluster_workspace_bytes bytes, 256-byte aligned.
 * Needs no bound buffers and no tables.  Enqueues on `stream`; does not synchronise.
 */
int csa_cluster_workspace_bytes(const csa_ctx *ctx, int32_t n_pre, size_t *bytes);
int csa_cluster_queries(csa_ctx *ctx, const void *q_pre_dev, int32_t n_pre, int32_t iters,
                        const float *u_seed_dev, const void *init_centroids_dev, void *centroids_out_dev,
                        float *mean_cos_dev, int32_t *assign_dev, void *work_dev, size_t work_bytes,
                        void *stream);
int csa_cluster_queries_minibatch(csa_ctx *ctx, const void *q_pre_dev, int32_t n_pre, int32_t iters,
                                  int32_t n_batches, const float *u_seed_dev, const void *init_centroids_dev,
                                  void *centroids_out_dev, float *mean_cos_dev, int32_t *assign_dev,
                                  void *work_dev, size_t work_bytes, void *stream);

/*
 * The whole offline prefill of Sec. 3.2 in one call, from the prefill queries and the keys in the
 * bound cache: (1) csa_cluster_queries_minibatch(q_pre_dev, n_pre, iters, n_batches, u_seed_dev) into
 * centroids_out_dev, then (2) csa_build_tables(centroids_out_dev, n_pre), on one stream.  Arguments
 * as in those two calls (centroids_out_dev, bf16 [B][Hkv][S][C][d/S], also serves the caller: it is
 * what csa_import_tables or an oracle of the build would take).  SYNCHRONISES `stream` (the table
 * build does); errors of either part are returned.
 */
int csa_prefill(csa_ctx *ctx, const void *q_pre_dev, int32_t n_pre, int32_t iters, int32_t n_batches,
                const float *u_seed_dev, void *centroids_out_dev, void *work_dev, size_t work_bytes, void *stream);

/*
 * Tables in the canonical layout, one KV head at a time or all at once:
 *   idx   int32 [S*C][L], score fp32 [S*C][L]; each row sorted by (score desc, idx asc)
 *   (Sec. 3.1 (iii) "sorted by score"); unused tail slots idx = -1, score = 0.
 * csa_export_tables writes the rows of KV head (b, g) to device buffers.
 * csa_import_tables reads centroids bf16 [B][Hkv][S][C][d/S] and canonical tables
 *   idx [B][Hkv][S*C][L], score [B][Hkv][S*C][L] (device), and makes them the ctx's tables; it
 *   needs score_frac_bits >= 0, SYNCHRONISES `stream`, and returns CSA_ERR_RANGE if a score is
 *   off the grid or too large, CSA_ERR_ARG if an index is outside [-1, n_pre).
 */
int csa_export_tables(const csa_ctx *ctx, int32_t b, int32_t g, int32_t *idx_dev,
                      float *score_dev, void *stream);
int csa_import_tables(csa_ctx *ctx, const void *centroids_dev, const int32_t *idx_dev,
                      const float *score_dev, int32_t n_pre, void *stream);

/*
 * Sec. 3.3 (5): append one key/value row per KV head at position n, n <- n+1.
 *   k_new_dev, v_new_dev: bf16 [B][Hkv][d].
 * stream_window = 0: appended keys are not inserted into the tables; every key in [n_pre, n) is
 * attended exactly by csa_decode_step (the "recent window" of Sec. 3.3 (4), covering all
 * decode-time keys).
 * stream_window = R > 0: the new key is also scored against every centroid of every subspace
 * (same fma chain and grid as the table build) and try-inserted into that centroid's
 * fixed-capacity list: a list with a free slot takes it, a full list takes it only if its score
 * beats the list's minimum (an equal score does not), which is evicted.  csa_decode_step then
 * attends the selected keys plus the last R positions [max(0, n - R), n); keys in that window
 * are not candidates of the Top-K.  A score outside the grid range is clamped (see
 * csa_streaming_status).
 * CSA_ERR_CAPACITY if n == max_ctx.
 */
int csa_append_kv(csa_ctx *ctx, const void *k_new_dev, const void *v_new_dev, void *stream);

/*
 * One decode step for every (sequence, query head), Sec. 3.3 (1)-(4) + App. A:
 *   1. in every subspace b, z_j = q^(b) . c_j^(b) (fp32 fma chain as above); the tau largest, ties
 *      to the lower j;
 *   2. the M = S * tau table rows are read;
 *   3. scores are summed per key index; U = keys present in at least one probed row;
 *   4. the min(k, |U|) keys of U with the largest sum, ties to the lower index;
 *   5. out = softmax(q K_A^T / sqrt(d)) V_A over A = selected keys + all keys in [n_pre, n)
 *      (Sec. 2.1), bf16 inputs, fp32 accumulation.  A empty -> out = 0.
 *   q_dev   bf16 [B][Hq][d]            out_dev fp32 [B][Hq][d]
 *   sel_idx_dev   int32 [B][Hq][k]  ascending, padded with -1   (may be NULL)
 *   sel_count_dev int32 [B][Hq]     = min(k, |U|)               (may be NULL)
 */
int csa_decode_step(csa_ctx *ctx, const void *q_dev, float *out_dev, int32_t *sel_idx_dev,
                    int32_t *sel_count_dev, void *stream);

/*
 * csa_decode_step for callers that cannot allocate or bring a workspace to the call - code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc: the same kernels, same
 * arguments and same results as csa_decode_step, but every per-step temporary (centroid scores,
 * probed rows, candidate words, bin offsets, Top-K records, split partials; and the index set
 * when sel_idx_dev / sel_count_dev are NULL) lives in a fixed array inside the library's own
 * device image instead of the scratch buffer given to csa_bind.  The call allocates nothing and
 * frees nothing (no hipMalloc, no hipFree, no library routine that allocates); it only launches
 * kernels on `stream`.
 *   Limit: the step's temporaries (csa_static_scratch_bytes reports them) must fit the array's
 *   32 MiB - e.g. batch 1, 32 query heads at a 128K context; CSA_ERR_WORKSPACE and nothing
 *   enqueued otherwise.  Tables and the K/V cache still come from csa_bind; inputs and outputs
 *   are the caller's as in csa_decode_step.
 *   Every GPU the library runs on holds its own copy of the array until the process ends.  All
 *   calls on one GPU, from any context, share it: nothing in it needs to start at zero and nothing
 *   is read from an earlier call, but two such calls that overlap in time on one GPU (different
 *   streams) race.  With both sel pointers NULL the index set stays in the array, so the next
 *   csa_decode_step_static of ANY context overwrites what csa_decode_step_reuse(NULL, NULL) would
 *   read.
 */
int csa_decode_step_static(csa_ctx *ctx, const void *q_dev, float *out_dev, int32_t *sel_idx_dev,
                           int32_t *sel_count_dev, void *stream);
/* Bytes of temporaries a step of this context needs, and the capacity of the static array. */
int csa_static_scratch_bytes(const csa_ctx *ctx, size_t *needed, size_t *capacity);

/*
 * A decode step inside a search period (App. "Schedules evaluation" and the complexity appendix:
 * with search period P the index set of the last searching step is reused for the next P-1
 * steps, e.g. the schedules 0.15-step-4 and 0.20-step-8): no centroid scoring, no table access,
 * no Top-K - step 5 of csa_decode_step over the given index set plus all keys in [n_pre, n),
 * with the current query.
 *   sel_idx_dev   int32 [B][Hq][k]  ascending, distinct, each < n_pre, padded with -1 (input)
 *   sel_count_dev int32 [B][Hq]     entries used per head, <= k                        (input)
 * Both NULL: the index set written by the last csa_decode_step on this ctx (whether into the
 * caller's buffers or into the scratch buffer, which must then be untouched since);
 * CSA_ERR_STATE if there was none since the tables were built.  An unsorted list is not
 * detected: keys may then be attended twice or not at all (never an invalid address).
 */
int csa_decode_step_reuse(csa_ctx *ctx, const void *q_dev, float *out_dev,
                          const int32_t *sel_idx_dev, const int32_t *sel_count_dev, void *stream);

/*
 * A whole decode iteration in one call: the step on the current context - csa_decode_step
 * (reuse = 0) or csa_decode_step_reuse (reuse != 0; sel_idx_dev / sel_count_dev are then inputs
 * or both NULL) - followed by csa_append_kv(k_new_dev, v_new_dev), Sec. 3.3 (1)-(5).  Same
 * results, same argument meaning and same errors as the two calls in that order; the append rides
 * in the step's last launch, which saves one kernel launch per iteration.  CSA_ERR_CAPACITY (and
 * nothing enqueued) when the context is full.
 */
int csa_decode_step_append(csa_ctx *ctx, const void *q_dev, const void *k_new_dev, const void *v_new_dev,
                           float *out_dev, int32_t *sel_idx_dev, int32_t *sel_count_dev, int32_t reuse,
                           void *stream);

/*
 * csa_decode_step_append in a form that a HIP graph can replay, one decode iteration (Sec. 3.3
 * (1)-(5)) per replay: no launch argument depends on the context length.  The library keeps a copy
 * of the context length in a word of the tables buffer (every appending call advances it); these
 * launches read the position there, attend the window [n_pre, n) it implies, write row n and
 * advance the word themselves, and their grids are sized for a full context (max_ctx - n_pre window
 * keys), so the same launches are right for every later position.  Same arguments and results as
 * csa_decode_step_append; q_dev, k_new_dev, v_new_dev, out_dev and the sel buffers are read and
 * written in place by every replay (refill the inputs between replays).  Only kernels are enqueued:
 * no allocation, no synchronisation, no memset or copy nodes.  Not available with streaming updates
 * (stream_window > 0: CSA_ERR_ARG).
 * The host-side count (csa_context_len, the capacity checks of the other calls) follows the CALLS
 * made on the context, not the replays of a graph: call csa_sync_context_len after capturing and
 * after replaying, before any other call that depends on the position.  A replay on a full context
 * appends nothing, leaves the count alone and is reported by csa_sync_context_len.
 */
int csa_decode_step_append_replayable(csa_ctx *ctx, const void *q_dev, const void *k_new_dev,
                                      const void *v_new_dev, float *out_dev, int32_t *sel_idx_dev,
                                      int32_t *sel_count_dev, int32_t reuse, void *stream);
/* SYNCHRONISES `stream`, sets the host-side context length to the device's count and returns
 * CSA_ERR_CAPACITY if a replayed append found the context full since the tables were built or the
 * length was last set, else CSA_OK. */
int csa_sync_context_len(csa_ctx *ctx, void *stream);

/* Streaming updates only: SYNCHRONISES `stream` and returns CSA_ERR_RANGE if a streamed key's
 * score did not fit the score grid since the tables were built (it was clamped), else CSA_OK. */
int csa_streaming_status(csa_ctx *ctx, void *stream);

/* Host-side counters: prefill length and current context length. */
int csa_context_len(const csa_ctx *ctx, int32_t *n_pre, int32_t *n);
/* Rewind / set the context length to n in [n_pre, max_ctx] (rows >= n are simply ignored), on the
 * host and - with a blocking copy - in the device's word.  With streaming updates the tables hold
 * the appended keys: CSA_ERR_STATE unless n is unchanged. */
int csa_set_context_len(csa_ctx *ctx, int32_t n);
/* The grid exponent F in use (valid after build/import). */
int csa_score_frac_bits(const csa_ctx *ctx, int32_t *frac_bits);
/* Copies the table rows (b * C + j) probed by the last csa_decode_step, int32 [B][Hq][S*tau]
 * (subspace-major; order within a subspace unspecified), into a device buffer.  Diagnostic for
 * step 1. */
int csa_last_probed_rows(const csa_ctx *ctx, int32_t *rows_dev, void *stream);

/*
 * Per-kernel timing with HIP events recorded on the caller's stream around each launch.
 * csa_profile_enable(ctx, 1) starts collecting; csa_profile_read synchronises the recorded
 * events, adds each stage's elapsed milliseconds into ms_sum[CSA_N_STAGES] and the number of
 * launches into launches[CSA_N_STAGES] (either may be NULL), and clears the record.
 * Events cost a few microseconds per stage: leave disabled when timing whole steps.
 */
#define CSA_N_STAGES 10
int csa_profile_enable(csa_ctx *ctx, int32_t on);
int csa_profile_read(csa_ctx *ctx, double *ms_sum, int64_t *launches);
const char *csa_stage_name(int32_t stage); /* NULL if out of range */

const char *csa_strerror(int status);
/* hipError_t of the last failing HIP call on this ctx (0 if none). */
int csa_last_hip_error(const csa_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* CSATTN_H */

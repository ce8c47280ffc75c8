// Host-callable launchers of the gfx950 kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace csa {

// A table entry in device memory is one 32-bit word: the grid integer q (signed, kQBits bits) above
// the low kUnitBits bits of the key index.  Rows are sorted by key index, and the per-row offsets
// of every block of kUnit (or fewer) key indices tell which block an entry belongs to, so the high
// bits of the index need not be stored.
constexpr int kUnitBits = 13;
constexpr int kUnit = 1 << kUnitBits;
constexpr int kQBits = 32 - kUnitBits;
constexpr int32_t kQLimit = (1 << (kQBits - 1)) - 1;  // |q| <= kQLimit

// Streaming updates: the rows that take a new key wait in queue segments of kScanNT rows each; what the
// try test of a key whose centroid scores are given needs (insert_try_segment in common.h).
constexpr int kScanNT = 1024;
struct TryArgs {
    const float *z_key;  // [B*Hkv][S][C]: centroid (s, j) . new key over subspace s, the table build's fma chain
    const int32_t *row_cnt, *row_min;
    int32_t *queue_n;
    int4 *queue;
    int32_t *clamped;  // set when a score left the grid and was clamped
    int C, L, nx, S;   // centroids per (KV head, subspace), list length, segments per (KV head, subspace), subspaces
    float up;          // 2^F
    int qmax;          // largest admissible |grid score|
};

// ---- tables.hip
void launch_pack_centroids(const void *cent, void *cent_t, int n_bg, int C, int S, hipStream_t st);
void launch_import_rows(const int32_t *idx, const float *score, void *ent, int32_t *part_off,
                        int32_t *flags, int64_t n_rows, int L, int Ls, int n_pre, int F, int qmax,
                        int Q, int PO, hipStream_t st);
void launch_export_rows(const void *ent, const int32_t *part_off, int32_t *idx, float *score,
                        int n_rows, int L, int Ls, int F, int Q, int PO, hipStream_t st);
void launch_build_scores(const void *kc, const int32_t *block_table, const void *cent, int32_t *qs,
                         int32_t *flags, int b, int g, int Hkv, int max_ctx, int n_pre, int S, int sub,
                         int jc, int F, int qmax, hipStream_t st);
void launch_build_select(const int32_t *qs, void *ent, int32_t *part_off, int jc, int n_pre, int L,
                         int Ls, int Q, int PO, hipStream_t st);
void launch_row_stats(const void *ent, const int32_t *part_off, int32_t *row_cnt, int32_t *row_min, int32_t *blk_min,
                      int64_t n_rows, int Ls, int PO, hipStream_t st);
// z_key != NULL: the new key's centroid scores are already there (k_score_centroids with KEY): the
// try test reads them instead of streaming the centroids (one subspace only)
// tried: that test has already run (in the merge launch of the step, see launch_attention_merge_append)
TryArgs insert_try_args(const float *z_key, const int32_t *row_cnt, const int32_t *row_min, int32_t *queue_n,
                        void *queue, int32_t *clamped, int C, int S, int L, int F, int qmax);
void launch_insert(const void *k_new, const float *z_key, bool tried, const void *cent_t, void *ent, int32_t *part_off, int32_t *row_cnt,
                   int32_t *row_min, int32_t *blk_min, int32_t *queue_n, void *queue, int32_t *clamped, int B, int Hkv, int C,
                   int S, int L, int Ls, int Q, int PO, int F, int qmax, int idx_new, hipStream_t st);
void launch_max_key_norm(const void *kc, const int32_t *block_table, float *out, int B, int Hkv,
                         int max_ctx, int n_pre, int S, hipStream_t st);

// ---- cluster.hip
// every (KV head, subspace) problem of one sequence side by side; n_batches > 1: mini-batch steps
size_t cluster_work_bytes(int n_prob, int n_all, int C, int db);
int cluster_sequence(const void *q_seq, int n_pre, int G, int Hkv, int S, int C, int iters, int n_batches,
                     const float *u_seed, const void *init, void *out, float *mean_cos_out,
                     int32_t *assign_out, void *work, hipStream_t st);

// ---- decode.hip
// z_key != NULL (one subspace only): also z_key[bg][j] = centroid j of KV head bg . k_new[bg]
void launch_score_centroids(const void *q, const void *cent_t, float *z, int B, int Hkv, int G,
                            int C, int S, const void *k_new, float *z_key, hipStream_t st);
// both of the above in one launch (several subspaces, C <= 256, few probes per subspace)
bool score_top_fused(int C, int S, int tau);
// z_key != NULL: also z_key[bg][s][j] = centroid (s, j) . k_new[bg] over subspace s
void launch_score_top_sub(const void *q, const void *cent_t, int32_t *rows, const int32_t *part_off,
                          int32_t *spans, int B, int Hkv, int G, int C, int S, int tau, int P, int nsub,
                          int PO, const void *k_new, float *z_key, hipStream_t st);
void launch_top_centroids(const float *z, int32_t *rows, const int32_t *part_off, int32_t *spans,
                          int n_heads, int C, int S, int tau, int G, int P, int nsub, int PO, hipStream_t st);
// candidates of (head, key range): cand_key (words grouped by coarse score bin, best first),
// bin_off[.][512] (start of every bin), seg_cnt (how many)
// self_top (see accumulate_self_top): the launch also chooses the probed rows from z (no
// launch_top_centroids before it; `spans` is not read, `rows` is written)
bool accumulate_self_top(int n_heads, int S, int C, int tau, int R, int P);
void launch_accumulate(const void *ent, int32_t *rows, const int32_t *spans, uint32_t *cand_key,
                       uint16_t *bin_off, int32_t *seg_cnt, int n_heads, int C,
                       int Ls, int m, int G, int R, int P, size_t cand_stride, uint32_t key_lo,
                       int key_sh, int excl_from, const float *z, const int32_t *part_off, int PO,
                       bool self_top, hipStream_t st);
// seg_run[head][p] = where the threshold's bin starts and ends among the candidates of range p
void launch_threshold(const uint32_t *cand_key, const int32_t *seg_cnt, const uint16_t *bin_off, int32_t *sel,
                      int32_t *sel_count, uint32_t *thr, void *seg_par, void *seg_run, int n_heads, int k,
                      int R, int P, size_t cand_stride, int key_sh, hipStream_t st);
void launch_emit(const uint32_t *cand_key, const void *seg_run, const int32_t *seg_cnt,
                 const uint32_t *thr, const void *seg_par, int32_t *sel, int n_heads, int k, int R, int P,
                 size_t cand_stride, hipStream_t st);

// ---- attention.hip
int attention_splits(int k, int P, int n_appended);
// cand_key != NULL: the kernel also does the second half of the Top-K for its key range (needs
// attention_can_emit(R)); else `sel` is read as given.  n_dev != NULL: the context length is read
// from that device word instead of `n` (a launch that can be replayed; S must then cover the
// longest window).
void launch_attention_split(const void *q, const void *kc, const void *vc,
                            const int32_t *block_table, int32_t *sel, const int32_t *sel_count,
                            const void *seg_par, float *part, int B, int Hq, int Hkv, int k, int n_pre,
                            int n, int max_ctx, int S, int P, const uint32_t *cand_key,
                            const void *seg_run, const int32_t *seg_cnt, const uint32_t *thr, int R,
                            size_t cand_stride, const int32_t *n_dev, hipStream_t st);
bool attention_can_emit(int R);
void launch_range_offsets(const int32_t *sel, const int32_t *sel_count, void *seg_par, int n_heads, int k,
                          int R, int P, hipStream_t st);
void launch_attention_merge(const float *part, float *out, int n_heads, int S, hipStream_t st);
// the merge, and in the same launch the append of row n; *n_word (the device's copy of the context
// length) becomes n + 1.  from_dev: the position is *n_word itself, not `n` (replayable); an append
// to a full context is skipped and recorded in *full_word.
// tr != NULL (streaming updates, the new key's centroid scores at hand): the try test of the key
// runs in further workgroups of this launch, one per queue segment.
void launch_attention_merge_append(const float *part, float *out, int n_heads, int S, void *kc, void *vc,
                                   const int32_t *block_table, const void *kn, const void *vn, int B,
                                   int Hkv, int n, int max_ctx, int32_t *n_word, int32_t *full_word,
                                   bool from_dev, const TryArgs *tr, hipStream_t st);
void launch_append(void *kc, void *vc, const int32_t *block_table, const void *kn, const void *vn,
                   int B, int Hkv, int n, int max_ctx, int32_t *n_word, hipStream_t st);

}  // namespace csa

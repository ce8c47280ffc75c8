// C ABI of the library (include/csattn.h): host object, workspace layout, call sequencing.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/csattn.h"
#include "kernels.h"

// Scratch memory of csa_decode_step_static: one array per GPU, part of the loaded code object (it
// exists on every device the library runs on until the process ends).  Host code never uses this
// name as an address: the device address is looked up once per device (static_scratch below).
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char g_static_scratch[kStaticScratchBytes];

namespace {

constexpr size_t kAlign = 256;
// Centroid rows scored per pass of the table build: their integer scores against every key wait in
// scratch for the Top-L selection (one workgroup per row), so more rows per pass fill the chip
// better (1024 instead of 256 rows: 0.57 -> 0.43 s for 32768 rows over 128K keys) until the scores
// reach 1 GiB; never fewer than 64.
int build_chunk(int max_ctx)
{
    int rows = 1024;
    while (rows > 64 && (size_t)rows * (size_t)max_ctx > ((size_t)1 << 28)) rows >>= 1;
    return rows;
}
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Region {
    size_t off = 0, bytes = 0;
};

struct Layout {
    // tables buffer
    Region cent_t, ent, part_off, row_cnt, row_min, blk_min;  // (the last three: streaming updates only)
    Region state;  // persistent device words: [0] = a streamed score was clamped since the build,
                   // [1] = the context length as the device knows it, [2] = a replayed append found the context full
    size_t tables_bytes = 0;
    // scratch buffer: what a decode step uses comes first (decode_bytes), then what only the table
    // build and the streaming insertion use
    Region z, rows, spans, cand, bin_off, cand_cnt, seg_par, seg_run, thr, sel, sel_count, part, flags, qs;
    Region queue_n, queue;  // rows waiting for the streaming insertion
    Region z_key;           // centroid scores of the key a streaming one-call iteration appends
    size_t scratch_bytes = 0, decode_bytes = 0;
    int P_max = 0, PO_max = 0, S_max = 0, Ls = 0;
    size_t cand_keys = 0;  // candidate slots per head
};

const char *kStageNames[CSA_N_STAGES] = {"score_centroids", "top_centroids",   "accumulate",      "select_threshold",
                                         "select_emit",     "attention_split", "attention_merge", "append_kv",
                                         "range_offsets",   "stream_insert"};
using csa::kUnit;

}  // namespace

struct csa_ctx {
    csa_config cfg;
    Layout lay;
    char *tables = nullptr, *scratch = nullptr;
    void *k_cache = nullptr, *v_cache = nullptr;
    const int32_t *block_table = nullptr;
    bool bound = false, have_tables = false;
    int n_pre = 0, n = 0, F = -1, R = 0, P = 0;
    int Q = 0, nsub = 0, PO = 0;  // block size min(R, kUnit), blocks per range, offsets per row
    uint32_t key_lo = 0;  // coarse score bins of the candidates: 512 bins of 2^key_sh keys starting at key_lo
    int key_sh = 0;
    int hip_err = 0;
    // profiling
    bool prof = false;
    struct Rec {
        hipEvent_t ev[CSA_N_STAGES + 1];  // stage i runs between ev[i] and ev[i + 1]
        bool done[CSA_N_STAGES];          // both events of stage i were recorded in this call
    };
    // the index set of the last searching step (reused by csa_decode_step_reuse)
    const int32_t *last_sel = nullptr, *last_sel_count = nullptr;
    const char *last_scratch = nullptr;  // where that step kept its temporaries (probed rows)
    std::vector<Rec> recs;
    size_t n_recs = 0;
};

namespace {

int min_R(const csa_config &c) { return c.partition_keys ? c.partition_keys : 1024; }

Layout make_layout(const csa_config &c)
{
    Layout l;
    const size_t BG = (size_t)c.batch * c.n_kv_heads, BH = (size_t)c.batch * c.n_q_heads;
    const size_t Ct = (size_t)c.n_subspaces * c.n_centroids;  // table rows per KV head
    const size_t M = (size_t)c.n_subspaces * c.n_probe;       // rows probed per query
    // choose_partition widens the key ranges until a head has at most 2048 of them, so neither the
    // ranges nor the block offsets of a row (P * nsub + 1, nsub = 2 only for ranges of 16384 keys,
    // of which there are at most 1024) outgrow these bounds however long the context is
    l.P_max = (c.max_ctx + min_R(c) - 1) / min_R(c);
    if (l.P_max > 2048) l.P_max = 2048;
    const int q_min = min_R(c) < kUnit ? min_R(c) : kUnit;
    l.PO_max = (c.max_ctx + q_min - 1) / q_min + 5;  // >= P * nsub + 1 for every admissible R
    if (l.PO_max > 2048 + 5) l.PO_max = 2048 + 5;
    l.Ls = (c.list_len + 3) / 4 * 4;                 // row stride: 16-byte aligned rows
    size_t off = 0;
    auto put = [&](Region &r, size_t bytes) {
        r.off = off;
        r.bytes = bytes;
        off = align_up(off + bytes);
    };
    put(l.cent_t, BG * c.n_centroids * c.head_dim * 2);
    put(l.ent, BG * Ct * (size_t)l.Ls * 4);
    put(l.part_off, BG * Ct * (size_t)l.PO_max * 4);
    if (c.stream_window > 0) {
        put(l.row_cnt, BG * Ct * 4);
        put(l.row_min, BG * Ct * 4);
        put(l.blk_min, BG * Ct * (size_t)l.PO_max * 4);  // per block of a row: its smallest score
    }
    put(l.state, 256);
    l.tables_bytes = off;
    off = 0;
    l.cand_keys = ((size_t)c.max_ctx + 16383) / 16384 * 16384;
    l.S_max = csa::attention_splits(c.budget_k, l.P_max, c.max_ctx);
    put(l.z, BH * Ct * 4);
    put(l.rows, BH * M * 4);
    put(l.spans, BH * M * 2 * l.PO_max * 4);  // P * (nsub + 1) <= 2 * PO offsets per row
    put(l.cand, BH * l.cand_keys * 4);       // candidate keys, R slots per (head, key range)
    put(l.cand_cnt, BH * (size_t)l.P_max * 4);  // candidates per (head, key range)
    put(l.seg_par, BH * (size_t)l.P_max * 8);   // (output offset, ties allowed) per (head, key range)
    put(l.seg_run, BH * (size_t)l.P_max * 8);   // candidates of the threshold's bin per (head, key range)
    put(l.thr, BH * 4);                         // Top-K threshold per head
    put(l.sel, BH * (size_t)(c.budget_k > 0 ? c.budget_k : 1) * 4);
    put(l.sel_count, BH * 4);
    put(l.part, BH * (size_t)(l.S_max > 0 ? l.S_max : 1) * (c.head_dim + 2) * 4);
    put(l.bin_off, BH * (size_t)l.P_max * 512 * 2);  // start of every coarse score bin per (head, key range)
    l.decode_bytes = off;
    put(l.flags, 256);
    put(l.qs, (size_t)(c.n_centroids < build_chunk(c.max_ctx) ? c.n_centroids : build_chunk(c.max_ctx)) * c.max_ctx * 4);
    if (c.stream_window > 0) {
        const size_t n_seg = (size_t)c.n_subspaces * ((c.n_centroids + 1023) / 1024);  // queue segments per KV head
        put(l.queue_n, BG * n_seg * 4);
        put(l.queue, BG * n_seg * 1024 * 16);
        put(l.z_key, BG * Ct * 4);  // the appended key's centroid scores
    }
    l.scratch_bytes = off;
    return l;
}

bool is_pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }

int validate(const csa_config &c)
{
    if (c.batch < 1 || c.n_kv_heads < 1 || c.n_q_heads < 1) return CSA_ERR_ARG;
    if (c.n_q_heads % c.n_kv_heads) return CSA_ERR_ARG;
    const int G = c.n_q_heads / c.n_kv_heads;
    if (G > 16) return CSA_ERR_ARG;
    if (c.head_dim != 128) return CSA_ERR_ARG;
    if (c.n_centroids < 1 || c.list_len < 1 || c.list_len > 8192) return CSA_ERR_ARG;
    const int S = c.n_subspaces;
    if (!(S == 1 || S == 2 || S == 4 || S == 8 || S == 16)) return CSA_ERR_ARG;
    if (c.n_probe < 1 || c.n_probe > c.n_centroids || (int64_t)S * c.n_probe > 63) return CSA_ERR_ARG;
    if (c.budget_k < 0) return CSA_ERR_ARG;
    if ((int64_t)S * c.n_centroids > (1 << 24)) return CSA_ERR_ARG;
    if (c.max_ctx < 1 || c.max_ctx > (1 << 24)) return CSA_ERR_ARG;
    if (c.page_size != 0 && c.page_size != 16) return CSA_ERR_ARG;
    if (c.page_size && c.max_ctx % c.page_size) return CSA_ERR_ARG;
    if (c.score_frac_bits > 30) return CSA_ERR_ARG;
    if (c.partition_keys &&
        (!is_pow2(c.partition_keys) || c.partition_keys < 1024 || c.partition_keys > 16384))
        return CSA_ERR_ARG;
    if ((int64_t)c.batch * c.n_q_heads > 65535) return CSA_ERR_ARG;  // grid.y
    if ((int64_t)c.batch * c.n_kv_heads > 65535) return CSA_ERR_ARG;  // grid.z
    if (c.stream_window < 0) return CSA_ERR_ARG;
    // the streaming update queues rows in segments of 1024 centroids, at most 64 per KV head
    if (c.stream_window > 0 && (int64_t)c.n_subspaces * ((c.n_centroids + 1023) / 1024) > 64) return CSA_ERR_ARG;
    return CSA_OK;
}

int hip_fail(csa_ctx *ctx, hipError_t e)
{
    ctx->hip_err = (int)e;
    return CSA_ERR_HIP;
}

int check_launch(csa_ctx *ctx)
{
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? CSA_OK : hip_fail(ctx, e);
}

// range of key indices per accumulation workgroup
void choose_partition(csa_ctx *ctx, int n_pre)
{
    const csa_config &c = ctx->cfg;
    if (c.stream_window > 0) n_pre = c.max_ctx;  // appended keys enter the tables: cover every index
    int R = c.partition_keys;
    if (!R) {
        // the accumulation kernel runs R/16 threads per key range, so the wave count does not
        // depend on R; larger ranges amortise per-row work, but at least ~512 workgroups are wanted
        // and 8192 keys (512 threads, three workgroups at a time per CU) measured best on MI355X
        // With few heads and a short context the step is a chain of small launches, and ranges of
        // at least 4096 keys keep that chain short (the accumulation launch then also chooses the
        // probed rows): 32 heads at 32K context, 43.8 us per step with 2048-key ranges, 38.8 with 4096
        const int heads = c.batch * c.n_q_heads;
        const int p_target = (512 + heads - 1) / heads;
        R = 8192;
        if ((n_pre + R - 1) / R < p_target) R = 4096;
    }
    while ((n_pre + R - 1) / R > 2048 && R < 16384) R <<= 1;  // at most 2048 key ranges per head
    ctx->R = R;
    ctx->P = (n_pre + R - 1) / R;
    if (ctx->P < 1) ctx->P = 1;
    ctx->Q = R < kUnit ? R : kUnit;
    ctx->nsub = R / ctx->Q;
    ctx->PO = ctx->P * ctx->nsub + 1;
}

template <class T>
T *at(char *base, const Region &r) { return reinterpret_cast<T *>(base + r.off); }

// device address of g_static_scratch on the current device (every GPU holds its own copy at its
// own address), looked up on the first call on that device
constexpr int kMaxDevices = 64;
std::mutex g_static_mu;
char *g_static_ptr[kMaxDevices] = {};

int static_scratch(csa_ctx *ctx, char **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(ctx, e);
    if (dev < 0 || dev >= kMaxDevices) return CSA_ERR_ARG;
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch));
        if (e != hipSuccess || !p) return hip_fail(ctx, e != hipSuccess ? e : hipErrorInvalidSymbol);
        g_static_ptr[dev] = (char *)p;
    }
    *out = g_static_ptr[dev];
    return CSA_OK;
}

// largest admissible |q|: m sums stay below 2^24 and q fits its field of a packed entry
int qmax_for(int m)
{
    const int a = ((1 << 24) - 1) / m, b = csa::kQLimit;
    return a < b ? a : b;
}

// The accumulated key of any key index is 2^24 + (sum of <= m table integers), so it lies within
// m * max|q| of 2^24: 512 equal bins over that span.
void set_key_range(csa_ctx *ctx, int qabs_max)
{
    // scores of keys inserted later are only known to respect the admissible maximum (a bound taken
    // from the prefill keys would be wrong for a short prefill followed by a long generation)
    if (ctx->cfg.stream_window > 0) qabs_max = qmax_for(ctx->cfg.n_probe * ctx->cfg.n_subspaces);
    const uint32_t span = (uint32_t)(ctx->cfg.n_probe * ctx->cfg.n_subspaces) * (uint32_t)qabs_max;  // < 2^24
    ctx->key_lo = (1u << 24) - span;
    int sh = 0;
    while (((2u * span) >> sh) >= 512u) ++sh;
    ctx->key_sh = sh;
}

int32_t *n_word(csa_ctx *ctx) { return at<int32_t>(ctx->tables, ctx->lay.state) + 1; }
int32_t *full_word(csa_ctx *ctx) { return at<int32_t>(ctx->tables, ctx->lay.state) + 2; }

// the device's copy of the context length (set-up paths only: the copy is synchronous)
int set_device_count(csa_ctx *ctx, int n)
{
    const int32_t words[2] = {n, 0};  // (count, no refused append)
    const hipError_t e = hipMemcpy(n_word(ctx), words, 8, hipMemcpyHostToDevice);
    return e == hipSuccess ? CSA_OK : hip_fail(ctx, e);
}

int window_start(const csa_ctx *ctx)
{
    if (ctx->cfg.stream_window <= 0) return ctx->n_pre;
    const int ws = ctx->n - ctx->cfg.stream_window;
    return ws > 0 ? ws : 0;
}

struct Prof {
    csa_ctx *ctx;
    hipStream_t st;
    csa_ctx::Rec *rec = nullptr;
    Prof(csa_ctx *c, hipStream_t s) : ctx(c), st(s)
    {
        if (!ctx->prof) return;
        if (ctx->n_recs == ctx->recs.size()) {
            csa_ctx::Rec r;
            for (auto &e : r.ev) (void)hipEventCreate(&e);
            ctx->recs.push_back(r);
        }
        rec = &ctx->recs[ctx->n_recs++];
        for (auto &u : rec->done) u = false;
    }
    // mark the boundary before stage `i` (and after stage i-1)
    void mark(int i)
    {
        if (!rec) return;
        (void)hipEventRecord(rec->ev[i], st);
    }
    // mark the end of stage `i` (= the boundary before stage i+1)
    void end(int i)
    {
        if (!rec) return;
        (void)hipEventRecord(rec->ev[i + 1], st);
        rec->done[i] = true;
    }
};

}  // namespace

extern "C" {

int csa_create(const csa_config *cfg, csa_ctx **out)
{
    if (!cfg || !out) return CSA_ERR_ARG;
    const int v = validate(*cfg);
    if (v != CSA_OK) return v;
    csa_ctx *ctx = new (std::nothrow) csa_ctx();
    if (!ctx) return CSA_ERR_ARG;
    ctx->cfg = *cfg;
    ctx->lay = make_layout(*cfg);
    *out = ctx;
    return CSA_OK;
}

void csa_destroy(csa_ctx *ctx)
{
    if (!ctx) return;
    for (auto &r : ctx->recs)
        for (auto &e : r.ev) (void)hipEventDestroy(e);
    delete ctx;
}

int csa_workspace_bytes(const csa_ctx *ctx, size_t *tables_bytes, size_t *scratch_bytes)
{
    if (!ctx) return CSA_ERR_ARG;
    if (tables_bytes) *tables_bytes = ctx->lay.tables_bytes;
    if (scratch_bytes) *scratch_bytes = ctx->lay.scratch_bytes;
    return CSA_OK;
}

int csa_bind(csa_ctx *ctx, void *tables_dev, size_t tables_bytes, void *scratch_dev,
             size_t scratch_bytes, void *k_cache_dev, void *v_cache_dev,
             const int32_t *block_table_dev)
{
    if (!ctx || !tables_dev || !scratch_dev || !k_cache_dev || !v_cache_dev) return CSA_ERR_ARG;
    if ((ctx->cfg.page_size != 0) != (block_table_dev != nullptr)) return CSA_ERR_ARG;
    for (const void *p : {(const void *)tables_dev, (const void *)scratch_dev,
                          (const void *)k_cache_dev, (const void *)v_cache_dev})
        if ((uintptr_t)p % kAlign) return CSA_ERR_ARG;
    if (tables_bytes < ctx->lay.tables_bytes || scratch_bytes < ctx->lay.scratch_bytes)
        return CSA_ERR_WORKSPACE;
    if (ctx->tables != (char *)tables_dev) ctx->have_tables = false;
    ctx->tables = (char *)tables_dev;
    ctx->scratch = (char *)scratch_dev;
    ctx->k_cache = k_cache_dev;
    ctx->v_cache = v_cache_dev;
    ctx->block_table = block_table_dev;
    ctx->last_sel = ctx->last_sel_count = nullptr;
    ctx->last_scratch = nullptr;
    ctx->bound = true;
    return CSA_OK;
}

int csa_build_tables(csa_ctx *ctx, const void *centroids_dev, int32_t n_pre, void *stream)
{
    if (!ctx || !centroids_dev) return CSA_ERR_ARG;
    if (!ctx->bound) return CSA_ERR_STATE;
    const csa_config &c = ctx->cfg;
    if (n_pre < 1 || n_pre > c.max_ctx) return CSA_ERR_ARG;
    hipStream_t st = (hipStream_t)stream;
    const Layout &l = ctx->lay;
    ctx->have_tables = false;
    ctx->last_sel = ctx->last_sel_count = nullptr;
    ctx->last_scratch = nullptr;
    int32_t *flags = at<int32_t>(ctx->scratch, l.flags);
    hipError_t e = hipMemsetAsync(flags, 0, 256, st);
    if (e == hipSuccess) e = hipMemsetAsync(at<void>(ctx->tables, l.state), 0, 256, st);
    if (e != hipSuccess) return hip_fail(ctx, e);

    int F = c.score_frac_bits;
    if (F < 0) {
        // finest grid with n_probe * (max|s| * 2^F + 1/2) < 2^24, |s| <= ||c|| ||k|| and
        // ||c|| <= 1.01 for unit centroids rounded to bf16
        csa::launch_max_key_norm(ctx->k_cache, ctx->block_table, (float *)(flags + 16), c.batch,
                                 c.n_kv_heads, c.max_ctx, n_pre, c.n_subspaces, st);
        float nn = 0.0f;
        e = hipMemcpyAsync(&nn, flags + 16, 4, hipMemcpyDeviceToHost, st);
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e != hipSuccess) return hip_fail(ctx, e);
        const double bound = 1.01 * std::sqrt((double)nn) + 1e-30;
        F = (int)std::floor(std::log2(((double)qmax_for(c.n_probe * c.n_subspaces) - 1.0) / bound));
        if (F > 30) F = 30;
        if (F < 0) return CSA_ERR_RANGE;
    }
    choose_partition(ctx, n_pre);
    if (ctx->PO > l.PO_max || ctx->P > l.P_max) return CSA_ERR_WORKSPACE;  // (cannot happen: see make_layout)
    const int BG = c.batch * c.n_kv_heads;
    const int S = c.n_subspaces, db = c.head_dim / S, M = S * c.n_probe;
    csa::launch_pack_centroids(centroids_dev, at<void>(ctx->tables, l.cent_t), BG, c.n_centroids, S, st);
    int32_t *qs = at<int32_t>(ctx->scratch, l.qs);
    char *ent = at<char>(ctx->tables, l.ent);
    int32_t *part_off = at<int32_t>(ctx->tables, l.part_off);
    const uint16_t *cent = (const uint16_t *)centroids_dev;
    const int chunk = build_chunk(c.max_ctx);
    for (int b = 0; b < c.batch; ++b)
        for (int g = 0; g < c.n_kv_heads; ++g)
            for (int sub = 0; sub < S; ++sub)
                for (int j0 = 0; j0 < c.n_centroids; j0 += chunk) {
                    const int jc = c.n_centroids - j0 < chunk ? c.n_centroids - j0 : chunk;
                    // table row of centroid (sub, j0) of KV head (b, g); its centroid vector
                    const size_t row0 = ((size_t)(b * c.n_kv_heads + g) * S + sub) * c.n_centroids + j0;
                    csa::launch_build_scores(ctx->k_cache, ctx->block_table, cent + row0 * db, qs, flags, b, g,
                                             c.n_kv_heads, c.max_ctx, n_pre, S, sub, jc, F, qmax_for(M), st);
                    csa::launch_build_select(qs, ent + row0 * l.Ls * 4, part_off + row0 * ctx->PO, jc, n_pre,
                                             c.list_len, l.Ls, ctx->Q, ctx->PO, st);
                }
    int rc = check_launch(ctx);
    if (rc != CSA_OK) return rc;
    int32_t hflags[2] = {0, 0};
    e = hipMemcpyAsync(hflags, flags, 8, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) return hip_fail(ctx, e);
    if (hflags[0] & 1) return CSA_ERR_RANGE;
    set_key_range(ctx, hflags[1]);
    if (c.stream_window > 0)
        csa::launch_row_stats(ent, part_off, at<int32_t>(ctx->tables, l.row_cnt), at<int32_t>(ctx->tables, l.row_min),
                              at<int32_t>(ctx->tables, l.blk_min),
                              (int64_t)BG * S * c.n_centroids, l.Ls, ctx->PO, st);
    ctx->F = F;
    ctx->n_pre = ctx->n = n_pre;
    rc = set_device_count(ctx, n_pre);
    if (rc != CSA_OK) return rc;
    ctx->have_tables = true;
    return CSA_OK;
}

int csa_cluster_workspace_bytes(const csa_ctx *ctx, int32_t n_pre, size_t *bytes)
{
    if (!ctx || !bytes || n_pre < 1) return CSA_ERR_ARG;
    const csa_config &c = ctx->cfg;
    const int64_t n_pool = (int64_t)(c.n_q_heads / c.n_kv_heads) * n_pre;
    if (n_pool > (1 << 30)) return CSA_ERR_ARG;
    *bytes = csa::cluster_work_bytes(c.n_kv_heads * c.n_subspaces, (int)n_pool, c.n_centroids,
                                     c.head_dim / c.n_subspaces);
    return CSA_OK;
}

int csa_cluster_queries_minibatch(csa_ctx *ctx, const void *q_pre_dev, int32_t n_pre, int32_t iters,
                                  int32_t n_batches, const float *u_seed_dev, const void *init_centroids_dev,
                                  void *centroids_out_dev, float *mean_cos_dev, int32_t *assign_dev,
                                  void *work_dev, size_t work_bytes, void *stream)
{
    if (!ctx || !q_pre_dev || !centroids_out_dev || !work_dev) return CSA_ERR_ARG;
    if (n_pre < 1 || iters < 0 || (!u_seed_dev && !init_centroids_dev)) return CSA_ERR_ARG;
    if ((uintptr_t)work_dev % kAlign) return CSA_ERR_ARG;
    const csa_config &c = ctx->cfg;
    const int G = c.n_q_heads / c.n_kv_heads, S = c.n_subspaces, C = c.n_centroids, db = c.head_dim / S;
    const int64_t n_pool64 = (int64_t)G * n_pre;
    if (n_pool64 > (1 << 30)) return CSA_ERR_ARG;
    const int n_pool = (int)n_pool64, n_prob = c.n_kv_heads * S;
    if (n_batches < 1 || n_batches > n_pool) return CSA_ERR_ARG;
    if (work_bytes < csa::cluster_work_bytes(n_prob, n_pool, C, db)) return CSA_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const int it_eff = iters > 0 ? iters : 1;
    for (int b = 0; b < c.batch; ++b) {
        const size_t p0 = (size_t)b * n_prob;  // the sequence's first problem
        const int rc = csa::cluster_sequence(
            (const uint16_t *)q_pre_dev + (size_t)b * c.n_q_heads * n_pre * c.head_dim, n_pre, G, c.n_kv_heads, S, C,
            iters, n_batches, u_seed_dev ? u_seed_dev + p0 * C : nullptr,
            init_centroids_dev ? (const uint16_t *)init_centroids_dev + p0 * C * db : nullptr,
            (uint16_t *)centroids_out_dev + p0 * C * db, mean_cos_dev ? mean_cos_dev + p0 * it_eff : nullptr,
            assign_dev ? assign_dev + p0 * n_pool : nullptr, work_dev, st);
        if (rc != 0) return hip_fail(ctx, (hipError_t)rc);
    }
    return CSA_OK;
}

int csa_cluster_queries(csa_ctx *ctx, const void *q_pre_dev, int32_t n_pre, int32_t iters,
                        const float *u_seed_dev, const void *init_centroids_dev, void *centroids_out_dev,
                        float *mean_cos_dev, int32_t *assign_dev, void *work_dev, size_t work_bytes,
                        void *stream)
{
    return csa_cluster_queries_minibatch(ctx, q_pre_dev, n_pre, iters, 1, u_seed_dev, init_centroids_dev,
                                         centroids_out_dev, mean_cos_dev, assign_dev, work_dev, work_bytes, stream);
}

int csa_prefill(csa_ctx *ctx, const void *q_pre_dev, int32_t n_pre, int32_t iters, int32_t n_batches,
                const float *u_seed_dev, void *centroids_out_dev, void *work_dev, size_t work_bytes, void *stream)
{
    if (!ctx) return CSA_ERR_ARG;
    if (!ctx->bound) return CSA_ERR_STATE;
    if (!u_seed_dev) return CSA_ERR_ARG;
    const int rc = csa_cluster_queries_minibatch(ctx, q_pre_dev, n_pre, iters, n_batches, u_seed_dev, nullptr,
                                                 centroids_out_dev, nullptr, nullptr, work_dev, work_bytes, stream);
    if (rc != CSA_OK) return rc;
    return csa_build_tables(ctx, centroids_out_dev, n_pre, stream);
}

int csa_import_tables(csa_ctx *ctx, const void *centroids_dev, const int32_t *idx_dev,
                      const float *score_dev, int32_t n_pre, void *stream)
{
    if (!ctx || !centroids_dev || !idx_dev || !score_dev) return CSA_ERR_ARG;
    if (!ctx->bound) return CSA_ERR_STATE;
    const csa_config &c = ctx->cfg;
    if (n_pre < 1 || n_pre > c.max_ctx || c.score_frac_bits < 0) return CSA_ERR_ARG;
    hipStream_t st = (hipStream_t)stream;
    const Layout &l = ctx->lay;
    ctx->have_tables = false;
    ctx->last_sel = ctx->last_sel_count = nullptr;
    ctx->last_scratch = nullptr;
    int32_t *flags = at<int32_t>(ctx->scratch, l.flags);
    hipError_t e = hipMemsetAsync(flags, 0, 256, st);
    if (e == hipSuccess) e = hipMemsetAsync(at<void>(ctx->tables, l.state), 0, 256, st);
    if (e != hipSuccess) return hip_fail(ctx, e);
    choose_partition(ctx, n_pre);
    if (ctx->PO > l.PO_max || ctx->P > l.P_max) return CSA_ERR_WORKSPACE;  // (cannot happen: see make_layout)
    const int BG = c.batch * c.n_kv_heads;
    const int64_t n_rows = (int64_t)BG * c.n_subspaces * c.n_centroids;
    csa::launch_pack_centroids(centroids_dev, at<void>(ctx->tables, l.cent_t), BG, c.n_centroids,
                               c.n_subspaces, st);
    csa::launch_import_rows(idx_dev, score_dev, at<void>(ctx->tables, l.ent), at<int32_t>(ctx->tables, l.part_off),
                            flags, n_rows, c.list_len, l.Ls, n_pre, c.score_frac_bits,
                            qmax_for(c.n_probe * c.n_subspaces), ctx->Q, ctx->PO, st);
    int rc = check_launch(ctx);
    if (rc != CSA_OK) return rc;
    int32_t hflags[2] = {0, 0};
    e = hipMemcpyAsync(hflags, flags, 8, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) return hip_fail(ctx, e);
    if (hflags[0] & 2) return CSA_ERR_ARG;
    if (hflags[0] & 1) return CSA_ERR_RANGE;
    set_key_range(ctx, hflags[1]);
    if (c.stream_window > 0)
        csa::launch_row_stats(at<void>(ctx->tables, l.ent), at<int32_t>(ctx->tables, l.part_off),
                              at<int32_t>(ctx->tables, l.row_cnt), at<int32_t>(ctx->tables, l.row_min),
                              at<int32_t>(ctx->tables, l.blk_min), n_rows, l.Ls, ctx->PO, st);
    ctx->F = c.score_frac_bits;
    ctx->n_pre = ctx->n = n_pre;
    rc = set_device_count(ctx, n_pre);
    if (rc != CSA_OK) return rc;
    ctx->have_tables = true;
    return CSA_OK;
}

int csa_export_tables(const csa_ctx *ctx, int32_t b, int32_t g, int32_t *idx_dev, float *score_dev,
                      void *stream)
{
    if (!ctx || !idx_dev || !score_dev) return CSA_ERR_ARG;
    if (!ctx->have_tables) return CSA_ERR_STATE;
    const csa_config &c = ctx->cfg;
    if (b < 0 || b >= c.batch || g < 0 || g >= c.n_kv_heads) return CSA_ERR_ARG;
    const int Ct = c.n_subspaces * c.n_centroids;
    const size_t row0 = (size_t)(b * c.n_kv_heads + g) * Ct;
    const int32_t *part_off = reinterpret_cast<const int32_t *>(ctx->tables + ctx->lay.part_off.off);
    csa::launch_export_rows(ctx->tables + ctx->lay.ent.off + row0 * ctx->lay.Ls * 4, part_off + row0 * ctx->PO,
                            idx_dev, score_dev, Ct, c.list_len, ctx->lay.Ls, ctx->F, ctx->Q,
                            ctx->PO, (hipStream_t)stream);
    return check_launch(const_cast<csa_ctx *>(ctx));
}

namespace {

// streaming update of the tables with the key just appended at position ctx->n (Sec. 3.3 (5))
// z_key: the new key's centroid scores if the step's scoring launch computed them, else NULL;
// tried: the try test on those scores has run already (in the step's merge launch)
void run_insert(csa_ctx *ctx, Prof &prof, const void *k_new_dev, const float *z_key, bool tried, hipStream_t st)
{
    const csa_config &c = ctx->cfg;
    const Layout &l = ctx->lay;
    prof.mark(9);
    csa::launch_insert(k_new_dev, z_key, tried, at<void>(ctx->tables, l.cent_t), at<void>(ctx->tables, l.ent),
                       at<int32_t>(ctx->tables, l.part_off), at<int32_t>(ctx->tables, l.row_cnt),
                       at<int32_t>(ctx->tables, l.row_min), at<int32_t>(ctx->tables, l.blk_min),
                       at<int32_t>(ctx->scratch, l.queue_n),
                       at<void>(ctx->scratch, l.queue), at<int32_t>(ctx->tables, l.state), c.batch,
                       c.n_kv_heads, c.n_centroids, c.n_subspaces, c.list_len, l.Ls, ctx->Q, ctx->PO, ctx->F,
                       qmax_for(c.n_probe * c.n_subspaces), ctx->n, st);
    prof.end(9);
}

// the split merge that ends a step; with k_new/v_new also the append of row n (same launch) and,
// with streaming updates, the try-insert
void finish_step(csa_ctx *ctx, Prof &prof, const float *part, float *out_dev, int S, const void *k_new_dev,
                 const void *v_new_dev, bool replayable, const float *z_key, hipStream_t st)
{
    const csa_config &c = ctx->cfg;
    const int BH = c.batch * c.n_q_heads;
    if (!k_new_dev) {
        csa::launch_attention_merge(part, out_dev, BH, S, st);
        prof.end(6);
        return;
    }
    const bool streaming = c.stream_window > 0;
    // with the new key's centroid scores at hand its try test rides in the merge launch (it reads the
    // tables' row states, which nothing in this launch writes)
    const bool try_here = streaming && z_key && !replayable;
    const Layout &l = ctx->lay;
    csa::TryArgs tr{};
    if (try_here)
        tr = csa::insert_try_args(z_key, at<int32_t>(ctx->tables, l.row_cnt), at<int32_t>(ctx->tables, l.row_min),
                                  at<int32_t>(ctx->scratch, l.queue_n), at<void>(ctx->scratch, l.queue),
                                  at<int32_t>(ctx->tables, l.state), c.n_centroids, c.n_subspaces, c.list_len, ctx->F,
                                  qmax_for(c.n_probe * c.n_subspaces));
    csa::launch_attention_merge_append(part, out_dev, BH, S, ctx->k_cache, ctx->v_cache, ctx->block_table,
                                       k_new_dev, v_new_dev, c.batch, c.n_kv_heads, ctx->n, c.max_ctx, n_word(ctx),
                                       full_word(ctx), replayable, try_here ? &tr : nullptr, st);
    prof.end(6);
    if (streaming) run_insert(ctx, prof, k_new_dev, z_key, try_here, st);
    ctx->n += 1;
}

}  // namespace

int csa_append_kv(csa_ctx *ctx, const void *k_new_dev, const void *v_new_dev, void *stream)
{
    if (!ctx || !k_new_dev || !v_new_dev) return CSA_ERR_ARG;
    if (!ctx->bound || !ctx->have_tables) return CSA_ERR_STATE;
    if (ctx->n >= ctx->cfg.max_ctx) return CSA_ERR_CAPACITY;
    hipStream_t st = (hipStream_t)stream;
    Prof prof(ctx, st);
    const csa_config &c = ctx->cfg;
    const bool streaming = c.stream_window > 0;
    prof.mark(7);
    csa::launch_append(ctx->k_cache, ctx->v_cache, ctx->block_table, k_new_dev, v_new_dev, c.batch,
                       c.n_kv_heads, ctx->n, c.max_ctx, n_word(ctx), st);
    prof.end(7);
    if (streaming) run_insert(ctx, prof, k_new_dev, nullptr, false, st);
    ctx->n += 1;
    return check_launch(ctx);
}

namespace {

// `scr`: the scratch memory of this step, laid out as Layout says (the bound scratch buffer, or
// the library's own static array)
// replayable: no launch argument depends on the context length - the kernels read the device's
// count, the window splits are sized for a full context (streaming updates excluded)
int search_step(csa_ctx *ctx, char *scr, const void *q_dev, float *out_dev, int32_t *sel_idx_dev,
                int32_t *sel_count_dev, const void *k_new_dev, const void *v_new_dev, bool replayable,
                void *stream)
{
    if (!ctx || !q_dev || !out_dev) return CSA_ERR_ARG;
    if (!ctx->bound || !ctx->have_tables) return CSA_ERR_STATE;
    if (k_new_dev && ctx->n >= ctx->cfg.max_ctx) return CSA_ERR_CAPACITY;
    if (replayable && ctx->cfg.stream_window > 0) return CSA_ERR_ARG;
    const csa_config &c = ctx->cfg;
    const Layout &l = ctx->lay;
    hipStream_t st = (hipStream_t)stream;
    const int BH = c.batch * c.n_q_heads, G = c.n_q_heads / c.n_kv_heads;
    const int S_sub = c.n_subspaces, Ct = S_sub * c.n_centroids, M = S_sub * c.n_probe;
    float *z = at<float>(scr, l.z);
    int32_t *rows = at<int32_t>(scr, l.rows);
    uint32_t *cand_key = at<uint32_t>(scr, l.cand);
    uint16_t *bin_off = at<uint16_t>(scr, l.bin_off);
    int32_t *cand_cnt = at<int32_t>(scr, l.cand_cnt);
    void *seg_par = at<void>(scr, l.seg_par);
    void *seg_run = at<void>(scr, l.seg_run);
    uint32_t *thr = at<uint32_t>(scr, l.thr);
    int32_t *sel = sel_idx_dev ? sel_idx_dev : at<int32_t>(scr, l.sel);
    int32_t *sel_count = sel_count_dev ? sel_count_dev : at<int32_t>(scr, l.sel_count);
    float *part = at<float>(scr, l.part);
    // the always-attended recent window [ws, n): every appended key, or - with streaming updates -
    // the last stream_window positions (older appended keys compete through the tables)
    const int ws = window_start(ctx);
    const int S = csa::attention_splits(c.budget_k, ctx->P, (replayable ? c.max_ctx : ctx->n) - ws);
    const int32_t *n_dev = replayable ? n_word(ctx) : nullptr;

    Prof prof(ctx, st);
    prof.mark(0);
    int32_t *spans = at<int32_t>(scr, l.spans);
    bool self_top = false;
    float *z_key = nullptr;
    if (csa::score_top_fused(c.n_centroids, S_sub, c.n_probe)) {
        // the paper's own geometry: scoring and the choice of the probed rows in one launch
        // with streaming updates the key this call appends is scored in the same pass over the centroids
        if (c.stream_window > 0 && k_new_dev) z_key = at<float>(ctx->scratch, l.z_key);
        csa::launch_score_top_sub(q_dev, at<void>(ctx->tables, l.cent_t), rows, at<int32_t>(ctx->tables, l.part_off),
                                  spans, c.batch, c.n_kv_heads, G, c.n_centroids, S_sub, c.n_probe, ctx->P,
                                  ctx->nsub, ctx->PO, k_new_dev, z_key, st);
        prof.end(0);
        prof.mark(2);
    } else {
        // with streaming updates the key this call appends is scored in the same pass over the centroids
        if (c.stream_window > 0 && k_new_dev && S_sub == 1) z_key = at<float>(ctx->scratch, l.z_key);
        csa::launch_score_centroids(q_dev, at<void>(ctx->tables, l.cent_t), z, c.batch, c.n_kv_heads, G,
                                    c.n_centroids, S_sub, k_new_dev, z_key, st);
        prof.end(0);
        // a small launch chooses the probed rows inside the accumulation launch (a kernel less in
        // the chain of dependent launches: 61 -> 57 us per step at batch 1, 128K)
        self_top = csa::accumulate_self_top(BH, S_sub, c.n_centroids, c.n_probe, ctx->R, ctx->P);
        if (!self_top) {
            csa::launch_top_centroids(z, rows, at<int32_t>(ctx->tables, l.part_off), spans, BH,
                                      c.n_centroids, S_sub, c.n_probe, G, ctx->P, ctx->nsub, ctx->PO, st);
            prof.end(1);
        } else {
            prof.mark(2);
        }
    }
    csa::launch_accumulate(at<void>(ctx->tables, l.ent), rows, spans, cand_key, bin_off, cand_cnt, BH,
                           Ct, l.Ls, M, G, ctx->R, ctx->P, l.cand_keys, ctx->key_lo, ctx->key_sh, ws, z,
                           at<int32_t>(ctx->tables, l.part_off), ctx->PO, self_top, st);
    prof.end(2);
    csa::launch_threshold(cand_key, cand_cnt, bin_off, sel, sel_count, thr, seg_par, seg_run, BH, c.budget_k,
                          ctx->R, ctx->P, l.cand_keys, ctx->key_sh, st);
    prof.end(3);
    // the second half of the Top-K runs in the prologue of the attention workgroups when a key
    // range has at most one bitmap word per attention thread and the launch is small (it then saves a
    // launch, 4 us of 66 at batch 1); with thousands of workgroups the prologue's latency delays
    // every workgroup's K/V stream and a kernel of its own measured 7 us of 390 faster
    const bool fused = c.budget_k > 0 && csa::attention_can_emit(ctx->R) && (int64_t)BH * S <= 2048;
    if (!fused) {
        csa::launch_emit(cand_key, seg_run, cand_cnt, thr, seg_par, sel, BH, c.budget_k, ctx->R, ctx->P,
                         l.cand_keys, st);
        prof.end(4);
    }
    prof.mark(5);
    csa::launch_attention_split(q_dev, ctx->k_cache, ctx->v_cache, ctx->block_table, sel, sel_count, seg_par,
                                part, c.batch, c.n_q_heads, c.n_kv_heads, c.budget_k, ws, ctx->n,
                                c.max_ctx, S, ctx->P, fused ? cand_key : nullptr, seg_run, cand_cnt, thr,
                                ctx->R, l.cand_keys, n_dev, st);
    prof.end(5);
    finish_step(ctx, prof, part, out_dev, S, k_new_dev, v_new_dev, replayable, z_key, st);
    ctx->last_sel = sel;
    ctx->last_scratch = scr;
    ctx->last_sel_count = sel_count;
    return check_launch(ctx);
}

int reuse_step(csa_ctx *ctx, const void *q_dev, float *out_dev, const int32_t *sel_idx_dev,
               const int32_t *sel_count_dev, const void *k_new_dev, const void *v_new_dev, bool replayable,
               void *stream)
{
    if (!ctx || !q_dev || !out_dev) return CSA_ERR_ARG;
    if (replayable && ctx->cfg.stream_window > 0) return CSA_ERR_ARG;
    if ((sel_idx_dev == nullptr) != (sel_count_dev == nullptr)) return CSA_ERR_ARG;
    if (!ctx->bound || !ctx->have_tables) return CSA_ERR_STATE;
    if (k_new_dev && ctx->n >= ctx->cfg.max_ctx) return CSA_ERR_CAPACITY;
    const int32_t *sel = sel_idx_dev ? sel_idx_dev : ctx->last_sel;
    const int32_t *sel_count = sel_count_dev ? sel_count_dev : ctx->last_sel_count;
    if (!sel || !sel_count) return CSA_ERR_STATE;  // no searching step yet
    const csa_config &c = ctx->cfg;
    const Layout &l = ctx->lay;
    hipStream_t st = (hipStream_t)stream;
    const int BH = c.batch * c.n_q_heads;
    void *seg_par = at<void>(ctx->scratch, l.seg_par);
    float *part = at<float>(ctx->scratch, l.part);
    const int ws = window_start(ctx);
    const int S = csa::attention_splits(c.budget_k, ctx->P, (replayable ? c.max_ctx : ctx->n) - ws);
    Prof prof(ctx, st);
    prof.mark(8);
    csa::launch_range_offsets(sel, sel_count, seg_par, BH, c.budget_k, ctx->R, ctx->P, st);
    prof.end(8);
    prof.mark(5);
    csa::launch_attention_split(q_dev, ctx->k_cache, ctx->v_cache, ctx->block_table,
                                const_cast<int32_t *>(sel), sel_count, seg_par, part, c.batch, c.n_q_heads,
                                c.n_kv_heads, c.budget_k, ws, ctx->n, c.max_ctx, S, ctx->P, nullptr, nullptr,
                                nullptr, nullptr, ctx->R, l.cand_keys, replayable ? n_word(ctx) : nullptr, st);
    prof.end(5);
    finish_step(ctx, prof, part, out_dev, S, k_new_dev, v_new_dev, replayable, nullptr, st);
    return check_launch(ctx);
}

}  // namespace

int csa_decode_step(csa_ctx *ctx, const void *q_dev, float *out_dev, int32_t *sel_idx_dev,
                    int32_t *sel_count_dev, void *stream)
{
    return search_step(ctx, ctx ? ctx->scratch : nullptr, q_dev, out_dev, sel_idx_dev, sel_count_dev, nullptr, nullptr, false, stream);
}

int csa_decode_step_static(csa_ctx *ctx, const void *q_dev, float *out_dev, int32_t *sel_idx_dev,
                           int32_t *sel_count_dev, void *stream)
{
    if (!ctx || !q_dev || !out_dev) return CSA_ERR_ARG;
    if (ctx->lay.decode_bytes > kStaticScratchBytes) return CSA_ERR_WORKSPACE;
    if (!ctx->bound || !ctx->have_tables) return CSA_ERR_STATE;  // (before the device is touched)
    char *scr = nullptr;
    const int rc = static_scratch(ctx, &scr);
    if (rc != CSA_OK) return rc;
    return search_step(ctx, scr, q_dev, out_dev, sel_idx_dev, sel_count_dev, nullptr, nullptr, false, stream);
}

int csa_static_scratch_bytes(const csa_ctx *ctx, size_t *needed, size_t *capacity)
{
    if (!ctx) return CSA_ERR_ARG;
    if (needed) *needed = ctx->lay.decode_bytes;
    if (capacity) *capacity = kStaticScratchBytes;
    return CSA_OK;
}

int csa_decode_step_reuse(csa_ctx *ctx, const void *q_dev, float *out_dev, const int32_t *sel_idx_dev,
                          const int32_t *sel_count_dev, void *stream)
{
    return reuse_step(ctx, q_dev, out_dev, sel_idx_dev, sel_count_dev, nullptr, nullptr, false, stream);
}

int csa_decode_step_append(csa_ctx *ctx, const void *q_dev, const void *k_new_dev, const void *v_new_dev,
                           float *out_dev, int32_t *sel_idx_dev, int32_t *sel_count_dev, int32_t reuse,
                           void *stream)
{
    if (!k_new_dev || !v_new_dev) return CSA_ERR_ARG;
    return reuse ? reuse_step(ctx, q_dev, out_dev, sel_idx_dev, sel_count_dev, k_new_dev, v_new_dev, false, stream)
                 : search_step(ctx, ctx ? ctx->scratch : nullptr, q_dev, out_dev, sel_idx_dev, sel_count_dev, k_new_dev,
                               v_new_dev, false, stream);
}

int csa_decode_step_append_replayable(csa_ctx *ctx, const void *q_dev, const void *k_new_dev,
                                      const void *v_new_dev, float *out_dev, int32_t *sel_idx_dev,
                                      int32_t *sel_count_dev, int32_t reuse, void *stream)
{
    if (!k_new_dev || !v_new_dev) return CSA_ERR_ARG;
    return reuse ? reuse_step(ctx, q_dev, out_dev, sel_idx_dev, sel_count_dev, k_new_dev, v_new_dev, true, stream)
                 : search_step(ctx, ctx ? ctx->scratch : nullptr, q_dev, out_dev, sel_idx_dev, sel_count_dev, k_new_dev,
                               v_new_dev, true, stream);
}

int csa_sync_context_len(csa_ctx *ctx, void *stream)
{
    if (!ctx) return CSA_ERR_ARG;
    if (!ctx->bound || !ctx->have_tables) return CSA_ERR_STATE;
    int32_t words[2] = {0, 0};
    hipError_t e = hipMemcpyAsync(words, n_word(ctx), 8, hipMemcpyDeviceToHost, (hipStream_t)stream);
    if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(ctx, e);
    if (words[0] < ctx->n_pre || words[0] > ctx->cfg.max_ctx) return CSA_ERR_STATE;  // (the word was overwritten)
    ctx->n = words[0];
    return words[1] ? CSA_ERR_CAPACITY : CSA_OK;
}

int csa_streaming_status(csa_ctx *ctx, void *stream)
{
    if (!ctx) return CSA_ERR_ARG;
    if (!ctx->bound || !ctx->have_tables) return CSA_ERR_STATE;
    if (ctx->cfg.stream_window <= 0) return CSA_OK;
    int32_t flag = 0;
    hipError_t e = hipMemcpyAsync(&flag, at<int32_t>(ctx->tables, ctx->lay.state), 4, hipMemcpyDeviceToHost,
                                  (hipStream_t)stream);
    if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(ctx, e);
    return flag ? CSA_ERR_RANGE : CSA_OK;
}

int csa_context_len(const csa_ctx *ctx, int32_t *n_pre, int32_t *n)
{
    if (!ctx) return CSA_ERR_ARG;
    if (!ctx->have_tables) return CSA_ERR_STATE;
    if (n_pre) *n_pre = ctx->n_pre;
    if (n) *n = ctx->n;
    return CSA_OK;
}

int csa_set_context_len(csa_ctx *ctx, int32_t n)
{
    if (!ctx) return CSA_ERR_ARG;
    if (!ctx->have_tables) return CSA_ERR_STATE;
    if (n < ctx->n_pre || n > ctx->cfg.max_ctx) return CSA_ERR_ARG;
    if (ctx->cfg.stream_window > 0 && n != ctx->n) return CSA_ERR_STATE;  // the tables hold the appended keys
    ctx->n = n;
    return ctx->bound ? set_device_count(ctx, n) : CSA_OK;
}

int csa_score_frac_bits(const csa_ctx *ctx, int32_t *frac_bits)
{
    if (!ctx || !frac_bits) return CSA_ERR_ARG;
    if (!ctx->have_tables) return CSA_ERR_STATE;
    *frac_bits = ctx->F;
    return CSA_OK;
}

int csa_last_probed_rows(const csa_ctx *ctx, int32_t *rows_dev, void *stream)
{
    if (!ctx || !rows_dev) return CSA_ERR_ARG;
    if (!ctx->bound || !ctx->have_tables) return CSA_ERR_STATE;
    const size_t bytes = (size_t)ctx->cfg.batch * ctx->cfg.n_q_heads * ctx->cfg.n_probe * ctx->cfg.n_subspaces * 4;
    if (!ctx->last_scratch) return CSA_ERR_STATE;  // no searching step since the tables were made
    const hipError_t e = hipMemcpyAsync(rows_dev, ctx->last_scratch + ctx->lay.rows.off, bytes,
                                        hipMemcpyDeviceToDevice, (hipStream_t)stream);
    return e == hipSuccess ? CSA_OK : hip_fail(const_cast<csa_ctx *>(ctx), e);
}

int csa_profile_enable(csa_ctx *ctx, int32_t on)
{
    if (!ctx) return CSA_ERR_ARG;
    ctx->prof = on != 0;
    return CSA_OK;
}

int csa_profile_read(csa_ctx *ctx, double *ms_sum, int64_t *launches)
{
    if (!ctx) return CSA_ERR_ARG;
    for (size_t r = 0; r < ctx->n_recs; ++r) {
        csa_ctx::Rec &rec = ctx->recs[r];
        for (int i = 0; i < CSA_N_STAGES; ++i) {
            if (!rec.done[i]) continue;
            hipError_t e = hipEventSynchronize(rec.ev[i + 1]);
            float ms = 0.0f;
            if (e == hipSuccess) e = hipEventElapsedTime(&ms, rec.ev[i], rec.ev[i + 1]);
            if (e != hipSuccess) return hip_fail(ctx, e);
            if (ms_sum) ms_sum[i] += ms;
            if (launches) launches[i] += 1;
        }
    }
    ctx->n_recs = 0;
    return CSA_OK;
}

const char *csa_stage_name(int32_t stage)
{
    return stage >= 0 && stage < CSA_N_STAGES ? kStageNames[stage] : nullptr;
}

const char *csa_strerror(int status)
{
    switch (status) {
    case CSA_OK: return "ok";
    case CSA_ERR_ARG: return "invalid argument or unsupported configuration";
    case CSA_ERR_STATE: return "call out of order (bind / build tables first)";
    case CSA_ERR_CAPACITY: return "context is at max_ctx";
    case CSA_ERR_WORKSPACE: return "bound buffer smaller than csa_workspace_bytes reports";
    case CSA_ERR_HIP: return "HIP runtime error";
    case CSA_ERR_RANGE: return "table score does not fit the score grid";
    default: return "unknown status";
    }
}

int csa_last_hip_error(const csa_ctx *ctx) { return ctx ? ctx->hip_err : 0; }

}  // extern "C"

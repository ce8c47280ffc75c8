// Offline query clustering (paper Sec. 3.2 (1)): cosine k-means on the l2-normalised prefill
// query sub-vectors of every (KV head, subspace) of a sequence, k-means++ seeding, Lloyd steps over
// all points or over mini-batches.  Centroids are held in bf16 between the steps - the form in which
// the table build consumes them.  All problems of a sequence run side by side (blockIdx.y = problem):
// the k-means++ draws are a chain of C dependent rounds, and one launch per round serves them all.
// The assignment step is the one dense contraction of the library ([points x d_b] . [d_b x C]) and
// runs on the matrix cores; everything else is bandwidth- or latency-bound bookkeeping.
#include "common.h"
#include "kernels.h"

namespace csa {

typedef short v4s __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// The pooled points of the problems of one sequence.  Problem p = (KV head g = p / S, subspace
// p % S); its point i < n_all = G * n_pre is prefill query i % n_pre of query head g * G + i / n_pre
// (q_seq is [Hq][n_pre][128] bf16: the heads of a group are consecutive, so i * 128 works), sub-vector
// [sub * DB, (sub + 1) * DB).  A launch works on a VIEW of the points - every stride-th one from
// `off` on (the whole pool: off 0, stride 1; a mini-batch: one residue class) - and numbers them
// v < n_view; per-point arrays that outlive a view (inv_norm) are indexed by the point itself.
struct Pool {
    const uint16_t *q_seq;
    int n_pre, G, S, DB;
    int n_all, off, stride, n_view;
    __device__ __forceinline__ int gid(int v) const { return off + v * stride; }
    __device__ __forceinline__ const uint16_t *row(int p, int i) const
    {
        const int g = p / S, sub = p - g * S;
        return q_seq + ((size_t)g * G * n_pre + (size_t)i) * kHeadDim + sub * DB;
    }
};

// inv_norm[p][i] = 1 / ||x_i|| of the subspace slice (0 for a zero vector), every point of every
// problem.  One thread per point; grid (ceil(n_all / 256), problems).
template <int DB>
__global__ void k_km_norms(Pool pool, float *__restrict__ inv_norm)
{
    const int i = blockIdx.x * 256 + threadIdx.x, p = blockIdx.y;
    if (i >= pool.n_all) return;
    const uint4 *r = (const uint4 *)pool.row(p, i);
    float nn = 0.0f;
#pragma unroll
    for (int c = 0; c < DB / 8; ++c) {
        const uint4 w = r[c];
        const float f[8] = {bf16_lo(w.x), bf16_hi(w.x), bf16_lo(w.y), bf16_hi(w.y),
                            bf16_lo(w.z), bf16_hi(w.z), bf16_lo(w.w), bf16_hi(w.w)};
#pragma unroll
        for (int e = 0; e < 8; ++e) nn = fmaf(f[e], f[e], nn);
    }
    inv_norm[(size_t)p * pool.n_all + i] = nn > 0.0f ? 1.0f / sqrtf(nn) : 0.0f;
}

// ---------------------------------------------------------------------------------------------
// k-means++ seeding, one round for every problem: seed j = the normalised point `pick` of the view,
// rounded to bf16; every point's squared distance to its nearest seed is brought up to date
// (||x~ - c||^2 = 1 + ||c||^2 - 2 x~.c) and the block's sum of them is written for the next draw.
// Round 0 takes point floor(u_0 * n_view); later rounds the one the previous draw left in pick_dev.
// grid (ceil(n_view / 1024), problems), block 256 (four points per thread).
// ---------------------------------------------------------------------------------------------
constexpr int kSeedPts = 1024;

struct SeedArgs {  // per-problem arrays: problem p's part starts at p * its stride
    const float *inv_norm;  // [n_all]
    float *dist;            // [n_view]
    float *part;            // [n_blk]
    uint16_t *cent16;       // [C * DB]
    int32_t *pick_dev;      // [1]
    const float *u;         // [C] uniforms
    int n_blk, C;
};

template <int DB, bool STRIDED>
__global__ __launch_bounds__(256) void k_km_seed_update(Pool pool, SeedArgs a, int j, int snake)
{
    __shared__ float s_c[DB];
    __shared__ float s_red[4];
    __shared__ float s_cn2;
    const int p = blockIdx.y;
    const float *inv_norm = a.inv_norm + (size_t)p * pool.n_all;
    float *dist = a.dist + (size_t)p * pool.n_view;
    // snake (pools too large for the last-level cache): odd rounds walk the points from the far end -
    // what the previous round read last is what this one reads first, while it is still cached
    const int blk = (snake && (j & 1)) ? (int)(gridDim.x - 1 - blockIdx.x) : (int)blockIdx.x;
    int pick = j == 0 ? (int)((double)a.u[(size_t)p * a.C] * (double)pool.n_view) : a.pick_dev[p];
    pick = min(max(pick, 0), pool.n_view - 1);
    if (threadIdx.x < DB) {
        const int gp = pool.gid(pick);
        const float v = __uint_as_float((uint32_t)pool.row(p, gp)[threadIdx.x] << 16) * inv_norm[gp];
        const uint16_t h = f32_to_bf16_rne(v);
        s_c[threadIdx.x] = __uint_as_float((uint32_t)h << 16);
        if (blockIdx.x == 0) a.cent16[((size_t)p * a.C + j) * DB + threadIdx.x] = h;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        float cn2 = 0.0f;
        for (int t = 0; t < DB; ++t) cn2 = fmaf(s_c[t], s_c[t], cn2);
        s_cn2 = cn2;
    }
    __syncthreads();
    const float cn2 = s_cn2;
    float local = 0.0f;
    if (STRIDED) {
        // a mini-batch: its rows are far apart and mostly cached - one point per thread with all of its
        // chunks requested at once measured faster (0.34 against 0.41 s for 4096 draws)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = blk * kSeedPts + u * 256 + threadIdx.x;
            if (i < pool.n_view) {
                const int gi = pool.gid(i);
                const uint4 *r = (const uint4 *)pool.row(p, gi);
                float dot = 0.0f;
#pragma unroll
                for (int c = 0; c < DB / 8; ++c) {
                    const uint4 w = r[c];
                    const float f[8] = {bf16_lo(w.x), bf16_hi(w.x), bf16_lo(w.y), bf16_hi(w.y),
                                        bf16_lo(w.z), bf16_hi(w.z), bf16_lo(w.w), bf16_hi(w.w)};
#pragma unroll
                    for (int e = 0; e < 8; ++e) dot = fmaf(f[e], s_c[c * 8 + e], dot);
                }
                const float inv = inv_norm[gi];
                float d = inv > 0.0f ? fmaxf(0.0f, 1.0f + cn2 - 2.0f * inv * dot) : cn2;
                if (j > 0) d = fminf(d, dist[i]);
                dist[i] = d;
                local += d;
            }
        }
    } else {
    // the whole pool, streamed from HBM: LPR lanes share a point (16 bytes of its sub-vector each), so a
    // wave instruction reads whole, consecutive rows - coalesced whatever the sub-vector's length
    constexpr int LPR = DB / 8, RPW = kWave / LPR, PER_WAVE = kSeedPts / 4;
    constexpr int UNR = PER_WAVE / RPW < 4 ? PER_WAVE / RPW : 4;  // rows requested ahead per lane
    const int c = lane_id() % LPR, rsub = lane_id() / LPR;
    float cf[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) cf[e] = s_c[c * 8 + e];
    const int base = blk * kSeedPts + (int)(threadIdx.x / kWave) * PER_WAVE + rsub;
    for (int it0 = 0; it0 < PER_WAVE / RPW; it0 += UNR) {
        uint4 w[UNR];
        int idx[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            idx[u] = base + (it0 + u) * RPW;
            w[u] = make_uint4(0, 0, 0, 0);
            if (idx[u] < pool.n_view) w[u] = *(const uint4 *)(pool.row(p, pool.gid(idx[u])) + c * 8);
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const float f[8] = {bf16_lo(w[u].x), bf16_hi(w[u].x), bf16_lo(w[u].y), bf16_hi(w[u].y),
                                bf16_lo(w[u].z), bf16_hi(w[u].z), bf16_lo(w[u].w), bf16_hi(w[u].w)};
            float dot = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) dot = fmaf(f[e], cf[e], dot);
#pragma unroll
            for (int o = 1; o < LPR; o <<= 1) dot += __shfl_xor(dot, o, kWave);
            if (c == 0 && idx[u] < pool.n_view) {
                const float inv = inv_norm[pool.gid(idx[u])];
                float d = inv > 0.0f ? fmaxf(0.0f, 1.0f + cn2 - 2.0f * inv * dot) : cn2;
                if (j > 0) d = fminf(d, dist[idx[u]]);
                dist[idx[u]] = d;
                local += d;
            }
        }
    }
    }
    local = __shfl_xor(local, 1, kWave) + local;
    local = __shfl_xor(local, 2, kWave) + local;
    local = __shfl_xor(local, 4, kWave) + local;
    local = __shfl_xor(local, 8, kWave) + local;
    local = __shfl_xor(local, 16, kWave) + local;
    local = __shfl_xor(local, 32, kWave) + local;
    if (lane_id() == 0) s_red[threadIdx.x / kWave] = local;
    __syncthreads();
    if (threadIdx.x == 0) a.part[(size_t)p * a.n_blk + blk] = (s_red[0] + s_red[1]) + (s_red[2] + s_red[3]);
}

// The draw: the first point whose running sum of distances exceeds u * total (the last point if
// none does).  Found in two levels: the block sums first, then the points of that block.
// grid problems, block 1024; j = the seed being drawn (its uniform is u[j]).
__global__ __launch_bounds__(1024) void k_km_seed_pick(SeedArgs a, int n_pool, int j)
{
    const int prob = blockIdx.x;
    const float *dist = a.dist + (size_t)prob * n_pool;
    const float *part = a.part + (size_t)prob * a.n_blk;
    const int n_blk = a.n_blk;
    const float u = a.u[(size_t)prob * a.C + j];
    int32_t *pick_dev = a.pick_dev + prob;
    __shared__ float s_tmp[1024 / kWave + 1];
    __shared__ float s_carry;
    __shared__ int s_hit;
    auto block_incl_scan_f = [&](float v, float &total) {
        float incl = v;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const float t = __shfl_up(incl, o, kWave);
            if (lane_id() >= o) incl += t;
        }
        if (lane_id() == kWave - 1) s_tmp[threadIdx.x / kWave] = incl;
        __syncthreads();
        float off = 0.0f, tot = 0.0f;
        for (int w = 0; w < 1024 / kWave; ++w) {
            const float t = s_tmp[w];
            if (w < (int)(threadIdx.x / kWave)) off += t;
            tot += t;
        }
        __syncthreads();
        total = tot;
        return off + incl;
    };
    // total of all block sums
    float acc = 0.0f;
    for (int b = threadIdx.x; b < n_blk; b += 1024) acc += part[b];
    float total;
    block_incl_scan_f(acc, total);
    const float target = u * total;
    // the block in which the running sum first exceeds the target
    constexpr int kNone = 0x7FFFFFFF;
    if (threadIdx.x == 0) { s_carry = 0.0f; s_hit = kNone; }
    __syncthreads();
    for (int b0 = 0; b0 < n_blk && s_hit == kNone; b0 += 1024) {
        const int b = b0 + threadIdx.x;
        float chunk_total;
        const float incl = s_carry + block_incl_scan_f(b < n_blk ? part[b] : 0.0f, chunk_total);
        if (b < n_blk && incl > target) atomicMin(&s_hit, b);
        __syncthreads();
        if (threadIdx.x == 0 && s_hit == kNone) s_carry += chunk_total;
        __syncthreads();
    }
    int pick = n_pool - 1;
    if (s_hit != kNone) {
        // prefix before the block = carry of the chunk + the partial sums before it in the chunk
        const int hit = s_hit;
        float before = 0.0f;
        {
            const int c0 = hit / 1024 * 1024;
            float v = 0.0f;
            const int b = c0 + threadIdx.x;
            if (b < hit) v = part[b];
            float t;
            block_incl_scan_f(v, t);
            before = s_carry + t;
        }
        const int i = hit * kSeedPts + threadIdx.x;
        float t;
        const float incl = before + block_incl_scan_f(i < n_pool ? dist[i] : 0.0f, t);
        __syncthreads();
        if (threadIdx.x == 0) s_hit = kNone;
        __syncthreads();
        if (i < n_pool && incl > target) atomicMin(&s_hit, i);
        __syncthreads();
        // (if rounding lets the running sum miss the target inside the block, its last point)
        pick = s_hit != kNone ? s_hit : min(hit * kSeedPts + kSeedPts - 1, n_pool - 1);
    }
    if (threadIdx.x == 0) *pick_dev = pick;
}

// ---------------------------------------------------------------------------------------------
// Lloyd step, first half: cosine assignment.  A workgroup takes 128 or 256 points, a wave one or
// two blocks of 32 of them, held as the B operands for the whole kernel (with two blocks every A
// operand read from LDS feeds two matrix instructions); the centroids pass through LDS 64 at a time (two
// buffers: the next tile is fetched while this one is used, one barrier per tile) and each 32 of
// them are one 32x32 block of inner products on the matrix cores (32x32x16 bf16: centroids as
// rows, points as columns, so a lane ends up with 16 centroid scores of ONE point and keeps a
// running arg-max in registers; the two lanes that share a point are merged at the end).  The
// arg-max first takes the block's maximum per lane and walks the 16 scores only when some lane's
// maximum beats its best so far - rare once a few tiles are done.  Ties go to the lower centroid.
// Positive scaling of a point does not change its arg-max, so the raw bf16 sub-vector is the B
// operand and the normalisation only enters the sums.
// What follows the assignment depends on the size of the sums.  When all C * d_b of them fit in
// LDS (few, short centroids: the paper's default geometry) every point adds its normalised
// sub-vector to its centroid's sum there and the workgroup flushes once (fp32 atomics: the order
// of these additions is not fixed).  Otherwise the kernel only records the assignment and counts
// the members; the sums are then taken per centroid over its member list (k_km_offsets,
// k_km_scatter, k_km_sum below) - adding 128 values per point with global atomics took three
// times as long as the matrix products.
// grid (point tiles of 128 or 256 - capped when the sums go through LDS - , problems), block 256, dynamic LDS lds_sums ? (C * DB + C) * 4 : 0 bytes.
// ---------------------------------------------------------------------------------------------
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
union Frag8 {  // eight bf16 values: as loaded (16 bytes) and as a matrix operand
    uint4 u;
    v8bf v;
};
constexpr int kKmTile = 64;  // centroids per LDS buffer

// blocks of 32 points per wave (one A read serves as many products): two for short sub-vectors, where
// the sums go through LDS and half as many workgroups flush them; one for long ones, where the
// registers of a second block cost more occupancy than the saved LDS reads bring
template <int DB>
constexpr int km_cols() { return DB <= 32 ? 2 : 1; }

struct StepArgs {  // per-problem arrays of a Lloyd step (problem p's part at p * its stride)
    const float *inv_norm;  // [n_all]
    uint16_t *cent16;       // [C * DB]
    float *sums;            // [C * DB]
    int32_t *counts;        // [C]   members in this step's view
    int32_t *run_cnt;       // [C]   members over all steps so far (mini-batches)
    float *cos_sum;         // [1]
    int32_t *assign_out;    // [n_all] or NULL (indexed by the point)
    int32_t *assign_work;   // [view_cap] (indexed within the view)
    int32_t *start, *cursor;  // [C + 1] each
    int32_t *member;        // [view_cap]
    float *mean_cos_out;    // [iters] or NULL
    int C, view_cap, iters;
};

template <int DB>
__global__ __launch_bounds__(256) void k_km_assign(Pool pool, StepArgs a, int write_assign, int lds_sums)
{
    const int prob = blockIdx.y, C = a.C;
    const float *inv_norm = a.inv_norm + (size_t)prob * pool.n_all;
    const uint16_t *cent16 = a.cent16 + (size_t)prob * C * DB;
    float *sums = a.sums + (size_t)prob * C * DB;
    int32_t *counts = a.counts + (size_t)prob * C;
    float *cos_sum = a.cos_sum + prob;
    int32_t *assign_out = write_assign && a.assign_out ? a.assign_out + (size_t)prob * pool.n_all : nullptr;
    int32_t *assign_work = a.assign_work + (size_t)prob * a.view_cap;
    extern __shared__ float s_sum[];             // [C * DB] sums, then [C] counts (as floats), if lds_sums
    constexpr int NK = (DB + 15) / 16;           // matrix instructions per 32x32 block
    constexpr int STRIDE = DB + 8;               // LDS row stride in elements (16-byte reads without conflicts)
    constexpr int CH = DB / 8;                   // 16-byte chunks of a centroid
    constexpr int PER = (kKmTile * CH + 255) / 256;  // chunks of a tile per thread
    constexpr int CB = km_cols<DB>();
    constexpr int kKmPts = 4 * 32 * CB;          // points per workgroup
    __shared__ __align__(16) uint16_t s_c[2][kKmTile * STRIDE];
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const int col = lane & 31, half = lane >> 5;
    if (lds_sums)
        for (int e = threadIdx.x; e < C * DB + C; e += 256) s_sum[e] = 0.0f;
    // a workgroup takes point tiles in turn (the grid is capped when the sums go through LDS, so that
    // few workgroups flush them: the flush is C * (DB + 1) global atomics per workgroup)
    float cs = 0.0f;
    const int n_tiles = (pool.n_view + kKmPts - 1) / kKmPts;
    for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        __syncthreads();  // (the centroid tiles of the previous point tile are done with)
        int pt[CB];
        bool live[CB];
        // operand element k of instruction kk is dimension 16 * kk + k; a lane holds k = 8 * half .. + 7
        // (zeros past d_b: only for 8-dimensional sub-vectors)
        Frag8 bq[CB][NK];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            pt[cb] = tile * kKmPts + (wave * CB + cb) * 32 + col;  // (within the view)
            live[cb] = pt[cb] < pool.n_view;
            const uint16_t *r = pool.row(prob, pool.gid(live[cb] ? pt[cb] : 0));
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) {
                const int e0 = 16 * kk + 8 * half;
                bq[cb][kk].u = make_uint4(0, 0, 0, 0);
                if (live[cb] && e0 < DB) bq[cb][kk].u = *(const uint4 *)(r + e0);
            }
        }
        uint4 pre[PER];
        auto fetch = [&](int t0) {  // this thread's chunks of the tile that starts at centroid t0 (zeros past C)
#pragma unroll
            for (int u = 0; u < PER; ++u) {
                const int e = u * 256 + (int)threadIdx.x, i = e / CH, c = e % CH;
                pre[u] = make_uint4(0, 0, 0, 0);
                if (e < kKmTile * CH && t0 + i < C) pre[u] = *(const uint4 *)(cent16 + (size_t)(t0 + i) * DB + c * 8);
            }
        };
        auto stash = [&](int buf) {
#pragma unroll
            for (int u = 0; u < PER; ++u) {
                const int e = u * 256 + (int)threadIdx.x, i = e / CH, c = e % CH;
                if (e < kKmTile * CH) *(uint4 *)(s_c[buf] + i * STRIDE + c * 8) = pre[u];
            }
        };
        fetch(0);
        stash(0);
        __syncthreads();
        float best[CB];
        int best_j[CB];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            best[cb] = -INFINITY;
            best_j[cb] = 0;
        }
        int buf = 0;
        for (int t0 = 0; t0 < C; t0 += kKmTile, buf ^= 1) {
            const bool more = t0 + kKmTile < C;
            if (more) fetch(t0 + kKmTile);
            v16f acc[2][CB];
#pragma unroll
            for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[rt][cb][r] = 0.0f;
#pragma unroll
            for (int kk = 0; kk < NK; ++kk) {
                const int e0 = 16 * kk + 8 * half;
#pragma unroll
                for (int rt = 0; rt < 2; ++rt) {  // (independent accumulation chains)
                    Frag8 a;
                    a.u = make_uint4(0, 0, 0, 0);
                    if (e0 < DB) a.u = *(const uint4 *)(s_c[buf] + (rt * 32 + col) * STRIDE + e0);
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb)
                        acc[rt][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, bq[cb][kk].v, acc[rt][cb], 0, 0, 0);
                }
            }
            // register r of this lane: centroid row (r % 4) + 8 * (r / 4) + 4 * half of the block,
            // column = its point
#pragma unroll
            for (int rt = 0; rt < 2; ++rt)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
                    float tm = acc[rt][cb][0];
#pragma unroll
                    for (int r = 1; r < 16; ++r) tm = fmaxf(tm, acc[rt][cb][r]);
                    if (__any(tm > best[cb])) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int j = t0 + rt * 32 + (r & 3) + 8 * (r >> 2) + 4 * half;
                            if (j < C && acc[rt][cb][r] > best[cb]) {
                                best[cb] = acc[rt][cb][r];
                                best_j[cb] = j;
                            }
                        }
                    }
                }
            if (more) stash(buf ^ 1);
            __syncthreads();
        }
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            {
                const float ob = __shfl_xor(best[cb], 32, kWave);
                const int oj = __shfl_xor(best_j[cb], 32, kWave);
                if (ob > best[cb] || (ob == best[cb] && oj < best_j[cb])) {
                    best[cb] = ob;
                    best_j[cb] = oj;
                }
            }
            const float inv = live[cb] ? inv_norm[pool.gid(pt[cb])] : 0.0f;
            if (live[cb]) {
                if (lds_sums) {
                    float *dst = s_sum + (size_t)best_j[cb] * DB;
#pragma unroll
                    for (int kk = 0; kk < NK; ++kk) {
                        const int e0 = 16 * kk + 8 * half;
                        if (e0 < DB) {
                            const uint32_t w[4] = {bq[cb][kk].u.x, bq[cb][kk].u.y, bq[cb][kk].u.z, bq[cb][kk].u.w};
#pragma unroll
                            for (int x = 0; x < 4; ++x) {
                                atomicAdd(dst + e0 + 2 * x, bf16_lo(w[x]) * inv);
                                atomicAdd(dst + e0 + 2 * x + 1, bf16_hi(w[x]) * inv);
                            }
                        }
                    }
                }
                if (half == 0) {
                    if (lds_sums) atomicAdd(s_sum + C * DB + best_j[cb], 1.0f);
                    else {
                        atomicAdd(counts + best_j[cb], 1);
                        assign_work[pt[cb]] = best_j[cb];
                    }
                    if (assign_out) assign_out[pool.gid(pt[cb])] = best_j[cb];
                }
            }
            cs += (live[cb] && half == 0) ? best[cb] * inv : 0.0f;
        }
    }
    if (lds_sums) {
        __syncthreads();
        for (int e = threadIdx.x; e < C * DB; e += 256) {
            const float v = s_sum[e];
            if (v != 0.0f) atomicAdd(sums + e, v);
        }
        for (int j = threadIdx.x; j < C; j += 256) {
            const float v = s_sum[C * DB + j];
            if (v != 0.0f) atomicAdd(counts + j, (int)v);   // (<= 256 members per workgroup: exact)
        }
    }
    for (int o = 32; o > 0; o >>= 1) cs += __shfl_xor(cs, o, kWave);
    if (lane == 0) atomicAdd(cos_sum, cs);
}

// Member lists for the sums of a Lloyd step with many or long centroids.
// k_km_offsets: exclusive scan of the member counts -> where each centroid's list starts (kept as
// the running write position of the scatter, and a second copy as the start).  One workgroup per
// problem.
__global__ __launch_bounds__(1024) void k_km_offsets(StepArgs a)
{
    const int prob = blockIdx.x, C = a.C;
    const int32_t *counts = a.counts + (size_t)prob * C;
    int32_t *start = a.start + (size_t)prob * (C + 1), *cursor = a.cursor + (size_t)prob * (C + 1);
    __shared__ int s_w[1024 / kWave + 1];
    __shared__ int s_carry;
    if (threadIdx.x == 0) s_carry = 0;
    __syncthreads();
    for (int j0 = 0; j0 < C; j0 += 1024) {
        const int j = j0 + threadIdx.x;
        const int v = j < C ? counts[j] : 0;
        int incl = v;
        for (int o = 1; o < kWave; o <<= 1) {
            const int t = __shfl_up(incl, o, kWave);
            if (lane_id() >= o) incl += t;
        }
        if (lane_id() == kWave - 1) s_w[threadIdx.x / kWave] = incl;
        __syncthreads();
        int before = s_carry;
        for (int w = 0; w < (int)threadIdx.x / kWave; ++w) before += s_w[w];
        if (j < C) {
            start[j] = before + incl - v;
            cursor[j] = before + incl - v;
        }
        __syncthreads();
        if (threadIdx.x == 1023) s_carry = before + incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) start[C] = s_carry;
}

// k_km_scatter: point v of the view goes to the next free place of its centroid's list.
// grid (ceil(n_view / 256), problems).
__global__ void k_km_scatter(StepArgs a, int n_view)
{
    const int v = blockIdx.x * 256 + threadIdx.x, prob = blockIdx.y;
    if (v >= n_view) return;
    const int32_t *assign = a.assign_work + (size_t)prob * a.view_cap;
    int32_t *cursor = a.cursor + (size_t)prob * (a.C + 1);
    int32_t *member = a.member + (size_t)prob * a.view_cap;
    member[atomicAdd(cursor + assign[v], 1)] = v;
}

// k_km_sum: sums[j][:] (+)= sum over the members i of centroid j of x_i / ||x_i||, one wave per
// centroid; a group of DB/8 lanes reads one member's sub-vector (16 bytes per lane), the groups of
// the wave take members in turn and are folded at the end.  No atomics.  keep: the sums run on over
// the steps (mini-batches) instead of starting over.  grid (ceil(C / 4), problems), block 256.
template <int DB>
__global__ __launch_bounds__(256) void k_km_sum(Pool pool, StepArgs a, int keep)
{
    constexpr int LPR = DB / 8;        // lanes per member row
    constexpr int GROUPS = kWave / LPR;  // members in flight per wave
    const int prob = blockIdx.y, C = a.C;
    const int j = blockIdx.x * 4 + threadIdx.x / kWave;
    if (j >= C) return;  // (whole waves)
    const float *inv_norm = a.inv_norm + (size_t)prob * pool.n_all;
    const int32_t *start = a.start + (size_t)prob * (C + 1);
    const int32_t *member = a.member + (size_t)prob * a.view_cap;
    float *sums = a.sums + (size_t)prob * C * DB;
    const int lane = lane_id(), grp = lane / LPR, c = lane % LPR;
    const int m0 = start[j], m1 = start[j + 1];
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
    for (int m = m0 + grp; m < m1; m += GROUPS) {
        const int i = pool.gid(member[m]);
        const float inv = inv_norm[i];
        const uint4 w = *(const uint4 *)(pool.row(prob, i) + c * 8);
        acc[0] = fmaf(bf16_lo(w.x), inv, acc[0]); acc[1] = fmaf(bf16_hi(w.x), inv, acc[1]);
        acc[2] = fmaf(bf16_lo(w.y), inv, acc[2]); acc[3] = fmaf(bf16_hi(w.y), inv, acc[3]);
        acc[4] = fmaf(bf16_lo(w.z), inv, acc[4]); acc[5] = fmaf(bf16_hi(w.z), inv, acc[5]);
        acc[6] = fmaf(bf16_lo(w.w), inv, acc[6]); acc[7] = fmaf(bf16_hi(w.w), inv, acc[7]);
    }
    // fold the groups: lanes c, c + LPR, c + 2 LPR, ...
#pragma unroll
    for (int o = LPR; o < kWave; o <<= 1)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += __shfl_xor(acc[e], o, kWave);
    if (grp == 0) {
        float4 *dst = (float4 *)(sums + (size_t)j * DB + c * 8);
        if (keep) {
            const float4 p0 = dst[0], p1 = dst[1];
            acc[0] += p0.x; acc[1] += p0.y; acc[2] += p0.z; acc[3] += p0.w;
            acc[4] += p1.x; acc[5] += p1.y; acc[6] += p1.z; acc[7] += p1.w;
        }
        dst[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
        dst[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
    }
}

// Lloyd step, second half: centroid <- its sum re-normalised and rounded to bf16 (a cluster without
// a member keeps its centroid); the step's mean best cosine is written out.  Full-batch steps start
// over: sums and counts are cleared.  Mini-batch steps (keep) run on: the sums stay, the view's
// counts go into the running counts, and "without a member" means none in any step so far.
// One wave per centroid.  grid (ceil(C / 4), problems), block 256.
template <int DB>
__global__ __launch_bounds__(256) void k_km_finish(StepArgs a, int step, int n_view, int keep)
{
    const int prob = blockIdx.y, C = a.C;
    float *sums = a.sums + (size_t)prob * C * DB;
    int32_t *counts = a.counts + (size_t)prob * C, *run_cnt = a.run_cnt + (size_t)prob * C;
    uint16_t *cent16 = a.cent16 + (size_t)prob * C * DB;
    const int j = blockIdx.x * 4 + threadIdx.x / kWave;
    const int lane = lane_id();
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        float *cos_sum = a.cos_sum + prob;
        if (a.mean_cos_out) a.mean_cos_out[(size_t)prob * a.iters + step] = n_view > 0 ? *cos_sum / (float)n_view : 0.0f;
        *cos_sum = 0.0f;
    }
    if (j >= C) return;
    float v[2] = {0.0f, 0.0f}, nn = 0.0f;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int e = u * kWave + lane;
        if (e < DB) {
            v[u] = sums[(size_t)j * DB + e];
            if (!keep) sums[(size_t)j * DB + e] = 0.0f;
            nn = fmaf(v[u], v[u], nn);
        }
    }
    for (int o = 32; o > 0; o >>= 1) nn += __shfl_xor(nn, o, kWave);
    const int cnt = counts[j] + (keep ? run_cnt[j] : 0);
    if (cnt > 0 && nn > 0.0f) {
        const float inv = 1.0f / sqrtf(nn);
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int e = u * kWave + lane;
            if (e < DB) cent16[(size_t)j * DB + e] = f32_to_bf16_rne(v[u] * inv);
        }
    }
    if (lane == 0) {
        if (keep) run_cnt[j] = cnt;
        counts[j] = 0;
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
namespace {

size_t up256(size_t x) { return (x + 255) / 256 * 256; }

struct WorkLayout {
    size_t inv_norm, dist, part, sums, counts, run_cnt, cent16, pick, cos_sum, assign_work, start, cursor, bytes;
    int n_blk, cap;
};

// n_prob problems of n_all points each; the largest view holds cap = ceil(n_all / n_batches) points
WorkLayout work_layout(int n_prob, int n_all, int C, int db, int n_batches)
{
    WorkLayout w;
    w.cap = (n_all + n_batches - 1) / n_batches;
    w.n_blk = (w.cap + kSeedPts - 1) / kSeedPts;
    size_t off = 0;
    auto put = [&](size_t &at, size_t bytes) { at = off; off += up256(bytes); };
    const size_t P = (size_t)n_prob;
    put(w.inv_norm, P * n_all * 4);
    put(w.dist, P * w.cap * 4);  // the seeding's distances; afterwards the member lists of the Lloyd steps
    put(w.part, P * w.n_blk * 4);
    put(w.sums, P * C * db * 4);  // sums, counts and running counts are cleared together
    put(w.counts, P * C * 4);
    put(w.run_cnt, P * C * 4);
    put(w.cent16, P * C * db * 2);
    put(w.pick, P * 4);
    put(w.cos_sum, P * 4);
    put(w.assign_work, P * w.cap * 4);
    put(w.start, P * (C + 1) * 4);
    put(w.cursor, P * (C + 1) * 4);
    w.bytes = off;
    return w;
}

template <int DB>
hipError_t cluster_sequence_db(const uint16_t *q_seq, int n_pre, int G, int Hkv, int S, int C, int iters,
                               int n_batches, const float *u_seed, const uint16_t *init, uint16_t *out,
                               float *mean_cos_out, int32_t *assign_out, char *work, hipStream_t st)
{
    const int n_prob = Hkv * S, n_all = G * n_pre;
    const WorkLayout w = work_layout(n_prob, n_all, C, DB, n_batches);
    float *inv_norm = (float *)(work + w.inv_norm);
    uint16_t *cent16 = (uint16_t *)(work + w.cent16);
    auto view = [&](int t) {  // the points of step t: every n_batches-th one from t % n_batches on
        Pool p{q_seq, n_pre, G, S, DB, n_all, t % n_batches, n_batches, 0};
        p.n_view = (n_all - p.off + n_batches - 1) / n_batches;
        return p;
    };
    hipError_t e = hipMemsetAsync(work + w.sums, 0, w.cent16 - w.sums, st);  // sums, counts, running counts
    if (e == hipSuccess) e = hipMemsetAsync(work + w.pick, 0, w.assign_work - w.pick, st);
    if (e != hipSuccess) return e;
    const Pool all = view(0);
    {
        Pool whole = all;
        whole.off = 0; whole.stride = 1; whole.n_view = n_all;
        k_km_norms<DB><<<dim3((n_all + 255) / 256, n_prob), 256, 0, st>>>(whole, inv_norm);
    }
    if (init) {
        e = hipMemcpyAsync(cent16, init, (size_t)n_prob * C * DB * 2, hipMemcpyDeviceToDevice, st);
        if (e != hipSuccess) return e;
    } else {
        // k-means++ over the first view; one launch per round serves every problem
        const SeedArgs sa{inv_norm, (float *)(work + w.dist), (float *)(work + w.part), cent16,
                          (int32_t *)(work + w.pick), u_seed, w.n_blk, C};
        const int snake = (size_t)all.n_view * DB * 2 * n_prob > ((size_t)64 << 20) ? 1 : 0;
        for (int j = 0; j < C; ++j) {
            if (all.stride > 1)
                k_km_seed_update<DB, true><<<dim3(w.n_blk, n_prob), 256, 0, st>>>(all, sa, j, snake);
            else
                k_km_seed_update<DB, false><<<dim3(w.n_blk, n_prob), 256, 0, st>>>(all, sa, j, snake);
            if (j + 1 < C) k_km_seed_pick<<<n_prob, 1024, 0, st>>>(sa, all.n_view, j + 1);
        }
    }
    if (assign_out && n_batches > 1) {  // points outside the last step's batch have no assignment: -1
        e = hipMemsetAsync(assign_out, 0xFF, (size_t)n_prob * n_all * 4, st);
        if (e != hipSuccess) return e;
    }
    // sums in LDS: up to 32 KiB of them, and within the 64 KiB a workgroup may use together with the
    // kernel's two centroid tiles
    const size_t tiles = 2 * (size_t)kKmTile * (DB + 8) * 2;
    const int lds_sums = ((size_t)C * DB + C <= 8192 && ((size_t)C * DB + C) * 4 + tiles <= 65536) ? 1 : 0;
    const size_t lds_bytes = lds_sums ? ((size_t)C * DB + C) * 4 : 0;
    const int keep = n_batches > 1 ? 1 : 0;
    const StepArgs a{inv_norm, cent16, (float *)(work + w.sums), (int32_t *)(work + w.counts),
                     (int32_t *)(work + w.run_cnt), (float *)(work + w.cos_sum), assign_out,
                     (int32_t *)(work + w.assign_work), (int32_t *)(work + w.start), (int32_t *)(work + w.cursor),
                     (int32_t *)(work + w.dist), mean_cos_out, C, w.cap, iters > 0 ? iters : 1};
    constexpr int kPts = 128 * km_cols<DB>();
    for (int it = 0; it < iters; ++it) {
        const Pool p = view(it);
        int tiles = (p.n_view + kPts - 1) / kPts;
        if (lds_sums) {  // about eight workgroups per CU in all
            const int cap = (2048 + n_prob - 1) / n_prob;
            if (tiles > cap) tiles = cap;
        }
        k_km_assign<DB><<<dim3(tiles, n_prob), 256, lds_bytes, st>>>(p, a, it + 1 == iters, lds_sums);
        if (!lds_sums) {
            k_km_offsets<<<n_prob, 1024, 0, st>>>(a);
            k_km_scatter<<<dim3((p.n_view + 255) / 256, n_prob), 256, 0, st>>>(a, p.n_view);
            k_km_sum<DB><<<dim3((C + 3) / 4, n_prob), 256, 0, st>>>(p, a, keep);
        }
        k_km_finish<DB><<<dim3((C + 3) / 4, n_prob), 256, 0, st>>>(a, it, p.n_view, keep);
    }
    e = hipMemcpyAsync(out, cent16, (size_t)n_prob * C * DB * 2, hipMemcpyDeviceToDevice, st);
    if (e != hipSuccess) return e;
    return hipGetLastError();
}

}  // namespace

size_t cluster_work_bytes(int n_prob, int n_all, int C, int db)
{
    return work_layout(n_prob, n_all, C, db, 1).bytes;  // (one batch: the largest views)
}

// All (KV head, subspace) problems of one sequence.  q_seq: [Hq][n_pre][128] bf16 of the sequence;
// u_seed: device fp32 [Hkv*S][C] or NULL; init / out: device bf16 [Hkv*S][C][128/S]; mean_cos_out: device
// [Hkv*S][max(iters,1)] or NULL; assign_out: device [Hkv*S][G*n_pre] or NULL.
int cluster_sequence(const void *q_seq, int n_pre, int G, int Hkv, int S, int C, int iters, int n_batches,
                     const float *u_seed, const void *init, void *out, float *mean_cos_out,
                     int32_t *assign_out, void *work, hipStream_t st)
{
#define CSA_KM(DB_)                                                                                      \
    return (int)cluster_sequence_db<DB_>((const uint16_t *)q_seq, n_pre, G, Hkv, S, C, iters, n_batches, \
                                         u_seed, (const uint16_t *)init, (uint16_t *)out, mean_cos_out,  \
                                         assign_out, (char *)work, st)
    switch (S) {
    case 1: CSA_KM(128);
    case 2: CSA_KM(64);
    case 4: CSA_KM(32);
    case 8: CSA_KM(16);
    default: CSA_KM(8);  // 16
    }
#undef CSA_KM
}

}  // namespace csa

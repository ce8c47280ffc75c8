// Offline query clustering (paper Sec. 3.2 (1)): cosine k-means on the l2-normalised prefill
// query sub-vectors of one (KV head, subspace), k-means++ seeding, full-batch Lloyd steps.
// Centroids are held in bf16 between the steps - the form in which the table build consumes them.
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

// The pooled points of KV head (b, g): point i < G * n_pre is prefill query i % n_pre of query
// head g * G + i / n_pre; q_pre is [B][Hq][n_pre][128] bf16.  Returns the point's subspace slice.
struct Pool {
    const uint16_t *q;  // q_pre + the first row of query head (b, g * G)
    int n_pre, n_pool, sub_off;
    __device__ __forceinline__ const uint16_t *row(int i) const
    {
        return q + (size_t)i * kHeadDim + sub_off;  // (heads of a group are consecutive: i*128 works)
    }
};

// inv_norm[i] = 1 / ||x_i|| of the subspace slice (0 for a zero vector).  One thread per point.
template <int DB>
__global__ void k_km_norms(Pool pool, float *__restrict__ inv_norm)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= pool.n_pool) return;
    const uint4 *r = (const uint4 *)pool.row(i);
    float nn = 0.0f;
#pragma unroll
    for (int c = 0; c < DB / 8; ++c) {
        const uint4 w = r[c];
        const float f[8] = {bf16_lo(w.x), bf16_hi(w.x), bf16_lo(w.y), bf16_hi(w.y),
                            bf16_lo(w.z), bf16_hi(w.z), bf16_lo(w.w), bf16_hi(w.w)};
#pragma unroll
        for (int e = 0; e < 8; ++e) nn = fmaf(f[e], f[e], nn);
    }
    inv_norm[i] = nn > 0.0f ? 1.0f / sqrtf(nn) : 0.0f;
}

// ---------------------------------------------------------------------------------------------
// k-means++ seeding, one round: seed j = the normalised point `pick` rounded to bf16; every
// point's squared distance to its nearest seed is brought up to date (||x~ - c||^2 =
// 1 + ||c||^2 - 2 x~.c) and the block's sum of them is written for the next draw.
// pick_host >= 0: the point to take; < 0: the one the previous draw left in *pick_dev.
// grid ceil(n_pool / 1024), block 256 (four points per thread).
// ---------------------------------------------------------------------------------------------
constexpr int kSeedPts = 1024;

template <int DB>
__global__ __launch_bounds__(256) void k_km_seed_update(Pool pool, const float *__restrict__ inv_norm,
                                                        float *__restrict__ dist,
                                                        float *__restrict__ part,
                                                        uint16_t *__restrict__ cent16,
                                                        const int32_t *__restrict__ pick_dev,
                                                        int pick_host, int j, int snake)
{
    __shared__ float s_c[DB];
    __shared__ float s_red[4];
    __shared__ float s_cn2;
    // snake (pools too large for the last-level cache): odd rounds walk the points from the far end -
    // what the previous round read last is what this one reads first, while it is still cached
    const int blk = (snake && (j & 1)) ? (int)(gridDim.x - 1 - blockIdx.x) : (int)blockIdx.x;
    int pick = pick_host >= 0 ? pick_host : *pick_dev;
    pick = min(max(pick, 0), pool.n_pool - 1);
    if (threadIdx.x < DB) {
        const float v = __uint_as_float((uint32_t)pool.row(pick)[threadIdx.x] << 16) * inv_norm[pick];
        const uint16_t h = f32_to_bf16_rne(v);
        s_c[threadIdx.x] = __uint_as_float((uint32_t)h << 16);
        if (blockIdx.x == 0) cent16[(size_t)j * DB + threadIdx.x] = h;
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
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int i = blk * kSeedPts + u * 256 + threadIdx.x;
        if (i < pool.n_pool) {
            const uint4 *r = (const uint4 *)pool.row(i);
            float dot = 0.0f;
#pragma unroll
            for (int c = 0; c < DB / 8; ++c) {
                const uint4 w = r[c];
                const float f[8] = {bf16_lo(w.x), bf16_hi(w.x), bf16_lo(w.y), bf16_hi(w.y),
                                    bf16_lo(w.z), bf16_hi(w.z), bf16_lo(w.w), bf16_hi(w.w)};
#pragma unroll
                for (int e = 0; e < 8; ++e) dot = fmaf(f[e], s_c[c * 8 + e], dot);
            }
            const float inv = inv_norm[i];
            float d = inv > 0.0f ? fmaxf(0.0f, 1.0f + cn2 - 2.0f * inv * dot) : cn2;
            if (j > 0) d = fminf(d, dist[i]);
            dist[i] = d;
            local += d;
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
    if (threadIdx.x == 0) part[blk] = (s_red[0] + s_red[1]) + (s_red[2] + s_red[3]);
}

// The draw: the first point whose running sum of distances exceeds u * total (the last point if
// none does).  Found in two levels: the block sums first, then the points of that block.
// grid 1, block 1024.
__global__ __launch_bounds__(1024) void k_km_seed_pick(const float *__restrict__ dist,
                                                       const float *__restrict__ part, int n_blk,
                                                       int n_pool, float u, int32_t *__restrict__ pick_dev)
{
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
// grid ceil(n_pool / (128 or 256)), block 256, dynamic LDS lds_sums ? (C * DB + C) * 4 : 0 bytes.
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

template <int DB>
__global__ __launch_bounds__(256) void k_km_assign(Pool pool, const float *__restrict__ inv_norm,
                                                   const uint16_t *__restrict__ cent16, int C,
                                                   float *__restrict__ sums, int32_t *__restrict__ counts,
                                                   float *__restrict__ cos_sum,
                                                   int32_t *__restrict__ assign_out,
                                                   int32_t *__restrict__ assign_work, int lds_sums)
{
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
    int pt[CB];
    bool live[CB];
    // operand element k of instruction kk is dimension 16 * kk + k; a lane holds k = 8 * half .. + 7
    // (zeros past d_b: only for 8-dimensional sub-vectors)
    Frag8 bq[CB][NK];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
        pt[cb] = blockIdx.x * kKmPts + (wave * CB + cb) * 32 + col;
        live[cb] = pt[cb] < pool.n_pool;
        const uint16_t *r = pool.row(live[cb] ? pt[cb] : 0);
#pragma unroll
        for (int kk = 0; kk < NK; ++kk) {
            const int e0 = 16 * kk + 8 * half;
            bq[cb][kk].u = make_uint4(0, 0, 0, 0);
            if (live[cb] && e0 < DB) bq[cb][kk].u = *(const uint4 *)(r + e0);
        }
    }
    if (lds_sums)
        for (int e = threadIdx.x; e < C * DB + C; e += 256) s_sum[e] = 0.0f;
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
    float cs = 0.0f;
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
        const float inv = live[cb] ? inv_norm[pt[cb]] : 0.0f;
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
                if (assign_out) assign_out[pt[cb]] = best_j[cb];
            }
        }
        cs += (live[cb] && half == 0) ? best[cb] * inv : 0.0f;
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
// the running write position of the scatter, and a second copy as the start).  One workgroup.
__global__ __launch_bounds__(1024) void k_km_offsets(const int32_t *__restrict__ counts, int C,
                                                     int32_t *__restrict__ start, int32_t *__restrict__ cursor)
{
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

// k_km_scatter: point i goes to the next free place of its centroid's list.  grid ceil(n / 256).
__global__ void k_km_scatter(const int32_t *__restrict__ assign, int n_pool, int32_t *__restrict__ cursor,
                             int32_t *__restrict__ member)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n_pool) return;
    member[atomicAdd(cursor + assign[i], 1)] = i;
}

// k_km_sum: sums[j][:] = sum over the members i of centroid j of x_i / ||x_i||, one wave per
// centroid; a group of DB/8 lanes reads one member's sub-vector (16 bytes per lane), the groups of
// the wave take members in turn and are folded at the end.  No atomics.  grid ceil(C / 4), block 256.
template <int DB>
__global__ __launch_bounds__(256) void k_km_sum(Pool pool, const float *__restrict__ inv_norm,
                                                const int32_t *__restrict__ start,
                                                const int32_t *__restrict__ member, int C,
                                                float *__restrict__ sums)
{
    constexpr int LPR = DB / 8;        // lanes per member row
    constexpr int GROUPS = kWave / LPR;  // members in flight per wave
    const int j = blockIdx.x * 4 + threadIdx.x / kWave;
    if (j >= C) return;  // (whole waves)
    const int lane = lane_id(), grp = lane / LPR, c = lane % LPR;
    const int m0 = start[j], m1 = start[j + 1];
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0f;
    for (int m = m0 + grp; m < m1; m += GROUPS) {
        const int i = member[m];
        const float inv = inv_norm[i];
        const uint4 w = *(const uint4 *)(pool.row(i) + c * 8);
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
        dst[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
        dst[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
    }
}

// Lloyd step, second half: centroid <- its sum re-normalised and rounded to bf16 (an empty cluster
// keeps its centroid); sums and counts are cleared for the next step; the step's mean best cosine
// is written out.  One wave per centroid.  grid ceil(C / 4), block 256.
template <int DB>
__global__ __launch_bounds__(256) void k_km_finish(float *__restrict__ sums, int32_t *__restrict__ counts,
                                                   uint16_t *__restrict__ cent16, int C,
                                                   float *__restrict__ cos_sum,
                                                   float *__restrict__ mean_cos_out, int n_pool)
{
    const int j = blockIdx.x * 4 + threadIdx.x / kWave;
    const int lane = lane_id();
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        if (mean_cos_out) *mean_cos_out = n_pool > 0 ? *cos_sum / (float)n_pool : 0.0f;
        *cos_sum = 0.0f;
    }
    if (j >= C) return;
    float v[2] = {0.0f, 0.0f}, nn = 0.0f;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int e = u * kWave + lane;
        if (e < DB) {
            v[u] = sums[(size_t)j * DB + e];
            sums[(size_t)j * DB + e] = 0.0f;
            nn = fmaf(v[u], v[u], nn);
        }
    }
    for (int o = 32; o > 0; o >>= 1) nn += __shfl_xor(nn, o, kWave);
    const int cnt = counts[j];
    if (cnt > 0 && nn > 0.0f) {
        const float inv = 1.0f / sqrtf(nn);
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int e = u * kWave + lane;
            if (e < DB) cent16[(size_t)j * DB + e] = f32_to_bf16_rne(v[u] * inv);
        }
    }
    if (lane == 0) counts[j] = 0;
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
size_t cluster_work_bytes(int n_pool, int C, int db)
{
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    const size_t n_blk = ((size_t)n_pool + kSeedPts - 1) / kSeedPts;
    return up((size_t)n_pool * 4) * 2 + up(n_blk * 4) + up((size_t)C * db * 4) + up((size_t)C * 4) +
           up((size_t)C * db * 2) + 512 +
           up((size_t)n_pool * 4) + 2 * up(((size_t)C + 1) * 4);  // assignments, list starts, write positions
}

template <int DB>
static hipError_t cluster_one(const uint16_t *q_group, int n_pre, int n_pool, int sub, int C, int iters,
                              const float *u_seed, const uint16_t *init, uint16_t *out,
                              float *mean_cos_out, int32_t *assign_out, char *work, hipStream_t st)
{
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    const int n_blk = (n_pool + kSeedPts - 1) / kSeedPts;
    float *inv_norm = (float *)work;
    float *dist = (float *)(work + up((size_t)n_pool * 4));
    float *part = (float *)(work + 2 * up((size_t)n_pool * 4));
    float *sums = (float *)((char *)part + up((size_t)n_blk * 4));
    int32_t *counts = (int32_t *)((char *)sums + up((size_t)C * DB * 4));
    uint16_t *cent16 = (uint16_t *)((char *)counts + up((size_t)C * 4));
    char *scal = (char *)cent16 + up((size_t)C * DB * 2);
    int32_t *pick_dev = (int32_t *)scal;
    float *cos_sum = (float *)(scal + 256);
    // member lists of the Lloyd steps (the seeding's distance array is free by then and holds them)
    int32_t *assign_work = (int32_t *)(scal + 512);
    int32_t *start = (int32_t *)((char *)assign_work + up((size_t)n_pool * 4));
    int32_t *cursor = (int32_t *)((char *)start + up(((size_t)C + 1) * 4));
    int32_t *member = (int32_t *)dist;
    Pool pool{q_group, n_pre, n_pool, sub * DB};
    hipError_t e = hipMemsetAsync(sums, 0, (size_t)((char *)cent16 - (char *)sums), st);  // sums + counts
    if (e != hipSuccess) return e;
    e = hipMemsetAsync(scal, 0, 512, st);
    if (e != hipSuccess) return e;
    k_km_norms<DB><<<(n_pool + 255) / 256, 256, 0, st>>>(pool, inv_norm);
    if (init) {
        e = hipMemcpyAsync(cent16, init, (size_t)C * DB * 2, hipMemcpyDeviceToDevice, st);
        if (e != hipSuccess) return e;
    } else {
        const int snake = (size_t)n_pool * DB * 2 > ((size_t)64 << 20) ? 1 : 0;
        int first = (int)((double)u_seed[0] * (double)n_pool);
        if (first >= n_pool) first = n_pool - 1;
        for (int j = 0; j < C; ++j) {
            k_km_seed_update<DB><<<n_blk, 256, 0, st>>>(pool, inv_norm, dist, part, cent16, pick_dev,
                                                        j == 0 ? first : -1, j, snake);
            if (j + 1 < C)
                k_km_seed_pick<<<1, 1024, 0, st>>>(dist, part, n_blk, n_pool, u_seed[j + 1], pick_dev);
        }
    }
    const int lds_sums = (size_t)C * DB + C <= 8192 ? 1 : 0;  // up to 32 KiB of LDS sums
    const size_t lds_bytes = lds_sums ? ((size_t)C * DB + C) * 4 : 0;
    for (int it = 0; it < iters; ++it) {
        k_km_assign<DB><<<(n_pool + 128 * km_cols<DB>() - 1) / (128 * km_cols<DB>()), 256, lds_bytes, st>>>(pool, inv_norm, cent16, C, sums, counts,
                                                                      cos_sum, it + 1 == iters ? assign_out : nullptr,
                                                                      assign_work, lds_sums);
        if (!lds_sums) {
            k_km_offsets<<<1, 1024, 0, st>>>(counts, C, start, cursor);
            k_km_scatter<<<(n_pool + 255) / 256, 256, 0, st>>>(assign_work, n_pool, cursor, member);
            k_km_sum<DB><<<(C + 3) / 4, 256, 0, st>>>(pool, inv_norm, start, member, C, sums);
        }
        k_km_finish<DB><<<(C + 3) / 4, 256, 0, st>>>(sums, counts, cent16, C, cos_sum,
                                                     mean_cos_out ? mean_cos_out + it : nullptr, n_pool);
    }
    e = hipMemcpyAsync(out, cent16, (size_t)C * DB * 2, hipMemcpyDeviceToDevice, st);
    if (e != hipSuccess) return e;
    return hipGetLastError();
}

// One (KV head, subspace) problem.  q_group: first row of the group's first query head.
int cluster_problem(const void *q_group, int n_pre, int n_pool, int S, int sub, int C, int iters,
                    const float *u_seed, const void *init, void *out, float *mean_cos_out,
                    int32_t *assign_out, void *work, hipStream_t st)
{
#define CSA_KM(DB_)                                                                                     \
    return (int)cluster_one<DB_>((const uint16_t *)q_group, n_pre, n_pool, sub, C, iters, u_seed,      \
                                 (const uint16_t *)init, (uint16_t *)out, mean_cos_out, assign_out,     \
                                 (char *)work, st)
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

// Search half of the decode step (paper Sec. 3.3 steps 1-4): centroid scoring, choice of the
// probed rows, row gather with per-key score accumulation, Top-K selection.
#include "common.h"
#include "kernels.h"

namespace csa {

// ---------------------------------------------------------------------------------------------
// Step 1a: z[b][h][j] = q[b][h] . c[b][g][j]   (Sec. 3.3 (1); q left un-normalised, which cannot
// change the ranking).  One lane per centroid; the centroid matrix is stored dimension-chunk
// major ([d/8][C][8] bf16) so that the 64 lanes of a wave read 1 KiB contiguous per load.  The
// sum is one fp32 fma chain over ascending dimension from +0: the order is part of the
// interface because it decides which rows are probed.
// grid (ceil(C/256), B*Hkv), block 256.
// ---------------------------------------------------------------------------------------------
template <int GH>
__global__ __launch_bounds__(256) void k_score_centroids(const uint16_t *__restrict__ q,
                                                         const uint4 *__restrict__ cent_t,
                                                         float *__restrict__ z, int C, int G)
{
    __shared__ float s_q[GH][kHeadDim];
    const int bg = blockIdx.y;
    const int j = blockIdx.x * 256 + threadIdx.x;
    const uint4 *ct = cent_t + (size_t)bg * (kHeadDim / 8) * C;
    for (int h0 = 0; h0 < G; h0 += GH) {
        __syncthreads();
        for (int e = threadIdx.x; e < GH * kHeadDim; e += 256) {
            const int hh = e / kHeadDim, t = e % kHeadDim;
            s_q[hh][t] = __uint_as_float((uint32_t)q[((size_t)bg * G + h0 + hh) * kHeadDim + t] << 16);
        }
        __syncthreads();
        if (j < C) {
            float acc[GH];
#pragma unroll
            for (int hh = 0; hh < GH; ++hh) acc[hh] = 0.0f;
#pragma unroll 4
            for (int c = 0; c < kHeadDim / 8; ++c) {
                const uint4 w = ct[(size_t)c * C + j];
                const float cf[8] = {bf16_lo(w.x), bf16_hi(w.x), bf16_lo(w.y), bf16_hi(w.y),
                                     bf16_lo(w.z), bf16_hi(w.z), bf16_lo(w.w), bf16_hi(w.w)};
#pragma unroll
                for (int e = 0; e < 8; ++e)
#pragma unroll
                    for (int hh = 0; hh < GH; ++hh)
                        acc[hh] = __builtin_fmaf(s_q[hh][c * 8 + e], cf[e], acc[hh]);
            }
#pragma unroll
            for (int hh = 0; hh < GH; ++hh)
                z[((size_t)bg * G + h0 + hh) * C + j] = acc[hh] + 0.0f;  // -0 -> +0
        }
    }
}

void launch_score_centroids(const void *q, const void *cent_t, float *z, int B, int Hkv, int G,
                            int C, hipStream_t st)
{
    dim3 grid((C + 255) / 256, B * Hkv), block(256);
    if (G % 8 == 0)
        k_score_centroids<8><<<grid, block, 0, st>>>((const uint16_t *)q, (const uint4 *)cent_t, z, C, G);
    else if (G % 4 == 0)
        k_score_centroids<4><<<grid, block, 0, st>>>((const uint16_t *)q, (const uint4 *)cent_t, z, C, G);
    else if (G % 2 == 0)
        k_score_centroids<2><<<grid, block, 0, st>>>((const uint16_t *)q, (const uint4 *)cent_t, z, C, G);
    else
        k_score_centroids<1><<<grid, block, 0, st>>>((const uint16_t *)q, (const uint4 *)cent_t, z, C, G);
}

// ---------------------------------------------------------------------------------------------
// Step 1b: the m centroids with the largest z, ties to the lower index (Sec. 3.3 (1) with the
// top-tau back-off of Sec. 4.4).  Radix threshold search on the order-preserving integer image
// of z, then an ordered pick: everything above the threshold, then threshold ties in
// ascending j.  grid B*Hq, block 256.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_top_centroids(const float *__restrict__ z,
                                                       int32_t *__restrict__ rows, int C, int m)
{
    __shared__ uint32_t s_hist[256 + 256 / kWave + 4];
    __shared__ int s_scan[256 / kWave + 1];
    const float *zh = z + (size_t)blockIdx.x * C;
    int32_t *out = rows + (size_t)blockIdx.x * m;
    int need = 0;
    const uint32_t T = block_radix_threshold<256, 8, 4>(
        [&](auto fn) {
            for (int j = threadIdx.x; j < C; j += 256) fn(orderable(zh[j]));
        },
        m, s_hist, need);
    // ordered emission, 256 centroids per round
    int n_out = 0, ties_taken = 0;
    for (int j0 = 0; j0 < C; j0 += 256) {
        const int j = j0 + threadIdx.x;
        const uint32_t key = j < C ? orderable(zh[j]) : 0u;
        const int is_tie = (j < C && key == T) ? 1 : 0;
        int tie_total;
        const int tie_rank = block_excl_scan<256>(is_tie, s_scan, tie_total) + ties_taken;
        const int take = (j < C && key > T) || (is_tie && tie_rank < need);
        int take_total;
        const int pos = block_excl_scan<256>(take, s_scan, take_total) + n_out;
        if (take) out[pos] = j;
        n_out += take_total;
        ties_taken += tie_total;
    }
}

void launch_top_centroids(const float *z, int32_t *rows, int n_heads, int C, int m, hipStream_t st)
{
    k_top_centroids<<<n_heads, 256, 0, st>>>(z, rows, C, m);
}

// ---------------------------------------------------------------------------------------------
// Steps 2+3: gather the m probed rows and sum scores per key (Sec. 3.3 (2)-(3), w_b = 1).
// Rows are stored sorted by key index with per-row offsets of every key range of R keys, so
// workgroup (head, p) reads only the slices of its range [p*R, (p+1)*R) - every table byte is
// read once - and keeps R direct-addressed integer accumulators in LDS.  Each entry adds
// q*64 + 1: exact integer sums, order-free, and "seen" == accumulator != 0 (U of Sec. 3.3 (3):
// a key absent from every probed row is not a candidate even if all sums are negative).
// Seen keys leave as (index, sum + 2^24) pairs in the head's candidate segment p.
// grid (P, B*Hq), block 256, dynamic LDS R*4 bytes.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_accumulate(const Entry *__restrict__ ent,
                                                    const int32_t *__restrict__ part_off,
                                                    const int32_t *__restrict__ rows,
                                                    Cand *__restrict__ cand,
                                                    int32_t *__restrict__ cand_cnt, int C, int L,
                                                    int m, int G, int R, int P, int PO)
{
    extern __shared__ int32_t s_acc[];  // [R]
    __shared__ int32_t s_lo[64], s_hi[64], s_row[64];
    __shared__ int s_count;
    const int p = blockIdx.x, head = blockIdx.y;
    const int bg = head / G;
    if (threadIdx.x < m) {
        const int r = rows[(size_t)head * m + threadIdx.x];
        const int32_t *po = part_off + ((size_t)bg * C + r) * PO;
        s_row[threadIdx.x] = r;
        s_lo[threadIdx.x] = po[p];
        s_hi[threadIdx.x] = po[p + 1];
    }
    if (threadIdx.x == 0) s_count = 0;
    for (int e = threadIdx.x; e < R; e += 256) s_acc[e] = 0;
    __syncthreads();
    const int base = p * R;
    const int wave = threadIdx.x / kWave, lane = lane_id();
    for (int r = wave; r < m; r += 256 / kWave) {
        const Entry *row = ent + ((size_t)bg * C + s_row[r]) * L;
        const int hi = s_hi[r];
        for (int e = s_lo[r] + lane; e < hi; e += kWave) {
            const Entry v = row[e];
            atomicAdd(&s_acc[v.idx - base], v.qe);
        }
    }
    __syncthreads();
    Cand *seg = cand + ((size_t)head * P + p) * R;
    for (int e0 = 0; e0 < R; e0 += 256) {
        const int e = e0 + threadIdx.x;
        const int32_t a = s_acc[e];
        const bool seen = a != 0;
        const uint64_t mask = __ballot(seen);
        int wbase = 0;
        if (lane == 0 && mask) wbase = atomicAdd(&s_count, __popcll(mask));
        wbase = __shfl(wbase, 0, kWave);
        if (seen) {
            Cand c;
            c.idx = base + e;
            c.key = (uint32_t)((a >> kCntBits) + kKeyBias);
            seg[wbase + mbcnt(mask)] = c;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) cand_cnt[(size_t)head * P + p] = s_count;
}

void launch_accumulate(const void *ent, const int32_t *part_off, const int32_t *rows, void *cand,
                       int32_t *cand_cnt, int n_heads, int C, int L, int m, int G, int R, int P,
                       int PO, hipStream_t st)
{
    dim3 grid(P, n_heads), block(256);
    static bool attr = false;
    if (!attr) {
        hipFuncSetAttribute((const void *)k_accumulate, hipFuncAttributeMaxDynamicSharedMemorySize, 16384 * 4);
        attr = true;
    }
    k_accumulate<<<grid, block, (size_t)R * 4, st>>>((const Entry *)ent, part_off, rows,
                                                     (Cand *)cand, cand_cnt, C, L, m, G, R, P, PO);
}

// ---------------------------------------------------------------------------------------------
// Step 4: Top-K over the candidates of one head (Sec. 3.3 (4)): the min(k, |U|) largest sums,
// ties to the lower key index, written in ascending index order and padded with -1.
// Radix threshold search over the 25-bit keys, then per chunk of kChunk key indices two LDS
// bitmaps ("above threshold", "equal to threshold") are filled, the lowest-index ties still
// needed are kept, and the set bits are emitted in order.
// grid B*Hq, block 1024.
// ---------------------------------------------------------------------------------------------
constexpr int kSelNT = 1024;
constexpr int kChunk = 32768;             // key indices per bitmap chunk
constexpr int kChunkWords = kChunk / 32;  // 1024 words = one per thread

__global__ __launch_bounds__(kSelNT) void k_select(const Cand *__restrict__ cand,
                                                   const int32_t *__restrict__ cand_cnt,
                                                   int32_t *__restrict__ sel,
                                                   int32_t *__restrict__ sel_count, int k, int R,
                                                   int P)
{
    __shared__ uint32_t s_hist[512 + kSelNT / kWave + 4];
    __shared__ int s_scan[kSelNT / kWave + 1];
    __shared__ uint32_t s_gt[kChunkWords], s_eq[kChunkWords];
    __shared__ int s_n;
    const int head = blockIdx.x;
    const Cand *hc = cand + (size_t)head * P * R;
    const int32_t *cnt = cand_cnt + (size_t)head * P;
    int32_t *out = sel + (size_t)head * k;

    // |U|
    int part = 0;
    for (int p = threadIdx.x; p < P; p += kSelNT) part += cnt[p];
    int n_total;
    block_excl_scan<kSelNT>(part, s_scan, n_total);
    const int k_eff = n_total < k ? n_total : k;
    if (threadIdx.x == 0) sel_count[head] = k_eff;
    for (int a = k_eff + threadIdx.x; a < k; a += kSelNT) out[a] = -1;
    if (k_eff == 0) return;

    uint32_t T = 0;  // keys are > 0, so T = 0 selects everything when k >= |U|
    int need = 0;
    if (n_total > k) {
        T = block_radix_threshold<kSelNT, 9, 3>(
            [&](auto fn) {
                for (int p = 0; p < P; ++p) {
                    const int c = cnt[p];
                    const Cand *seg = hc + (size_t)p * R;
                    for (int e = threadIdx.x; e < c; e += kSelNT) fn(seg[e].key);
                }
            },
            k, s_hist, need);
    }

    // ordered emission, kChunk key indices at a time (R divides kChunk or kChunk divides R)
    int n_out = 0;
    const int n_keys = P * R;
    for (int c0 = 0; c0 < n_keys; c0 += kChunk) {
        s_gt[threadIdx.x] = 0;
        s_eq[threadIdx.x] = 0;
        __syncthreads();
        // candidate segments intersecting [c0, c0 + kChunk)
        const int p_lo = c0 / R;
        const int p_hi = min(P, (c0 + kChunk + R - 1) / R);
        for (int p = p_lo; p < p_hi; ++p) {
            const int c = cnt[p];
            const Cand *seg = hc + (size_t)p * R;
            for (int e = threadIdx.x; e < c; e += kSelNT) {
                const Cand v = seg[e];
                const int rel = v.idx - c0;
                if (rel < 0 || rel >= kChunk) continue;  // R > kChunk: other chunk of this segment
                if (v.key > T)
                    atomicOr(&s_gt[rel >> 5], 1u << (rel & 31));
                else if (v.key == T)
                    atomicOr(&s_eq[rel >> 5], 1u << (rel & 31));
            }
        }
        __syncthreads();
        // keep the lowest-index `need` ties
        uint32_t eq = s_eq[threadIdx.x];
        int tie_total;
        const int tie_before = block_excl_scan<kSelNT>(__popc(eq), s_scan, tie_total);
        int allow = need - tie_before;
        if (allow <= 0)
            eq = 0;
        else
            while (__popc(eq) > allow) eq &= ~(0x80000000u >> __clz(eq));  // drop highest bit
        need = max(0, need - tie_total);
        uint32_t bits = s_gt[threadIdx.x] | eq;
        int take_total;
        int pos = block_excl_scan<kSelNT>(__popc(bits), s_scan, take_total) + n_out;
        const int kbase = c0 + threadIdx.x * 32;
        while (bits) {
            const int b = __ffs(bits) - 1;
            out[pos++] = kbase + b;
            bits &= bits - 1;
        }
        n_out += take_total;
        __syncthreads();
    }
}

void launch_select(const void *cand, const int32_t *cand_cnt, int32_t *sel, int32_t *sel_count,
                   int n_heads, int k, int R, int P, hipStream_t st)
{
    k_select<<<n_heads, kSelNT, 0, st>>>((const Cand *)cand, cand_cnt, sel, sel_count, k, R, P);
}

}  // namespace csa

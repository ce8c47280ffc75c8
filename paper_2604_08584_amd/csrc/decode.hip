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
            uint4 wv[kHeadDim / 8];
#pragma unroll
            for (int c = 0; c < kHeadDim / 8; ++c) wv[c] = ct[(size_t)c * C + j];
#pragma unroll
            for (int c = 0; c < kHeadDim / 8; ++c) {
                const uint4 w = wv[c];
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
// top-tau back-off of Sec. 4.4), on the order-preserving integer image of z.
// Fast path (m small against C): every thread takes the maximum of its own slice; the m-th
// largest of the 256 thread maxima is a lower bound on the m-th largest overall, so only the few
// values >= that bound are candidates; they are ranked against each other by (z desc, j asc) and
// ranks < m are written in rank order.  If there are too many candidates (many equal values) a
// radix threshold search with an ordered tie pick does the job instead.
// Also clears the head's coarse score histogram and looks up, for every key range p, the slice
// [lo, hi) of each probed row, so that the accumulation kernel starts with one coalesced read.
// grid B*Hq, block 256.
// ---------------------------------------------------------------------------------------------
constexpr int kTopNT = 256;
constexpr int kCoarseBins = 512;  // per-head histogram of accumulated scores, filled by k_accumulate
constexpr int kTopReg = 16;     // keys per thread held in registers
constexpr int kTopCand = 1024;  // candidate capacity of the fast path

__global__ __launch_bounds__(kTopNT) void k_top_centroids(const float *__restrict__ z,
                                                          int32_t *__restrict__ rows,
                                                          const int32_t *__restrict__ part_off,
                                                          int2 *__restrict__ spans,
                                                          uint32_t *__restrict__ hist_g, int C,
                                                          int m, int G, int P)
{
    __shared__ int32_t s_rows[64];
    __shared__ __align__(16) uint32_t s_hist[256 + kTopNT / kWave + 4];
    __shared__ int s_scan[kTopNT / kWave + 1];
    __shared__ __align__(16) uint64_t s_ck[kTopCand + 2];  // (key << 32) | ~j : larger = better, distinct
    __shared__ int s_slot;
    __shared__ uint32_t s_bound;
    const float *zh = z + (size_t)blockIdx.x * C;
    int32_t *out = rows + (size_t)blockIdx.x * m;
    if (threadIdx.x == 0) s_slot = 0;
    for (int i = threadIdx.x; i < kCoarseBins; i += kTopNT) hist_g[(size_t)blockIdx.x * kCoarseBins + i] = 0;
    const bool in_regs = C <= kTopNT * kTopReg;
    uint32_t kreg[kTopReg];
    if (in_regs) {
#pragma unroll
        for (int u = 0; u < kTopReg; ++u) {
            const int j = u * kTopNT + threadIdx.x;
            kreg[u] = j < C ? orderable(zh[j]) : 0u;
        }
    }
    const int rounds = (C + kTopNT - 1) / kTopNT;
    // visit(fn): fn(j, key, valid) for every centroid slot of this thread, uniformly per wave
    auto visit = [&](auto fn) {
        if (in_regs) {
#pragma unroll
            for (int u = 0; u < kTopReg; ++u)
                if (u < rounds) {
                    const int j = u * kTopNT + threadIdx.x;
                    fn(j, kreg[u], j < C);
                }
        } else {
            for (int u = 0; u < rounds; ++u) {
                const int j = u * kTopNT + threadIdx.x;
                fn(j, j < C ? orderable(zh[j]) : 0u, j < C);
            }
        }
    };
    if (m <= kTopNT / 4 && C >= kTopNT) {  // every lane holds at least one value
        // ---- fast path
        uint32_t best = 0;  // orderable(z) of a finite z is never 0
        visit([&](int, uint32_t key, bool valid) { if (valid && key > best) best = key; });
        // a lower bound on the m-th largest value overall: in each wave the r-th largest of the
        // 64 lane maxima, r = ceil(m / waves) (found by r rounds of max-and-remove); the smallest
        // of these over the waves has at least m values at or above it
        {
            constexpr int NWT = kTopNT / kWave;
            const int r = (m + NWT - 1) / NWT;  // <= 16 of the 64 lane maxima; NWT * r >= m
            uint64_t cur = ((uint64_t)best << 32) | (uint32_t)~threadIdx.x;  // distinct per lane
            uint64_t wmax = 0ull;
            for (int round = 0; round < r; ++round) {
                wmax = cur;
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) {
                    const uint64_t t = __shfl_xor(wmax, o, kWave);
                    wmax = t > wmax ? t : wmax;
                }
                if (cur == wmax) cur = 0ull;  // remove the winner
            }
            if (lane_id() == 0) s_hist[threadIdx.x / kWave] = (uint32_t)(wmax >> 32);
            __syncthreads();
            if (threadIdx.x == 0) {
                uint32_t bnd = 0xFFFFFFFFu;
                for (int w = 0; w < NWT; ++w) bnd = min(bnd, s_hist[w]);
                s_bound = bnd;
            }
        }
        __syncthreads();
        const uint32_t bound = s_bound;
        visit([&](int j, uint32_t key, bool valid) {
            if (valid && key >= bound) {
                const int slot = atomicAdd(&s_slot, 1);
                if (slot < kTopCand) s_ck[slot] = ((uint64_t)key << 32) | (uint32_t)~j;
            }
        });
        __syncthreads();
        const int nc = s_slot;
        if (nc <= kTopCand && nc >= m) {  // (nc >= m always holds; checked so that no row is ever left unset)
            if (threadIdx.x == 0) s_ck[nc] = 0;  // pad to an even count (0 beats nothing)
            __syncthreads();
            const ulonglong2 *c2 = (const ulonglong2 *)s_ck;
            for (int a = threadIdx.x; a < nc; a += kTopNT) {
                const uint64_t mine = s_ck[a];
                int r = 0;
#pragma unroll 4
                for (int t2 = 0; t2 < (nc + 1) / 2; ++t2) {
                    const ulonglong2 o = c2[t2];
                    r += (o.x > mine) + (o.y > mine);
                }
                if (r < m) s_rows[r] = (int32_t)~(uint32_t)mine;
            }
            goto publish;
        }
        __syncthreads();
        if (threadIdx.x == 0) s_slot = 0;
    }
    {
    // ---- general path: radix threshold, winners above it take any slot, ties in index order
    int need = 0;
    const uint32_t T = block_radix_threshold<kTopNT, 8, 4>(
        [&](auto fn) { visit([&](int, uint32_t key, bool valid) { fn(key, valid); }); }, m, s_hist,
        need);
    visit([&](int j, uint32_t key, bool valid) {
        if (valid && key > T) s_rows[atomicAdd(&s_slot, 1)] = j;
    });
    int ties_taken = 0;
    const int base = m - need;
    visit([&](int j, uint32_t key, bool valid) {
        const int is_tie = (valid && key == T) ? 1 : 0;
        int round_total;
        const int rank = block_excl_scan<kTopNT>(is_tie, s_scan, round_total) + ties_taken;
        if (is_tie && rank < need) s_rows[base + rank] = j;
        ties_taken += round_total;
    });
    }
publish:
    // the probed rows, and for every key range p the slice [lo, hi) of each probed row
    __syncthreads();
    if (threadIdx.x < m) out[threadIdx.x] = s_rows[threadIdx.x];
    const int bg = blockIdx.x / G;
    int2 *sp = spans + (size_t)blockIdx.x * P * m;
    for (int t = threadIdx.x; t < P * m; t += kTopNT) {
        const int p = t / m, r = t - p * m;
        const int32_t *po = part_off + ((size_t)bg * C + s_rows[r]) * (P + 1);
        sp[t] = make_int2(po[p], po[p + 1]);
    }
}

void launch_top_centroids(const float *z, int32_t *rows, const int32_t *part_off, void *spans,
                          uint32_t *hist_g, int n_heads, int C, int m, int G, int P, hipStream_t st)
{
    k_top_centroids<<<n_heads, kTopNT, 0, st>>>(z, rows, part_off, (int2 *)spans, hist_g, C, m, G, P);
}

// ---------------------------------------------------------------------------------------------
// Steps 2+3: gather the m probed rows and sum scores per key (Sec. 3.3 (2)-(3), w_b = 1).
// Rows are stored sorted by key index with per-row offsets of every key range of R keys, so
// workgroup (head, p) reads only the slices of its range [p*R, (p+1)*R) - every table byte is
// read once - and keeps R direct-addressed integer accumulators in LDS.  Each entry adds
// q*64 + 1: exact integer sums, order-free, and "seen" == accumulator != 0 (U of Sec. 3.3 (3):
// a key absent from every probed row is not a candidate even if all sums are negative).
// The kernel is bound by instruction issue as much as by HBM, so the per-entry and per-slot
// paths are kept minimal: a wave owns whole rows (row constants are scalar), keeps eight
// 512-byte loads in flight (two rows at a time), and the sparse accumulator array is first compacted
// into LDS; only the dense survivors are turned into (sum + 2^24, index), counted into the
// head's coarse histogram and written out, in segment p of the head's candidate arrays.
// grid (P, B*Hq), block NT = R/16, dynamic LDS R*4 bytes.
// ---------------------------------------------------------------------------------------------
constexpr int kAccUnroll = 4;

template <int NT>
__global__ __launch_bounds__(NT) void k_accumulate(const Entry *__restrict__ ent,
                                                   const int32_t *__restrict__ rows,
                                                   const int2 *__restrict__ spans,
                                                   uint32_t *__restrict__ cand_key,
                                                   int32_t *__restrict__ cand_idx,
                                                   int32_t *__restrict__ seg_cnt,
                                                   uint32_t *__restrict__ hist_g, int C, int L,
                                                   int m, int G, int P, size_t cand_stride,
                                                   uint32_t key_lo, int key_sh)
{
    constexpr int NW = NT / kWave;
    constexpr int R = NT * 16;
    extern __shared__ __align__(16) int32_t s_acc[];  // [R]
    __shared__ int32_t s_lo[64], s_hi[64], s_row[64];
    __shared__ uint32_t s_h[kCoarseBins];
    __shared__ int s_scan[NW + 1];
    const int p = blockIdx.x, head = blockIdx.y;
    const int bg = head / G;
    const int wave = threadIdx.x / kWave, lane = lane_id();
    if (threadIdx.x < m) {
        const int2 sp = spans[((size_t)head * P + p) * m + threadIdx.x];
        s_row[threadIdx.x] = rows[(size_t)head * m + threadIdx.x];
        s_lo[threadIdx.x] = sp.x;
        s_hi[threadIdx.x] = sp.y;
    }
    {
        int4 *z4 = (int4 *)s_acc;
#pragma unroll
        for (int u = 0; u < 4; ++u) z4[u * NT + threadIdx.x] = make_int4(0, 0, 0, 0);
        for (int e = threadIdx.x; e < kCoarseBins; e += NT) s_h[e] = 0;
    }
    __syncthreads();
    const int base = p * R;
    // two rows per wave at a time, kAccUnroll 512-byte loads in flight for each
    for (int r = wave; r < m; r += 2 * NW) {
        const int r2 = r + NW < m ? r + NW : r;
        const int lo_a = __builtin_amdgcn_readfirstlane(s_lo[r]);
        const int hi_a = __builtin_amdgcn_readfirstlane(s_hi[r]);
        const int lo_b = __builtin_amdgcn_readfirstlane(s_lo[r2]);
        const int hi_b = r2 != r ? __builtin_amdgcn_readfirstlane(s_hi[r2]) : lo_b;  // empty if no 2nd row
        const Entry *rp_a = ent + ((size_t)bg * C + __builtin_amdgcn_readfirstlane(s_row[r])) * L;
        const Entry *rp_b = ent + ((size_t)bg * C + __builtin_amdgcn_readfirstlane(s_row[r2])) * L;
        for (int ea = lo_a, eb = lo_b; ea < hi_a || eb < hi_b;
             ea += kWave * kAccUnroll, eb += kWave * kAccUnroll) {
            Entry va[kAccUnroll], vb[kAccUnroll];
#pragma unroll
            for (int u = 0; u < kAccUnroll; ++u) {
                const int xa = ea + u * kWave + lane, xb = eb + u * kWave + lane;
                va[u].idx = -1;
                vb[u].idx = -1;
                if (xa < hi_a) va[u] = rp_a[xa];
                if (xb < hi_b) vb[u] = rp_b[xb];
            }
#pragma unroll
            for (int u = 0; u < kAccUnroll; ++u) {
                if (va[u].idx >= 0) atomicAdd(&s_acc[va[u].idx - base], va[u].qe);
                if (vb[u].idx >= 0) atomicAdd(&s_acc[vb[u].idx - base], vb[u].qe);
            }
        }
    }
    __syncthreads();
    // sparse -> dense: thread t owns the 16 slots 4*(u*NT + t) .. +3, u < 4 (128-bit LDS reads)
    int4 a[4];
    int mine = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        a[u] = ((const int4 *)s_acc)[u * NT + threadIdx.x];
        mine += (a[u].x != 0) + (a[u].y != 0) + (a[u].z != 0) + (a[u].w != 0);
    }
    int total;
    const int pos = block_excl_scan<NT>(mine, s_scan, total);  // (barriers: all slots are in registers)
    uint32_t *dk = cand_key + (size_t)head * cand_stride + (size_t)p * R;
    int32_t *di = cand_idx + (size_t)head * cand_stride + (size_t)p * R;
    uint2 *s_stage = (uint2 *)s_acc;  // R/2 (accumulator, local slot) pairs at a time
    constexpr int half = R / 2;
    for (int w0 = 0; w0 < total; w0 += half) {
        if (w0) __syncthreads();  // previous window consumed
        int q = pos - w0;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int slot = 4 * (u * NT + threadIdx.x);
            const int av[4] = {a[u].x, a[u].y, a[u].z, a[u].w};
#pragma unroll
            for (int x = 0; x < 4; ++x)
                if (av[x] != 0) {
                    if ((unsigned)q < (unsigned)half) s_stage[q] = make_uint2((uint32_t)av[x], (uint32_t)(slot + x));
                    ++q;
                }
        }
        __syncthreads();
        const int n_here = min(half, total - w0);
        for (int i = threadIdx.x; i < n_here; i += NT) {
            const uint2 c = s_stage[i];
            const uint32_t key = (uint32_t)(((int32_t)c.x >> kCntBits) + kKeyBias);
            dk[w0 + i] = key;
            di[w0 + i] = base + (int32_t)c.y;
            atomicAdd(&s_h[(key - key_lo) >> key_sh], 1u);
        }
    }
    if (threadIdx.x == 0) seg_cnt[(size_t)head * P + p] = total;
    // histogram complete once every wave's LDS atomics have landed: wait for LDS traffic only
    // (a full __syncthreads would also wait for the candidate stores above)
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0), vmcnt / expcnt untouched
    __builtin_amdgcn_s_barrier();
    for (int e = threadIdx.x; e < kCoarseBins; e += NT) {
        const uint32_t c = s_h[e];
        if (c) atomicAdd(&hist_g[(size_t)head * kCoarseBins + e], c);
    }
}

void launch_accumulate(const void *ent, const int32_t *rows, const void *spans, uint32_t *cand_key,
                       int32_t *cand_idx, int32_t *seg_cnt, uint32_t *hist_g, int n_heads, int C,
                       int L, int m, int G, int R, int P, size_t cand_stride, uint32_t key_lo,
                       int key_sh, hipStream_t st)
{
    dim3 grid(P, n_heads);
    static bool attr = false;
    if (!attr) {
        (void)hipFuncSetAttribute((const void *)k_accumulate<1024>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                  16384 * 4);
        attr = true;
    }
#define CSA_ACC(NT_)                                                                             \
    k_accumulate<NT_><<<grid, NT_, (size_t)R * 4, st>>>((const Entry *)ent, rows, (const int2 *)spans, \
                                                        cand_key, cand_idx, seg_cnt, hist_g, C, L, m, \
                                                        G, P, cand_stride, key_lo, key_sh)
    switch (R) {
    case 1024: CSA_ACC(64); break;
    case 2048: CSA_ACC(128); break;
    case 4096: CSA_ACC(256); break;
    case 8192: CSA_ACC(512); break;
    default: CSA_ACC(1024); break;  // 16384
    }
#undef CSA_ACC
}

// ---------------------------------------------------------------------------------------------
// Step 4: Top-K over the candidates of one head (Sec. 3.3 (4)): the min(k, |U|) largest sums,
// ties to the lower key index, written in ascending index order and padded with -1.
// Threshold search by range refinement: the live key range [lo, hi] is cut into <= 512 equal
// bins and a histogram of the candidate keys over them is taken (the first one arrives
// ready-made from the accumulation kernel, a further one costs a streaming pass and is rarely
// needed); the bin holding the k-th largest becomes the new range; once it holds few enough
// keys they are gathered into LDS (with their indices) and finished there with a radix search.
// Winners are marked in two LDS bitmaps over the key indices ("above threshold", "equal to
// threshold"), the lowest-index ties still needed are kept, and the set bits are emitted in
// ascending order.  When all key indices fit one bitmap chunk (n <= 131072) the gather pass
// marks the sure winners on the fly, so the candidates are streamed exactly once.
// grid B*Hq, block 1024.
// ---------------------------------------------------------------------------------------------
constexpr int kSelNT = 1024;
constexpr int kSelCap = 4096;                       // contenders finished in LDS
constexpr int kSelMaxP = 2048;                      // key ranges (segments) per head
constexpr int kChunk = 131072;                      // key indices per bitmap chunk
constexpr int kChunkWords = kChunk / 32;            // 4096 words
constexpr int kWordsPerThread = kChunkWords / kSelNT;  // 4 consecutive words per thread

__global__ __launch_bounds__(kSelNT) void k_select(const uint32_t *__restrict__ cand_key,
                                                   const int32_t *__restrict__ cand_idx,
                                                   const int32_t *__restrict__ seg_cnt,
                                                   int32_t *__restrict__ sel,
                                                   int32_t *__restrict__ sel_count,
                                                   const uint32_t *__restrict__ hist_g, int k, int R,
                                                   int P, size_t cand_stride, uint32_t key_lo,
                                                   int key_sh)
{
    constexpr int NW = kSelNT / kWave;
    __shared__ uint32_t s_hist[512 + kSelNT / kWave + 2];
    __shared__ int s_scan[kSelNT / kWave + 1];
    __shared__ __align__(16) uint32_t s_gt[kChunkWords], s_eq[kChunkWords];
    __shared__ uint2 s_ck[kSelCap];  // contenders: (key - lo, key index)
    __shared__ int32_t s_cnt[kSelMaxP];
    __shared__ int s_n;
    const int head = blockIdx.x;
    const uint32_t *hk = cand_key + (size_t)head * cand_stride;
    const int32_t *hi_ = cand_idx + (size_t)head * cand_stride;
    int32_t *out = sel + (size_t)head * k;
    const int wave = threadIdx.x / kWave, lane = lane_id();
    // segment counts; |U| = their sum
    int part = 0;
    for (int p = threadIdx.x; p < P; p += kSelNT) {
        const int c = seg_cnt[(size_t)head * P + p];
        s_cnt[p] = c;
        part += c;
    }
    if (threadIdx.x == 0) s_n = 0;
#pragma unroll
    for (int u = 0; u < kWordsPerThread; ++u) {
        s_gt[u * kSelNT + threadIdx.x] = 0;
        s_eq[u * kSelNT + threadIdx.x] = 0;
    }
    int n_total;
    block_excl_scan<kSelNT>(part, s_scan, n_total);  // (its barriers also publish the LDS writes)
    const int k_eff = n_total < k ? n_total : k;
    if (threadIdx.x == 0) sel_count[head] = k_eff;
    for (int a = k_eff + threadIdx.x; a < k; a += kSelNT) out[a] = -1;
    if (k_eff == 0) return;

    // stream(fn): fn(key, key_index, valid) over the candidates of every segment.  A wave walks
    // whole segments, four consecutive slots per lane and load, keys and indices both read with
    // full-width loads issued up front (a dependent index load per winner would serialise the
    // walk); fn may use wave-level operations only (trip counts differ between waves).
    auto stream = [&](auto fn) {
        for (int p = wave; p < P; p += NW) {
            const int c = s_cnt[p];
            const int s0 = p * R;
            for (int e0 = 0; e0 < c; e0 += kWave * 16) {
                uint4 kk[4];
                int4 ii[4];
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const int e = e0 + (x * kWave + lane) * 4;
                    kk[x] = e < c ? *(const uint4 *)(hk + s0 + e) : make_uint4(0, 0, 0, 0);
                    ii[x] = e < c ? *(const int4 *)(hi_ + s0 + e) : make_int4(0, 0, 0, 0);
                }
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const int e = e0 + (x * kWave + lane) * 4;
                    if (e0 + x * kWave * 4 < c) {  // wave-uniform
                        fn(kk[x].x, ii[x].x, e + 0 < c);
                        fn(kk[x].y, ii[x].y, e + 1 < c);
                        fn(kk[x].z, ii[x].z, e + 2 < c);
                        fn(kk[x].w, ii[x].w, e + 3 < c);
                    }
                }
            }
        }
    };
    auto mark = [&](uint32_t *bitmap, int key_index, int c0) {
        const int rel = key_index - c0;
        if ((unsigned)rel < (unsigned)kChunk) atomicOr(&bitmap[rel >> 5], 1u << (rel & 31));
    };

    const bool single = P * R <= kChunk;  // one bitmap chunk covers every key index
    bool marked = false;                  // bitmaps of chunk 0 already hold the final marks
    uint32_t T = 0;  // keys are > 0, so T = 0 selects everything when k >= |U|
    int need = 0;
    if (n_total > k) {
        // first round: the head's coarse histogram, filled by the accumulation kernel
        uint32_t lo = key_lo, hi = key_lo + ((uint32_t)kCoarseBins << key_sh) - 1u;
        int sh = key_sh;
        for (int i = threadIdx.x; i < kCoarseBins; i += kSelNT)
            s_hist[i] = hist_g[(size_t)head * kCoarseBins + i];
        __syncthreads();
        int want = k;
        for (bool have_hist = true;; have_hist = false) {
            if (!have_hist) {
                sh = 0;
                while (((hi - lo) >> sh) >= 512u) ++sh;
                for (int i = threadIdx.x; i < 512; i += kSelNT) s_hist[i] = 0;
                __syncthreads();
                stream([&](uint32_t key, int, bool valid) {
                    const bool in = valid && key >= lo && key <= hi;
                    hist_add(s_hist, in ? (key - lo) >> sh : 0u, in);
                });
                __syncthreads();
            }
            int above;
            const int bin = block_pick_bin<kSelNT, 512>(s_hist, want, s_hist + 512, above);
            const int in_bin = (int)s_hist[bin];
            want -= above;
            lo += (uint32_t)bin << sh;
            hi = min(hi, lo + ((1u << sh) - 1u));
            if (sh == 0) {  // the bin is a single key value
                T = lo;
                need = want;
                break;
            }
            if (in_bin <= kSelCap) {
                // gather the contenders (key - lo < 2^sh <= 2^16) with their key indices; with a
                // single bitmap chunk, keys above the bin are sure winners and are marked now
                __syncthreads();
                stream([&](uint32_t key, int key_index, bool valid) {
                    const bool in = valid && key >= lo && key <= hi;
                    const uint64_t mask = __ballot(in);
                    if (mask) {
                        int wbase = 0;
                        if (mbcnt(mask) == 0 && in) wbase = atomicAdd(&s_n, __popcll(mask));
                        wbase = __builtin_amdgcn_readlane(wbase, __ffsll((unsigned long long)mask) - 1);
                        if (in) s_ck[wbase + mbcnt(mask)] = make_uint2(key - lo, (uint32_t)key_index);
                    }
                    if (single && valid && key > hi) mark(s_gt, key_index, 0);
                });
                __syncthreads();
                const int nc = s_n;
                const uint32_t Tl = block_radix_threshold<kSelNT, 8, 2>(
                    [&](auto fn) {
                        for (int a0 = 0; a0 < nc; a0 += kSelNT) {
                            const int a = a0 + threadIdx.x;
                            fn(a < nc ? s_ck[a].x : 0u, a < nc);
                        }
                    },
                    want, s_hist, need);
                T = lo + Tl;
                if (single) {
                    for (int a = threadIdx.x; a < nc; a += kSelNT) {
                        const uint2 c = s_ck[a];
                        if (c.x > Tl)
                            mark(s_gt, (int)c.y, 0);
                        else if (c.x == Tl)
                            mark(s_eq, (int)c.y, 0);
                    }
                    marked = true;
                }
                break;
            }
            __syncthreads();  // s_hist[bin] was read above; the next round clears the histogram
        }
    }

    // ordered emission, kChunk key indices at a time
    int n_out = 0;
    for (int c0 = 0; c0 < P * R; c0 += kChunk) {
        if (!marked) {
            if (c0) {
#pragma unroll
                for (int u = 0; u < kWordsPerThread; ++u) {
                    s_gt[u * kSelNT + threadIdx.x] = 0;
                    s_eq[u * kSelNT + threadIdx.x] = 0;
                }
            }
            __syncthreads();
            stream([&](uint32_t key, int key_index, bool valid) {
                if (valid && key >= T) mark(key > T ? s_gt : s_eq, key_index, c0);
            });
        }
        marked = false;
        __syncthreads();
        // keep the lowest-index `need` ties; thread t owns words [4t, 4t+4)
        uint32_t eq[kWordsPerThread], bits[kWordsPerThread];
        int n_eq = 0;
        {
            const uint4 e4 = ((const uint4 *)s_eq)[threadIdx.x];
            eq[0] = e4.x; eq[1] = e4.y; eq[2] = e4.z; eq[3] = e4.w;
            n_eq = __popc(e4.x) + __popc(e4.y) + __popc(e4.z) + __popc(e4.w);
        }
        int tie_total;
        int allow = need - block_excl_scan<kSelNT>(n_eq, s_scan, tie_total);
        int n_bits = 0;
        const uint4 g4 = ((const uint4 *)s_gt)[threadIdx.x];
        const uint32_t gt[kWordsPerThread] = {g4.x, g4.y, g4.z, g4.w};
#pragma unroll
        for (int u = 0; u < kWordsPerThread; ++u) {
            uint32_t e = eq[u];
            if (allow <= 0)
                e = 0;
            else
                while (__popc(e) > allow) e &= ~(0x80000000u >> __clz(e));  // drop the highest bit
            allow -= __popc(e);
            bits[u] = gt[u] | e;
            n_bits += __popc(bits[u]);
        }
        need = max(0, need - tie_total);
        int take_total;
        int pos = block_excl_scan<kSelNT>(n_bits, s_scan, take_total) + n_out;
#pragma unroll
        for (int u = 0; u < kWordsPerThread; ++u) {
            uint32_t b = bits[u];
            const int kbase = c0 + (threadIdx.x * kWordsPerThread + u) * 32;
            while (b) {
                out[pos++] = kbase + __ffs(b) - 1;
                b &= b - 1;
            }
        }
        n_out += take_total;
        __syncthreads();
    }
}

void launch_select(const uint32_t *cand_key, const int32_t *cand_idx, const int32_t *seg_cnt,
                   int32_t *sel, int32_t *sel_count, const uint32_t *hist_g, int n_heads, int k, int R,
                   int P, size_t cand_stride, uint32_t key_lo, int key_sh, hipStream_t st)
{
    k_select<<<n_heads, kSelNT, 0, st>>>(cand_key, cand_idx, seg_cnt, sel, sel_count, hist_g, k, R, P,
                                         cand_stride, key_lo, key_sh);
}

}  // namespace csa

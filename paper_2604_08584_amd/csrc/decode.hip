// Search half of the decode step (paper Sec. 3.3 steps 1-4): centroid scoring, choice of the
// probed rows, row gather with per-key score accumulation, Top-K selection.
#include <type_traits>

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
// EARLY (a launch of few workgroups, where latency is everything): the centroid is requested before
// the queries are staged - one memory round trip instead of two; on a full chip the early loads only
// hold back the staging (16 -> 26 us at batch 8).
// KEY (streaming updates, one-call iteration): the key about to be appended is scored against the
// same centroids in the same pass - z_key[bg][j] = c[bg][j] . k_new[bg], the same fma chain - so the
// try-insert after the step need not stream the centroid matrix again.
template <int GH, bool EARLY, bool KEY>
__global__ __launch_bounds__(256) void k_score_centroids(const uint16_t *__restrict__ q,
                                                         const uint4 *__restrict__ cent_t,
                                                         float *__restrict__ z, int C, int G,
                                                         const uint16_t *__restrict__ k_new,
                                                         float *__restrict__ z_key)
{
    constexpr int NV = GH + (KEY ? 1 : 0);  // vectors scored per pass: GH queries (+ the new key, as the last)
    __shared__ float s_q[NV][kHeadDim];
    const int bg = blockIdx.y;
    const int j = blockIdx.x * 256 + threadIdx.x;
    const uint4 *ct = cent_t + (size_t)bg * (kHeadDim / 8) * C;
    uint4 wv[kHeadDim / 8];
    if (EARLY) {
#pragma unroll
        for (int c = 0; c < kHeadDim / 8; ++c) wv[c] = j < C ? ct[(size_t)c * C + j] : make_uint4(0, 0, 0, 0);
    }
    for (int h0 = 0; h0 < G; h0 += GH) {
        __syncthreads();
        for (int e = threadIdx.x; e < GH * kHeadDim; e += 256) {
            const int hh = e / kHeadDim, t = e % kHeadDim;
            s_q[hh][t] = __uint_as_float((uint32_t)q[((size_t)bg * G + h0 + hh) * kHeadDim + t] << 16);
        }
        if (KEY && threadIdx.x < kHeadDim)  // (scored again in every pass over the heads: G > 8 is rare)
            s_q[NV - 1][threadIdx.x] = __uint_as_float((uint32_t)k_new[(size_t)bg * kHeadDim + threadIdx.x] << 16);
        __syncthreads();
        if (j < C) {
            float acc[NV];
#pragma unroll
            for (int hh = 0; hh < NV; ++hh) acc[hh] = 0.0f;
            if (!EARLY) {
#pragma unroll
                for (int c = 0; c < kHeadDim / 8; ++c) wv[c] = ct[(size_t)c * C + j];
            }
#pragma unroll
            for (int c = 0; c < kHeadDim / 8; ++c) {
                const uint4 w = wv[c];
                const float cf[8] = {bf16_lo(w.x), bf16_hi(w.x), bf16_lo(w.y), bf16_hi(w.y),
                                     bf16_lo(w.z), bf16_hi(w.z), bf16_lo(w.w), bf16_hi(w.w)};
#pragma unroll
                for (int e = 0; e < 8; ++e)
#pragma unroll
                    for (int hh = 0; hh < NV; ++hh)
                        acc[hh] = __builtin_fmaf(s_q[hh][c * 8 + e], cf[e], acc[hh]);
            }
#pragma unroll
            for (int hh = 0; hh < GH; ++hh)
                z[((size_t)bg * G + h0 + hh) * C + j] = acc[hh] + 0.0f;  // -0 -> +0
            if (KEY) z_key[(size_t)bg * C + j] = acc[NV - 1];
        }
    }
}

// The same for S > 1 subspaces of db = 128/S dimensions (Sec. 3.1 (i), 3.3 (1)): lane j of block
// (x, s, bg) scores centroid (s, j) against dimensions [s*db, (s+1)*db) of the G queries.
// cent_t is [bg][S][db/8][C][8]; z is [b][h][S][C].
// grid (ceil(C/256), S, B*Hkv), block 256.
template <int GH>
__global__ __launch_bounds__(256) void k_score_centroids_sub(const uint16_t *__restrict__ q,
                                                             const uint4 *__restrict__ cent_t,
                                                             float *__restrict__ z, int C, int G, int S)
{
    __shared__ float s_q[GH][kHeadDim / 2];
    const int sub = blockIdx.y, bg = blockIdx.z;
    const int db = kHeadDim / S, nch = db / 8;  // nch <= 8
    const int j = blockIdx.x * 256 + threadIdx.x;
    const uint4 *ct = cent_t + ((size_t)bg * S + sub) * nch * C;
    uint4 wv[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) wv[c] = (c < nch && j < C) ? ct[(size_t)c * C + j] : make_uint4(0, 0, 0, 0);
    for (int h0 = 0; h0 < G; h0 += GH) {
        __syncthreads();
        for (int e = threadIdx.x; e < GH * db; e += 256) {
            const int hh = e / db, t = e % db;
            s_q[hh][t] = __uint_as_float((uint32_t)q[((size_t)bg * G + h0 + hh) * kHeadDim + sub * db + t] << 16);
        }
        __syncthreads();
        if (j < C) {
            float acc[GH];
#pragma unroll
            for (int hh = 0; hh < GH; ++hh) acc[hh] = 0.0f;
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                if (c < nch) {
                    const uint4 w = wv[c];
                    const float cf[8] = {bf16_lo(w.x), bf16_hi(w.x), bf16_lo(w.y), bf16_hi(w.y),
                                         bf16_lo(w.z), bf16_hi(w.z), bf16_lo(w.w), bf16_hi(w.w)};
#pragma unroll
                    for (int e = 0; e < 8; ++e)
#pragma unroll
                        for (int hh = 0; hh < GH; ++hh)
                            acc[hh] = __builtin_fmaf(s_q[hh][c * 8 + e], cf[e], acc[hh]);
                }
            }
#pragma unroll
            for (int hh = 0; hh < GH; ++hh)
                z[(((size_t)bg * G + h0 + hh) * S + sub) * C + j] = acc[hh] + 0.0f;  // -0 -> +0
        }
    }
}

// Steps 1a + 1b in one launch for the paper's own geometry - several subspaces with few centroids
// each (C <= 256) and few probes per subspace (tau <= kFusedTau): the workgroup that scores
// subspace s of a KV head holds every centroid score of that subspace for the GH query heads in
// registers, so it also picks the tau best per head (tau rounds of "largest, ties to the lower
// centroid, remove") and publishes the probed rows and their block offsets, as k_top_centroids
// does.  No z array, no second launch.
// grid (1, S, B*Hkv), block 256.
constexpr int kFusedTau = 4;

template <int GH, bool KEY>
__global__ __launch_bounds__(256) void k_score_top_sub(const uint16_t *__restrict__ q,
                                                       const uint4 *__restrict__ cent_t,
                                                       int32_t *__restrict__ rows,
                                                       const int32_t *__restrict__ part_off,
                                                       int32_t *__restrict__ spans, int C, int G, int S,
                                                       int tau, int P, int nsub, int PO,
                                                       const uint16_t *__restrict__ k_new,
                                                       float *__restrict__ z_key)
{
    // KEY (streaming updates, one-call iteration): the key about to be appended is scored as one more
    // vector of the pass, z_key[bg][sub][j] = centroid (sub, j) . k_new[bg] over the subspace's dimensions
    constexpr int NV = GH + (KEY ? 1 : 0);
    __shared__ float s_q[NV][kHeadDim / 2];
    __shared__ unsigned long long s_best[256 / kWave][GH];  // per wave and head: (key, ~centroid)
    __shared__ int32_t s_rows[GH][kFusedTau];
    const int sub = blockIdx.y, bg = blockIdx.z;
    const int db = kHeadDim / S, nch = db / 8;  // nch <= 8
    const int j = threadIdx.x;
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const int M = S * tau, nb = nsub + 1;
    const uint4 *ct = cent_t + ((size_t)bg * S + sub) * nch * C;
    uint4 wv[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) wv[c] = (c < nch && j < C) ? ct[(size_t)c * C + j] : make_uint4(0, 0, 0, 0);
    for (int h0 = 0; h0 < G; h0 += GH) {
        __syncthreads();
        for (int e = threadIdx.x; e < GH * db; e += 256) {
            const int hh = e / db, t = e % db;
            s_q[hh][t] = __uint_as_float((uint32_t)q[((size_t)bg * G + h0 + hh) * kHeadDim + sub * db + t] << 16);
        }
        if (KEY && (int)threadIdx.x < db)  // (scored again in every pass over the heads: G > 8 is rare)
            s_q[NV - 1][threadIdx.x] = __uint_as_float((uint32_t)k_new[(size_t)bg * kHeadDim + sub * db + threadIdx.x] << 16);
        __syncthreads();
        uint32_t key[GH];  // order-preserving image of z; 0 = no centroid / already taken
        {
            float acc[NV];
#pragma unroll
            for (int hh = 0; hh < NV; ++hh) acc[hh] = 0.0f;
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                if (c < nch) {
                    const uint4 w = wv[c];
                    const float cf[8] = {bf16_lo(w.x), bf16_hi(w.x), bf16_lo(w.y), bf16_hi(w.y),
                                         bf16_lo(w.z), bf16_hi(w.z), bf16_lo(w.w), bf16_hi(w.w)};
#pragma unroll
                    for (int e = 0; e < 8; ++e)
#pragma unroll
                        for (int hh = 0; hh < NV; ++hh)
                            acc[hh] = __builtin_fmaf(s_q[hh][c * 8 + e], cf[e], acc[hh]);
                }
            }
#pragma unroll
            for (int hh = 0; hh < GH; ++hh) key[hh] = j < C ? orderable(acc[hh] + 0.0f) : 0u;  // -0 -> +0
            if (KEY && j < C) z_key[((size_t)bg * S + sub) * C + j] = acc[NV - 1];
        }
        for (int r = 0; r < tau; ++r) {
#pragma unroll
            for (int hh = 0; hh < GH; ++hh) {
                const uint32_t wm = wave_max(key[hh]);
                const int first = __ffsll((unsigned long long)__ballot(key[hh] == wm)) - 1;  // lowest centroid
                if (lane == 0)
                    s_best[wave][hh] = ((unsigned long long)wm << 32) | (uint32_t)~(uint32_t)(wave * kWave + first);
            }
            __syncthreads();
#pragma unroll
            for (int hh = 0; hh < GH; ++hh) {
                unsigned long long b = s_best[0][hh];
#pragma unroll
                for (int w = 1; w < 256 / kWave; ++w) b = max(b, s_best[w][hh]);
                const int win = (int)~(uint32_t)b;
                if (j == win) {
                    key[hh] = 0u;
                    s_rows[hh][r] = win;
                }
            }
            __syncthreads();
        }
        // the probed rows, and for every key range p the nsub + 1 block offsets of each probed row
        for (int t = threadIdx.x; t < GH * tau; t += 256) {
            const int hh = t / tau, r = t - hh * tau;
            rows[((size_t)bg * G + h0 + hh) * M + sub * tau + r] = sub * C + s_rows[hh][r];
        }
        for (int t = threadIdx.x; t < GH * P * tau * nb; t += 256) {
            const int x = t % nb, pr = t / nb;
            const int r = pr % tau, ph = pr / tau;
            const int p = ph % P, hh = ph / P;
            const size_t head = (size_t)bg * G + h0 + hh;
            spans[((head * P + p) * M + sub * tau + r) * nb + x] =
                part_off[((size_t)bg * S * C + (size_t)sub * C + s_rows[hh][r]) * PO + p * nsub + x];
        }
    }
}

// query heads of a KV head scored per pass over its centroids: the largest divisor of G up to 8
static int heads_per_pass(int G)
{
    for (int gh = 8; gh > 1; --gh)
        if (G % gh == 0) return gh;
    return 1;
}

bool score_top_fused(int C, int S, int tau) { return S > 1 && C <= 256 && tau <= kFusedTau; }

void launch_score_top_sub(const void *q, const void *cent_t, int32_t *rows, const int32_t *part_off,
                          int32_t *spans, int B, int Hkv, int G, int C, int S, int tau, int P, int nsub,
                          int PO, const void *k_new, float *z_key, hipStream_t st)
{
    dim3 grid(1, S, B * Hkv), block(256);
#define CSA_ST(GH_)                                                                                    \
    do {                                                                                               \
        if (z_key)                                                                                     \
            k_score_top_sub<GH_, true><<<grid, block, 0, st>>>((const uint16_t *)q, (const uint4 *)cent_t, rows, part_off, \
                                                               spans, C, G, S, tau, P, nsub, PO, (const uint16_t *)k_new, z_key); \
        else                                                                                           \
            k_score_top_sub<GH_, false><<<grid, block, 0, st>>>((const uint16_t *)q, (const uint4 *)cent_t, rows, part_off, \
                                                                spans, C, G, S, tau, P, nsub, PO, nullptr, nullptr); \
    } while (0)
    switch (heads_per_pass(G)) {
    case 8: CSA_ST(8); break;
    case 7: CSA_ST(7); break;
    case 6: CSA_ST(6); break;
    case 5: CSA_ST(5); break;
    case 4: CSA_ST(4); break;
    case 3: CSA_ST(3); break;
    case 2: CSA_ST(2); break;
    default: CSA_ST(1); break;
    }
#undef CSA_ST
}

void launch_score_centroids(const void *q, const void *cent_t, float *z, int B, int Hkv, int G,
                            int C, int S, const void *k_new, float *z_key, hipStream_t st)
{
    dim3 block(256);
    const int gh = heads_per_pass(G);
    if (S == 1) {
        dim3 grid((C + 255) / 256, B * Hkv);
        const bool early = (int64_t)grid.x * grid.y <= 256;
#define CSA_SC(GH_)                                                                                            \
    do {                                                                                                       \
        if (z_key && early)                                                                                    \
            k_score_centroids<GH_, true, true><<<grid, block, 0, st>>>((const uint16_t *)q, (const uint4 *)cent_t, z, C, G, (const uint16_t *)k_new, z_key); \
        else if (z_key)                                                                                        \
            k_score_centroids<GH_, false, true><<<grid, block, 0, st>>>((const uint16_t *)q, (const uint4 *)cent_t, z, C, G, (const uint16_t *)k_new, z_key); \
        else if (early)                                                                                        \
            k_score_centroids<GH_, true, false><<<grid, block, 0, st>>>((const uint16_t *)q, (const uint4 *)cent_t, z, C, G, nullptr, nullptr); \
        else                                                                                                   \
            k_score_centroids<GH_, false, false><<<grid, block, 0, st>>>((const uint16_t *)q, (const uint4 *)cent_t, z, C, G, nullptr, nullptr); \
    } while (0)
        switch (gh) {
        case 8: CSA_SC(8); break;
        case 7: CSA_SC(7); break;
        case 6: CSA_SC(6); break;
        case 5: CSA_SC(5); break;
        case 4: CSA_SC(4); break;
        case 3: CSA_SC(3); break;
        case 2: CSA_SC(2); break;
        default: CSA_SC(1); break;
        }
#undef CSA_SC
        return;
    }
    dim3 grid((C + 255) / 256, S, B * Hkv);
#define CSA_SC(GH_) \
    k_score_centroids_sub<GH_><<<grid, block, 0, st>>>((const uint16_t *)q, (const uint4 *)cent_t, z, C, G, S)
    switch (gh) {
    case 8: CSA_SC(8); break;
    case 7: CSA_SC(7); break;
    case 6: CSA_SC(6); break;
    case 5: CSA_SC(5); break;
    case 4: CSA_SC(4); break;
    case 3: CSA_SC(3); break;
    case 2: CSA_SC(2); break;
    default: CSA_SC(1); break;
    }
#undef CSA_SC
}

// ---------------------------------------------------------------------------------------------
// Step 1b: in one subspace of one head, the m = tau centroids with the largest z, ties to the
// lower index (Sec. 3.3 (1) with the top-tau back-off of Sec. 4.4), on the order-preserving
// integer image of z; they become table rows sub*C + j, slots [sub*tau, (sub+1)*tau) of the head's
// M = S*tau probed rows.
// Fast path (m small against C): every thread takes the maximum of its own slice; a lower bound
// on the m-th largest overall follows from the thread maxima, so only the few values >= that
// bound are candidates; they are ranked against each other by (z desc, j asc) and ranks < m are
// kept.  If there are too many candidates (many equal values) a radix threshold search with an
// ordered tie pick does the job instead.  With C <= 256 every value is a candidate.
// Also looks up, for every key range p, the
// nsub + 1 offsets that cut the slice of each probed row into its blocks, so that the
// accumulation kernel starts with one coalesced read.
// grid B*Hq*S, block 256 (1024 for a small launch of long score arrays).
// ---------------------------------------------------------------------------------------------
constexpr int kTopReg = 16;     // keys per thread held in registers
constexpr int kTopCand = 1024;  // candidate capacity of the fast path

template <int NT>
struct TopSmem {
    int32_t rows[64];  // the result: the m chosen centroids (valid after the barrier that follows select_top)
    alignas(16) uint32_t hist[256 + NT / kWave + 4];
    int scan[NT / kWave + 1];
    alignas(16) uint64_t ck[kTopCand + 2];  // (key << 32) | ~j : larger = better, distinct
    int slot;
    uint32_t bound;
};

// The m centroids of zh[0..C) with the largest score, ties to the lower index, into sm.rows (in
// no particular order on the fast path).  All NT threads of the workgroup must call; the caller
// puts a barrier between this call and its reads of sm.rows; sm may hold anything on entry.
template <int NT>
__device__ __forceinline__ void select_top(const float *__restrict__ zh, int C, int m, TopSmem<NT> &sm)
{
    if (threadIdx.x == 0) sm.slot = 0;
    // rank the nc candidates in sm.ck[0..nc) (distinct words, larger = better) against each other and
    // keep ranks < m.  A candidate is shared by tpc adjacent lanes, each counting over a slice of the
    // others, so that the chain of LDS reads is short however many threads the workgroup has.
    // (sm.ck[nc] must be 0 - the pad to an even count, 0 beats nothing - and the candidates visible)
    auto rank_candidates = [&](int nc) {
        int sh = 0;
        while (sh < 4 && ((nc * 2) << sh) <= NT) ++sh;  // tpc = 2^sh lanes per candidate (uniform)
        const int tpc = 1 << sh, part = (int)threadIdx.x & (tpc - 1);
        const int n2 = (nc + 1) / 2, per = (n2 + tpc - 1) >> sh;
        const int t_lo = part * per, t_hi = min(n2, t_lo + per);
        const ulonglong2 *c2 = (const ulonglong2 *)sm.ck;
        for (int a0 = 0; a0 < nc; a0 += NT >> sh) {  // (uniform trip count)
            const int a = a0 + ((int)threadIdx.x >> sh);
            const uint64_t mine = a < nc ? sm.ck[a] : ~0ull;
            int r = 0;
#pragma unroll 4
            for (int t2 = t_lo; t2 < t_hi; ++t2) {
                const ulonglong2 o = c2[t2];
                r += (o.x > mine) + (o.y > mine);
            }
            for (int x = 1; x < tpc; x <<= 1) r += __shfl_xor(r, x, kWave);
            if (a < nc && part == 0 && r < m) sm.rows[r] = (int32_t)~(uint32_t)mine;
        }
    };
    if (C <= 256) {
        // ---- few centroids: every value is a candidate
        for (int j = threadIdx.x; j <= C; j += NT)
            sm.ck[j] = j < C ? ((uint64_t)orderable(zh[j]) << 32) | (uint32_t)~(uint32_t)j : 0ull;
        __syncthreads();
        rank_candidates(C);
        return;
    }
    // (the candidate array starts out as zeros: whatever the count turns out to be, its pad is there)
    for (int e = threadIdx.x; e < kTopCand + 2; e += NT) sm.ck[e] = 0ull;
    const bool in_regs = C <= NT * kTopReg;
    uint32_t kreg[kTopReg];
    if (in_regs) {
#pragma unroll
        for (int u = 0; u < kTopReg; ++u) {
            const int j = u * NT + threadIdx.x;
            kreg[u] = j < C ? orderable(zh[j]) : 0u;
        }
    }
    const int rounds = (C + NT - 1) / NT;
    // visit(fn): fn(j, key, valid) for every centroid slot of this thread, uniformly per wave
    auto visit = [&](auto fn) {
        if (in_regs) {
#pragma unroll
            for (int u = 0; u < kTopReg; ++u)
                if (u < rounds) {
                    const int j = u * NT + threadIdx.x;
                    fn(j, kreg[u], j < C);
                }
        } else {
            for (int u = 0; u < rounds; ++u) {
                const int j = u * NT + threadIdx.x;
                fn(j, j < C ? orderable(zh[j]) : 0u, j < C);
            }
        }
    };
    if (m <= NT / 4 && C >= NT) {  // every lane holds at least one value
        // ---- fast path
        uint32_t best = 0;  // orderable(z) of a finite z is never 0
        visit([&](int, uint32_t key, bool valid) { if (valid && key > best) best = key; });
        // a lower bound on the m-th largest value overall: in each wave the r-th largest of the
        // 64 lane maxima, r = ceil(m / waves) (found by r rounds of max-and-remove); the smallest
        // of these over the waves has at least m values at or above it
        {
            constexpr int NWT = NT / kWave;
            const int r = (m + NWT - 1) / NWT;  // <= 16 of the 64 lane maxima; NWT * r >= m
            uint32_t cur = best, wmax = 0u;
            for (int round = 0; round < r; ++round) {
                wmax = wave_max(cur);
                const uint64_t holders = __ballot(cur == wmax);
                if (lane_id() == __ffsll((unsigned long long)holders) - 1) cur = 0u;  // remove one winner
            }
            if (lane_id() == 0) sm.hist[threadIdx.x / kWave] = wmax;
            __syncthreads();
            if (threadIdx.x < kWave) {
                uint32_t bnd = (int)threadIdx.x < NWT ? sm.hist[threadIdx.x] : 0xFFFFFFFFu;
                bnd = ~wave_max(~bnd);  // the smallest
                if (threadIdx.x == 0) sm.bound = bnd;
            }
        }
        __syncthreads();
        const uint32_t bound = sm.bound;
        visit([&](int j, uint32_t key, bool valid) {
            const bool in = valid && key >= bound;
            const uint64_t mask = __ballot(in);
            if (mask) {  // (uniform over the wave) one counter update per wave and round
                int base = 0;
                if (lane_id() == 0) base = atomicAdd(&sm.slot, (int)__popcll(mask));
                const int slot = __builtin_amdgcn_readfirstlane(base) + mbcnt(mask);
                if (in && slot < kTopCand) sm.ck[slot] = ((uint64_t)key << 32) | (uint32_t)~j;
            }
        });
        __syncthreads();
        const int nc = sm.slot;
        if (nc <= kTopCand && nc >= m) {  // (nc >= m always holds; checked so that no row is ever left unset)
            rank_candidates(nc);
            return;
        }
        __syncthreads();
        if (threadIdx.x == 0) sm.slot = 0;
    }
    // ---- general path: radix threshold, winners above it take any slot, ties in index order
    int need = 0;
    const uint32_t T = block_radix_threshold<NT, 8, 4>(
        [&](auto fn) { visit([&](int, uint32_t key, bool valid) { fn(key, valid); }); }, m, sm.hist,
        need);
    visit([&](int j, uint32_t key, bool valid) {
        if (valid && key > T) sm.rows[atomicAdd(&sm.slot, 1)] = j;
    });
    int ties_taken = 0;
    const int base = m - need;
    visit([&](int j, uint32_t key, bool valid) {
        const int is_tie = (valid && key == T) ? 1 : 0;
        int round_total;
        const int rank = block_excl_scan<NT>(is_tie, sm.scan, round_total) + ties_taken;
        if (is_tie && rank < need) sm.rows[base + rank] = j;
        ties_taken += round_total;
    });
}

template <int kTopNT>
__global__ __launch_bounds__(kTopNT) void k_top_centroids(const float *__restrict__ z,
                                                          int32_t *__restrict__ rows,
                                                          const int32_t *__restrict__ part_off,
                                                          int32_t *__restrict__ spans, int C, int S,
                                                          int m, int G, int P, int nsub, int PO)
{
    const int head = blockIdx.x / S, sub = blockIdx.x - head * S;
    const int M = S * m;
    __shared__ TopSmem<kTopNT> sm;
    int32_t *out = rows + (size_t)head * M + sub * m;
    select_top<kTopNT>(z + (size_t)blockIdx.x * C, C, m, sm);
    // the probed rows, and for every key range p the nsub + 1 block offsets of each probed row
    __syncthreads();
    const int32_t *s_rows = sm.rows;
    if ((int)threadIdx.x < m) out[threadIdx.x] = sub * C + s_rows[threadIdx.x];
    const int bg = head / G;
    const int nb = nsub + 1;
    int32_t *sp = spans + (size_t)head * P * M * nb;
    // (four independent loads in flight per thread before the first store)
    for (int t0 = threadIdx.x; t0 < P * m * nb; t0 += 4 * kTopNT) {
        int32_t v[4];
        size_t dst[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int t = min(t0 + u * kTopNT, P * m * nb - 1);
            const int x = t % nb, pr = t / nb;
            const int p = pr / m, r = pr - p * m;
            dst[u] = ((size_t)p * M + sub * m + r) * nb + x;
            v[u] = part_off[((size_t)bg * S * C + (size_t)sub * C + s_rows[r]) * PO + p * nsub + x];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (t0 + u * kTopNT < P * m * nb) sp[dst[u]] = v[u];
    }
}

void launch_top_centroids(const float *z, int32_t *rows, const int32_t *part_off, int32_t *spans,
                          int n_heads, int C, int S, int tau, int G, int P, int nsub, int PO, hipStream_t st)
{
    // a small launch (fewer workgroups than CUs) of long score arrays: 1024 threads per head shorten
    // every phase of this chain of latencies
    if (n_heads * S <= 256 && C >= 1024)
        k_top_centroids<1024><<<n_heads * S, 1024, 0, st>>>(z, rows, part_off, spans, C, S, tau, G, P, nsub, PO);
    else
        k_top_centroids<256><<<n_heads * S, 256, 0, st>>>(z, rows, part_off, spans, C, S, tau, G, P, nsub, PO);
}

// ---------------------------------------------------------------------------------------------
// Steps 2+3: gather the m probed rows and sum scores per key (Sec. 3.3 (2)-(3), w_b = 1).
// Rows are stored sorted by key index with per-row offsets of every block of key indices, so
// workgroup (head, p) reads only the slices of its range [p*R, (p+1)*R) - every table byte is
// read once - and keeps R direct-addressed integer accumulators in LDS.  Each entry adds
// q*64 + 1: exact integer sums, order-free, and "seen" == accumulator != 0 (U of Sec. 3.3 (3):
// a key absent from every probed row is not a candidate even if all sums are negative).
// A wave owns whole rows (row constants are scalar) and keeps the slices of four rows in
// flight, 16 bytes (4 packed entries) per lane and round.  The kernel is bound by instruction
// issue and the LDS atomic rate, so the per-entry and per-slot paths are kept minimal.  What
// leaves the workgroup are the range's candidates as 32-bit words grouped by coarse bin of
// their sum, best bin first (a counting sort through LDS), and the start offset of every bin:
// the selection kernels then read offsets and one bin instead of every candidate.
// grid (P, B*Hq), block NT = R/16, dynamic LDS R*4 bytes.
// ---------------------------------------------------------------------------------------------
constexpr int kAccRows = 4;  // rows in flight per wave

// SELF_TOP (one subspace, small launches): no launch of k_top_centroids came before - the workgroup
// first picks the head's m best centroids from the scores z itself (every range's workgroup repeats
// that choice; with few workgroups the repeated work is cheaper than a launch in the chain) and
// looks up its block offsets in part_off; the workgroup of range 0 publishes the probed rows.
template <int NT, bool SELF_TOP>
__global__ __launch_bounds__(NT) void k_accumulate(const uint32_t *__restrict__ ent,
                                                   int32_t *__restrict__ rows,
                                                   const int32_t *__restrict__ spans,
                                                   uint32_t *__restrict__ cand_key,
                                                   uint16_t *__restrict__ bin_off,
                                                   int32_t *__restrict__ seg_cnt, int C, int Ls,
                                                   int m, int G, int P, size_t cand_stride,
                                                   uint32_t key_lo, int key_sh, int excl_from,
                                                   const float *__restrict__ z,
                                                   const int32_t *__restrict__ part_off, int PO, int c_sh)
{
    constexpr int NW = NT / kWave;
    constexpr int R = NT * 16;
    constexpr int NSUB = R > kUnit ? R / kUnit : 1;  // blocks of a range (1, 2 or 4)
    constexpr int NB = NSUB + 1;
    extern __shared__ __align__(16) int32_t s_acc[];  // [R]
    __shared__ int32_t s_b[64 * NB], s_row[64];
    __shared__ uint32_t s_h[kCoarseBins], s_pos[kCoarseBins];
    __shared__ int s_scan[NW + 1];
    const int p = blockIdx.x, head = blockIdx.y;
    const int bg = head / G;
    const int wave = threadIdx.x / kWave, lane = lane_id();
    {
        int4 *z4 = (int4 *)s_acc;
#pragma unroll
        for (int u = 0; u < 4; ++u) z4[u * NT + threadIdx.x] = make_int4(0, 0, 0, 0);
        for (int e = threadIdx.x; e < kCoarseBins; e += NT) s_h[e] = 0;
    }
    if (SELF_TOP) {
        static_assert(!SELF_TOP || 2 * NT >= 64 * NB, "two offsets per thread cover m * NB");
        // (LDS of its own - 10 KiB, three workgroups per CU instead of four, which a launch this small
        // does not fill anyway - so that the accumulators are zeroed while the scores are on their way)
        __shared__ typename std::conditional<SELF_TOP, TopSmem<NT>, int>::type s_top;
        TopSmem<NT> &sm = *reinterpret_cast<TopSmem<NT> *>(&s_top);
        select_top<NT>(z + (size_t)head * C, C, m, sm);
        __syncthreads();
        if ((int)threadIdx.x < m) {
            const int my_row = sm.rows[threadIdx.x];
            s_row[threadIdx.x] = my_row;
            if (p == 0) rows[(size_t)head * m + threadIdx.x] = my_row;
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int e = u * NT + (int)threadIdx.x;
            const int r = e / NB, x = e - r * NB;
            if (e < m * NB) s_b[e] = part_off[((size_t)bg * C + sm.rows[r]) * PO + p * NSUB + x];
        }
    } else {
        const int32_t *sp = spans + ((size_t)head * P + p) * m * NB;
        for (int e = threadIdx.x; e < m * NB; e += NT) s_b[e] = sp[e];
        if ((int)threadIdx.x < m) s_row[threadIdx.x] = rows[(size_t)head * m + threadIdx.x];
    }
    __syncthreads();
    // slot of an entry = (its block within the range) * kUnit + (low index bits) - off0
    const int off0 = (p * R) & (kUnit - 1);  // non-zero only for ranges smaller than a block
    constexpr int kChunk = kWave * 4;  // entries of one round of 16-byte loads
    // With few probed rows (the paper's geometry: one long row per subspace) a row's slice is cut into
    // 2^c_sh pieces that are walked as rows of their own, so that the workgroup still has kAccRows * NW
    // loads in flight instead of a few waves walking long slices round after round.
    const int mv = m << c_sh;
    for (int r0 = wave; r0 < mv; r0 += kAccRows * NW) {
        int lo[kAccRows], hi[kAccRows], b1[kAccRows], b2[kAccRows], b3[kAccRows];
        int n_wide[kAccRows], n_tail[kAccRows];
        const uint32_t *rp[kAccRows];
        int rounds = 0;
        // the constants of the wave's rows come out of LDS with ONE read - lane (what, j) fetches
        // constant `what` of row j - and are handed out by lane reads; a read per constant would be a
        // chain of two dozen LDS round trips
        int gv = 0;
        {
            const int jj = lane % kAccRows, what = lane / kAccRows;  // what: lo, hi, b1, b2, b3, row
            const int r = r0 + jj * NW;
            const int rr = (r < mv ? r : r0) >> c_sh;
            const int within = what == 1 ? NSUB : what == 0 ? 0 : what - 1;
            const int32_t *src = what == 5 ? s_row + rr : s_b + rr * NB + min(within, NSUB);
            if (what <= 5) gv = *src;
        }
#pragma unroll
        for (int j = 0; j < kAccRows; ++j) {
            const bool on = r0 + j * NW < mv;
            lo[j] = __builtin_amdgcn_readlane(gv, 0 * kAccRows + j);
            hi[j] = on ? __builtin_amdgcn_readlane(gv, 1 * kAccRows + j) : lo[j];  // empty if no such row
            b1[j] = NSUB > 1 ? __builtin_amdgcn_readlane(gv, 2 * kAccRows + j) : 0x7FFFFFFF;
            b2[j] = NSUB > 2 ? __builtin_amdgcn_readlane(gv, 3 * kAccRows + j) : 0x7FFFFFFF;
            b3[j] = NSUB > 2 ? __builtin_amdgcn_readlane(gv, 4 * kAccRows + j) : 0x7FFFFFFF;
            rp[j] = ent + ((size_t)bg * C + __builtin_amdgcn_readlane(gv, 5 * kAccRows + j)) * Ls;
            lo[j] = min(lo[j], hi[j]);
            if (c_sh) {  // this piece of the slice
                const int piece = (r0 + j * NW) & ((1 << c_sh) - 1), len = hi[j] - lo[j];
                hi[j] = lo[j] + ((len * (piece + 1)) >> c_sh);
                lo[j] = lo[j] + ((len * piece) >> c_sh);
            }
            // the slice from its 16-byte boundary: rounds of 16 bytes per lane, and - when what is
            // left after them fits one entry per lane - one such round instead of a mostly idle wide
            // one (a slice of a 1/P share of a row is typically a little over one wide round)
            const int n = hi[j] - (lo[j] & ~3);
            const int left = n % kChunk;
            n_wide[j] = n / kChunk + (left > kWave ? 1 : 0);
            n_tail[j] = left > kWave ? 0 : left;
            rounds = max(rounds, n_wide[j]);
        }
        auto add = [&](uint32_t e, int pos, int j) {
            if ((uint32_t)(pos - lo[j]) < (uint32_t)(hi[j] - lo[j])) {
                int slot = (int)(e & (uint32_t)(kUnit - 1)) - off0;
                if (NSUB > 1) slot += (pos >= b1[j]) ? kUnit : 0;
                if (NSUB > 2) slot += ((pos >= b2[j]) ? kUnit : 0) + ((pos >= b3[j]) ? kUnit : 0);
                const int32_t val = entry_q(e) * (1 << kCntBits) + 1;
                if ((unsigned)slot < (unsigned)R) atomicAdd(&s_acc[slot], val);
            }
        };
        uint32_t vt[kAccRows];  // the one-per-lane leftovers: requested first, used last
#pragma unroll
        for (int j = 0; j < kAccRows; ++j)
            vt[j] = lane < n_tail[j] ? rp[j][(lo[j] & ~3) + n_wide[j] * kChunk + lane] : 0u;
        for (int it = 0; it < rounds; ++it) {
            uint4 va[kAccRows];
#pragma unroll
            for (int j = 0; j < kAccRows; ++j) {
                const int x = (lo[j] & ~3) + it * kChunk + lane * 4;
                va[j] = it < n_wide[j] && x < hi[j] ? *(const uint4 *)(rp[j] + x) : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < kAccRows; ++j) {
                const int x = (lo[j] & ~3) + it * kChunk + lane * 4;
                if (it < n_wide[j]) {  // (scalar)
                    add(va[j].x, x, j);
                    add(va[j].y, x + 1, j);
                    add(va[j].z, x + 2, j);
                    add(va[j].w, x + 3, j);
                }
            }
        }
#pragma unroll
        for (int j = 0; j < kAccRows; ++j)
            if (lane < n_tail[j]) add(vt[j], (lo[j] & ~3) + n_wide[j] * kChunk + lane, j);
    }
    __syncthreads();
    // thread t owns the slot groups 4*(u*NT + t) .. +3, u < 4 (128-bit LDS reads)
    int4 a[4];
    // key indices at or above excl_from (the always-attended recent window, which streaming updates
    // may have put into the tables) are not candidates; only the last range(s) can hold any
    const bool has_excl = p * R + R > excl_from;  // (uniform over the workgroup)
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        a[u] = ((const int4 *)s_acc)[u * NT + threadIdx.x];
        if (has_excl) {
            const int i0 = p * R + 4 * (u * NT + (int)threadIdx.x);
            if (i0 + 0 >= excl_from) a[u].x = 0;
            if (i0 + 1 >= excl_from) a[u].y = 0;
            if (i0 + 2 >= excl_from) a[u].z = 0;
            if (i0 + 3 >= excl_from) a[u].w = 0;
        }
    }
    // The candidates leave grouped by coarse bin of their accumulated score, best bin first (a
    // counting sort through LDS): word = (score bits below the bin) << kIdxBits | slot in the range.
    // The Top-K threshold then needs the per-range bin offsets and the one bin it falls in, and a
    // range's winners are a prefix of its candidates plus part of that bin.
    // every accumulator becomes d = (its score key) - key_lo once (kEmpty for an untouched slot): the
    // two passes below then need a shift each
    constexpr uint32_t kEmpty = 0xFFFFFFFFu;  // (a real d is below 2^25)
    const int32_t rebase = kKeyBias - (int32_t)key_lo;
    uint32_t d[16];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int av[4] = {a[u].x, a[u].y, a[u].z, a[u].w};
#pragma unroll
        for (int x = 0; x < 4; ++x) d[4 * u + x] = av[x] != 0 ? (uint32_t)((av[x] >> kCntBits) + rebase) : kEmpty;
    }
    // pass 1: occupancy of the bins (s_h is indexed by the bin itself, the output by the reversed
    // bin: output bin 0 holds the largest scores)
    const uint32_t low_mask = (1u << key_sh) - 1u;
#pragma unroll
    for (int i = 0; i < 16; ++i)
        if (d[i] != kEmpty) atomicAdd(&s_h[d[i] >> key_sh], 1u);
    __syncthreads();
    // exclusive scan over the reversed bins: where each bin's run starts (kept in LDS as the running
    // write position of the bin, and written out for the selection kernels)
    constexpr int BPT = NT >= kCoarseBins ? 1 : kCoarseBins / NT;  // bins per owning thread
    const bool owner = (int)threadIdx.x * BPT < kCoarseBins;
    int cnt[BPT], mine = 0;
#pragma unroll
    for (int j = 0; j < BPT; ++j) {
        cnt[j] = owner ? (int)s_h[(kCoarseBins - 1) - (threadIdx.x * BPT + j)] : 0;
        mine += cnt[j];
    }
    int total;
    int start = block_excl_scan<NT>(mine, (int *)s_scan, total);
    uint16_t *bo = bin_off + ((size_t)head * P + p) * kCoarseBins;
    if (owner) {
#pragma unroll
        for (int j = 0; j < BPT; ++j) {
            s_pos[(kCoarseBins - 1) - (threadIdx.x * BPT + j)] = (uint32_t)start;
            bo[threadIdx.x * BPT + j] = (uint16_t)start;
            start += cnt[j];
        }
    }
    __syncthreads();
    // pass 2: every candidate takes the next position of its bin (every accumulator is in
    // registers by now, so the accumulator array is free to hold the sorted words)
    uint32_t *s_out = (uint32_t *)s_acc;
#pragma unroll
    for (int i = 0; i < 16; ++i)
        if (d[i] != kEmpty) {
            const uint32_t at = atomicAdd(&s_pos[d[i] >> key_sh], 1u);
            // slot of accumulator i = 4 * ((i / 4) * NT + thread) + i % 4
            s_out[at] = ((d[i] & low_mask) << kIdxBits) | (uint32_t)(4 * ((i >> 2) * NT + (int)threadIdx.x) + (i & 3));
        }
    __syncthreads();
    uint32_t *dk = cand_key + (size_t)head * cand_stride + (size_t)p * R;
    for (int i = threadIdx.x; i < total; i += NT) dk[i] = s_out[i];
    if (threadIdx.x == 0) seg_cnt[(size_t)head * P + p] = total;
}

// does the accumulation launch choose the probed rows itself (no k_top_centroids launch)?
bool accumulate_self_top(int n_heads, int S, int C, int tau, int R, int P)
{
    return S == 1 && R >= 4096 && (int64_t)n_heads * P <= 1024;
}

void launch_accumulate(const void *ent, int32_t *rows, const int32_t *spans, uint32_t *cand_key,
                       uint16_t *bin_off, int32_t *seg_cnt, int n_heads, int C,
                       int Ls, int m, int G, int R, int P, size_t cand_stride, uint32_t key_lo,
                       int key_sh, int excl_from, const float *z, const int32_t *part_off, int PO,
                       bool self_top, hipStream_t st)
{
    dim3 grid(P, n_heads);
    // pieces per row slice: as many as keep every wave's row slots busy, while a piece still holds at
    // least ~128 entries
    int c_sh = 0;
    {
        const int slots = kAccRows * (R / 16 / kWave);
        const int per_slice = Ls / (P > 0 ? P : 1);
        while (c_sh < 5 && (m << (c_sh + 1)) <= slots && (per_slice >> (c_sh + 1)) >= 128) ++c_sh;
    }
    static bool attr = false;
    if (!attr) {
        (void)hipFuncSetAttribute((const void *)k_accumulate<1024, false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                  16384 * 4);
        (void)hipFuncSetAttribute((const void *)k_accumulate<1024, true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                  16384 * 4);
        attr = true;
    }
#define CSA_ACC(NT_, SELF_)                                                                                \
    k_accumulate<NT_, SELF_><<<grid, NT_, (size_t)R * 4, st>>>((const uint32_t *)ent, rows, spans, cand_key, \
                                                               bin_off, seg_cnt, C, Ls, m, G, P, cand_stride, \
                                                               key_lo, key_sh, excl_from, z, part_off, PO, c_sh)
    if (self_top) {  // (R >= 4096: see accumulate_self_top)
        switch (R) {
        case 4096: CSA_ACC(256, true); break;
        case 8192: CSA_ACC(512, true); break;
        default: CSA_ACC(1024, true); break;  // 16384
        }
        return;
    }
    switch (R) {
    case 1024: CSA_ACC(64, false); break;
    case 2048: CSA_ACC(128, false); break;
    case 4096: CSA_ACC(256, false); break;
    case 8192: CSA_ACC(512, false); break;
    default: CSA_ACC(1024, false); break;  // 16384
    }
#undef CSA_ACC
}

// ---------------------------------------------------------------------------------------------
// Step 4, first half: the Top-K threshold of one head (Sec. 3.3 (4)).  The accumulation kernel
// left every key range's candidates grouped by coarse score bin (best first) with the bins' start
// offsets, so the head's histogram is a sum of offset differences, the bin B holding the k-th
// largest score follows from it, and everything in better bins is selected without being looked
// at.  Only the candidates of bin B (a run per key range) are read: their scores within the bin
// are searched for the value T such that the winners are every candidate above T plus the `need`
// lowest-index candidates equal to T - in LDS by a radix search when the bin holds few enough,
// else by refining the range with histogram passes over the runs first.  Output:
//   thr[head] = B << kThrShift | T   (0xFFFFFFFF: nothing selected; B = 512: every candidate),
//   seg_par[head][p] = (first output slot of range p, ties range p may keep).
// grid B*Hq, block NT.
// ---------------------------------------------------------------------------------------------
// grid B*Hq, block NT.
template <int kThrNT>
__global__ __launch_bounds__(kThrNT) void k_threshold(const uint32_t *__restrict__ cand_key,
                                                      const int32_t *__restrict__ seg_cnt,
                                                      const uint16_t *__restrict__ bin_off,
                                                      int32_t *__restrict__ sel,
                                                      int32_t *__restrict__ sel_count,
                                                      uint32_t *__restrict__ thr,
                                                      int2 *__restrict__ seg_par,
                                                      int2 *__restrict__ seg_run, int k, int R, int P,
                                                      size_t cand_stride, int key_sh)
{
    __shared__ ThrSmem<kThrNT, kSelMaxP> sm;
    const int head = blockIdx.x;
    int k_eff;
    const uint32_t T = head_threshold<kThrNT, kSelMaxP>(
        cand_key + (size_t)head * cand_stride, seg_cnt + (size_t)head * P,
        bin_off + (size_t)head * P * kCoarseBins, k, R, P, key_sh, sm, k_eff, [&](int p, int off, int al) {
            seg_par[(size_t)head * P + p] = make_int2(off, al);
            // (sm.beg / sm.end are only set when something is selected)
            if (k_eff > 0) seg_run[(size_t)head * P + p] = make_int2((int)sm.beg[p], (int)sm.end[p]);
        });
    if (threadIdx.x == 0) {
        sel_count[head] = k_eff;
        thr[head] = T;
    }
    int32_t *out = sel + (size_t)head * k;
    for (int a = k_eff + threadIdx.x; a < k; a += kThrNT) out[a] = -1;
}

void launch_threshold(const uint32_t *cand_key, const int32_t *seg_cnt, const uint16_t *bin_off, int32_t *sel,
                      int32_t *sel_count, uint32_t *thr, void *seg_par, void *seg_run, int n_heads, int k,
                      int R, int P, size_t cand_stride, int key_sh, hipStream_t st)
{
    // two 512-thread workgroups fit a CU: with more heads than CUs all heads run at once
    if (n_heads > 256)
        k_threshold<512><<<n_heads, 512, 0, st>>>(cand_key, seg_cnt, bin_off, sel, sel_count, thr,
                                                  (int2 *)seg_par, (int2 *)seg_run, k, R, P, cand_stride,
                                                  key_sh);
    else
        k_threshold<1024><<<n_heads, 1024, 0, st>>>(cand_key, seg_cnt, bin_off, sel, sel_count, thr,
                                                    (int2 *)seg_par, (int2 *)seg_run, k, R, P, cand_stride,
                                                    key_sh);
}

// ---------------------------------------------------------------------------------------------
// Step 4, second half as a kernel of its own (see emit_range in common.h): used when the gathered
// attention cannot do it in its prologue.
// grid (P, B*Hq), block NT = max(64, R/32).
// ---------------------------------------------------------------------------------------------
template <int NT>
__global__ __launch_bounds__(NT) void k_emit(const uint32_t *__restrict__ cand_key,
                                             const int2 *__restrict__ seg_run,
                                             const int32_t *__restrict__ seg_cnt,
                                             const uint32_t *__restrict__ thr,
                                             const int2 *__restrict__ seg_par,
                                             int32_t *__restrict__ sel, int k, int R, int P,
                                             size_t cand_stride)
{
    __shared__ uint32_t s_bits[2 * NT];  // NT >= R/32 words each for the winners and the ties
    __shared__ int s_scan[NT / kWave + 1];
    int first;
    (void)emit_range<NT>(cand_key, seg_run, seg_cnt, thr, seg_par, sel, k, R, P, cand_stride, blockIdx.y,
                         blockIdx.x, s_bits, s_scan, first);
}

void launch_emit(const uint32_t *cand_key, const void *seg_run, const int32_t *seg_cnt,
                 const uint32_t *thr, const void *seg_par, int32_t *sel, int n_heads, int k, int R, int P,
                 size_t cand_stride, hipStream_t st)
{
    if (k <= 0) return;
    dim3 grid(P, n_heads);
#define CSA_EMIT(NT_)                                                                               \
    k_emit<NT_><<<grid, NT_, 0, st>>>(cand_key, (const int2 *)seg_run, seg_cnt, thr, (const int2 *)seg_par, sel, k, R, P, \
                                      cand_stride)
    switch (R) {
    case 1024: CSA_EMIT(64); break;
    case 2048: CSA_EMIT(64); break;
    case 4096: CSA_EMIT(128); break;
    case 8192: CSA_EMIT(256); break;
    default: CSA_EMIT(512); break;  // 16384
    }
#undef CSA_EMIT
}

}  // namespace csa

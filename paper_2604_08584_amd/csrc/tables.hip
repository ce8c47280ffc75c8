// Offline side: lookup-table construction (paper Sec. 3.2 (2)), conversion between the canonical
// table layout (rows sorted by score, Sec. 3.1 (iii)) and the library's private device layout
// (rows sorted by key index + per-row offsets of every key range), centroid repacking.
#include "common.h"
#include "kernels.h"

namespace csa {

// cent [n_bg][S][C][db] bf16 -> cent_t [n_bg][S][db/8][C][8] bf16 (one 16-byte chunk per thread;
// db = 128 / S dimensions per subspace)
__global__ void k_pack_centroids(const uint4 *__restrict__ cent, uint4 *__restrict__ cent_t, int C, int S)
{
    const int bg = blockIdx.y;
    const int e = blockIdx.x * 256 + threadIdx.x;  // = ((s * C) + j) * nch + c
    if (e >= C * 16) return;
    const int nch = 16 / S;
    const int c = e % nch, sj = e / nch;
    const int s = sj / C, j = sj - s * C;
    cent_t[(((size_t)bg * S + s) * nch + c) * C + j] = cent[(size_t)bg * C * 16 + e];
}

void launch_pack_centroids(const void *cent, void *cent_t, int n_bg, int C, int S, hipStream_t st)
{
    dim3 grid((C * 16 + 255) / 256, n_bg);
    k_pack_centroids<<<grid, 256, 0, st>>>((const uint4 *)cent, (uint4 *)cent_t, C, S);
}

// in-LDS bitonic sort of NP (power of two) 64-bit keys, ascending; all threads of the block
template <int NT>
__device__ __forceinline__ void bitonic_sort_u64(uint64_t *s, int NP)
{
    for (int k2 = 2; k2 <= NP; k2 <<= 1) {
        for (int j = k2 >> 1; j > 0; j >>= 1) {
            __syncthreads();
            for (int i = threadIdx.x; i < NP; i += NT) {
                const int x = i ^ j;
                if (x > i) {
                    const uint64_t a = s[i], b = s[x];
                    const bool up = (i & k2) == 0;
                    if ((a > b) == up) { s[i] = b; s[x] = a; }
                }
            }
        }
    }
    __syncthreads();
}

// first position in the ascending array a[0, n) whose value is >= bound
template <class T>
__device__ __forceinline__ int lower_bound_pos(const T *a, int n, T bound)
{
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (a[mid] < bound) lo = mid + 1; else hi = mid;
    }
    return lo;
}

// ---------------------------------------------------------------------------------------------
// Canonical rows -> device rows.  One workgroup per row: checks every (idx, score), converts
// score to its grid integer q (exact or flagged), sorts by key index, writes packed entries
// (row stride Ls, unused slots zero) and the row's offsets part_off[u] = number of entries with
// key index < u * Q, u < PO.
// flags[0] |= 1: score off the grid or too large; |= 2: index outside [-1, n_pre).
// flags[1] = max |q| over all entries (atomicMax).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_import_rows(const int32_t *__restrict__ idx,
                                                     const float *__restrict__ score,
                                                     uint32_t *__restrict__ ent,
                                                     int32_t *__restrict__ part_off,
                                                     int32_t *__restrict__ flags, int L, int Ls,
                                                     int NP, int n_pre, float up, int qmax, int Q,
                                                     int PO)
{
    extern __shared__ uint64_t s_keys[];
    const size_t row = blockIdx.x;
    int bad = 0, qabs = 0;
    for (int p = threadIdx.x; p < NP; p += 256) {
        uint64_t key = ~0ull;
        if (p < L) {
            const int32_t i = idx[row * L + p];
            if (i >= n_pre || i < -1) {
                bad |= 2;
            } else if (i >= 0) {
                const float qf = score[row * L + p] * up;
                if (!(fabsf(qf) <= (float)qmax) || qf != rintf(qf)) bad |= 1;
                const int32_t q = bad ? 0 : (int32_t)qf;
                qabs = max(qabs, abs(q));
                key = ((uint64_t)(uint32_t)i << 32) | (uint32_t)q;
            }
        }
        s_keys[p] = key;
    }
    if (bad) atomicOr(flags, bad);
    for (int o = 32; o > 0; o >>= 1) qabs = max(qabs, __shfl_xor(qabs, o, kWave));
    if (lane_id() == 0 && !bad) atomicMax(flags + 1, qabs);
    bitonic_sort_u64<256>(s_keys, NP);
    for (int p = threadIdx.x; p < Ls; p += 256) {
        const uint64_t key = p < NP ? s_keys[p] : ~0ull;
        ent[row * Ls + p] = key == ~0ull ? 0u : pack_entry((int32_t)(key >> 32), (int32_t)(uint32_t)key);
    }
    for (int u = threadIdx.x; u < PO; u += 256)
        part_off[row * PO + u] = lower_bound_pos<uint64_t>(s_keys, NP, (uint64_t)u * (uint64_t)Q << 32);
}

static int next_pow2(int x) { int p = 1; while (p < x) p <<= 1; return p; }

void launch_import_rows(const int32_t *idx, const float *score, void *ent, int32_t *part_off,
                        int32_t *flags, int64_t n_rows, int L, int Ls, int n_pre, int F, int qmax,
                        int Q, int PO, hipStream_t st)
{
    const int NP = next_pow2(L);
    static bool attr = false;
    if (!attr) {
        (void)hipFuncSetAttribute((const void *)k_import_rows, hipFuncAttributeMaxDynamicSharedMemorySize, 8192 * 8);
        attr = true;
    }
    k_import_rows<<<(unsigned)n_rows, 256, (size_t)NP * 8, st>>>(idx, score, (uint32_t *)ent, part_off, flags,
                                                                 L, Ls, NP, n_pre, ldexpf(1.0f, F), qmax, Q, PO);
}

// Device rows -> canonical rows: sort by (score desc, idx asc), unused slots last.  The block of
// an entry (hence the high bits of its key index) follows from its position and the row offsets.
__global__ __launch_bounds__(256) void k_export_rows(const uint32_t *__restrict__ ent,
                                                     const int32_t *__restrict__ part_off,
                                                     int32_t *__restrict__ idx,
                                                     float *__restrict__ score, int L, int Ls, int NP,
                                                     float down, int Q, int PO)
{
    extern __shared__ uint64_t s_keys[];
    const size_t row = blockIdx.x;
    const int32_t *po = part_off + row * PO;
    const int count = po[PO - 1];
    for (int p = threadIdx.x; p < NP; p += 256) {
        uint64_t key = ~0ull;
        if (p < count && p < L) {
            const uint32_t e = ent[row * Ls + p];
            // block u: the last one whose first entry is at or before p
            int lo = 0, hi = PO - 1;  // po[lo] <= p < po[hi]
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (po[mid] <= p) lo = mid; else hi = mid;
            }
            const uint32_t i = (((uint32_t)lo * (uint32_t)Q) & ~(uint32_t)(kUnit - 1)) | (e & (uint32_t)(kUnit - 1));
            const int32_t q = entry_q(e);
            key = ((uint64_t)(~((uint32_t)q ^ 0x80000000u)) << 32) | i;
        }
        s_keys[p] = key;
    }
    bitonic_sort_u64<256>(s_keys, NP);
    for (int p = threadIdx.x; p < L; p += 256) {
        const uint64_t key = s_keys[p];
        if (key == ~0ull) {
            idx[row * L + p] = -1;
            score[row * L + p] = 0.0f;
        } else {
            const int32_t q = (int32_t)((~(uint32_t)(key >> 32)) ^ 0x80000000u);
            idx[row * L + p] = (int32_t)(uint32_t)key;
            score[row * L + p] = (float)q * down;
        }
    }
}

void launch_export_rows(const void *ent, const int32_t *part_off, int32_t *idx, float *score,
                        int n_rows, int L, int Ls, int F, int Q, int PO, hipStream_t st)
{
    const int NP = next_pow2(L);
    static bool attr = false;
    if (!attr) {
        (void)hipFuncSetAttribute((const void *)k_export_rows, hipFuncAttributeMaxDynamicSharedMemorySize, 8192 * 8);
        attr = true;
    }
    k_export_rows<<<n_rows, 256, (size_t)NP * 8, st>>>((const uint32_t *)ent, part_off, idx, score, L, Ls, NP,
                                                       ldexpf(1.0f, -F), Q, PO);
}

// ---------------------------------------------------------------------------------------------
// Table build, part 1: grid integers q[jj][i] = round-half-even(2^F * (c . k_i^(s))) for one KV
// head, one subspace s (dimensions [s*DB, (s+1)*DB) of the head) and a chunk of that subspace's
// centroids (Sec. 3.2 (2)).  One lane per key (its sub-vector lives in registers as DB fp32),
// centroids staged through LDS 64 at a time and broadcast.  The inner product is one fma chain
// over ascending dimension from +0 - the same definition as the decode-time centroid scores - so
// the table contents are reproducible bit for bit.
// grid ceil(n_pre/256), block 256.  cent points at the chunk's first centroid ([jc][DB] bf16).
// ---------------------------------------------------------------------------------------------
constexpr int kBuildTile = 64;

template <bool PAGED, int DB>
__global__ __launch_bounds__(256) void k_build_scores(const uint16_t *__restrict__ kc,
                                                      const int32_t *__restrict__ block_table,
                                                      const uint16_t *__restrict__ cent,
                                                      int32_t *__restrict__ qs,
                                                      int32_t *__restrict__ flags, int b, int g,
                                                      int Hkv, int max_ctx, int n_pre, int sub,
                                                      int jc, float up, int qmax)
{
    constexpr int NCH = DB / 8;
    __shared__ uint4 s_c[kBuildTile][NCH];
    const int i = blockIdx.x * 256 + threadIdx.x;
    const int ic = i < n_pre ? i : n_pre - 1;  // clamp: tail lanes compute a duplicate, store nothing
    int64_t row;
    if (PAGED) {
        const int page = block_table[(size_t)b * (max_ctx >> 4) + (ic >> 4)];
        row = ((int64_t)page * Hkv + g) * 16 + (ic & 15);
    } else {
        row = ((int64_t)b * Hkv + g) * max_ctx + ic;
    }
    float kf[DB];
    {
        const uint4 *kr = (const uint4 *)(kc + row * kHeadDim + sub * DB);
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const uint4 w = kr[c];
            kf[c * 8 + 0] = bf16_lo(w.x); kf[c * 8 + 1] = bf16_hi(w.x);
            kf[c * 8 + 2] = bf16_lo(w.y); kf[c * 8 + 3] = bf16_hi(w.y);
            kf[c * 8 + 4] = bf16_lo(w.z); kf[c * 8 + 5] = bf16_hi(w.z);
            kf[c * 8 + 6] = bf16_lo(w.w); kf[c * 8 + 7] = bf16_hi(w.w);
        }
    }
    const uint4 *cg = (const uint4 *)cent;
    int bad = 0;
    float qabs = 0.0f;
    for (int t0 = 0; t0 < jc; t0 += kBuildTile) {
        const int nt = min(kBuildTile, jc - t0);
        __syncthreads();
        for (int e = threadIdx.x; e < nt * NCH; e += 256)
            s_c[e / NCH][e % NCH] = cg[(size_t)t0 * NCH + e];
        __syncthreads();
        for (int jj = 0; jj < nt; ++jj) {
            float acc = 0.0f;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const uint4 w = s_c[jj][c];
                acc = __builtin_fmaf(bf16_lo(w.x), kf[c * 8 + 0], acc);
                acc = __builtin_fmaf(bf16_hi(w.x), kf[c * 8 + 1], acc);
                acc = __builtin_fmaf(bf16_lo(w.y), kf[c * 8 + 2], acc);
                acc = __builtin_fmaf(bf16_hi(w.y), kf[c * 8 + 3], acc);
                acc = __builtin_fmaf(bf16_lo(w.z), kf[c * 8 + 4], acc);
                acc = __builtin_fmaf(bf16_hi(w.z), kf[c * 8 + 5], acc);
                acc = __builtin_fmaf(bf16_lo(w.w), kf[c * 8 + 6], acc);
                acc = __builtin_fmaf(bf16_hi(w.w), kf[c * 8 + 7], acc);
            }
            const float qf = rintf(acc * up);
            if (!(fabsf(qf) <= (float)qmax)) bad = 1;
            qabs = fmaxf(qabs, fabsf(qf));
            if (i < n_pre) qs[(size_t)(t0 + jj) * n_pre + i] = bad ? 0 : (int32_t)qf;
        }
    }
    if (bad) atomicOr(flags, 1);
    for (int o = 32; o > 0; o >>= 1) qabs = fmaxf(qabs, __shfl_xor(qabs, o, kWave));
    if (lane_id() == 0 && !bad) atomicMax(flags + 1, (int)qabs);  // max |q| (a bound: every score of the
                                                                  // chunk counts, kept or not)
}

template <int DB>
static void launch_build_scores_db(const void *kc, const int32_t *block_table, const void *cent,
                                   int32_t *qs, int32_t *flags, int b, int g, int Hkv, int max_ctx,
                                   int n_pre, int sub, int jc, int F, int qmax, hipStream_t st)
{
    const int grid = (n_pre + 255) / 256;
    if (block_table)
        k_build_scores<true, DB><<<grid, 256, 0, st>>>((const uint16_t *)kc, block_table, (const uint16_t *)cent,
                                                       qs, flags, b, g, Hkv, max_ctx, n_pre, sub, jc,
                                                       ldexpf(1.0f, F), qmax);
    else
        k_build_scores<false, DB><<<grid, 256, 0, st>>>((const uint16_t *)kc, nullptr, (const uint16_t *)cent, qs,
                                                        flags, b, g, Hkv, max_ctx, n_pre, sub, jc,
                                                        ldexpf(1.0f, F), qmax);
}

void launch_build_scores(const void *kc, const int32_t *block_table, const void *cent, int32_t *qs,
                         int32_t *flags, int b, int g, int Hkv, int max_ctx, int n_pre, int S, int sub,
                         int jc, int F, int qmax, hipStream_t st)
{
#define CSA_BS(DB_) launch_build_scores_db<DB_>(kc, block_table, cent, qs, flags, b, g, Hkv, max_ctx, n_pre, sub, jc, F, qmax, st)
    switch (S) {
    case 1: CSA_BS(128); break;
    case 2: CSA_BS(64); break;
    case 4: CSA_BS(32); break;
    case 8: CSA_BS(16); break;
    default: CSA_BS(8); break;  // 16
    }
#undef CSA_BS
}

// ---------------------------------------------------------------------------------------------
// Table build, part 2: Top-L of one row of grid integers (largest first, ties to the lower key
// index, Sec. 3.2 (2) "keep Top-L pairs"), written directly in the device layout (packed entries
// in ascending key index, row stride Ls) together with the row's block offsets.  Radix threshold
// search, then each wave walks a contiguous range of keys in order and compacts the winners with
// ballots; a wave's output offset and its share of the threshold ties follow from per-wave
// counts.  The winners' key indices are also kept in LDS so that the offsets
// part_off[u] = number of entries with key index < u * Q can be looked up afterwards.
// grid = rows of the chunk, block 1024.  ent / part_off point at the chunk's first row.
// ---------------------------------------------------------------------------------------------
constexpr int kBsNT = 1024;
constexpr int kBsWaves = kBsNT / kWave;
constexpr int kMaxL = 8192;

__global__ __launch_bounds__(kBsNT) void k_build_select(const int32_t *__restrict__ qs,
                                                        uint32_t *__restrict__ ent,
                                                        int32_t *__restrict__ part_off, int n_pre,
                                                        int L, int Ls, int Q, int PO)
{
    __shared__ uint32_t s_hist[256 + kBsWaves + 4];
    __shared__ int s_gt[kBsWaves], s_eq[kBsWaves];
    __shared__ int32_t s_idx[kMaxL];
    const int32_t *qr = qs + (size_t)blockIdx.x * n_pre;
    uint32_t *out = ent + (size_t)blockIdx.x * Ls;
    const int want = min(L, n_pre);
    uint32_t T = 0;
    int need = 0;
    if (n_pre > L) {
        T = block_radix_threshold<kBsNT, 8, 4>(
            [&](auto fn) {
                for (int i0 = 0; i0 < n_pre; i0 += kBsNT) {
                    const int i = i0 + threadIdx.x;
                    fn(i < n_pre ? ((uint32_t)qr[i] ^ 0x80000000u) : 0u, i < n_pre);
                }
            },
            want, s_hist, need);
    }
    const int wave = threadIdx.x / kWave, lane = lane_id();
    const int per_wave = ((n_pre + kBsWaves - 1) / kBsWaves + kWave - 1) / kWave * kWave;
    const int lo = min(n_pre, wave * per_wave), hi = min(n_pre, lo + per_wave);
    int n_gt = 0, n_eq = 0;
    for (int i0 = lo; i0 < hi; i0 += kWave) {
        const int i = i0 + lane;
        const uint32_t key = i < hi ? ((uint32_t)qr[i] ^ 0x80000000u) : 0u;
        n_gt += __popcll(__ballot(i < hi && key > T));
        n_eq += __popcll(__ballot(i < hi && key == T && n_pre > L));
    }
    if (lane == 0) { s_gt[wave] = n_gt; s_eq[wave] = n_eq; }
    __syncthreads();
    int pos = 0, ties_before = 0;
    for (int w = 0; w < wave; ++w) {
        const int e = s_eq[w];
        pos += s_gt[w] + max(0, min(e, need - ties_before));
        ties_before += e;
    }
    int tie_rank = ties_before;
    for (int i0 = lo; i0 < hi; i0 += kWave) {
        const int i = i0 + lane;
        const int32_t q = i < hi ? qr[i] : 0;
        const uint32_t key = (uint32_t)q ^ 0x80000000u;
        const bool gt = i < hi && key > T;
        const bool eq = i < hi && key == T && n_pre > L;
        const uint64_t eq_mask = __ballot(eq);
        const bool take = gt || (eq && tie_rank + mbcnt(eq_mask) < need);
        const uint64_t take_mask = __ballot(take);
        if (take) {
            const int o = pos + mbcnt(take_mask);
            if (o < want) {  // (always: the counts above add up to `want`)
                out[o] = pack_entry(i, q);
                s_idx[o] = i;
            }
        }
        pos += __popcll(take_mask);
        tie_rank += __popcll(eq_mask);
    }
    for (int p = want + threadIdx.x; p < Ls; p += kBsNT) out[p] = 0u;
    __syncthreads();
    int32_t *po = part_off + (size_t)blockIdx.x * PO;
    for (int u = threadIdx.x; u < PO; u += kBsNT) {
        const int64_t bound = (int64_t)u * Q;
        po[u] = bound >= n_pre ? want : lower_bound_pos<int32_t>(s_idx, want, (int32_t)bound);
    }
}

void launch_build_select(const int32_t *qs, void *ent, int32_t *part_off, int jc, int n_pre, int L,
                         int Ls, int Q, int PO, hipStream_t st)
{
    k_build_select<<<jc, kBsNT, 0, st>>>(qs, (uint32_t *)ent, part_off, n_pre, L, Ls, Q, PO);
}

// ---------------------------------------------------------------------------------------------
// Streaming updates (Sec. 3.3 (5)): per-row state, try test, insertion.
// ---------------------------------------------------------------------------------------------

// row_cnt[row] = valid entries of the row, row_min[row] = their smallest q (INT_MAX if none),
// blk_min[row][u] = the smallest q within block u of the row (INT_MAX for an empty block): an
// insertion then reads the one block that holds the minimum instead of the whole row.
// One wave per row.  grid ceil(n_rows / 4), block 256.
__global__ __launch_bounds__(256) void k_row_stats(const uint32_t *__restrict__ ent,
                                                   const int32_t *__restrict__ part_off,
                                                   int32_t *__restrict__ row_cnt,
                                                   int32_t *__restrict__ row_min,
                                                   int32_t *__restrict__ blk_min, int64_t n_rows,
                                                   int Ls, int PO)
{
    const int64_t row = (int64_t)blockIdx.x * 4 + threadIdx.x / kWave;
    if (row >= n_rows) return;
    const int32_t *po = part_off + row * PO;
    int all = 0x7FFFFFFF;
    for (int u = 0; u + 1 < PO; ++u) {
        const int b0 = po[u], b1 = po[u + 1];
        int mn = 0x7FFFFFFF;
        for (int p = b0 + lane_id(); p < b1; p += kWave) mn = min(mn, entry_q(ent[row * Ls + p]));
        for (int o = 32; o > 0; o >>= 1) mn = min(mn, __shfl_xor(mn, o, kWave));
        if (lane_id() == 0) blk_min[row * PO + u] = mn;
        all = min(all, mn);
    }
    if (lane_id() == 0) {
        row_cnt[row] = po[PO - 1];
        row_min[row] = all;
    }
}

void launch_row_stats(const void *ent, const int32_t *part_off, int32_t *row_cnt, int32_t *row_min,
                      int32_t *blk_min, int64_t n_rows, int Ls, int PO, hipStream_t st)
{
    k_row_stats<<<(unsigned)((n_rows + 3) / 4), 256, 0, st>>>((const uint32_t *)ent, part_off, row_cnt, row_min,
                                                              blk_min, n_rows, Ls, PO);
}

// Try test: lane j of block (x, s, bg) scores the new key of KV head bg against centroid (s, j)
// - the fma chain and grid of the table build - and, if the row has a free slot or the score beats
// the row minimum, queues (row, q) for insertion.  A score outside the grid range is clamped and
// reported in *clamped.  cent_t is [bg][S][db/8][C][8]; k_new is [bg][128] bf16.
// Every workgroup owns a queue segment of kScanNT slots and its count (written, not added to): no
// global atomics - on this multi-die part thousands of returning atomics on a few addresses cost
// more than the scan itself - and nothing to clear between steps.
// grid (ceil(C/1024), S, B*Hkv), block 1024; segment id = (bg*S + s) * gridDim.x + x.

__global__ __launch_bounds__(kScanNT) void k_insert_scan(const uint16_t *__restrict__ k_new,
                                                     const uint4 *__restrict__ cent_t,
                                                     const int32_t *__restrict__ row_cnt,
                                                     const int32_t *__restrict__ row_min,
                                                     int32_t *__restrict__ queue_n,
                                                     int4 *__restrict__ queue,
                                                     int32_t *__restrict__ clamped, int C, int S, int L,
                                                     float up, int qmax)
{
    __shared__ float s_k[kHeadDim];
    __shared__ int s_n;
    const int sub = blockIdx.y, bg = blockIdx.z;
    const int db = kHeadDim / S, nch = db / 8;
    const int j = blockIdx.x * kScanNT + threadIdx.x;
    if (threadIdx.x == 0) s_n = 0;
    if ((int)threadIdx.x < db)
        s_k[threadIdx.x] = __uint_as_float((uint32_t)k_new[(size_t)bg * kHeadDim + sub * db + threadIdx.x] << 16);
    __syncthreads();
    const bool live = j < C;
    const int jc = live ? j : C - 1;  // (tail lanes compute a duplicate and queue nothing)
    const uint4 *ct = cent_t + ((size_t)bg * S + sub) * nch * C;
    const int64_t row = ((int64_t)bg * S + sub) * C + jc;
    const int cnt = row_cnt[row], mn = row_min[row];
    uint4 wv[kHeadDim / 8];  // every load is requested before the first use
#pragma unroll
    for (int c = 0; c < kHeadDim / 8; ++c) wv[c] = c < nch ? ct[(size_t)c * C + jc] : make_uint4(0, 0, 0, 0);
    float acc = 0.0f;
#pragma unroll
    for (int c = 0; c < kHeadDim / 8; ++c) {
        if (c < nch) {
            const uint4 w = wv[c];
            const float cf[8] = {bf16_lo(w.x), bf16_hi(w.x), bf16_lo(w.y), bf16_hi(w.y),
                                 bf16_lo(w.z), bf16_hi(w.z), bf16_lo(w.w), bf16_hi(w.w)};
#pragma unroll
            for (int e = 0; e < 8; ++e) acc = __builtin_fmaf(cf[e], s_k[c * 8 + e], acc);
        }
    }
    float qf = rintf(acc * up);
    if (!(fabsf(qf) <= (float)qmax)) {
        atomicOr(clamped, 1);
        qf = qf > 0.0f ? (float)qmax : -(float)qmax;  // (a NaN cannot occur: inputs are finite)
    }
    const int q = (int)qf;
    // one LDS counter update per wave
    const size_t seg = ((size_t)bg * S + sub) * gridDim.x + blockIdx.x;
    const bool take = live && (cnt < L || q > mn);
    const uint64_t mask = __ballot(take);
    if (mask) {
        int base = 0;
        if (lane_id() == __ffsll((unsigned long long)mask) - 1) base = atomicAdd(&s_n, __popcll(mask));
        base = __builtin_amdgcn_readlane(base, __ffsll((unsigned long long)mask) - 1);
        if (take)  // (the row's state travels along)
            queue[seg * kScanNT + base + mbcnt(mask)] = make_int4((int)row, q, cnt, mn);
    }
    __syncthreads();
    if (threadIdx.x == 0) queue_n[seg] = s_n;
}

// Insertion: one wave per queued row.  Rows are grouped by blocks of Q key indices (the order
// inside a block carries no meaning: the accumulation kernel scatters by index).  The new key has
// the largest index so far, so it belongs to the last block.  A row with a free slot takes it at
// its end.  A full row first loses its minimum - the entry with the smallest q, among equals the
// one with the largest key index, found by reading only the block whose recorded minimum it is -
// and the hole travels to the last block one block at a time: the last entry of a block moves into
// the hole, which leaves the hole in front of the next block; the new entry fills it in front of
// the last block.  That is one entry move per block instead of shifting the rest of the row, and
// about 1/P of the row read instead of all of it.  Block offsets, block minima, count and row
// minimum are brought up to date.  The work is a chain of memory latencies, so a row gets a
// wave, not a workgroup, nothing waits at a barrier, and a wave is tied to a queue slot (segment
// s, slots w, w + W, ...), so the segment's count and the slot's content are requested together.
// One wave per workgroup: a wave without work (most segments hold fewer rows than they have
// waves) gives its place up at once.
// grid (W, n_seg, B*Hkv), block 64.
constexpr int kInsPo = 1024;  // block offsets and minima of a row kept in LDS when they fit

__global__ __launch_bounds__(kWave) void k_insert_rows(uint32_t *__restrict__ ent,
                                                       int32_t *__restrict__ part_off,
                                                       int32_t *__restrict__ row_cnt,
                                                       int32_t *__restrict__ row_min,
                                                       int32_t *__restrict__ blk_min,
                                                       const int32_t *__restrict__ queue_n,
                                                       const int4 *__restrict__ queue, int n_seg, int L,
                                                       int Ls, int Q, int PO, int idx_new)
{
    __shared__ int32_t s_po[kInsPo];
    const int lane = lane_id();
    const size_t seg = (size_t)blockIdx.z * n_seg + blockIdx.y;
    const int4 *qseg = queue + seg * kScanNT;
    const int first = blockIdx.x;
    const int4 it0 = qseg[first < kScanNT ? first : 0];  // (a stale slot when the segment holds fewer)
    const int n_items = queue_n[seg];
    const int u_new = idx_new / Q;  // the new key's block
    const bool po_lds = PO <= kInsPo;
    for (int item = first; item < n_items; item += gridDim.x) {
        const int4 it = item == first ? it0 : qseg[item];
        const int64_t row = it.x;
        const int q_new = it.y, cnt = it.z, mn = it.w;
        uint32_t *re = ent + row * Ls;
        int32_t *po = part_off + row * PO;
        int32_t *bm = blk_min + row * PO;
        const uint32_t e_new = pack_entry(idx_new, q_new);
        if (cnt < L) {  // (uniform over the wave)
            if (lane == 0) {
                re[cnt] = e_new;
                row_cnt[row] = cnt + 1;
                row_min[row] = min(mn, q_new);
                bm[u_new] = min(bm[u_new], q_new);
            }
            for (int u = lane; u < PO; u += kWave)
                if ((int64_t)u * Q > idx_new) po[u] += 1;
            continue;
        }
        if (po_lds)
            for (int u = lane; u < PO; u += kWave) s_po[u] = po[u];
        const int32_t *pol = po_lds ? s_po : po;  // the offsets as they are before this insertion
        // the block that holds the entry to evict: the last one whose minimum is the row minimum;
        // the smallest of the other blocks' minima goes into the new row minimum
        int ue = -1, others = 0x7FFFFFFF;
        for (int u0 = 0; u0 + 1 < PO; u0 += kWave) {
            const int u = u0 + lane;
            const int v = u + 1 < PO ? bm[u] : 0x7FFFFFFF;
            const unsigned long long hit = __ballot(v == mn);
            if (hit) {
                if (ue >= 0) others = min(others, mn);  // (an earlier block also holds the minimum)
                ue = u0 + 63 - __clzll(hit);
            }
            int o = (v == mn && u == ue) ? 0x7FFFFFFF : v;
            for (int d = 32; d > 0; d >>= 1) o = min(o, __shfl_xor(o, d, kWave));
            others = min(others, o);
        }
        if (ue < 0) continue;  // (cannot happen: row_min is the minimum of a full row)
        // that block: the evicted entry (q == mn, largest index = largest low index bits within a
        // block) and the smallest q of what stays in the block
        const int b0 = pol[ue], b1 = pol[ue + 1];
        unsigned long long best = 0ull;  // (low index bits + 1, position): larger wins
        int n_min = 0, min2 = 0x7FFFFFFF;
        // (eight entries per lane requested together: with long rows - the paper's geometry keeps a tenth
        // of the context per row - a block holds hundreds of entries, and one request per round trip
        // would make this read the longest part of the insertion)
        constexpr int kBlkFlight = 8;
        for (int p0 = b0 + lane; p0 < b1; p0 += kBlkFlight * kWave) {
            uint32_t ev[kBlkFlight];
#pragma unroll
            for (int u = 0; u < kBlkFlight; ++u) {
                const int p = p0 + u * kWave;
                ev[u] = p < b1 ? re[p] : 0u;
            }
#pragma unroll
            for (int u = 0; u < kBlkFlight; ++u) {
                const int p = p0 + u * kWave;
                if (p < b1) {
                    const uint32_t e = ev[u];
                    const int q = entry_q(e);
                    if (q == mn) {
                        ++n_min;
                        const unsigned long long cand =
                            ((unsigned long long)((e & (uint32_t)(kUnit - 1)) + 1u) << 32) | (uint32_t)p;
                        best = cand > best ? cand : best;
                    } else {
                        min2 = min(min2, q);
                    }
                }
            }
        }
        for (int o = 32; o > 0; o >>= 1) {
            const unsigned long long t = __shfl_xor(best, o, kWave);
            best = t > best ? t : best;
            min2 = min(min2, __shfl_xor(min2, o, kWave));
        }
        n_min = wave_sum(n_min);
        if (best == 0ull) continue;  // (cannot happen: the block's minimum is recorded as mn)
        const int pe = (int)(uint32_t)best;
        const int blk_left = n_min >= 2 ? mn : min2;  // the block's minimum without the evicted entry
        // the hole's way: block w in [ue, u_new) gives its last entry (at pol[w+1] - 1) to the hole
        // (at pe in block ue, else in front of block w at pol[w] - 1); all reads of a round of 64
        // blocks first, then its writes - the source of one move is the target of the next
        for (int w0 = ue; w0 < u_new; w0 += kWave) {  // (uniform bounds)
            const int w = w0 + lane;
            const bool on = w < u_new;
            int src = 0, dst = 0;
            uint32_t val = 0u;
            if (on) {
                src = pol[w + 1] - 1;
                // (without the LDS copy, the first block of a later round already has its lowered offset)
                dst = w == ue ? pe : (!po_lds && w == w0 ? pol[w] : pol[w] - 1);
                val = re[src];
            }
            __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the reads have returned
            if (on && src != dst) re[dst] = val;
            if (on) po[w + 1] = src;  // one entry fewer before block w + 1
            __builtin_amdgcn_s_waitcnt(0x0F70);  // (the next round reads what this one wrote)
        }
        if (lane == 0) {
            // the new entry: in place of the evicted one if that sat in the last block, else in the
            // hole now in front of the last block
            re[ue == u_new ? pe : (po_lds ? s_po[u_new] - 1 : po[u_new])] = e_new;
            int last_min;  // the last block's minimum with the new entry
            if (ue == u_new) {
                last_min = min(blk_left, q_new);
            } else {
                bm[ue] = blk_left;
                last_min = min(bm[u_new], q_new);
            }
            bm[u_new] = last_min;
            // (`others` counted block u_new with its old minimum when it is not the evicted one's)
            row_min[row] = min(min(others, blk_left), q_new);
        }
    }
}

// The try test with the new key's centroid scores given (insert_try_segment), as a launch of its own.
// grid (ceil(C / kScanNT), S, B*Hkv), block kScanNT.
__global__ __launch_bounds__(kScanNT) void k_insert_try(TryArgs a)
{
    __shared__ int s_n;
    insert_try_segment<kScanNT>(a, (int)(blockIdx.z * gridDim.y + blockIdx.y), (int)blockIdx.x, &s_n);
}

TryArgs insert_try_args(const float *z_key, const int32_t *row_cnt, const int32_t *row_min, int32_t *queue_n,
                        void *queue, int32_t *clamped, int C, int S, int L, int F, int qmax)
{
    return TryArgs{z_key, row_cnt, row_min, queue_n, (int4 *)queue, clamped, C, L, (C + kScanNT - 1) / kScanNT, S,
                   ldexpf(1.0f, F), qmax};
}

void launch_insert(const void *k_new, const float *z_key, bool tried, const void *cent_t, void *ent, int32_t *part_off, int32_t *row_cnt,
                   int32_t *row_min, int32_t *blk_min, int32_t *queue_n, void *queue, int32_t *clamped, int B, int Hkv, int C,
                   int S, int L, int Ls, int Q, int PO, int F, int qmax, int idx_new, hipStream_t st)
{
    const int nx = (C + kScanNT - 1) / kScanNT, n_seg = S * nx;  // (n_seg <= 64: checked at create)
    dim3 grid(nx, S, B * Hkv);
    if (tried) {
        // (the try test rode in an earlier launch of the step: the queues are filled)
    } else if (z_key)
        k_insert_try<<<grid, kScanNT, 0, st>>>(insert_try_args(z_key, row_cnt, row_min, queue_n, queue, clamped, C, S, L, F, qmax));
    else
        k_insert_scan<<<grid, kScanNT, 0, st>>>((const uint16_t *)k_new, (const uint4 *)cent_t, row_cnt, row_min, queue_n,
                                                (int4 *)queue, clamped, C, S, L, ldexpf(1.0f, F), qmax);
    // the queue lengths are only known on the device: enough waves for one row each in the usual
    // case (a few percent of the rows take a new key), striding when there are more
    // A row takes the new key with probability about L / (context length): one wave per 8 rows covers
    // the 3 % of 128K-context tables with lists of 4096; long lists in few rows (the paper's geometry:
    // a tenth of the rows) get three waves per expected row, up to one per row
    const int per_seg = C < kScanNT ? C : kScanNT;  // rows behind a segment
    int waves = per_seg / 8 < 1 ? 1 : per_seg / 8;
    const int64_t expect3 = 3 * (int64_t)per_seg * L / (idx_new > 0 ? idx_new : 1);
    if (expect3 > waves) waves = (int)(expect3 < per_seg ? expect3 : per_seg);
    k_insert_rows<<<dim3(waves, n_seg, B * Hkv), kWave, 0, st>>>((uint32_t *)ent, part_off, row_cnt, row_min, blk_min, queue_n,
                                                      (const int4 *)queue, n_seg, L, Ls, Q, PO, idx_new);
}

// max over prefill keys and subspaces of ||k^(s)||^2 (nch 16-byte chunks per subspace), as the bit
// pattern of a non-negative fp32 (atomicMax on int).  Used to pick the score grid.  out must be
// zeroed.
template <bool PAGED>
__global__ void k_max_key_norm(const uint16_t *__restrict__ kc, const int32_t *__restrict__ block_table,
                               int *__restrict__ out, int Hkv, int max_ctx, int n_pre, int64_t total,
                               int nch)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    float best = 0.0f;
    if (t < total) {
        const int i = (int)(t % n_pre);
        const int bg = (int)(t / n_pre), b = bg / Hkv, g = bg % Hkv;
        int64_t row;
        if (PAGED) {
            const int page = block_table[(size_t)b * (max_ctx >> 4) + (i >> 4)];
            row = ((int64_t)page * Hkv + g) * 16 + (i & 15);
        } else {
            row = (int64_t)bg * max_ctx + i;
        }
        const uint4 *kr = (const uint4 *)(kc + row * kHeadDim);
        float nn = 0.0f;
        for (int c = 0; c < kHeadDim / 8; ++c) {
            const uint4 w = kr[c];
            const float f[8] = {bf16_lo(w.x), bf16_hi(w.x), bf16_lo(w.y), bf16_hi(w.y),
                                bf16_lo(w.z), bf16_hi(w.z), bf16_lo(w.w), bf16_hi(w.w)};
            for (int e = 0; e < 8; ++e) nn = fmaf(f[e], f[e], nn);
            if ((c + 1) % nch == 0) {
                best = fmaxf(best, nn);
                nn = 0.0f;
            }
        }
    }
    for (int o = 32; o > 0; o >>= 1) best = fmaxf(best, __shfl_xor(best, o, kWave));
    if (lane_id() == 0) atomicMax(out, __float_as_int(best));
}

void launch_max_key_norm(const void *kc, const int32_t *block_table, float *out, int B, int Hkv,
                         int max_ctx, int n_pre, int S, hipStream_t st)
{
    const int64_t total = (int64_t)B * Hkv * n_pre;
    const unsigned grid = (unsigned)((total + 255) / 256);
    if (block_table)
        k_max_key_norm<true><<<grid, 256, 0, st>>>((const uint16_t *)kc, block_table, (int *)out, Hkv, max_ctx, n_pre, total, 16 / S);
    else
        k_max_key_norm<false><<<grid, 256, 0, st>>>((const uint16_t *)kc, nullptr, (int *)out, Hkv, max_ctx, n_pre, total, 16 / S);
}

}  // namespace csa

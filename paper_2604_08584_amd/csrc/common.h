// Shared device helpers for the gfx950 kernels (wave64 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace csa {

constexpr int kWave = 64;
constexpr int kHeadDim = 128;
// accumulator packing: each table entry contributes q * 64 + 1, so a key's accumulator is
// (sum of q) * 64 + (number of probed rows that list it); non-zero iff the key was seen.
constexpr int kCntBits = 6;
constexpr int32_t kKeyBias = 1 << 24;  // accumulated |sum q| < 2^24  ->  key in (0, 2^25)

__device__ __forceinline__ uint32_t pack_entry(int32_t idx, int32_t q)
{
    return ((uint32_t)q << kUnitBits) | ((uint32_t)idx & (uint32_t)(kUnit - 1));
}
__device__ __forceinline__ int32_t entry_q(uint32_t e) { return (int32_t)e >> kUnitBits; }

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// order-preserving image of an fp32 (after -0 -> +0 canonicalisation by the caller)
__device__ __forceinline__ uint32_t orderable(float f)
{
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// workgroup barrier that orders LDS accesses only: outstanding global loads and stores are not
// waited for (what __syncthreads() would do)
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// number of set bits of `mask` below this lane
__device__ __forceinline__ int mbcnt(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// Inclusive prefix sum over the 64 lanes with data-parallel-primitive moves (no LDS traffic):
// shifts by 1, 2, 4, 8 inside each row of 16 lanes, then the last lane of row 0 / 2 is broadcast
// into row 1 / 3, then lane 31 into the upper half.
__device__ __forceinline__ int wave_incl_scan(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, true);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, true);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, true);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, true);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);  // row_bcast:15 into rows 1, 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);  // row_bcast:31 into rows 2, 3
    return v;
}

// Exclusive prefix sum over the block in thread order; returns this thread's prefix and the
// block total.  s_tmp: at least NT/64 + 1 ints of LDS.  Contains two barriers.
template <int NT>
__device__ __forceinline__ int block_excl_scan(int v, int *s_tmp, int &total)
{
    constexpr int NW = NT / kWave;
    const int w = threadIdx.x / kWave;
    int incl = wave_incl_scan(v);
    if (lane_id() == kWave - 1) s_tmp[w] = incl;
    __syncthreads();
    int off = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        int t = s_tmp[i];
        if (i < w) off += t;
        tot += t;
    }
    __syncthreads();
    total = tot;
    return off + incl - v;
}

// The same for four 16-bit counters packed in a 64-bit word (every running total must stay
// below 65536): one scan, four prefix sums.
template <int NT>
__device__ __forceinline__ unsigned long long block_excl_scan_4x16(unsigned long long v,
                                                                    unsigned long long *s_tmp,
                                                                    unsigned long long &total)
{
    constexpr int NW = NT / kWave;
    const int w = threadIdx.x / kWave;
    // (no field overflows, so the two 32-bit halves scan independently)
    const unsigned long long incl =
        ((unsigned long long)(uint32_t)wave_incl_scan((int)(uint32_t)(v >> 32)) << 32) |
        (uint32_t)wave_incl_scan((int)(uint32_t)v);
    if (lane_id() == kWave - 1) s_tmp[w] = incl;
    __syncthreads();
    unsigned long long off = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        const unsigned long long t = s_tmp[i];
        if (i < w) off += t;
        tot += t;
    }
    __syncthreads();
    total = tot;
    return off + incl - v;
}

// sum over the wave, result in every lane
__device__ __forceinline__ int wave_sum(int v)
{
    return __builtin_amdgcn_readlane(wave_incl_scan(v), kWave - 1);
}

// largest value over the wave, result in every lane (the same moves as the scan; a lane that
// receives nothing keeps its value: 0 is the identity)
__device__ __forceinline__ uint32_t wave_max(uint32_t v)
{
    int x = (int)v;
    auto mx = [](int a, int b) { return (int)max((uint32_t)a, (uint32_t)b); };
    x = mx(x, __builtin_amdgcn_update_dpp(0, x, 0x111, 0xF, 0xF, true));
    x = mx(x, __builtin_amdgcn_update_dpp(0, x, 0x112, 0xF, 0xF, true));
    x = mx(x, __builtin_amdgcn_update_dpp(0, x, 0x114, 0xF, 0xF, true));
    x = mx(x, __builtin_amdgcn_update_dpp(0, x, 0x118, 0xF, 0xF, true));
    x = mx(x, __builtin_amdgcn_update_dpp(0, x, 0x142, 0xA, 0xF, false));
    x = mx(x, __builtin_amdgcn_update_dpp(0, x, 0x143, 0xC, 0xF, false));
    return (uint32_t)__builtin_amdgcn_readlane(x, kWave - 1);
}

// Wave-aggregated histogram increment: lanes that hit the same bin as the first pending lane
// are counted with one LDS atomic (keys cluster heavily in the leading digits); after two such
// rounds the remaining lanes fall back to one atomic each.
__device__ __forceinline__ void hist_add(uint32_t *hist, uint32_t bin, bool active)
{
#pragma unroll
    for (int round = 0; round < 2; ++round) {
        if (active) {  // exec = the pending lanes
            const uint32_t lb = (uint32_t)__builtin_amdgcn_readfirstlane((int)bin);
            const bool same = bin == lb;
            const uint64_t mask = __ballot(same);
            if (same) {
                if (mbcnt(mask) == 0) atomicAdd(&hist[lb], (uint32_t)__popcll(mask));
                active = false;
            }
        }
    }
    if (active) atomicAdd(&hist[bin], 1u);
}

// Given a histogram of NB bins in LDS, finds the bin in which the `want`-th largest element
// falls when bins are walked from the top: returns that bin, `above` = number of elements in
// higher bins (above < want <= above + hist[bin]).  All NT threads must call; NB % NT == 0 or
// NT >= NB.  s_aux: NT/64 + 2 uint32 of LDS.  Ends with a barrier (hist may be reused after).
template <int NT, int NB>
__device__ __forceinline__ int block_pick_bin(const uint32_t *s_hist, int want, uint32_t *s_aux,
                                              int &above)
{
    constexpr int BPT = NB >= NT ? NB / NT : 1;  // bins per owning thread
    static_assert(NB >= NT ? NB % NT == 0 : true, "bins must divide evenly");
    uint32_t *s_res = s_aux + NT / kWave;
    // thread t owns bins NB-1-t*BPT downwards; inclusive scan from the top bin
    int v = 0;
    const int top = NB - 1 - (int)threadIdx.x * BPT;
    if (top >= 0)
#pragma unroll
        for (int u = 0; u < BPT; ++u) v += (int)s_hist[top - u];
    int incl = wave_incl_scan(v);
    if (lane_id() == kWave - 1) s_aux[threadIdx.x / kWave] = (uint32_t)incl;
    __syncthreads();
    int off = 0;
    for (int i = 0; i < (int)(threadIdx.x / kWave); ++i) off += (int)s_aux[i];
    incl += off;
    int excl = incl - v;
    if (top >= 0 && excl < want && want <= incl) {
#pragma unroll
        for (int u = 0; u < BPT; ++u) {
            const int h = (int)s_hist[top - u];
            if (excl < want && want <= excl + h) {
                s_res[0] = (uint32_t)(top - u);
                s_res[1] = (uint32_t)excl;
            }
            excl += h;
        }
    }
    __syncthreads();
    const int bin = (int)s_res[0];
    above = (int)s_res[1];
    __syncthreads();
    return bin;
}

// Radix threshold search over a set of keys visited through `for_each(fn)`, which must call
// fn(key, valid) from every thread (valid = false for padding).
// Finds T such that   count(key > T) < want <= count(key >= T)     (requires 1 <= want <= n).
// Returns T; `need` = want - count(key > T) = how many keys equal to T are still wanted.
// Keys must be < 2^(RB*PASSES).  s_hist: 2^RB + NT/64 + 2 uint32 of LDS.
template <int NT, int RB, int PASSES, class ForEach>
__device__ __forceinline__ uint32_t block_radix_threshold(ForEach for_each, int want,
                                                          uint32_t *s_hist, int &need)
{
    constexpr int NB = 1 << RB;
    uint32_t prefix = 0, pmask = 0;
    int remaining = want;
    for (int pass = 0; pass < PASSES; ++pass) {
        const int shift = RB * (PASSES - 1 - pass);
        for (int i = threadIdx.x; i < NB; i += NT) s_hist[i] = 0;
        __syncthreads();
        for_each([&](uint32_t key, bool valid) {
            hist_add(s_hist, (key >> shift) & (NB - 1), valid && (key & pmask) == prefix);
        });
        __syncthreads();
        int above;
        const int bin = block_pick_bin<NT, NB>(s_hist, remaining, s_hist + NB, above);
        prefix |= (uint32_t)bin << shift;
        pmask |= (uint32_t)(NB - 1) << shift;
        remaining -= above;
    }
    need = remaining;
    return prefix;
}


// ---------------------------------------------------------------------------------------------
// Streaming updates (Sec. 3.3 (5)), the try test with the new key's centroid scores given: row j of
// (KV head, subspace) pair bg takes the key if it has room or the key's grid score beats the row's minimum.  Rows
// that take it are queued, with their state, in the queue segment of their 1024 rows (kScanNT);
// the segment's count is written, not added to.  All NT threads of a workgroup call (NT divides
// kScanNT); *s_n is an LDS word of the workgroup.
// ---------------------------------------------------------------------------------------------
template <int NT>
__device__ __forceinline__ void insert_try_segment(const TryArgs &a, int bg, int x, int *s_n)
{
    constexpr int PER = kScanNT / NT;
    if (threadIdx.x == 0) *s_n = 0;
    __syncthreads();
    float zk[PER];
    int cnt[PER], mn[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {  // (every load before the first use)
        const int j = x * kScanNT + u * NT + (int)threadIdx.x;
        const int64_t row = (int64_t)bg * a.C + (j < a.C ? j : a.C - 1);
        zk[u] = a.z_key[row];
        cnt[u] = a.row_cnt[row];
        mn[u] = a.row_min[row];
    }
    const size_t seg = (size_t)bg * a.nx + x;
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int j = x * kScanNT + u * NT + (int)threadIdx.x;
        const bool live = j < a.C;
        float qf = rintf(zk[u] * a.up);
        if (!(fabsf(qf) <= (float)a.qmax)) {
            if (live) atomicOr(a.clamped, 1);
            qf = qf > 0.0f ? (float)a.qmax : -(float)a.qmax;  // (a NaN cannot occur: inputs are finite)
        }
        const int q = (int)qf;
        const bool take = live && (cnt[u] < a.L || q > mn[u]);
        const uint64_t mask = __ballot(take);
        if (mask) {  // one LDS counter update per wave
            int base = 0;
            if (lane_id() == __ffsll((unsigned long long)mask) - 1) base = atomicAdd(s_n, __popcll(mask));
            base = __builtin_amdgcn_readlane(base, __ffsll((unsigned long long)mask) - 1);
            if (take)  // (the row's state travels along)
                a.queue[seg * kScanNT + base + mbcnt(mask)] = make_int4((int)((int64_t)bg * a.C + j), q, cnt[u], mn[u]);
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) a.queue_n[seg] = *s_n;
}

// ---------------------------------------------------------------------------------------------
// Candidate words.  The accumulation kernel leaves the candidates of (head, key range) grouped by
// coarse bin of their accumulated score, best bin first: word = (score bits below the bin) <<
// kIdxBits | key index within the range, with the start offset of every bin in bin_off[.][512]
// (uint16; bin 512 would start at the range's candidate count).  The head's threshold is
// B << kThrShift | T: candidates of bins before B are selected, of bin B those whose score bits
// exceed T plus some whose bits equal T.
// ---------------------------------------------------------------------------------------------
constexpr int kCoarseBins = 512;
constexpr int kIdxBits = 14;   // key index within a range of <= 16384 keys
constexpr int kThrShift = 22;  // score bits within a bin: < 2^18

// ---------------------------------------------------------------------------------------------
// Top-K, first half (paper Sec. 3.3 (4)): the threshold of one head.  Every key range's candidates
// are grouped by coarse score bin (best first) with the bins' start offsets, so the head's histogram
// is a sum of offset differences, the bin B holding the k-th largest score follows from it, and
// everything in better bins is selected without being looked at.  Only the candidates of bin B (a
// run per key range) are read: their scores within the bin are searched for the value T such that
// the winners are every candidate above T plus the `need` lowest-index candidates equal to T - in
// LDS by a radix search when the bin holds few enough, else by refining the range with histogram
// passes over the runs first.  The result is B << kThrShift | T (0xFFFFFFFF: nothing selected;
// B = 512: every candidate) and, per range, its first output slot and the ties it may keep.
// ---------------------------------------------------------------------------------------------
constexpr int kSelCap = 4096;   // contenders finished in LDS
constexpr int kSelMaxP = 2048;  // key ranges (segments) per head
constexpr int kSegBits = 11;    // a contender is (score within the bin) << kSegBits | p
static_assert((1 << kSegBits) >= kSelMaxP, "segment tag too narrow");

// LDS of head_threshold for workgroups of NT threads and heads of up to MAXP key ranges
template <int NT, int MAXP>
struct ThrSmem {
    uint32_t hist[512 + NT / kWave + 2];
    int scan[NT / kWave + 1];
    uint32_t ck[kSelCap];
    int32_t cnt[MAXP], gt[MAXP], eq[MAXP];
    uint16_t beg[MAXP], end[MAXP];  // the run of the threshold's bin in every range
    int n;
};

// The threshold of one head from its ranges' candidates (hk), counts (seg_cnt) and bin offsets (bo);
// all NT threads of the workgroup call.  Returns T (see above) and k_eff = min(k, candidates); for
// every range p, on_range(p, first output slot, ties allowed) is called by one thread, and sm.beg[p] /
// sm.end[p] / sm.cnt[p] hold the run of the threshold's bin and the range's candidate count.  Ends
// with the calls to on_range, not with a barrier.  P <= MAXP.
template <int kThrNT, int MAXP, class OnRange>
__device__ __forceinline__ uint32_t head_threshold(const uint32_t *__restrict__ hk,
                                                   const int32_t *__restrict__ seg_cnt,
                                                   const uint16_t *__restrict__ bo, int k, int R, int P,
                                                   int key_sh, ThrSmem<kThrNT, MAXP> &sm, int &k_eff_out,
                                                   OnRange on_range)
{
    constexpr int NW = kThrNT / kWave;
    uint32_t *s_hist = sm.hist;
    int *s_scan = sm.scan;
    uint32_t *s_ck = sm.ck;
    int32_t *s_cnt = sm.cnt, *s_gt = sm.gt, *s_eq = sm.eq;
    uint16_t *s_beg = sm.beg, *s_end = sm.end;
    int &s_n = sm.n;
    static_assert(kCoarseBins == 512 && (512 % kThrNT == 0 || kThrNT % 512 == 0), "whole bins per thread");
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave), lane = lane_id();
    // the head's histogram, bin j = sum over the ranges of (start of bin j+1) - (start of bin j):
    // a wave reads a range's 512 offsets with one 16-byte load per lane (lane = eight consecutive
    // bins); the first two ranges of every wave are requested before anything is waited for
    static_assert(kCoarseBins == 8 * kWave, "one 16-byte load per lane covers a range's offsets");
    auto hist_load = [&](int p) {
        return p < P ? *(const uint4 *)(bo + (size_t)p * kCoarseBins + lane * 8) : make_uint4(0, 0, 0, 0);
    };
    const uint4 hpre[4] = {hist_load(wave), hist_load(wave + NW), hist_load(wave + 2 * NW), hist_load(wave + 3 * NW)};
    int part = 0;
    for (int p = threadIdx.x; p < MAXP; p += kThrNT) {
        const int c = p < P ? min(seg_cnt[p], R) : 0;
        s_cnt[p] = c;
        s_gt[p] = 0;
        s_eq[p] = 0;
        part += c;
    }
    for (int i = threadIdx.x; i < 512; i += kThrNT) s_hist[i] = 0;  // (walked top = best by block_pick_bin)
    if (threadIdx.x == 0) s_n = 0;
    int n_total;
    block_excl_scan<kThrNT>(part, s_scan, n_total);  // (its barriers also publish the LDS writes)
    const int k_eff = n_total < k ? n_total : k;
    k_eff_out = k_eff;

    uint32_t T = 0xFFFFFFFFu;
    int need = 0;
    if (k_eff > 0 && n_total <= k) {
        T = (uint32_t)kCoarseBins << kThrShift;  // every candidate wins
        for (int p = threadIdx.x; p < P; p += kThrNT) {
            s_gt[p] = s_cnt[p];
            s_beg[p] = s_end[p] = (uint16_t)s_cnt[p];
        }
    } else if (k_eff > 0) {
        for (int p = wave, it = 0; p < P; p += NW, ++it) {
            const uint4 v = it < 4 ? hpre[it] : hist_load(p);
            // start of the bin after this lane's eight: the next lane's first, or the range's count
            uint32_t nxt = (uint32_t)__shfl_down((int)(v.x & 0xFFFFu), 1, kWave);
            if (lane == kWave - 1) nxt = (uint32_t)s_cnt[p];
            const uint32_t o[9] = {v.x & 0xFFFFu, v.x >> 16, v.y & 0xFFFFu, v.y >> 16, v.z & 0xFFFFu,
                                   v.z >> 16, v.w & 0xFFFFu, v.w >> 16, nxt};
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (o[i + 1] > o[i]) atomicAdd(&s_hist[(kCoarseBins - 1) - (lane * 8 + i)], o[i + 1] - o[i]);
        }
        __syncthreads();
        int above;
        const int top_bin = block_pick_bin<kThrNT, 512>(s_hist, k, s_hist + 512, above);
        const int B = (kCoarseBins - 1) - top_bin;  // as the accumulation kernel numbers the bins
        int in_bin = (int)s_hist[top_bin];
        int want = k - above;  // how many of bin B's candidates are selected (>= 1)
        if (P <= 4 * NW) {
            // every range's offsets are still in the registers of the wave that loaded them: the
            // lane that holds bin B hands out the run, no second trip to memory
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int p = wave + it * NW;
                if (p >= P) break;
                const uint4 v = hpre[it];
                uint32_t nxt = (uint32_t)__shfl_down((int)(v.x & 0xFFFFu), 1, kWave);
                if (lane == kWave - 1) nxt = (uint32_t)s_cnt[p];
                if (lane == (B >> 3)) {
                    const uint32_t o[9] = {v.x & 0xFFFFu, v.x >> 16, v.y & 0xFFFFu, v.y >> 16, v.z & 0xFFFFu,
                                           v.z >> 16, v.w & 0xFFFFu, v.w >> 16, nxt};
                    uint32_t b0 = o[0], b1 = o[1];
#pragma unroll
                    for (int i = 1; i < 8; ++i)
                        if ((B & 7) == i) { b0 = o[i]; b1 = o[i + 1]; }
                    s_beg[p] = (uint16_t)b0;
                    s_end[p] = (uint16_t)b1;
                    s_gt[p] = (int)b0;  // every candidate of a better bin
                }
            }
        } else {
            for (int p = threadIdx.x; p < P; p += kThrNT) {
                const int c = s_cnt[p];
                const int b0 = c > 0 ? (int)bo[(size_t)p * kCoarseBins + B] : 0;
                const int b1 = c > 0 ? (B + 1 < kCoarseBins ? (int)bo[(size_t)p * kCoarseBins + B + 1] : c) : 0;
                s_beg[p] = (uint16_t)b0;
                s_end[p] = (uint16_t)b1;
                s_gt[p] = b0;  // every candidate of a better bin
            }
        }
        __syncthreads();
        // runs(fn, seg_end): fn(score within the bin, valid, p) for the candidates of bin B of every
        // range p (a wave walks whole runs, one candidate per lane and round), then seg_end(p)
        auto runs = [&](auto fn, auto seg_end) {
            for (int p = wave; p < P; p += NW) {
                const int b0 = __builtin_amdgcn_readfirstlane((int)s_beg[p]);
                const int b1 = __builtin_amdgcn_readfirstlane((int)s_end[p]);
                for (int e0 = b0; e0 < b1; e0 += kWave) {
                    const bool valid = e0 + lane < b1;
                    const uint32_t w = valid ? hk[(size_t)p * R + e0 + lane] : 0u;
                    fn(w >> kIdxBits, valid, p);
                }
                seg_end(p);
            }
        };
        // the live score range [lo, hi] within the bin, narrowed until few enough candidates remain
        uint32_t lo = 0, hi = (1u << key_sh) - 1u;
        for (;;) {
            if (in_bin <= kSelCap) {
                // gather the contenders, tagged with their range; candidates above the live range are
                // sure winners of their range
                int n_gt = 0;  // (wave-uniform)
                runs([&](uint32_t key, bool valid, int p) {
                         n_gt += __popcll(__ballot(valid && key > hi));
                         const bool in = valid && key >= lo && key <= hi;
                         const unsigned long long m = __ballot(in);
                         if (m) {
                             int o = 0;
                             if (lane == 0) o = atomicAdd(&s_n, __popcll(m));
                             o = __builtin_amdgcn_readfirstlane(o) + mbcnt(m);
                             if (in && o < kSelCap) s_ck[o] = ((key - lo) << kSegBits) | (uint32_t)p;
                         }
                     },
                     [&](int p) {
                         if (lane == 0 && n_gt) s_gt[p] += n_gt;
                         n_gt = 0;
                     });
                __syncthreads();
                const int nc = min(s_n, kSelCap);
                const uint32_t Tl = block_radix_threshold<kThrNT, 8, 2>(
                    [&](auto fn) {
                        for (int a0 = 0; a0 < nc; a0 += kThrNT) {
                            const int a = a0 + threadIdx.x;
                            fn(a < nc ? s_ck[a] >> kSegBits : 0u, a < nc);
                        }
                    },
                    want, s_hist, need);
                T = ((uint32_t)B << kThrShift) | (lo + Tl);
                for (int a = threadIdx.x; a < nc; a += kThrNT) {
                    const uint32_t c = s_ck[a];
                    const uint32_t kk = c >> kSegBits;
                    const int p = (int)(c & ((1u << kSegBits) - 1u));
                    if (kk > Tl)
                        atomicAdd(&s_gt[p], 1);
                    else if (kk == Tl)
                        atomicAdd(&s_eq[p], 1);
                }
                break;
            }
            if (lo == hi) {
                // a single score value: count, per range, the candidates above and equal to it
                T = ((uint32_t)B << kThrShift) | lo;
                need = want;
                int n_gt = 0, n_eq = 0;
                runs([&](uint32_t key, bool valid, int) {
                         n_gt += __popcll(__ballot(valid && key > lo));
                         n_eq += __popcll(__ballot(valid && key == lo));
                     },
                     [&](int p) {
                         if (lane == 0) {
                             s_gt[p] += n_gt;
                             s_eq[p] = n_eq;
                         }
                         n_gt = 0;
                         n_eq = 0;
                     });
                break;
            }
            // too many: histogram of the live range over <= 512 equal bins, keep the bin with the
            // want-th largest
            int sh = 0;
            while (((hi - lo) >> sh) >= 512u) ++sh;
            __syncthreads();
            for (int i = threadIdx.x; i < 512; i += kThrNT) s_hist[i] = 0;
            __syncthreads();
            runs([&](uint32_t key, bool valid, int) {
                     const bool in = valid && key >= lo && key <= hi;
                     hist_add(s_hist, in ? (key - lo) >> sh : 0u, in);
                 },
                 [&](int) {});
            __syncthreads();
            const int bin = block_pick_bin<kThrNT, 512>(s_hist, want, s_hist + 512, above);
            in_bin = (int)s_hist[bin];
            want -= above;
            lo += (uint32_t)bin << sh;
            hi = min(hi, lo + ((1u << sh) - 1u));
        }
    }
    __syncthreads();
    // per range: its share of the ties (lowest ranges first) and its first output slot; thread t
    // owns the RPT consecutive ranges starting at t * RPT (threads past MAXP / RPT own none)
    constexpr int RPT = MAXP >= kThrNT ? MAXP / kThrNT : 1;
    const int p0 = RPT * (int)threadIdx.x;
    const bool own = p0 < MAXP;
    int e_mine = 0;
#pragma unroll
    for (int i = 0; i < RPT; ++i) e_mine += own ? s_eq[p0 + i] : 0;
    int dummy;
    int ties_before = block_excl_scan<kThrNT>(e_mine, s_scan, dummy);
    int al[RPT], take_mine = 0;
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
        const int e = own ? s_eq[p0 + i] : 0;
        al[i] = max(0, min(e, need - ties_before));
        ties_before += e;
        take_mine += (own ? s_gt[p0 + i] : 0) + al[i];
    }
    int off = block_excl_scan<kThrNT>(take_mine, s_scan, dummy);
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
        if (own && p0 + i < P) on_range(p0 + i, off, al[i]);
        off += (own ? s_gt[p0 + i] : 0) + al[i];
    }
    return T;
}


// ---------------------------------------------------------------------------------------------
// Top-K, second half (paper Sec. 3.3 (4)) for key range p of one head: the range writes its winners
// - its candidates in bins better than the threshold's, those of the threshold's bin above the
// threshold, plus its allowed number of lowest-index candidates equal to it - as ascending key
// indices into sel[head], starting at its output slot.  The winners (a prefix of the range's
// candidate words and part of one bin's run) set their bits in an LDS bitmap over the range; thread
// t then owns bitmap word t and writes its indices at the rank of its bits.  The first words are
// requested before the threshold is known: they are almost always the ones needed.
// All NT >= R/32 threads of the workgroup must call.  s_bits: 2 * R/32 words, s_scan: NT/64 + 1.
// Returns the number of winners written (uniform); `first` = the range's first output slot.
// s_list (optional, LDS): also receives the first list_cap winners, in the same order.
// Ends with every thread past the last barrier but NOT with a barrier after the global writes.
// ---------------------------------------------------------------------------------------------
constexpr int kEmitPre = 2;  // candidate words per thread requested up front

// the range's first candidate words, requested before its threshold is known
template <int NT>
__device__ __forceinline__ void emit_prefetch(const uint32_t *__restrict__ dk, int R, uint32_t (&pre)[kEmitPre])
{
#pragma unroll
    for (int u = 0; u < kEmitPre; ++u) {
        const int i = u * NT + (int)threadIdx.x;
        pre[u] = i < R ? dk[i] : 0u;  // (slots past the count hold stale words; masked below)
    }
}

// dk: the range's candidate words; c: how many; T: the head's threshold; par = (first output slot,
// ties allowed); run = (start, end) of the threshold's bin among the words (unused when T says
// nothing is selected); pre: emit_prefetch(dk).
template <int NT>
__device__ __forceinline__ int emit_range_core(const uint32_t *__restrict__ dk, const uint32_t (&pre)[kEmitPre],
                                               int c, uint32_t T, int2 par, int2 run,
                                               int32_t *__restrict__ out, int k, int R, int p,
                                               uint32_t *s_bits, int *s_scan, int &first,
                                               int32_t *s_list, int list_cap)
{
    const int W = R / 32;
    uint32_t *s_tie = s_bits + W;
    first = par.x;
    if (c <= 0 || T == 0xFFFFFFFFu) return 0;  // (uniform over the workgroup)
    const uint32_t Tl = T & ((1u << kThrShift) - 1u);
    const int o0 = min(run.x, c);  // winners without a look: [0, o0)
    const int o1 = min(run.y, c);  // the threshold's bin: [o0, o1)
    if ((int)threadIdx.x < W) {
        s_bits[threadIdx.x] = 0;
        s_tie[threadIdx.x] = 0;
    }
    __syncthreads();
    auto place = [&](int i, uint32_t w) {
        if (i < o1) {
            const uint32_t idx = w & ((1u << kIdxBits) - 1u), bit = 1u << (idx & 31);
            const uint32_t sc = w >> kIdxBits;
            if (i < o0 || sc > Tl)
                atomicOr(&s_bits[idx >> 5], bit);
            else if (sc == Tl)
                atomicOr(&s_tie[idx >> 5], bit);
        }
    };
#pragma unroll
    for (int u = 0; u < kEmitPre; ++u) place(u * NT + (int)threadIdx.x, pre[u]);
    for (int i = kEmitPre * NT + (int)threadIdx.x; i < o1; i += NT) place(i, dk[i]);
    __syncthreads();
    uint32_t bits = (int)threadIdx.x < W ? s_bits[threadIdx.x] : 0u;
    uint32_t eq = (int)threadIdx.x < W ? s_tie[threadIdx.x] : 0u;
    int total;
    // keep the lowest-index ties this range is allowed
    if (par.y <= 0) {
        eq = 0;
    } else {
        const int allow = par.y - block_excl_scan<NT>(__popc(eq), s_scan, total);
        if (allow <= 0)
            eq = 0;
        else
            while ((int)__popc(eq) > allow) eq &= ~(0x80000000u >> __clz(eq));  // drop the highest bit
    }
    bits |= eq;
    int pos = par.x + block_excl_scan<NT>(__popc(bits), s_scan, total);
    const int kbase = p * R + (int)threadIdx.x * 32;
    for (; bits; bits &= bits - 1) {
        const int key = kbase + __ffs(bits) - 1;
        if (pos < k) out[pos] = key;
        if (pos - par.x < list_cap) s_list[pos - par.x] = key;  // (the caller's copy of the first winners)
        ++pos;
    }
    return total;
}

// The same with the range's records read from memory (written by k_threshold).
template <int NT>
__device__ __forceinline__ int emit_range(const uint32_t *__restrict__ cand_key,
                                          const int2 *__restrict__ seg_run,
                                          const int32_t *__restrict__ seg_cnt,
                                          const uint32_t *__restrict__ thr,
                                          const int2 *__restrict__ seg_par, int32_t *__restrict__ sel,
                                          int k, int R, int P, size_t cand_stride, int head, int p,
                                          uint32_t *s_bits, int *s_scan, int &first,
                                          int32_t *s_list = nullptr, int list_cap = 0)
{
    const uint32_t *dk = cand_key + (size_t)head * cand_stride + (size_t)p * R;
    uint32_t pre[kEmitPre];
    emit_prefetch<NT>(dk, R, pre);
    const int c = min(seg_cnt[(size_t)head * P + p], R);
    const uint32_t T = thr[head];
    const int2 par = seg_par[(size_t)head * P + p];
    const int2 run = seg_run[(size_t)head * P + p];  // (holds stale values when nothing is selected)
    return emit_range_core<NT>(dk, pre, c, T, par, run, sel + (size_t)head * k, k, R, p, s_bits, s_scan, first,
                               s_list, list_cap);
}

}  // namespace csa

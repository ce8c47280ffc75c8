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
    const int W = R / 32;
    uint32_t *s_tie = s_bits + W;
    uint32_t pre[kEmitPre];
#pragma unroll
    for (int u = 0; u < kEmitPre; ++u) {
        const int i = u * NT + (int)threadIdx.x;
        pre[u] = i < R ? dk[i] : 0u;  // (slots past the count hold stale words; masked below)
    }
    const int c = min(seg_cnt[(size_t)head * P + p], R);
    const uint32_t T = thr[head];
    const int2 par = seg_par[(size_t)head * P + p];
    const int2 run = seg_run[(size_t)head * P + p];  // (holds stale values when nothing is selected)
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
    int32_t *out = sel + (size_t)head * k;
    const int kbase = p * R + (int)threadIdx.x * 32;
    for (; bits; bits &= bits - 1) {
        const int key = kbase + __ffs(bits) - 1;
        if (pos < k) out[pos] = key;
        if (pos - par.x < list_cap) s_list[pos - par.x] = key;  // (the caller's copy of the first winners)
        ++pos;
    }
    return total;
}

}  // namespace csa

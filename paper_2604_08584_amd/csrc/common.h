// Shared device helpers for the gfx950 kernels (wave64 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace csa {

constexpr int kWave = 64;
constexpr int kHeadDim = 128;
// accumulator packing: each table entry contributes q * 64 + 1, so a key's accumulator is
// (sum of q) * 64 + (number of probed rows that list it); non-zero iff the key was seen.
constexpr int kCntBits = 6;
constexpr int32_t kKeyBias = 1 << 24;  // accumulated |sum q| < 2^24  ->  key in (0, 2^25)

struct __align__(8) Entry {
    int32_t idx;  // key index, -1 = unused slot
    int32_t qe;   // q * 64 + 1
};

struct __align__(8) Cand {
    int32_t idx;
    uint32_t key;  // (sum of q) + kKeyBias
};

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// order-preserving image of an fp32 (after -0 -> +0 canonicalisation by the caller)
__device__ __forceinline__ uint32_t orderable(float f)
{
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// number of set bits of `mask` below this lane
__device__ __forceinline__ int mbcnt(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

__device__ __forceinline__ int wave_incl_scan(int v)
{
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        int t = __shfl_up(v, o, kWave);
        if (lane_id() >= o) v += t;
    }
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

// Radix threshold search over n keys (visited through `for_each(fn)`, which must call
// fn(key) once per element, from any thread).  Finds T such that
//   count(key > T) < want <= count(key >= T)            (requires 1 <= want <= n)
// Returns T; `need` = want - count(key > T) = how many keys equal to T are still wanted.
// Keys must be < 2^(RB*PASSES).  s_hist: (1<<RB) + NT/64 + 4 uint32 of LDS.  NT >= (1<<RB).
template <int NT, int RB, int PASSES, class ForEach>
__device__ __forceinline__ uint32_t block_radix_threshold(ForEach for_each, int want,
                                                          uint32_t *s_hist, int &need)
{
    constexpr int NB = 1 << RB;
    static_assert(NT >= NB, "one thread per histogram bin");
    uint32_t *s_aux = s_hist + NB;  // [NT/64] wave totals, then [2] result
    uint32_t *s_res = s_aux + NT / kWave;
    uint32_t prefix = 0, pmask = 0;
    int remaining = want;
    for (int pass = 0; pass < PASSES; ++pass) {
        const int shift = RB * (PASSES - 1 - pass);
        for (int i = threadIdx.x; i < NB; i += NT) s_hist[i] = 0;
        __syncthreads();
        for_each([&](uint32_t key) {
            if ((key & pmask) == prefix) atomicAdd(&s_hist[(key >> shift) & (NB - 1)], 1u);
        });
        __syncthreads();
        // thread t owns bin NB-1-t; inclusive scan from the top bin downwards
        int v = threadIdx.x < NB ? (int)s_hist[NB - 1 - threadIdx.x] : 0;
        int incl = wave_incl_scan(v);
        if (lane_id() == kWave - 1) s_aux[threadIdx.x / kWave] = (uint32_t)incl;
        __syncthreads();
        int off = 0;
        for (int i = 0; i < (int)(threadIdx.x / kWave); ++i) off += (int)s_aux[i];
        incl += off;
        const int excl = incl - v;
        if (threadIdx.x < NB && excl < remaining && remaining <= incl) {
            s_res[0] = (uint32_t)(NB - 1 - threadIdx.x);
            s_res[1] = (uint32_t)excl;
        }
        __syncthreads();
        prefix |= s_res[0] << shift;
        pmask |= (uint32_t)(NB - 1) << shift;
        remaining -= (int)s_res[1];
        __syncthreads();
    }
    need = remaining;
    return prefix;
}

}  // namespace csa

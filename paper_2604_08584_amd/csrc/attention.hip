// Attention half of the decode step: exact softmax attention over the selected keys plus every
// key appended since prefill (paper Sec. 2.1 restricted to the kept set, Sec. 3.3 (4), App. A
// "standard attention over selected KV"), and the K/V append (Sec. 3.3 (5), first sentence).
#include "common.h"
#include "kernels.h"

namespace csa {

// sum over the 16 lanes of a DPP row (result in every lane of the row)
__device__ __forceinline__ float row16_sum(float v)
{
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true));  // row_half_mirror
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, true));  // row_mirror
    return v;
}

constexpr int kXcd = 8;                          // accelerator dies, each with a private L2
constexpr int kAttNT = 256;                     // 4 waves
constexpr int kAttWaves = kAttNT / kWave;
constexpr int kItemsPerWave = 128;              // two index registers per lane
constexpr int kSplit = kAttWaves * kItemsPerWave;  // 512 attended keys per workgroup

// ---------------------------------------------------------------------------------------------
// Split-KV gathered attention.  The attended keys of a head are cut the way the search half cut
// them: split s < P_sel holds the selected keys whose index lies in key range s (their slice of
// the head's ascending `sel` list starts at seg_par[head][s].x), split s >= P_sel holds a run of
// kSplit keys appended since prefill.  Cutting by key range rather than by rank means the G query
// heads of a KV head walk the same stretch of K/V in the same split, so a row picked by several of
// them is fetched from HBM once and hits in L2 for the others.  A K or V row (256 B) is read by
// 16 lanes x 16 B, so one wave load instruction fetches 4 whole rows; each 16-lane group keeps
// its own online-softmax state for the rows it sees, merged at the end.  Logits are taken in
// the log2 domain (q pre-scaled by log2(e)/sqrt(d)).  Output: un-normalised partial
// (max, sum, o[128]) per (head, split).
// EMIT: the workgroup of a key range first finishes the Top-K for that range itself (second half of
// Sec. 3.3 (4): compare the range's candidates with the head's threshold, write the winners'
// indices into `sel`) and then attends what it wrote - possible when a range has at most one bitmap
// word per thread (R <= 8192); it saves a launch, and this latency-bound piece runs while other
// workgroups stream K/V.  Otherwise `sel` is read as given (Top-K done by a kernel before, or a
// reused / caller-made index set).
// grid ceil8(B*Hkv*S) * G workgroups (1-D, see the id mapping below), block 256.
// ---------------------------------------------------------------------------------------------
struct EmitArgs {  // what the prologue of an EMIT launch needs (see emit_range)
    const uint32_t *cand_key, *thr;
    const int2 *seg_run;
    const int32_t *seg_cnt;
    int R;
    size_t cand_stride;
};

template <bool PAGED, bool EMIT>
__global__ __launch_bounds__(kAttNT) void k_attention_split(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ kc, const uint16_t *__restrict__ vc,
    const int32_t *__restrict__ block_table, int32_t *__restrict__ sel,
    const int32_t *__restrict__ sel_count, const int2 *__restrict__ seg_par,
    float *__restrict__ part, int k, int n_pre, int n, int Hq, int G, int Hkv, int max_ctx, int S,
    int P, int P_sel, int n_units, float qscale, EmitArgs ea, const int32_t *__restrict__ n_dev)
{
    // a replayable launch has no context length among its arguments: it reads the device's count
    // (and was sized for the longest window, so some window splits may be empty)
    if (n_dev) n = min(*n_dev, max_ctx);
    __shared__ float s_m[kAttWaves], s_l[kAttWaves], s_o[kAttWaves][kHeadDim];
    __shared__ uint32_t s_bits[EMIT ? 2 * kAttNT : 4];  // winners' and ties' bitmaps of the key range
    __shared__ int s_scan[kAttWaves + 1];
    __shared__ int32_t s_list[EMIT ? kSplit : 1];  // the range's first winners (what one pass attends)
    // XCD-aware order: the chip deals consecutive workgroup ids round-robin to its 8 XCDs (each
    // with its own L2).  The G workgroups that handle the same split of the same KV head get ids
    // 8 apart: same XCD, same moment.
    const int id = blockIdx.x;
    const int unit = (id / (kXcd * G)) * kXcd + id % kXcd;  // (KV head, split) pair
    if (unit >= n_units) return;                            // grid padded to a multiple of 8 * G
    const int s = unit % S;
    const int head = (unit / S) * G + (id % (kXcd * G)) / kXcd;
    const int b = head / Hq, g = (head % Hq) / G;
    const int lane = lane_id(), wave = threadIdx.x / kWave;
    const int sub = lane >> 4, c = lane & 15;
    float *pout = part + ((size_t)head * S + s) * (kHeadDim + 2);
    // this workgroup's items: [first, first + count) of the head's sel list, or of the appended keys
    const bool from_sel = s < P_sel;
    int first, count;
    if (from_sel && EMIT) {
        count = emit_range<kAttNT>(ea.cand_key, ea.seg_run, ea.seg_cnt, ea.thr, seg_par, sel, k, ea.R, P,
                                   ea.cand_stride, head, s, s_bits, s_scan, first, s_list, kSplit);
        count = max(0, min(count, k - first));
        // the winners are read back below by other threads: the first kSplit from LDS (no wait for
        // the stores to `sel`), any further ones - an unusually popular range - from `sel`
        if (count > kSplit) __syncthreads(); else lds_barrier();
    } else if (from_sel) {
        const int n_sel = min(sel_count[head], k);
        first = min(seg_par[(size_t)head * P + s].x, n_sel);
        const int end = s + 1 < P ? min(seg_par[(size_t)head * P + s + 1].x, n_sel) : n_sel;
        count = max(end - first, 0);
    } else {
        first = n_pre + (s - P_sel) * kSplit;
        count = max(min(kSplit, n - first), 0);
    }

    // this lane's 8 query dimensions, pre-scaled
    float qv[8];
    {
        const uint4 w = *(const uint4 *)(q + (size_t)head * kHeadDim + c * 8);
        qv[0] = bf16_lo(w.x) * qscale; qv[1] = bf16_hi(w.x) * qscale;
        qv[2] = bf16_lo(w.y) * qscale; qv[3] = bf16_hi(w.y) * qscale;
        qv[4] = bf16_lo(w.z) * qscale; qv[5] = bf16_hi(w.z) * qscale;
        qv[6] = bf16_lo(w.w) * qscale; qv[7] = bf16_hi(w.w) * qscale;
    }
    float m_run = -INFINITY, l_run = 0.0f, o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = 0.0f;

    // kSplit items per pass over the workgroup (one pass unless a key range is unusually popular).
    // The four waves interleave: group j of 8 consecutive items belongs to wave j % 4, so the
    // workgroup moves through its (ascending) keys as one front - and the workgroups of the other
    // heads of the KV head, started at the same moment on the same XCD, move with it.
    for (int base = 0; base < count; base += kSplit) {
        const int rem = count - base;             // items left for the workgroup
        if (wave * 8 >= rem) break;               // nothing for this wave (wave-uniform)
        // this wave's slot t < 128 is item base + ((t / 8) * 4 + wave) * 8 + t % 8; a prefix of
        // the slots is valid.  Row numbers (in units of 256-byte rows of the cache / pool) of slots
        // lane and 64 + lane:
        int64_t rown[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int t = u * kWave + lane;
            const int a = ((t >> 3) * kAttWaves + wave) * 8 + (t & 7);
            int key = 0;
            if (a < rem) {
                if (EMIT && from_sel && base == 0)
                    key = s_list[a];
                else
                    key = from_sel ? sel[(size_t)head * k + first + base + a] : first + base + a;
            }
            if ((unsigned)key >= (unsigned)n) key = 0;  // never form an address from a bad index
            if (PAGED) {
                const int page = block_table[(size_t)b * (max_ctx >> 4) + (key >> 4)];
                rown[u] = ((int64_t)page * Hkv + g) * 16 + (key & 15);
            } else {
                rown[u] = ((int64_t)b * Hkv + g) * max_ctx + key;
            }
        }
        // valid slots of this wave: full groups of 8 plus the ragged last one
        int n_here = 0;
        {
            const int groups = (rem + 7) / 8;                              // groups of the workgroup
            const int mine = (groups - wave + kAttWaves - 1) / kAttWaves;  // groups of this wave (>= 1)
            const int last = ((mine - 1) * kAttWaves + wave) * 8;          // first item of its last group
            n_here = min(kItemsPerWave, (mine - 1) * 8 + min(8, rem - last));
        }
        // rows of iteration `it`: items it*8 + sub and it*8 + 4 + sub; the next iteration's rows are
        // requested before this one's are used, so that eight row loads per lane group stay in flight
        auto fetch = [&](int it, uint4 &k0, uint4 &k1, uint4 &v0, uint4 &v1) {
            const int i0 = it * 8 + sub, i1 = i0 + 4;
            const int64_t src = it < 8 ? rown[0] : rown[1];
            const int64_t r0 = __shfl(src, i0 & 63, kWave), r1 = __shfl(src, i1 & 63, kWave);
            k0 = *(const uint4 *)(kc + r0 * kHeadDim + c * 8);
            k1 = *(const uint4 *)(kc + r1 * kHeadDim + c * 8);
            v0 = *(const uint4 *)(vc + r0 * kHeadDim + c * 8);
            v1 = *(const uint4 *)(vc + r1 * kHeadDim + c * 8);
        };
        uint4 k0, k1, v0, v1, nk0, nk1, nv0, nv1;
        fetch(0, k0, k1, v0, v1);
        for (int it = 0; it * 8 < n_here; ++it) {
            const int i0 = it * 8 + sub, i1 = i0 + 4;
            // (unconditional, so that the wait below can leave exactly these four loads in flight;
            // after the last iteration it re-requests the rows just used, which hit in cache)
            fetch((it + 1) * 8 < n_here ? it + 1 : it, nk0, nk1, nv0, nv1);
            float d0 = qv[0] * bf16_lo(k0.x), d1 = qv[0] * bf16_lo(k1.x);
            d0 = fmaf(qv[1], bf16_hi(k0.x), d0); d1 = fmaf(qv[1], bf16_hi(k1.x), d1);
            d0 = fmaf(qv[2], bf16_lo(k0.y), d0); d1 = fmaf(qv[2], bf16_lo(k1.y), d1);
            d0 = fmaf(qv[3], bf16_hi(k0.y), d0); d1 = fmaf(qv[3], bf16_hi(k1.y), d1);
            d0 = fmaf(qv[4], bf16_lo(k0.z), d0); d1 = fmaf(qv[4], bf16_lo(k1.z), d1);
            d0 = fmaf(qv[5], bf16_hi(k0.z), d0); d1 = fmaf(qv[5], bf16_hi(k1.z), d1);
            d0 = fmaf(qv[6], bf16_lo(k0.w), d0); d1 = fmaf(qv[6], bf16_lo(k1.w), d1);
            d0 = fmaf(qv[7], bf16_hi(k0.w), d0); d1 = fmaf(qv[7], bf16_hi(k1.w), d1);
            d0 = row16_sum(d0);
            d1 = row16_sum(d1);
            if (i0 >= n_here) d0 = -INFINITY;
            if (i1 >= n_here) d1 = -INFINITY;
            const float m_new = fmaxf(m_run, fmaxf(d0, d1));
            if (m_new != -INFINITY) {  // this 16-lane group has seen at least one real item
                const float sc = exp2f(m_run - m_new);
                const float p0 = exp2f(d0 - m_new), p1 = exp2f(d1 - m_new);
                l_run = l_run * sc + p0 + p1;
                const float vf0[8] = {bf16_lo(v0.x), bf16_hi(v0.x), bf16_lo(v0.y), bf16_hi(v0.y),
                                      bf16_lo(v0.z), bf16_hi(v0.z), bf16_lo(v0.w), bf16_hi(v0.w)};
                const float vf1[8] = {bf16_lo(v1.x), bf16_hi(v1.x), bf16_lo(v1.y), bf16_hi(v1.y),
                                      bf16_lo(v1.z), bf16_hi(v1.z), bf16_lo(v1.w), bf16_hi(v1.w)};
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = fmaf(p1, vf1[e], fmaf(p0, vf0[e], o[e] * sc));
                m_run = m_new;
            }
            k0 = nk0; k1 = nk1; v0 = nv0; v1 = nv1;
        }
    }
    // merge the four 16-lane groups of the wave (lanes c, c+16, c+32, c+48)
#pragma unroll
    for (int x = 16; x <= 32; x <<= 1) {
        const float m_o = __shfl_xor(m_run, x, kWave), l_o = __shfl_xor(l_run, x, kWave);
        const float m_new = fmaxf(m_run, m_o);
        const float sa = m_run == -INFINITY ? 0.0f : exp2f(m_run - m_new);
        const float sb = m_o == -INFINITY ? 0.0f : exp2f(m_o - m_new);
        l_run = l_run * sa + l_o * sb;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = o[e] * sa + __shfl_xor(o[e], x, kWave) * sb;
        m_run = m_new;
    }
    if (lane < 16) {
#pragma unroll
        for (int e = 0; e < 8; ++e) s_o[wave][c * 8 + e] = o[e];
        if (lane == 0) { s_m[wave] = m_run; s_l[wave] = l_run; }
    }
    __syncthreads();
    if (threadIdx.x < kHeadDim) {
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < kAttWaves; ++w) M = fmaxf(M, s_m[w]);
        float acc = 0.0f, l = 0.0f;
#pragma unroll
        for (int w = 0; w < kAttWaves; ++w) {
            const float f = s_m[w] == -INFINITY ? 0.0f : exp2f(s_m[w] - M);
            acc += s_o[w][threadIdx.x] * f;
            l += s_l[w] * f;
        }
        pout[2 + threadIdx.x] = acc;
        if (threadIdx.x == 0) { pout[0] = M; pout[1] = l; }
    }
}

// Where the key ranges start in an ascending index list (a search-period step reuses an index set
// instead of searching, so the per-range output offsets of the Top-K kernels do not exist):
// seg_par[head][p].x = number of listed indices below p*R.  One thread per range, binary search.
// grid B*Hq, block 256.
__global__ void k_range_offsets(const int32_t *__restrict__ sel, const int32_t *__restrict__ sel_count,
                                int2 *__restrict__ seg_par, int k, int R, int P)
{
    const int head = blockIdx.x;
    const int n_sel = max(0, min(sel_count[head], k));
    const int32_t *list = sel + (size_t)head * k;
    for (int p = threadIdx.x; p < P; p += blockDim.x) {
        const int64_t bound = (int64_t)p * R;
        int lo = 0, hi = n_sel;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (list[mid] < bound) lo = mid + 1; else hi = mid;
        }
        seg_par[(size_t)head * P + p] = make_int2(lo, 0);
    }
}

void launch_range_offsets(const int32_t *sel, const int32_t *sel_count, void *seg_par, int n_heads, int k,
                          int R, int P, hipStream_t st)
{
    if (k <= 0) return;
    k_range_offsets<<<n_heads, 256, 0, st>>>(sel, sel_count, (int2 *)seg_par, k, R, P);
}

// Merge of the S split partials of a head (a separate launch: publishing partials to a "last
// workgroup" inside the split kernel needs device-scope fences in every workgroup, which cost far
// more on this multi-die part than one small launch).
// out[head][e] = sum_s o_s[e] 2^(m_s - M) / sum_s l_s 2^(m_s - M); no attended key -> 0.
// grid B*Hq, block 128.
// APPEND: B*Hkv further workgroups write row n of K and V (Sec. 3.3 (5)) - the append that follows
// a step, folded into this launch (the attention kernel, which has finished, never read row n).
struct AppendArgs {
    uint16_t *kc, *vc;
    const int32_t *block_table;
    const uint16_t *kn, *vn;
    int n, Hkv, max_ctx;
    // the context length as the device knows it (a word of the tables buffer) and the word that
    // records an append refused on the device.  from_dev: the position is read there instead of
    // taken from `n` (a launch that can be replayed), and n_bg rows are appended by one workgroup,
    // which then advances the count; otherwise the count is set to n + 1.
    int32_t *n_word, *full_word;
    int from_dev, n_bg;
    // streaming updates: n_try further workgroups (one per queue segment) run the try test of the key
    // being appended against the tables (its centroid scores were taken by the step's scoring launch)
    int n_try;
    TryArgs tr;
};

template <bool PAGED>
__device__ __forceinline__ void append_row(const AppendArgs &a, int n, int bg, int t)
{
    // row n of (sequence, KV head) bg: 16 lanes copy K, 16 lanes V, 16 bytes each
    const int b = bg / a.Hkv, g = bg % a.Hkv;
    int64_t row;
    if (PAGED) {
        const int page = a.block_table[(size_t)b * (a.max_ctx >> 4) + (n >> 4)];
        row = ((int64_t)page * a.Hkv + g) * 16 + (n & 15);
    } else {
        row = (int64_t)bg * a.max_ctx + n;
    }
    const int c = t & 15;
    const uint16_t *src = (t < 16 ? a.kn : a.vn) + (size_t)bg * kHeadDim + c * 8;
    uint16_t *dst = (t < 16 ? a.kc : a.vc) + row * kHeadDim + c * 8;
    *(uint4 *)dst = *(const uint4 *)src;
}

template <int APPEND>  // 0: merge only, 1: + append (contiguous cache), 2: + append (paged cache)
__global__ __launch_bounds__(kHeadDim) void k_attention_merge(const float *__restrict__ part,
                                                              float *__restrict__ out, int S,
                                                              int n_heads, AppendArgs ap)
{
    __shared__ float s_f[kHeadDim];  // per-split scale (S <= 128 per pass)
    __shared__ float s_red[2];
    if (APPEND && (int)blockIdx.x >= n_heads) {  // (uniform over the workgroup)
        if (ap.from_dev) {
            // one workgroup appends every row at the device's own count and then advances it: nothing
            // else in this launch reads the count.  A full context is recorded, not written to.
            const int n = *ap.n_word;
            if (n < ap.max_ctx)
                for (int bg = threadIdx.x / 32; bg < ap.n_bg; bg += kHeadDim / 32)
                    append_row<APPEND == 2>(ap, n, bg, (int)threadIdx.x & 31);
            __syncthreads();
            if (threadIdx.x == 0) {
                if (n < ap.max_ctx) *ap.n_word = n + 1; else *ap.full_word = 1;
            }
            return;
        }
        const int extra = (int)blockIdx.x - n_heads;
        if (extra >= ap.n_bg) {  // (never in a replayable launch: streaming updates exclude it)
            __shared__ int s_try_n;
            const int seg = extra - ap.n_bg;
            insert_try_segment<kHeadDim>(ap.tr, seg / ap.tr.nx, seg % ap.tr.nx, &s_try_n);
            return;
        }
        if (threadIdx.x < 32) append_row<APPEND == 2>(ap, ap.n, extra, (int)threadIdx.x);
        if (extra == 0 && threadIdx.x == 0) *ap.n_word = ap.n + 1;
        return;
    }
    const float *ph = part + (size_t)blockIdx.x * S * (kHeadDim + 2);
    // this thread's value of the first kMergePre splits, requested together with the splits' maxima
    // and sums instead of after them: the launch is a chain of memory round trips, one less this way
    constexpr int kMergePre = 32;
    float pv[kMergePre];
#pragma unroll
    for (int t = 0; t < kMergePre; ++t) pv[t] = t < S ? ph[(size_t)t * (kHeadDim + 2) + 2 + threadIdx.x] : 0.0f;
    float acc = 0.0f, l = 0.0f, M = -INFINITY;
    for (int s0 = 0; s0 < S; s0 += kHeadDim) {
        const int s = s0 + threadIdx.x;
        const float ms = s < S ? ph[(size_t)s * (kHeadDim + 2)] : -INFINITY;
        const float ls = s < S ? ph[(size_t)s * (kHeadDim + 2) + 1] : 0.0f;
        float mx = ms;
        for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, kWave));
        __syncthreads();
        if (lane_id() == 0) s_red[threadIdx.x / kWave] = mx;
        __syncthreads();
        const float M_new = fmaxf(M, fmaxf(s_red[0], s_red[1]));
        const float rescale = M == -INFINITY ? 0.0f : exp2f(M - M_new);
        acc *= rescale;
        l *= rescale;
        M = M_new;
        s_f[threadIdx.x] = ms == -INFINITY ? 0.0f : exp2f(ms - M);
        float lw = ls * s_f[threadIdx.x];
        for (int o = 32; o > 0; o >>= 1) lw += __shfl_xor(lw, o, kWave);
        __syncthreads();
        if (lane_id() == 0) s_red[threadIdx.x / kWave] = lw;
        __syncthreads();
        l += s_red[0] + s_red[1];
        const int ns = min(kHeadDim, S - s0);
        int t_first = 0;
        if (s0 == 0) {  // (the same additions in the same order, from the values already here)
#pragma unroll
            for (int t = 0; t < kMergePre; ++t)
                if (t < ns) acc += pv[t] * s_f[t];
            t_first = kMergePre;
        }
        for (int t = t_first; t < ns; ++t)
            acc += ph[(size_t)(s0 + t) * (kHeadDim + 2) + 2 + threadIdx.x] * s_f[t];
    }
    out[(size_t)blockIdx.x * kHeadDim + threadIdx.x] = l > 0.0f ? acc / l : 0.0f;
}

// number of splits: one per key range for the selected keys (none when k = 0), one per kSplit
// appended keys
int attention_splits(int k, int P, int n_appended)
{
    return (k > 0 ? P : 0) + (n_appended + kSplit - 1) / kSplit;
}

void launch_attention_split(const void *q, const void *kc, const void *vc,
                            const int32_t *block_table, int32_t *sel, const int32_t *sel_count,
                            const void *seg_par, float *part, int B, int Hq, int Hkv, int k, int n_pre,
                            int n, int max_ctx, int S, int P, const uint32_t *cand_key,
                            const void *seg_run, const int32_t *seg_cnt, const uint32_t *thr, int R,
                            size_t cand_stride, const int32_t *n_dev, hipStream_t st)
{
    if (S <= 0) return;
    const float qscale = 1.4426950408889634f / sqrtf((float)kHeadDim);
    const int G = Hq / Hkv;
    const int n_units = B * Hkv * S;
    const int P_sel = k > 0 ? P : 0;
    const bool emit = cand_key != nullptr;  // (the caller has checked attention_can_emit(R))
    const EmitArgs ea{cand_key, thr, (const int2 *)seg_run, seg_cnt, R, cand_stride};
    dim3 grid((n_units + kXcd - 1) / kXcd * kXcd * G), block(kAttNT);
#define CSA_ATT(PAGED_, EMIT_)                                                                            \
    k_attention_split<PAGED_, EMIT_><<<grid, block, 0, st>>>(                                             \
        (const uint16_t *)q, (const uint16_t *)kc, (const uint16_t *)vc, block_table, sel, sel_count,     \
        (const int2 *)seg_par, part, k, n_pre, n, Hq, G, Hkv, max_ctx, S, P, P_sel, n_units, qscale, ea, n_dev)
    if (block_table) {
        if (emit) CSA_ATT(true, true); else CSA_ATT(true, false);
    } else {
        if (emit) CSA_ATT(false, true); else CSA_ATT(false, false);
    }
#undef CSA_ATT
}

bool attention_can_emit(int R) { return R <= 32 * kAttNT; }

void launch_attention_merge(const float *part, float *out, int n_heads, int S, hipStream_t st)
{
    k_attention_merge<0><<<n_heads, kHeadDim, 0, st>>>(part, out, S, n_heads, AppendArgs{});
}

void launch_attention_merge_append(const float *part, float *out, int n_heads, int S, void *kc, void *vc,
                                   const int32_t *block_table, const void *kn, const void *vn, int B,
                                   int Hkv, int n, int max_ctx, int32_t *n_word, int32_t *full_word,
                                   bool from_dev, const TryArgs *tr, hipStream_t st)
{
    const int n_try = tr && !from_dev ? B * Hkv * tr->S * tr->nx : 0;
    const AppendArgs ap{(uint16_t *)kc, (uint16_t *)vc, block_table, (const uint16_t *)kn,
                        (const uint16_t *)vn, n, Hkv, max_ctx, n_word, full_word, from_dev ? 1 : 0, B * Hkv,
                        n_try, n_try ? *tr : TryArgs{}};
    const int grid = n_heads + (from_dev ? 1 : B * Hkv) + n_try;
    if (block_table)
        k_attention_merge<2><<<grid, kHeadDim, 0, st>>>(part, out, S, n_heads, ap);
    else
        k_attention_merge<1><<<grid, kHeadDim, 0, st>>>(part, out, S, n_heads, ap);
}

// K/V append: row n of every (sequence, KV head).  grid B*Hkv, block 32 (16 lanes K, 16 lanes V).
template <bool PAGED>
__global__ void k_append(AppendArgs ap)
{
    append_row<PAGED>(ap, ap.n, (int)blockIdx.x, (int)threadIdx.x);
    if (blockIdx.x == 0 && threadIdx.x == 0) *ap.n_word = ap.n + 1;
}

void launch_append(void *kc, void *vc, const int32_t *block_table, const void *kn, const void *vn,
                   int B, int Hkv, int n, int max_ctx, int32_t *n_word, hipStream_t st)
{
    const AppendArgs ap{(uint16_t *)kc, (uint16_t *)vc, block_table, (const uint16_t *)kn,
                        (const uint16_t *)vn, n, Hkv, max_ctx, n_word, nullptr, 0, B * Hkv, 0, TryArgs{}};
    if (block_table)
        k_append<true><<<B * Hkv, 32, 0, st>>>(ap);
    else
        k_append<false><<<B * Hkv, 32, 0, st>>>(ap);
}

}  // namespace csa

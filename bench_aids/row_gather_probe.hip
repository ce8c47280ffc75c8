// Measurement aid of bench.py --row-gather-floor; no part of the CSAttention library and not
// linked into it.  It reads, and only reads, 256-byte rows of two device buffers at given indices
// the way a gathered-attention kernel fetches K and V rows: a group of 16 lanes owns 64 consecutive
// indices and reads row idx[i] (16 bytes per lane) of both buffers, eight rows of each in flight;
// what it read is folded into one XOR word per group, so that the reads are real and checkable.
// Timed over a decode step's distinct attended rows it gives the floor for any kernel that has
// to fetch them.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr int kProbeRows = 64, kProbeFlight = 8;

// grid ceil(n_idx / 1024), block 256
__global__ __launch_bounds__(256) void k_probe_row_gather(const uint4 *__restrict__ kr,
                                                          const uint4 *__restrict__ vr, long long n_rows,
                                                          const int32_t *__restrict__ idx, long long n_idx,
                                                          uint32_t *__restrict__ check)
{
    const long long grp = ((long long)blockIdx.x * 256 + threadIdx.x) / 16;
    const int l = threadIdx.x & 15;
    const long long i0 = grp * kProbeRows;
    uint32_t x = 0;
    if (i0 >= n_idx) return;  // (whole lane groups; the shuffles below stay within a group)
    // every load is unconditional (a skipped index reads row 0 and its words are dropped): no
    // branch stands between the loads, so all of a round's rows are in flight together
#pragma unroll 1
    for (int r = 0; r < kProbeRows; r += kProbeFlight) {
        long long row[kProbeFlight];
        bool ok[kProbeFlight];
#pragma unroll
        for (int u = 0; u < kProbeFlight; ++u) {
            const long long i = i0 + r + u;
            row[u] = (long long)idx[i < n_idx ? i : n_idx - 1];
            ok[u] = i < n_idx && row[u] >= 0 && row[u] < n_rows;
            row[u] = ok[u] ? row[u] : 0;
        }
        uint4 a[kProbeFlight], b[kProbeFlight];
#pragma unroll
        for (int u = 0; u < kProbeFlight; ++u) {
            a[u] = kr[row[u] * 16 + l];
            b[u] = vr[row[u] * 16 + l];
        }
#pragma unroll
        for (int u = 0; u < kProbeFlight; ++u) {
            const uint32_t w = a[u].x ^ a[u].y ^ a[u].z ^ a[u].w ^ b[u].x ^ b[u].y ^ b[u].z ^ b[u].w;
            x ^= ok[u] ? w : 0u;
        }
    }
#pragma unroll
    for (int d = 8; d >= 1; d >>= 1) x ^= (uint32_t)__shfl_xor((int)x, d, 16);
    if (l == 0) check[grp] = x;
}

}  // namespace

// k_rows_dev, v_rows_dev: device buffers of n_rows rows of 256 bytes; idx_dev: int32 [n_idx];
// check_dev: uint32 [ceil(n_idx / 64)], word j = XOR of all 32-bit words read for indices
// [64 j, 64 j + 64); indices outside [0, n_rows) are skipped.  Enqueues on `stream`.
// Returns 0, or -1 for NULL pointers / non-positive n_rows, -5 if the launch failed.
extern "C" int probe_row_gather(const void *k_rows_dev, const void *v_rows_dev, int64_t n_rows,
                                const int32_t *idx_dev, int64_t n_idx, uint32_t *check_dev, void *stream)
{
    if (!k_rows_dev || !v_rows_dev || !idx_dev || !check_dev) return -1;
    if (n_rows <= 0 || n_idx < 0 || n_idx > ((int64_t)1 << 40)) return -1;
    const int64_t blocks = (n_idx + 16 * kProbeRows - 1) / (16 * kProbeRows);
    if (blocks > 0)
        k_probe_row_gather<<<(unsigned)blocks, 256, 0, (hipStream_t)stream>>>(
            (const uint4 *)k_rows_dev, (const uint4 *)v_rows_dev, n_rows, idx_dev, n_idx, check_dev);
    return hipGetLastError() == hipSuccess ? 0 : -5;
}

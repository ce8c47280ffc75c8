"""bench.py's measurement aid (bench_aids/row_gather_probe.hip, a library of its own: it is no part
of libcsattn.so): the bare K/V row fetch reads exactly the rows it is given."""
import numpy as np
import pytest
import torch

import bench_aids

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(120)]


def test_row_gather_probe_reads_the_rows_it_is_given():
    """Its XOR words equal those of the K and V rows named by the indices (numpy), indices outside
    the buffers are skipped, the last group is ragged."""
    g = torch.Generator().manual_seed(3)
    n_rows, n_idx = 5000, 64 * 37 + 21
    k = torch.randn(n_rows, 128, generator=g).to(torch.bfloat16)
    v = torch.randn(n_rows, 128, generator=g).to(torch.bfloat16)
    idx = torch.randint(0, n_rows, (n_idx,), generator=g, dtype=torch.int32)
    idx[5], idx[70], idx[700], idx[-1] = -1, n_rows, 2 ** 31 - 1, -(2 ** 31)
    n_grp = (n_idx + 63) // 64
    check = torch.full((n_grp + 1,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
    bench_aids.probe_row_gather(k.cuda(), v.cuda(), idx.cuda(), check)
    torch.cuda.synchronize()
    got = check.cpu().numpy().view(np.uint32)
    kw = k.view(torch.int32).numpy().view(np.uint32)          # [n_rows][64]
    vw = v.view(torch.int32).numpy().view(np.uint32)
    rows = idx.numpy().astype(np.int64)
    for j in range(n_grp):
        r = rows[64 * j:64 * j + 64]
        r = r[(r >= 0) & (r < n_rows)]
        want = np.bitwise_xor.reduce(np.concatenate([kw[r].ravel(), vw[r].ravel()])) if len(r) else 0
        assert got[j] == want, j
    assert got[n_grp] == 0x5A5A5A5A                           # nothing past the last group is written


def test_row_gather_probe_rejects_null_arguments():
    bench_aids.probe_row_gather   # loads lazily; call the C entry directly with NULLs
    import ctypes as C
    lib = C.CDLL(bench_aids.LIB)
    lib.probe_row_gather.restype = C.c_int
    assert lib.probe_row_gather(None, None, C.c_int64(1), None, C.c_int64(0), None, None) == -1

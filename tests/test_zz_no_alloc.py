"""csa_decode_step_static - the decode step whose temporaries live in the library's own static
device array, for callers that cannot allocate - against csa_decode_step on the same context and
query: two calls in a row, the second on a smaller input, which finds the array full of the first
call's leftovers.  Indices and counts must be identical, outputs within the output tolerance (they
are the same kernels, so in fact equal).  Collected last: a failure here must not hide other tests.
"""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2604_08584_amd import binding
from paper_2604_08584_amd.workload import CONFIGS

from harness import TOL_OUT, Case, small

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(300)]


def _both_ways(case, step):
    """(out, sel, cnt, rows) of csa_decode_step and of csa_decode_step_static for one query."""
    ctx, q = case.ctx, case.inp["q_steps"][step]
    res = []
    for fn in (binding.csa_decode_step, binding.csa_decode_step_static):
        out = torch.full_like(ctx.out, float("nan"))
        sel = torch.full_like(ctx.sel, -7)
        cnt = torch.full_like(ctx.sel_count, -7)
        fn(ctx.ctx, q, out, sel, cnt)
        rows = ctx.probed_rows()
        torch.cuda.synchronize()
        res.append((out.cpu().numpy(), sel.cpu().numpy(), cnt.cpu().numpy(), rows.cpu().numpy()))
    return res


def _compare(tag, ref, got, k):
    assert np.array_equal(ref[2], got[2]), f"{tag}: counts differ"
    if k:
        assert np.array_equal(ref[1], got[1]), f"{tag}: selected indices differ"
    assert np.array_equal(np.sort(ref[3], axis=-1), np.sort(got[3], axis=-1)), f"{tag}: probed rows differ"
    assert np.isfinite(got[0]).all()
    err = float(np.abs(ref[0] - got[0]).max())
    assert err <= TOL_OUT, f"{tag}: |out_static - out| = {err}"
    return err


def test_static_scratch_step_matches_the_workspace_step_twice_in_a_row():
    big = Case(small("static_big", n_q_heads=8, n_kv_heads=2, n_pre=40000, C=96, L=1500, m=7, k=2000, steps=3),
               F=13, partition_keys=4096)
    big.build_on_gpu()
    need, cap = binding.csa_static_scratch_bytes(big.ctx.ctx)
    assert 0 < need <= cap == 32 << 20
    big.append(2)                                   # appended keys take part in the attention
    ref, got = _both_ways(big, 2)
    print("static scratch, first call: err", _compare("first call", ref, got, big.w.k))
    # the oracle agrees with both (the static step is a decode step like any other)
    heads = [(0, h) for h in range(big.w.n_q_heads)]
    o_rows, o_sel, o_cnt, o_out = big.oracle_decode(2, heads)
    for t, (b, h) in enumerate(heads):
        assert got[2][b, h] == o_cnt[t] and np.array_equal(got[1][b, h][:big.w.k], o_sel[t])
        assert float(np.abs(got[0][b, h] - o_out[t]).max()) <= TOL_OUT

    tiny = Case(small("static_tiny", n_pre=1500, C=20, L=90, m=3, k=70, steps=1), F=13)
    tiny.build_on_gpu()
    ref, got = _both_ways(tiny, 0)
    print("static scratch, second (smaller) call: err", _compare("second call", ref, got, tiny.w.k))
    o_rows, o_sel, o_cnt, o_out = tiny.oracle_decode(0, [(0, h) for h in range(tiny.w.n_q_heads)])
    for h in range(tiny.w.n_q_heads):
        assert got[2][0, h] == o_cnt[h] and np.array_equal(got[1][0, h][:tiny.w.k], o_sel[h])
        assert float(np.abs(got[0][0, h] - o_out[h]).max()) <= TOL_OUT
    # and the first context again, after the smaller one has used the array
    ref, got = _both_ways(big, 1)
    _compare("first context again", ref, got, big.w.k)


def test_static_scratch_step_refuses_what_does_not_fit():
    w = CONFIGS["cfg4"]
    ctx = binding.csa_create(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, n_centroids=w.C,
                             list_len=w.L, n_probe=w.m, budget_k=w.k, max_ctx=w.max_ctx)
    need, cap = binding.csa_static_scratch_bytes(ctx)
    assert need > cap
    rc = binding.lib().csa_decode_step_static(ctx, C.c_void_p(256), C.c_void_p(256), None, None, None)
    assert rc == binding.CSA_ERR_WORKSPACE
    binding.csa_destroy(ctx)

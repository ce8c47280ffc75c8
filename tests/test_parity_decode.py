"""GPU parity: the HIP library (through the C ABI) against the CPU oracle on the same seeded
inputs.  Selected indices, counts and probed rows must match exactly; attention outputs within
2e-2 max-abs (bf16 inputs, fp32 accumulation on the GPU, fp64 in the oracle)."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2604_08584_amd import binding
from paper_2604_08584_amd.workload import CONFIGS

from harness import Case, small

pytestmark = pytest.mark.gpu


def test_cfg0_build_matches_oracle_bit_for_bit_and_decodes():
    """Benchmark configuration 0: tables built on the GPU equal the oracle's tables exactly (same fma
    chain, same grid, same tie rule), then one decode step matches."""
    case = Case(CONFIGS["cfg0"], F=14)
    case.build_on_gpu()
    idx, score = case.export(0, 0)
    o_idx, o_score, mx = case.oracle_tables(0, 0)
    assert mx * case.w.m < 2 ** 24
    assert np.array_equal(idx, o_idx)
    assert np.array_equal(score, o_score)
    err = case.check_step(0)
    print("cfg0 max |out - oracle| =", err)


def test_cfg0_automatic_grid():
    """score_frac_bits < 0: the library picks F itself; the tables then equal the oracle's at
    that F and F is the finest grid its bound allows."""
    case = Case(CONFIGS["cfg0"], F=-1)
    case.build_on_gpu()
    assert 8 <= case.F <= 22
    idx, score = case.export(0, 0)
    o_idx, o_score, mx = case.oracle_tables(0, 0)
    assert np.array_equal(idx, o_idx) and np.array_equal(score, o_score)
    limit = min(2 ** 24 / case.w.m, 2 ** 18)      # exact sums of m scores; 19-bit packed scores
    assert mx < limit and mx * 8 > limit          # within 3 bits of the limit
    case.check_step(0)


@pytest.mark.parametrize("G,part", [(1, 0), (2, 1024), (4, 2048), (8, 1024), (3, 2048), (7, 1024), (12, 0)])
def test_ragged_shapes_import_and_build(G, part):
    """Sizes that are not multiples of any tile (n_pre = 5003, C = 100, L = 300, m = 7, k = 333),
    several key ranges, appended keys crossing the 8-item iteration and wave boundaries."""
    w = small(f"ragged{G}", n_q_heads=2 * G, n_kv_heads=2, n_pre=5003, C=100, L=300, m=7, k=333,
              steps=4, pre_appended=0)
    case = Case(w, seed=G, F=13, partition_keys=part)
    case.import_oracle_tables()
    case.check_step(0)
    case.append(1)
    case.check_step(1)
    case.append(2)
    case.check_step(2)
    # tables built on the GPU agree with the imported oracle tables
    case2 = Case(w, seed=G, F=13, partition_keys=part)
    case2.build_on_gpu()
    for g in range(2):
        idx, score = case2.export(0, g)
        assert np.array_equal(idx, case.oracle_rows(0, g)[0])
        assert np.array_equal(score, case.oracle_rows(0, g)[1])


@pytest.mark.parametrize("part", [4096, 8192, 16384])
def test_key_ranges_spanning_several_index_blocks(part):
    """Key ranges of half a block, one block and two blocks of 8192 key indices (a packed table entry
    keeps only the low 13 index bits; the block follows from the entry's position), ragged last range."""
    w = small(f"blocks{part}", n_q_heads=4, n_kv_heads=2, n_pre=20011, C=30, L=700, m=9, k=1500,
              steps=2)
    case = Case(w, seed=part, F=13, partition_keys=part)
    case.build_on_gpu()
    for g in range(2):
        idx, score = case.export(0, g)
        o_idx, o_score, _ = case.oracle_tables(0, g)
        assert np.array_equal(idx, o_idx) and np.array_equal(score, o_score)
    case.check_step(0)
    case.append(1)
    case.check_step(1)


@pytest.mark.parametrize("S,tau,C", [(2, 3, 300), (8, 1, 37), (8, 2, 64), (16, 3, 20), (4, 2, 600)])
def test_subspace_geometry(S, tau, C):
    """S uniform subspaces with tau probes each (S = 8, tau = 1 is the paper's default; tau > 1 its
    centroid back-off): tables built on the GPU equal the oracle's bit for bit, probed rows, selected
    indices and outputs match over two steps with an append in between."""
    w = small(f"sub{S}x{tau}", n_q_heads=8, n_kv_heads=2, n_pre=5003, C=C, L=200, m=tau, k=333,
              steps=2, n_sub=S)
    case = Case(w, seed=S * 10 + tau, F=13, partition_keys=2048)
    case.build_on_gpu()
    for g in range(2):
        idx, score = case.export(0, g)
        o_idx, o_score, mx = case.oracle_tables(0, g)
        assert mx * S * tau < 2 ** 24
        assert idx.shape == (S * C, 200)
        assert np.array_equal(idx, o_idx) and np.array_equal(score, o_score)
    case.check_step(0)
    case.append(1)
    case.check_step(1)
    # the import path carries the same tables
    case2 = Case(w, seed=S * 10 + tau, F=13, partition_keys=1024)
    case2.import_oracle_tables()
    case2.check_step(0)


@pytest.mark.parametrize("S,tau,L,part", [(1, 2, 2000, 8192), (8, 1, 1800, 8192), (1, 1, 3000, 16384), (2, 3, 1100, 4096)])
def test_few_long_rows_are_walked_in_pieces(S, tau, L, part):
    """Few probed rows with long lists (the paper's geometry has one row of 0.1 N entries per
    subspace): the accumulation launch walks a row's slice of a key range as 2, 4, 8 or more pieces
    handled like rows of their own.  Selected indices and outputs must not change with that: every
    head, two steps with an append in between, ragged last range."""
    w = small(f"pieces{S}x{tau}", n_q_heads=4, n_kv_heads=2, n_pre=9001, C=24, L=L, m=tau, k=700,
              steps=2, n_sub=S)
    case = Case(w, seed=S * 100 + tau, F=13, partition_keys=part)
    case.build_on_gpu()
    case.check_step(0)
    case.append(1)
    case.check_step(1)


def test_subspace_geometry_automatic_grid_uses_subvector_norms():
    """With S = 8 the scores are inner products of 16-dimensional sub-vectors, so the automatic
    grid is finer than the one a whole-vector norm bound would allow."""
    w = small("sub_auto", n_q_heads=4, n_kv_heads=1, n_pre=3000, C=32, L=128, m=1, k=100, steps=1, n_sub=8)
    case = Case(w, seed=3, F=-1)
    case.build_on_gpu()
    w1 = small("sub_auto1", n_q_heads=4, n_kv_heads=1, n_pre=3000, C=32, L=128, m=8, k=100, steps=1)
    case1 = Case(w1, seed=3, F=-1)
    case1.build_on_gpu()
    assert case.F > case1.F
    idx, score = case.export(0, 0)
    o_idx, o_score, mx = case.oracle_tables(0, 0)
    assert np.array_equal(idx, o_idx) and np.array_equal(score, o_score)
    assert mx * 8 < 2 ** 24 and mx < 2 ** 18
    case.check_step(0)


def _tie_heavy_tables(w, rng, qmax, fill):
    idx = np.full((w.batch, w.n_kv_heads, w.C, w.L), -1, np.int32)
    score = np.zeros((w.batch, w.n_kv_heads, w.C, w.L), np.float32)
    for b in range(w.batch):
        for g in range(w.n_kv_heads):
            for j in range(w.C):
                n = int(rng.integers(fill[0], fill[1] + 1))
                ids = rng.choice(w.n_pre, n, replace=False).astype(np.int32)
                q = rng.integers(-qmax, qmax + 1, n)
                order = np.lexsort((ids, -q))
                idx[b, g, j, :n] = ids[order]
                score[b, g, j, :n] = q[order] * 2.0 ** -10
    return idx, score


@pytest.mark.parametrize("k,part", [(1, 1024), (64, 1024), (700, 1024), (5000, 1024), (700, 8192),
                                    (3000, 16384)])
def test_tie_breaking_with_few_distinct_sums(k, part):
    """Tables with integer scores in [-2, 2]: the k-th sum is shared by hundreds of keys, so the
    result is decided by the lowest-index rule, across key ranges and bitmap words; partially
    filled rows (unused slots) are skipped."""
    w = small("ties", n_q_heads=4, n_kv_heads=2, n_pre=9000, C=20, L=400, m=6, k=k, steps=1)
    case = Case(w, seed=7, F=10, partition_keys=part)
    idx, score = _tie_heavy_tables(w, np.random.default_rng(k), 2, (250, 400))
    case.import_tables(idx, score)
    case.check_step(0)


def test_budget_larger_than_union_and_rows_longer_than_prefill():
    """k > |U| -> count = |U|, padding with -1; L > n_pre -> rows padded with unused slots."""
    w = small("pad", n_pre=150, C=6, L=256, m=2, k=400, steps=2)
    case = Case(w, seed=3, F=12)
    case.build_on_gpu()
    idx, score = case.export(0, 0)
    o_idx, o_score, _ = case.oracle_tables(0, 0)
    assert np.array_equal(idx, o_idx) and np.array_equal(score, o_score)
    assert (idx[:, 150:] == -1).all()
    out, sel, cnt, rows = case.decode(0)
    assert (cnt == 150).all() and (sel[..., 150:] == -1).all()
    assert (sel[0, 0, :150] == np.arange(150)).all()
    case.check_step(0)


def test_zero_budget_and_empty_attention():
    w = small("k0", k=0, steps=3)
    case = Case(w, seed=4, F=12)
    case.import_oracle_tables()
    out, sel, cnt, rows = case.decode(0)
    assert (cnt == 0).all() and (out == 0).all()          # nothing selected, nothing appended
    case.append(3)
    case.check_step(1)                                    # dense attention over the 3 appended keys


@pytest.mark.parametrize("m", [1, 12])
def test_single_probe_and_probe_all(m):
    w = small(f"m{m}", C=12, m=m, L=128, k=100, steps=1)
    case = Case(w, seed=5, F=12)
    case.import_oracle_tables()
    case.check_step(0)


def test_many_appended_keys_fill_several_splits():
    """600 appended keys + k = 150: the attended set spans two 512-item splits with a ragged tail."""
    w = small("long_tail", steps=1, pre_appended=600)
    case = Case(w, seed=6, F=12)
    case.import_oracle_tables()
    case.append(600)
    case.check_step(600)


def test_paged_cache_matches_contiguous_and_oracle():
    """16-token pages in shuffled physical order (config 3's storage), appends crossing a page
    boundary; the build reads K through the block table."""
    w = small("paged", batch=2, n_q_heads=4, n_kv_heads=2, n_pre=2000, C=40, L=128, m=4, k=100,
              steps=3, pre_appended=20, page_size=16)
    case = Case(w, seed=8, F=12)
    assert not torch.equal(case.k_store.view(-1)[:4096], case.inp["k_cache"].view(-1)[:4096])
    case.build_on_gpu()
    for b in range(2):
        for g in range(2):
            idx, score = case.export(b, g)
            o_idx, o_score, _ = case.oracle_tables(b, g)
            assert np.array_equal(idx, o_idx) and np.array_equal(score, o_score)
    case.append(20)
    for step in range(3):
        case.check_step(20 + step)
        case.append(1)


@pytest.mark.parametrize("paged", [False, True])
def test_search_period_steps_reuse_the_index_set(paged):
    """Schedule with search period 4: step 0 searches, steps 1-3 reuse its index set for their own
    queries while keys keep being appended (they are always attended), step 4 searches again.
    Both ways of naming the index set (the library's own copy / caller's buffers) are checked."""
    w = small("period", batch=2, n_q_heads=8, n_kv_heads=2, n_pre=6000, C=40, L=300, m=6, k=500,
              steps=6, page_size=16 if paged else 0)
    case = Case(w, seed=12, F=12, partition_keys=2048)
    case.import_oracle_tables()
    with pytest.raises(binding.CsaError) as e:          # nothing to reuse yet
        case.ctx.decode_step_reuse(case.inp["q_steps"][0])
    assert e.value.status == binding.CSA_ERR_STATE
    case.check_step(0)                                  # leaves the library holding step 0's index set
    sel, cnt = case.oracle_index_set(0)                 # the oracle's own copy of it (checked equal above)
    for step in (1, 2, 3):
        case.append(1)
        case.check_reuse_step(step, sel, cnt, pass_buffers=(step == 2))
    case.append(1)
    case.check_step(4)
    # a caller-made ascending list (not a search result) is attended as given
    mine = np.full_like(sel, -1)
    mine[..., :7] = np.array([0, 5, 2047, 2048, 4095, 4096, 5999], np.int32)
    mcnt = np.full_like(cnt, 7)
    case.check_reuse_step(5, mine, mcnt, pass_buffers=True)
    # an empty list leaves the appended keys only
    case.check_reuse_step(5, mine, np.zeros_like(cnt), pass_buffers=True)


@pytest.mark.parametrize("S,L,part,paged", [(1, 200, 1024, False), (4, 96, 2048, True), (1, 700, 8192, False)])
def test_streaming_updates_try_insert_and_recent_window(S, L, part, paged):
    """stream_window = 8: every appended key is try-inserted into the Top-L lists on the GPU and,
    by the oracle, into the host copy; after 1, 9 and 30 appends the exported tables are identical
    and decode steps (window = last 8 positions, excluded from the Top-K candidates) match.  L = 700
    with n_pre = 600 starts from lists with free slots; the other cases evict."""
    n_pre = 600 if L == 700 else 3000
    w = small(f"stream{S}", n_q_heads=4, n_kv_heads=2, n_pre=n_pre, C=24, L=L, m=2, k=150, steps=32,
              n_sub=S, page_size=16 if paged else 0)
    case = Case(w, seed=20 + S, F=12, partition_keys=part, stream_window=8)
    case.build_on_gpu()
    for g in range(2):
        case.check_tables(0, g)
    case.check_step(0)
    done = 0
    for upto in (1, 9, 30):
        case.append(upto - done)
        done = upto
        for g in range(2):
            case.check_tables(0, g)
        case.check_step(upto)
    binding.csa_streaming_status(case.ctx.ctx)                 # no score left the grid
    # the newest keys really are in the tables, and rewinding is refused
    assert (case.oracle_rows(0, 0)[0] >= w.n_pre).any()
    with pytest.raises(binding.CsaError) as e:
        binding.csa_set_context_len(case.ctx.ctx, w.n_pre)
    assert e.value.status == binding.CSA_ERR_STATE


@pytest.mark.parametrize("paged,stream_window", [(False, 0), (True, 0), (False, 6), (True, 6)])
def test_one_call_iteration_equals_step_then_append(paged, stream_window):
    """csa_decode_step_append = csa_decode_step (or the reuse step) followed by csa_append_kv: every
    step's outputs match the oracle on the context before the append, the appended rows are attended
    by the following steps, the tables follow the appends when streaming updates are on, a reuse
    step can be the fused one too, and a full context is refused with nothing changed."""
    w = small("onecall", batch=2, n_q_heads=4, n_kv_heads=2, n_pre=2504, C=32, L=150, m=4, k=200, steps=8,
              page_size=16 if paged else 0)
    assert w.max_ctx == w.n_pre + 8
    case = Case(w, seed=50, F=12, partition_keys=1024, stream_window=stream_window)
    case.build_on_gpu()
    for step in range(5):
        case.check_step(step, fused_append=True)
    assert binding.csa_context_len(case.ctx.ctx) == (w.n_pre, w.n_pre + 5)
    if stream_window:
        for b in range(2):
            for g in range(2):
                case.check_tables(b, g)
        binding.csa_streaming_status(case.ctx.ctx)
    # a reuse step in the one-call form: the oracle's index set of a searching step on this context
    case.check_step(5)
    sel, cnt = case.oracle_index_set(5)
    q = case.inp["q_steps"][6]
    out = case.ctx.decode_step_reuse_append(q, case.inp["k_new"][case.t], case.inp["v_new"][case.t],
                                            torch.from_numpy(sel).cuda(), torch.from_numpy(cnt).cuda())
    torch.cuda.synchronize()
    out = out.cpu().numpy()
    qh, n = oracle.bf16_bits(q), w.n_pre + case.t
    for b in range(2):
        for h in range(4):
            want = oracle.attend_selected(np.ascontiguousarray(qh[b, h]), case.K_host[b, h // 2], case.V_host[b, h // 2],
                                          sel[b, h][:cnt[b, h]], case.window_start(), n)
            assert np.abs(out[b, h] - want).max() <= 2e-2
    case._mirror_append()
    case.check_step(6, fused_append=True)               # attends the rows appended by the one-call steps
    case.check_step(7, fused_append=True)
    assert binding.csa_context_len(case.ctx.ctx)[1] == w.max_ctx
    before = case.ctx.out.clone()
    with pytest.raises(binding.CsaError) as e:          # full: refused before anything is enqueued
        case.ctx.decode_step_append(case.inp["q_steps"][7], case.inp["k_new"][7], case.inp["v_new"][7])
    assert e.value.status == binding.CSA_ERR_CAPACITY
    torch.cuda.synchronize()
    assert torch.equal(before, case.ctx.out) and binding.csa_context_len(case.ctx.ctx)[1] == w.max_ctx
    case.check_step(7)                                   # the plain step still works on the full context


@pytest.mark.parametrize("n_pre,C,steps", [(70000, 8, 12), (1100000, 64, 40)])
def test_streaming_updates_with_many_blocks_per_row(n_pre, C, steps):
    """Key ranges of 1024 over 70K and 1.1M keys: a row is cut into 69 and 1075 blocks, so an
    eviction's hole travels over more than one round of 64 blocks, and (1.1M) the row's offsets no
    longer fit the on-chip copy.  Lists of the maximum length so that a fair share of the appended
    keys enters some list; tables and steps are compared after every few appends."""
    w = small(f"blocks{n_pre}", n_q_heads=2, n_kv_heads=1, n_pre=n_pre, n_comp=8, C=C, L=8192, m=2, k=100,
              steps=steps)
    case = Case(w, seed=60, F=11, partition_keys=1024, stream_window=4, gen_device="cuda")
    case.build_on_gpu()
    case.check_tables(0, 0)
    for upto in (1, steps // 2, steps):
        case.append(upto - case.t)
        case.check_tables(0, 0)
        case.check_step(upto - 1)
    binding.csa_streaming_status(case.ctx.ctx)
    assert (case.oracle_rows(0, 0)[0] >= w.n_pre).sum() >= 3


@pytest.mark.parametrize("n_pre,S,C", [(1, 1, 1), (2, 8, 5), (17, 2, 64)])
def test_streaming_updates_after_a_very_short_prefill(n_pre, S, C):
    """A prefill of one, two or seventeen keys, then generation with streaming updates: lists start
    almost empty and fill up; appended keys score well above anything the prefill held, and none of
    that may be clamped or reported."""
    w = small(f"short{n_pre}", n_q_heads=6, n_kv_heads=2, n_pre=n_pre, n_comp=2, C=C, L=16, m=1, k=50, steps=24,
              n_sub=S)
    case = Case(w, seed=80 + n_pre, F=10, partition_keys=16384, stream_window=3)
    case.build_on_gpu()
    for step in range(24):
        case.check_step(step, fused_append=(step % 2 == 0))
        if step % 2:
            case.append(1)
        if step % 6 == 5:
            for g in range(2):
                case.check_tables(0, g)
    binding.csa_streaming_status(case.ctx.ctx)


@pytest.mark.parametrize("S,tau,C,paged", [(4, 2, 40, False), (8, 1, 128, True), (2, 3, 300, False)])
def test_streaming_one_call_iterations_with_subspaces(S, tau, C, paged):
    """Streaming updates through the one-call iteration with several subspaces: full lists, so every
    accepted key evicts one; the tables of every KV head are compared with the oracle's after four
    and after eight iterations, the steps themselves at every iteration.  (C = 300 takes the scoring
    launch that leaves the try test its own pass over the centroids.)"""
    w = small(f"stream_sub{S}", batch=2, n_q_heads=4, n_kv_heads=2, n_pre=2100, C=C, L=100, m=tau, k=150, steps=8,
              n_sub=S, page_size=16 if paged else 0)
    case = Case(w, seed=300 + S, F=12, partition_keys=2048, stream_window=5)
    case.build_on_gpu()
    for step in range(8):
        case.check_step(step, fused_append=True)
        if step % 4 == 3:
            for b in range(2):
                for g in range(2):
                    case.check_tables(b, g)
    binding.csa_streaming_status(case.ctx.ctx)
    assert (case.oracle_rows(0, 0)[0] >= w.n_pre).any()


def test_streaming_updates_report_scores_that_leave_the_grid():
    w = small("stream_ovf", n_q_heads=4, n_kv_heads=1, n_pre=500, C=8, L=64, m=2, k=50, steps=2)
    case = Case(w, seed=31, F=-1, stream_window=4)
    case.build_on_gpu()
    binding.csa_streaming_status(case.ctx.ctx)
    huge = (case.inp["k_new"][0].float() * 64).to(torch.bfloat16)   # far outside the prefill keys' norms
    case.ctx.append_kv(huge, case.inp["v_new"][0])
    with pytest.raises(binding.CsaError) as e:
        binding.csa_streaming_status(case.ctx.ctx)
    assert e.value.status == binding.CSA_ERR_RANGE


def test_maximum_list_length_and_probe_count():
    """L = 8192 (the largest list: whole-row sorts and the build's index copy fill their LDS) with
    rows shorter and longer than the prefill, and M = 63 probed rows (the most the 6-bit occurrence
    count of an accumulator allows)."""
    w = small("maxL", n_q_heads=2, n_kv_heads=1, n_pre=9000, C=5, L=8192, m=3, k=4000, steps=1)
    case = Case(w, seed=40, F=12, partition_keys=4096)
    case.build_on_gpu()
    idx, score = case.export(0, 0)
    o_idx, o_score, _ = case.oracle_tables(0, 0)
    assert np.array_equal(idx, o_idx) and np.array_equal(score, o_score)
    case.check_step(0)
    case2 = Case(w, seed=40, F=12)
    case2.import_tables(o_idx[None, None], o_score[None, None])
    case2.check_step(0)
    w = small("maxM", n_q_heads=16, n_kv_heads=1, n_pre=2000, C=64, L=100, m=63, k=900, steps=1)   # G = 16
    case = Case(w, seed=41, F=10)
    case.import_oracle_tables()
    case.check_step(0)


def test_result_does_not_depend_on_the_key_range_size():
    """The key-range size is a launch parameter, not part of the method: the selections of the same
    inputs are bit-identical for every admissible size, the outputs equal up to fp32 summation order."""
    w = small("ranges", n_q_heads=4, n_kv_heads=2, n_pre=20000, C=30, L=500, m=6, k=900, steps=1, pre_appended=3)
    ref = None
    for part in (1024, 2048, 4096, 8192, 16384):
        case = Case(w, seed=42, F=12, partition_keys=part)
        case.build_on_gpu()
        case.append(3)
        out, sel, cnt, _ = case.decode(3)
        if ref is None:
            ref = (out, sel, cnt)
            case.check_step(3)
        else:
            assert np.array_equal(sel, ref[1]) and np.array_equal(cnt, ref[2])
            # (outputs: the attention splits follow the key ranges, so fp32 summation order differs)
            np.testing.assert_allclose(out, ref[0], rtol=0, atol=1e-5)


def test_repeated_steps_are_deterministic():
    w = small("det", n_q_heads=8, n_kv_heads=2, steps=1, pre_appended=9)
    case = Case(w, seed=9, F=12, partition_keys=1024)
    case.import_oracle_tables()
    case.append(9)
    first = case.decode(9)
    for _ in range(3):
        again = case.decode(9)
        for a, b in zip(first, again):
            if a is first[3]:
                assert np.array_equal(np.sort(a, -1), np.sort(b, -1))
            else:
                assert np.array_equal(a.view(np.uint8), b.view(np.uint8))


@pytest.mark.parametrize("R,paged", [(8192, False), (1024, True)])
def test_decode_step_is_capturable_in_a_hip_graph(R, paged):
    """A serving loop can capture csa_decode_step (every launch goes to the caller's stream, nothing
    allocates, nothing synchronises, no memset nodes): the graph is replayed with new queries in the
    captured buffer, with eager steps and synchronisations between the replays, and every replay
    matches the oracle and the eager result bit for bit.  (R = 8192 with a small launch takes the path
    that finishes the Top-K inside the attention kernel, R = 1024 the separate kernel.)"""
    w = small("graph", batch=2, n_q_heads=4, n_kv_heads=2, n_pre=9000, C=40, L=400, m=4, k=300, steps=4,
              pre_appended=3, page_size=16 if paged else 0)
    case = Case(w, seed=70, F=12, partition_keys=R)
    case.import_oracle_tables()
    case.append(3)
    q_static = case.inp["q_steps"][3].clone()
    case.ctx.decode_step(q_static)                       # warm-up outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()                           # (default priority)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            case.ctx.decode_step(q_static)
    torch.cuda.synchronize()
    heads = [(b, h) for b in range(w.batch) for h in range(w.n_q_heads)]
    for step in (3, 4, 5, 3):
        q_static.copy_(case.inp["q_steps"][step])
        graph.replay()
        torch.cuda.synchronize()
        out = case.ctx.out.cpu().numpy().copy()
        sel = case.ctx.sel.cpu().numpy().copy()
        cnt = case.ctx.sel_count.cpu().numpy().copy()
        e_out, e_sel, e_cnt, _ = case.decode(step)      # eager work between the replays
        assert np.array_equal(out.view(np.uint8), e_out.view(np.uint8))
        assert np.array_equal(sel, e_sel) and np.array_equal(cnt, e_cnt)
        _, o_sel, o_cnt, o_out = case.oracle_decode(step, heads)
        for t, (b, h) in enumerate(heads):
            assert cnt[b, h] == o_cnt[t] and np.array_equal(sel[b, h][:w.k], o_sel[t])
            assert np.abs(out[b, h] - o_out[t]).max() <= 2e-2


def test_device_side_errors_are_reported():
    w = small("err", n_pre=500, C=8, L=64, m=2, k=10, steps=1)
    case = Case(w, seed=10, F=12)
    idx = np.full((1, 1, 8, 64), -1, np.int32)
    score = np.zeros((1, 1, 8, 64), np.float32)
    idx[0, 0, :, 0] = 3
    score[0, 0, :, 0] = 0.3                                   # not a multiple of 2^-12
    with pytest.raises(binding.CsaError) as e:
        case.import_tables(idx, score)
    assert e.value.status == binding.CSA_ERR_RANGE
    score[0, 0, :, 0] = 2.0 ** 23                             # on the grid, far too large
    with pytest.raises(binding.CsaError) as e:
        case.import_tables(idx, score)
    assert e.value.status == binding.CSA_ERR_RANGE
    score[:] = 0
    idx[0, 0, 1, 5] = 500                                     # key index == n_pre
    with pytest.raises(binding.CsaError) as e:
        case.import_tables(idx, score)
    assert e.value.status == binding.CSA_ERR_ARG
    with pytest.raises(binding.CsaError) as e:                # tables invalid after a failed import
        case.decode(0)
    assert e.value.status == binding.CSA_ERR_STATE
    idx[0, 0, 1, 5] = 499
    case.import_tables(idx, score)
    n_free = w.max_ctx - w.n_pre
    for t in range(n_free):
        case.ctx.append_kv(case.inp["k_new"][0], case.inp["v_new"][0])
    with pytest.raises(binding.CsaError) as e:
        case.ctx.append_kv(case.inp["k_new"][0], case.inp["v_new"][0])
    assert e.value.status == binding.CSA_ERR_CAPACITY
    assert binding.csa_context_len(case.ctx.ctx) == (500, w.max_ctx)


def test_profile_counters_cover_every_stage():
    # 64 heads of 40 key ranges each: too many workgroups for the accumulation launch to choose the probed
    # rows itself or for the attention launch to write the winners, so every stage is a launch of its own
    w = small("prof", batch=4, n_q_heads=16, n_kv_heads=4, n_pre=40000, L=900, k=2000, steps=2, pre_appended=0)
    case = Case(w, seed=11, F=12, partition_keys=1024)
    case.import_oracle_tables()
    binding.csa_profile_enable(case.ctx.ctx, True)
    case.decode(0)
    case.append(1)
    case.decode(1)
    prof = binding.csa_profile_read(case.ctx.ctx)
    binding.csa_profile_enable(case.ctx.ctx, False)
    assert prof["append_kv"][1] == 1
    for name in ("score_centroids", "top_centroids", "accumulate", "select_threshold", "select_emit", "attention_split",
                 "attention_merge"):
        assert prof[name][1] == 2 and prof[name][0] > 0
    assert all(v == (0.0, 0) for v in binding.csa_profile_read(case.ctx.ctx).values())


def test_two_contexts_interleaved_on_two_streams():
    """Two contexts of different shapes take turns, each on a stream of its own: nothing in the
    library is shared between contexts, so every step still matches the oracle."""
    wa = small("ctx_a", n_q_heads=8, n_kv_heads=2, n_pre=9000, C=64, L=300, m=4, k=500, steps=4)
    wb = small("ctx_b", batch=2, n_q_heads=6, n_kv_heads=2, n_pre=2000, C=32, L=64, m=2, k=40, steps=4,
               n_sub=4, page_size=16)
    a = Case(wa, seed=1, F=12, partition_keys=1024)
    b = Case(wb, seed=2, F=10, stream_window=3)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    with torch.cuda.stream(sa):
        a.build_on_gpu()
    with torch.cuda.stream(sb):
        b.build_on_gpu()
    for step in range(4):
        with torch.cuda.stream(sa):
            a.check_step(step, fused_append=(step % 2 == 0))
            if step % 2:
                a.append(1)
        with torch.cuda.stream(sb):
            b.check_step(step, fused_append=(step % 2 == 1))
            if step % 2 == 0:
                b.append(1)
    with torch.cuda.stream(sb):
        for g in range(2):
            b.check_tables(0, g)
            b.check_tables(1, g)


@pytest.mark.parametrize("stream", [0, 4])
def test_a_context_is_reused_for_new_sequences(stream):
    """A serving loop keeps one context and its buffers: after some steps on one sequence the caller
    overwrites the K/V cache with the prefill of another (shorter, then longer) and calls
    csa_build_tables again with new centroids.  Nothing of the earlier sequence may survive: tables,
    context length, key ranges and the score grid all follow the new build."""
    shape = dict(n_q_heads=8, n_kv_heads=2, C=48, L=200, m=3, k=150, steps=6)
    first = Case(small("seq0", n_pre=9000, **shape), seed=1, F=-1, stream_window=stream)
    first.build_on_gpu()
    first.check_step(0, fused_append=True)
    first.check_step(1, fused_append=True)
    shared = first.ctx
    for i, n_pre in enumerate((2500, 8800)):
        nxt = Case(small(f"seq{i + 1}", n_pre=n_pre, **shape), seed=10 + i, F=-1, stream_window=stream)
        nxt.ctx.close()
        nxt.ctx = shared                                    # the first sequence's context and buffers
        n_rows = nxt.w.max_ctx
        first.inp["k_cache"][:, :, :n_rows] = nxt.inp["k_cache"]
        first.inp["v_cache"][:, :, :n_rows] = nxt.inp["v_cache"]
        nxt.build_on_gpu()
        assert binding.csa_context_len(shared.ctx) == (n_pre, n_pre)
        for g in range(2):
            nxt.check_tables(0, g)
        for step in range(3):
            nxt.check_step(step, fused_append=(step != 1))
            if step == 1:
                nxt.append(1)
        if stream:
            for g in range(2):
                nxt.check_tables(0, g)
        nxt.ctx = None                                      # (the context belongs to `first`)

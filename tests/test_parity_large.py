"""GPU parity at the full sizes of benchmark configurations 1-4, in the launch configuration bench.py
times (automatic key-range size, automatic score grid).  The oracle recomputes sampled table
rows and sampled (sequence, head) decode steps one by one, building for each sampled head the
table rows it probes itself (nothing the oracle reads comes from the GPU).  Centroid synthesis is
shortened (fewer
Lloyd iterations on a sample of the prefill queries): centroids are inputs to both sides."""
import dataclasses

import numpy as np
import pytest

from paper_2604_08584_amd import binding
from paper_2604_08584_amd.workload import CONFIGS, Workload

from harness import Case

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


def _check_rows(case, b, g, rows):
    idx, score = case.export(b, g)
    o_idx, o_score, mx = case.oracle_tables(b, g, rows)
    assert mx * case.w.m * case.w.n_sub < 2 ** 24
    assert np.array_equal(idx[rows], o_idx), f"table rows {rows} of ({b},{g}) differ"
    assert np.array_equal(score[rows], o_score)
    # row invariants at full size: distinct, in range, sorted by score
    assert all(len(set(r.tolist())) == case.w.L for r in idx[rows])
    assert (np.diff(score[rows], axis=1) <= 0).all()


def _light(name, steps, **kw):
    return dataclasses.replace(CONFIGS[name], kmeans_iters=3, steps=steps, **kw)


def test_cfg1_full_size():
    w = _light("cfg1", 1)
    case = Case(w, F=-1, gen_device="cuda", kmeans_sample=16 * w.C)
    case.build_on_gpu()
    _check_rows(case, 0, 3, [0, 511, 1023])
    print("cfg1 all 32 heads err", case.check_step(0))


def test_cfg2_full_size_with_appends():
    w = _light("cfg2", 4)
    case = Case(w, F=-1, gen_device="cuda", kmeans_sample=16 * w.C)
    case.build_on_gpu()
    _check_rows(case, 0, 5, [7, 2047])
    heads = [(0, h) for h in (0, 3, 20, 21, 22, 23)]
    for step in range(3):       # the one-call iteration bench.py times, and the two-call form
        print("cfg2 step", step, "err", case.check_step(step, heads, fused_append=(step != 1)))
        if step == 1:
            case.append(1)


def test_cfg3_paged_batch():
    w = _light("cfg3", 2)
    case = Case(w, F=-1, gen_device="cuda", kmeans_sample=16 * w.C)
    case.build_on_gpu()
    _check_rows(case, 9, 2, [5, 1000])
    case.append(w.pre_appended)
    heads = [(0, 0), (0, 31), (9, 8), (9, 9), (15, 4), (15, 31)]
    print("cfg3 err", case.check_step(w.pre_appended, heads))
    case.append(1)
    print("cfg3 err", case.check_step(w.pre_appended + 1, heads))


def test_cfg4_70b_shape():
    w = _light("cfg4", 3)
    case = Case(w, F=-1, gen_device="cuda", kmeans_sample=8 * w.C)
    case.build_on_gpu()
    _check_rows(case, 7, 7, [4095])
    heads = [(0, 0), (0, 7), (3, 40), (7, 56), (7, 63)]
    for step in range(2):       # the one-call iteration (step, then append) that bench.py times
        print("cfg4 step", step, "err", case.check_step(step, heads, fused_append=True))


def _sampled_rows(case, n_groups, per_group, seed):
    """per_group table rows of each of n_groups (sequence, KV head) pairs, seeded; compared one export
    per pair."""
    w = case.w
    rng = np.random.default_rng(seed)
    pairs = rng.choice(w.batch * w.n_kv_heads, size=n_groups, replace=False)
    for pr in pairs:
        b, g = divmod(int(pr), w.n_kv_heads)
        rows = sorted(set(rng.choice(w.n_sub * w.C, size=per_group, replace=False).tolist()) | {0, w.n_sub * w.C - 1})
        _check_rows(case, b, g, rows)


def test_cfg2_every_head_first_and_last_step():
    """Config 2 as defined (batch 1, 128K, 64 steps): 34+ sampled table rows, EVERY head at the first
    step and EVERY head at the last one (63 keys appended), in the one-call form bench.py times."""
    w = _light("cfg2", 64)
    case = Case(w, F=-1, gen_device="cuda", kmeans_sample=16 * w.C)
    case.build_on_gpu()
    _sampled_rows(case, 4, 8, seed=2)
    print("cfg2 all heads, step 0: err", case.check_step(0, fused_append=True))
    case.append(62)
    assert case.t == 63
    print("cfg2 all heads, step 63: err", case.check_step(63, fused_append=True))
    assert binding.csa_context_len(case.ctx.ctx) == (w.n_pre, w.n_pre + 64)


def test_cfg4_every_head_and_the_last_step():
    """Config 4 as defined (batch 8, 64 query heads, 128K, 256 steps): 40 sampled table rows, EVERY
    one of the 512 heads at the first step and at the last one (255 keys appended, context 131327);
    the oracle builds the table rows they probe, about 16 thousand per step."""
    w = _light("cfg4", 256)
    case = Case(w, F=-1, gen_device="cuda", kmeans_sample=8 * w.C)
    case.build_on_gpu()
    _sampled_rows(case, 4, 8, seed=4)
    print("cfg4 all 512 heads, step 0: err", case.check_step(0, fused_append=True))
    case.append(254)
    assert case.t == 255
    print("cfg4 all 512 heads, step 255: err", case.check_step(255, fused_append=True))
    assert binding.csa_context_len(case.ctx.ctx) == (w.n_pre, w.n_pre + 256)


def test_paper_default_geometry_full_size():
    """The paper's default geometry (8 subspaces, one probe each, C = 128, L = 0.1 N_pre,
    k = 0.05 N_pre) at 64K context, batch 8: sampled table rows of several subspaces and sampled
    heads over two steps."""
    w = _light("paper_s8", 2)
    case = Case(w, F=-1, gen_device="cuda", kmeans_sample=64 * w.C)
    case.build_on_gpu()
    _check_rows(case, 3, 5, [0, 127, 128 * 3 + 17, 128 * 7 + 127])
    heads = [(0, 0), (0, 3), (3, 20), (7, 28), (7, 31)]
    for step in range(2):
        print("paper_s8 step", step, "err", case.check_step(step, heads))
        case.append(1)


def test_cfg3_every_head_paged():
    """All 512 (sequence, query head) pairs of config 3 (paged K/V through a scattered block table, 256
    keys appended before the step) in one step, and 32 sampled table rows."""
    w = _light("cfg3", 1)
    case = Case(w, F=-1, gen_device="cuda", kmeans_sample=8 * w.C)
    case.build_on_gpu()
    _sampled_rows(case, 4, 8, seed=31)
    case.append(w.pre_appended)
    print("cfg3 all 512 heads err", case.check_step(w.pre_appended))


def test_paper_geometry_every_head():
    """All 256 (sequence, query head) pairs of the paper's default geometry at 64K context, one step."""
    w = _light("paper_s8", 1)
    case = Case(w, F=-1, gen_device="cuda", kmeans_sample=64 * w.C)
    case.build_on_gpu()
    print("paper_s8 all 256 heads err", case.check_step(0))


def test_long_context_with_the_widest_key_ranges():
    """A 144K context in ranges of 16384 keys (the widest the library offers: 1024-thread accumulation
    workgroups with two blocks per range, 512-thread workgroups writing the winners); every head of
    two KV heads, two steps."""
    w = Workload("long144k", 1, 8, 2, 128, 147000, 64, 512, 2048, 16, 7350, 2, 0, 0, kmeans_iters=3)
    case = Case(w, F=-1, partition_keys=16384, gen_device="cuda", kmeans_sample=16 * w.C)
    case.build_on_gpu()
    heads = [(0, h) for h in range(8)]
    for step in range(2):
        print("long144k step", step, "err", case.check_step(step, heads))
        case.append(1)


def test_cfg2_streaming_updates_full_size():
    """Config 2's shape with streaming updates (recent window R = 32): 40 appended keys are
    try-inserted on the GPU and by the oracle into KV head 5's tables; tables and sampled decode
    steps (before the window is full, and after keys have left it) must match."""
    w = _light("cfg2", 41)
    case = Case(w, F=-1, gen_device="cuda", kmeans_sample=16 * w.C, stream_window=32)
    case.build_on_gpu()
    heads = [(0, 20), (0, 21), (0, 23)]
    print("stream step 0 err", case.check_step(0, heads))
    for upto in (3, 40):
        case.append(upto - case.t, groups=[(0, 5)])
        case.check_tables(0, 5)
        print("stream step", upto, "err", case.check_step(upto, heads))
    idx = case.oracle_rows(0, 5)[0]
    print("rows holding appended keys:", int((idx >= w.n_pre).any(axis=1).sum()), "of", idx.shape[0])

"""GPU parity of the offline query clustering (paper Sec. 3.2 (1)): the library's k-means++ seeding
and Lloyd steps (assignment on the matrix cores) against the oracle's two-part bf16 form.

Where floating point decides an integer (an assignment, a seed draw) both sides are compared on
what is unique: assignments may differ only where the oracle's own decision gap is at rounding
level; centroids of clusters with identical members may differ by one bf16 step (fp32 atomics vs
fp64 sums); seeds must be data points and follow the D^2 weighting."""
import random

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2604_08584_amd import binding

from harness import Case, small

pytestmark = pytest.mark.gpu


def _queries(B, Hq, n_pre, n_comp, seed, spread=0.5):
    """Mixture-of-Gaussians prefill queries [B][Hq][n_pre][128] bf16 (data synthesis only)."""
    g = torch.Generator().manual_seed(seed)
    means = torch.randn(n_comp, 128, generator=g)
    comp = torch.randint(0, n_comp, (B, Hq, n_pre), generator=g)
    x = means[comp] + spread * torch.randn(B, Hq, n_pre, 128, generator=g)
    return x.to(torch.bfloat16)


def _ctx(B, Hq, Hkv, C, S):
    return binding.csa_create(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, n_centroids=C, list_len=64, n_probe=1,
                              budget_k=10, max_ctx=4096, n_subspaces=S)


def _pool(q_bits, b, g, G, sub, db):
    """Pooled sub-vectors of KV head (b, g) as fp32 [G*n_pre][db]."""
    x = oracle.bits_to_f32(q_bits[b, g * G:(g + 1) * G])          # [G][n_pre][128]
    return np.ascontiguousarray(x.reshape(-1, 128)[:, sub * db:(sub + 1) * db])


def _check_lloyd_step(B, Hkv, G, n_pre, S, C, seed, max_diff=2):
    """One Lloyd step from random unit centroids on both sides; returns nothing, asserts parity."""
    Hq, db = G * Hkv, 128 // S
    q = _queries(B, Hq, n_pre, 12, 100 + seed)
    rng = np.random.default_rng(seed)
    init = rng.standard_normal((B, Hkv, S, C, db)).astype(np.float32)
    init /= np.linalg.norm(init, axis=-1, keepdims=True)
    init_t = torch.from_numpy(init).to(torch.bfloat16).cuda()
    ctx = _ctx(B, Hq, Hkv, C, S)
    out = torch.empty_like(init_t)
    mean_cos = torch.zeros(B, Hkv, S, 1, device="cuda")
    assign = torch.empty(B, Hkv, S, G * n_pre, dtype=torch.int32, device="cuda")
    binding.csa_cluster_queries(ctx, q.cuda(), n_pre, 1, None, init_t, out, mean_cos, assign)
    binding.csa_destroy(ctx)
    q_bits, init_bits, out_bits = oracle.bf16_bits(q), oracle.bf16_bits(init_t), oracle.bf16_bits(out)
    assign, mean_cos = assign.cpu().numpy(), mean_cos.cpu().numpy()
    n_diff = 0
    for b in range(B):
        for g in range(Hkv):
            for s in range(S):
                x = _pool(q_bits, b, g, G, s, db)
                want, asg, gap, mc = oracle.kmeans_step(x, init_bits[b, g, s])
                diff = np.nonzero(assign[b, g, s] != asg)[0]
                n_diff += len(diff)
                assert (gap[diff] < 1e-5).all(), f"assignments differ where the decision was clear: {gap[diff]}"
                assert mean_cos[b, g, s, 0] == pytest.approx(mc, abs=1e-4)
                got_f, want_f = oracle.bits_to_f32(out_bits[b, g, s]), oracle.bits_to_f32(want)
                touched = set(assign[b, g, s][diff].tolist()) | set(asg[diff].tolist())
                for j in range(C):
                    if j in touched:
                        continue
                    np.testing.assert_allclose(got_f[j], want_f[j], rtol=2.0 ** -7, atol=1e-6,
                                               err_msg=f"centroid {j} of ({b},{g},{s})")
                np.testing.assert_allclose(np.linalg.norm(got_f.astype(np.float64), axis=1), 1.0, atol=1e-2)
    assert n_diff <= max_diff


@pytest.mark.parametrize("S,C", [(1, 37), (4, 64), (16, 20), (8, 130)])
def test_lloyd_step_matches_the_oracle(S, C):
    _check_lloyd_step(B=2, Hkv=2, G=2, n_pre=700, S=S, C=C, seed=S)


def test_lloyd_step_on_random_shapes():
    """Pools of 1 to 24000 points and 1 to 1030 centroids around every tile edge of the assignment
    kernel (32-point and 32-centroid MFMA tiles, 128 points per workgroup), all sub-space widths,
    more centroids than points."""
    rng = random.Random(5)
    for ci in range(24):
        S = rng.choice([1, 2, 4, 8, 16])
        C = rng.choice([1, 2, 3, 31, 32, 33, 63, 64, 65, 127, 128, 129, 200, 257, 600, 1030])
        B, Hkv, G = rng.choice([1, 2]), rng.choice([1, 2]), rng.choice([1, 2, 3, 8])
        n_pre = rng.choice([1, 5, 31, 64, 127, 128, 129, 700, 1111, 3000])
        print(ci, dict(S=S, C=C, B=B, Hkv=Hkv, G=G, n_pre=n_pre), flush=True)
        _check_lloyd_step(B, Hkv, G, n_pre, S, C, seed=1000 + ci, max_diff=4)
    # the widest sub-vectors with the most centroids whose sums still go through LDS, and one more
    for C in (56, 57, 63, 64):
        _check_lloyd_step(1, 2, 2, 300, 1, C, seed=2000 + C, max_diff=4)


def test_seeds_are_data_points_drawn_by_squared_distance():
    """8 tight groups of 150 points and C = 8: D^2 sampling lands in a new group at (almost) every
    draw, every seed is one of the normalised points rounded to bf16, the first seed is point
    floor(u_0 n), and the whole seed set matches the oracle's (fp64) draw."""
    B, Hq, Hkv, n_pre, C = 1, 2, 1, 600, 8
    g = torch.Generator().manual_seed(7)
    dirs = torch.nn.functional.normalize(torch.randn(8, 128, generator=g), dim=1)
    comp = torch.arange(B * Hq * n_pre).view(B, Hq, n_pre) % 8
    x = (dirs[comp] * (1 + torch.rand(B, Hq, n_pre, 1, generator=g)) +
         0.01 * torch.randn(B, Hq, n_pre, 128, generator=g)).to(torch.bfloat16)
    u = np.random.default_rng(1).uniform(size=(B, Hkv, 1, C)).astype(np.float32)
    ctx = _ctx(B, Hq, Hkv, C, 1)
    out = torch.empty(B, Hkv, 1, C, 128, dtype=torch.bfloat16, device="cuda")
    binding.csa_cluster_queries(ctx, x.cuda(), n_pre, 0, u, None, out)
    binding.csa_destroy(ctx)
    seeds = oracle.bits_to_f32(oracle.bf16_bits(out))[0, 0, 0]
    pool = _pool(oracle.bf16_bits(x), 0, 0, 2, 0, 128)
    pn = pool / np.linalg.norm(pool, axis=1, keepdims=True)
    pn_bf16 = oracle.bits_to_f32(oracle.round_bf16(pn.astype(np.float32)))
    which = [int(np.argmax(pn @ s)) for s in seeds]
    for s, i in zip(seeds, which):
        assert np.abs(pn_bf16[i] - s).max() <= 2.0 ** -8          # a data point (fp32 vs fp64 normalisation)
    assert which[0] == int(np.float64(u[0, 0, 0, 0]) * len(pool))
    groups = {int(np.argmax(dirs.numpy() @ s)) for s in seeds}
    assert len(groups) >= 7
    _compare_seeds(seeds, pool, C, u[0, 0, 0])


def _compare_seeds(seeds, pool, C, u, tol=2e-5):
    """The library's seeds (fp32 [C][d]) against the oracle's draws on the same points and uniforms:
    equal seed by seed up to the first draw whose target sat within `tol` of the total from the edge
    of the picked point's stretch of the running sum (the oracle reports that margin; the library sums
    in fp32, block by block) - at such a draw the library may take a neighbouring point, and the
    later draws are then not comparable.  Returns the number of seeds compared equal."""
    want_bits, picks, margin = oracle.kmeans_seed(pool, C, np.asarray(u, np.float64), with_draws=True)
    want = oracle.bits_to_f32(want_bits)
    for j in range(C):
        if np.abs(want[j] - seeds[j]).max() <= 2.0 ** -8:
            continue
        assert margin[j] < tol, f"seed {j} differs from the oracle's (point {picks[j]}) although the draw was clear: margin {margin[j]}"
        print(f"seed {j}: a draw at rounding level (margin {margin[j]:.2e}); {j} of {C} seeds compared")
        return j
    return C


@pytest.mark.parametrize("S,C,n_pre,G", [(1, 40, 900, 2), (8, 17, 333, 3), (4, 100, 2100, 1)])
def test_seeding_matches_the_oracle_draw_by_draw(S, C, n_pre, G):
    """Generic mixtures (no structure that would make the draws easy), several problems side by side:
    every problem's seeds follow the oracle's draws; a difference is accepted only at a draw the
    oracle itself marks as rounding-level, and at most one problem may have one."""
    B, Hkv = 2, 2
    Hq, db = Hkv * G, 128 // S
    q = _queries(B, Hq, n_pre, 9, 40 + S)
    u = np.random.default_rng(S).uniform(size=(B, Hkv, S, C)).astype(np.float32)
    ctx = _ctx(B, Hq, Hkv, C, S)
    out = torch.empty(B, Hkv, S, C, db, dtype=torch.bfloat16, device="cuda")
    binding.csa_cluster_queries(ctx, q.cuda(), n_pre, 0, u, None, out)
    binding.csa_destroy(ctx)
    seeds = oracle.bits_to_f32(oracle.bf16_bits(out))
    q_bits = oracle.bf16_bits(q)
    short = 0
    for b in range(B):
        for g in range(Hkv):
            for s in range(S):
                short += _compare_seeds(seeds[b, g, s], _pool(q_bits, b, g, G, s, db), C, u[b, g, s]) < C
    assert short <= 1


def test_minibatch_steps_match_the_oracle():
    """Three mini-batch steps over three classes of points (i % 3), from given centroids: after every
    step the running-mean centroids equal the oracle's wherever no rounding-level assignment
    difference touched the cluster; assignments of the last step are -1 outside its class."""
    B, Hkv, G, n_pre, S, C, nb = 1, 2, 2, 900, 2, 24, 3
    Hq, db = Hkv * G, 128 // S
    q = _queries(B, Hq, n_pre, 10, 77)
    rng = np.random.default_rng(9)
    init = rng.standard_normal((B, Hkv, S, C, db)).astype(np.float32)
    init /= np.linalg.norm(init, axis=-1, keepdims=True)
    init_t = torch.from_numpy(init).to(torch.bfloat16).cuda()
    q_bits, init_bits = oracle.bf16_bits(q), oracle.bf16_bits(init_t)
    for iters in (1, 2, 3):
        ctx = _ctx(B, Hq, Hkv, C, S)
        out = torch.empty_like(init_t)
        mean_cos = torch.zeros(B, Hkv, S, iters, device="cuda")
        assign = torch.empty(B, Hkv, S, G * n_pre, dtype=torch.int32, device="cuda")
        binding.csa_cluster_queries(ctx, q.cuda(), n_pre, iters, None, init_t, out, mean_cos, assign, n_batches=nb)
        binding.csa_destroy(ctx)
        out_bits, assign_h, mc_h = oracle.bf16_bits(out), assign.cpu().numpy(), mean_cos.cpu().numpy()
        for g in range(Hkv):
            for s in range(S):
                x = _pool(q_bits, 0, g, G, s, db)
                cent = init_bits[0, g, s]
                rs, rc = np.zeros((C, db)), np.zeros(C, np.int64)
                touched = set()
                for it in range(iters):
                    cls = np.arange(it % nb, len(x), nb)
                    cent, asg, gap, mc = oracle.kmeans_minibatch_step(x[cls], cent, rs, rc)
                    assert mc_h[0, g, s, it] == pytest.approx(mc, abs=2e-4)
                got = assign_h[0, g, s]
                outside = np.setdiff1d(np.arange(len(x)), cls)
                assert (got[outside] == -1).all()
                diff = np.nonzero(got[cls] != asg)[0]
                assert (gap[diff] < 1e-5).all() and len(diff) <= 2
                # (a rounding-level difference in an earlier step cannot be seen here; the centroid
                # comparison below then skips nothing it should not: such a difference moves a sum by
                # one point of hundreds, far inside the tolerance for all but tiny clusters)
                touched |= set(got[cls][diff].tolist()) | set(asg[diff].tolist())
                got_f, want_f = oracle.bits_to_f32(out_bits[0, g, s]), oracle.bits_to_f32(cent)
                for j in range(C):
                    if j in touched or rc[j] < 8:
                        continue
                    np.testing.assert_allclose(got_f[j], want_f[j], rtol=2.0 ** -7, atol=2e-3,
                                               err_msg=f"centroid {j} of ({g},{s}) after {iters} steps")


def test_prefill_in_one_call_matches_oracle_clustering_and_build():
    """csa_prefill = clustering + table build.  The clustering half follows the oracle's seeds and
    steps (draw by draw / up to rounding-level assignments); the tables are then compared bit for bit
    with the oracle's build from the centroids the library produced (centroids are an input of the
    build), and a decode step on them matches the oracle."""
    w = small("prefill", n_q_heads=4, n_kv_heads=2, n_pre=1800, C=20, L=96, m=2, k=100, steps=1, n_sub=2)
    case = Case(w, seed=31, F=12)
    G, db, iters = w.group, 64, 2
    q = _queries(1, 4, w.n_pre, 8, 19)
    u = np.random.default_rng(5).uniform(size=(1, 2, 2, w.C)).astype(np.float32)
    cent = torch.empty(1, 2, 2, w.C, db, dtype=torch.bfloat16, device="cuda")
    q_bits = oracle.bf16_bits(q)
    # seeding alone (no Lloyd step): draw by draw
    binding.csa_prefill(case.ctx.ctx, q.cuda(), w.n_pre, 0, 1, u, cent)
    seeds = oracle.bits_to_f32(oracle.bf16_bits(cent))
    followed = {(g, s) for g in range(2) for s in range(2)
                if _compare_seeds(seeds[0, g, s], _pool(q_bits, 0, g, G, s, db), w.C, u[0, g, s]) == w.C}
    assert len(followed) >= 3
    # the whole prefill: the same seeds (the seeding is deterministic), then two Lloyd steps
    binding.csa_prefill(case.ctx.ctx, q.cuda(), w.n_pre, iters, 1, u, cent)
    torch.cuda.synchronize()
    assert binding.csa_context_len(case.ctx.ctx) == (w.n_pre, w.n_pre)
    got = oracle.bits_to_f32(oracle.bf16_bits(cent))
    for g, s in sorted(followed):
        x = _pool(q_bits, 0, g, G, s, db)
        c = oracle.kmeans_seed(x, w.C, u[0, g, s].astype(np.float64))
        for _ in range(iters):
            c, _, _, _ = oracle.kmeans_step(x, c)
        want = oracle.bits_to_f32(c)
        # a point whose two best centroids tie at rounding level may sit in another cluster on the GPU:
        # that moves two centroids by one member of hundreds; all others agree to a bf16 step
        close = [np.allclose(got[0, g, s, j], want[j], rtol=2.0 ** -7, atol=1e-6) for j in range(w.C)]
        assert sum(close) >= w.C - 4, f"({g},{s}): only {sum(close)} of {w.C} centroids follow the oracle"
        assert np.abs(got[0, g, s] - want).max() < 0.05
    # the build half: the oracle builds from the library's centroids
    case.inp["centroids"] = cent
    case.cent_host = oracle.bf16_bits(cent)
    case.F = binding.csa_score_frac_bits(case.ctx.ctx)
    for g in range(2):
        case.check_tables(0, g)
    print("prefill in one call: decode err", case.check_step(0))


def test_full_clustering_improves_monotonically_and_matches_the_oracle_quality():
    B, Hq, Hkv, n_pre, C, S, iters = 1, 4, 1, 1500, 24, 2, 6
    q = _queries(B, Hq, n_pre, 20, 5)
    u = np.random.default_rng(2).uniform(size=(B, Hkv, S, C)).astype(np.float32)
    ctx = _ctx(B, Hq, Hkv, C, S)
    out = torch.empty(B, Hkv, S, C, 128 // S, dtype=torch.bfloat16, device="cuda")
    mean_cos = torch.zeros(B, Hkv, S, iters, device="cuda")
    binding.csa_cluster_queries(ctx, q.cuda(), n_pre, iters, u, None, out, mean_cos)
    binding.csa_destroy(ctx)
    mean_cos = mean_cos.cpu().numpy()
    q_bits = oracle.bf16_bits(q)
    for s in range(S):
        mc = mean_cos[0, 0, s]
        assert (np.diff(mc) >= -1e-4).all(), mc
        x = _pool(q_bits, 0, 0, 4, s, 64)
        cent = oracle.kmeans_seed(x, C, u[0, 0, s].astype(np.float64))
        for _ in range(iters):
            cent, _, _, o_mc = oracle.kmeans_step(x, cent)
        assert mc[-1] >= o_mc - 0.01, (mc[-1], o_mc)
        # the quality of the centroids the library returned, from the definition (mean over the points
        # of the best cosine; plain numpy - nothing the library produced is handed to the oracle)
        c = out[0, 0, s].float().cpu().numpy().astype(np.float64)
        xn = x.astype(np.float64) / np.linalg.norm(x.astype(np.float64), axis=1, keepdims=True)
        final = float((xn @ (c / np.linalg.norm(c, axis=1, keepdims=True)).T).max(axis=1).mean())
        assert final >= o_mc - 0.01


def test_clustered_centroids_feed_the_table_build_and_decode():
    """Prefill queries -> csa_cluster_queries -> csa_build_tables -> decode, all on the GPU, the
    centroid buffer handed on as it was written.  The centroids here are the library's own output, so
    the oracle takes no part: the test checks, from the definitions, what holds whatever the
    centroids are (Sec. 3.2 (2): the head of every list is the key with the largest sub-space inner
    product with its centroid and carries that product rounded to the grid; lists hold distinct,
    valid keys in non-increasing score order) and that the step returns k distinct prefill keys."""
    w = small("e2e", n_q_heads=4, n_kv_heads=2, n_pre=2500, C=32, L=128, m=2, k=120, steps=1, n_sub=4)
    case = Case(w, seed=77, F=12)
    q = _queries(1, 4, w.n_pre, 16, 9).cuda()
    u = np.random.default_rng(3).uniform(size=(1, 2, 4, 32)).astype(np.float32)
    cent = torch.empty(1, 2, 4, 32, 32, dtype=torch.bfloat16, device="cuda")
    binding.csa_cluster_queries(case.ctx.ctx, q, w.n_pre, 4, u, None, cent)
    case.inp["centroids"] = cent
    case.build_on_gpu()
    cent_f = cent.float().cpu().numpy().astype(np.float64)                       # [1][2][S][C][32]
    np.testing.assert_allclose(np.linalg.norm(cent_f, axis=-1), 1.0, atol=1e-2)
    K = case.inp["k_cache"].float().cpu().numpy().astype(np.float64)             # [1][2][n][128]
    for g in range(2):
        idx, score = case.export(0, g)                                           # [S*C][L]
        assert ((idx >= 0) & (idx < w.n_pre)).all()
        assert (np.diff(score, axis=1) <= 0).all()
        for s in range(4):
            ip = cent_f[0, g, s] @ K[0, g, :w.n_pre, 32 * s:32 * s + 32].T       # [C][n_pre]
            for j in range(32):
                row = s * 32 + j
                assert len(set(idx[row].tolist())) == w.L
                assert ip[j, idx[row, 0]] >= ip[j].max() - 2.0 ** -case.F
                assert abs(score[row, 0] - ip[j].max()) <= 2.0 ** -case.F
    out, sel, cnt, rows = case.decode(0)
    assert np.isfinite(out).all() and (cnt == w.k).all()
    for h in range(4):
        assert (np.diff(sel[0, h]) > 0).all() and sel[0, h, 0] >= 0 and sel[0, h, -1] < w.n_pre
        assert sorted(r // 32 for r in rows[0, h]) == [0, 0, 1, 1, 2, 2, 3, 3]   # tau = 2 rows per sub-space

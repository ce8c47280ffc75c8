"""Pins for the CPU oracle: checks against what the paper's definitions and the mathematics
fix, none of which call back into the oracle's own arithmetic.

Each test names the mistake it is meant to catch.  The paper prints no worked numeric example;
tests/golden/ holds a hand-worked one derived from Sec. 3.3's definitions.
"""
import fractions
import math
import os

import numpy as np
import pytest

from oracle import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ helpers (independent)

def to_bits(x):
    """float array whose values are exactly representable in bf16 -> uint16 bit patterns."""
    x = np.ascontiguousarray(x, np.float32)
    u = x.view(np.uint32)
    assert np.all((u & 0xFFFF) == 0), "test value not representable in bf16"
    return (u >> 16).astype(np.uint16)


def rand_bf16(rng, shape, scale=1.0):
    x = (rng.standard_normal(shape) * scale).astype(np.float32)
    u = x.view(np.uint32)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return (u >> 16).astype(np.uint16)


def f32(bits):
    return oracle.bits_to_f32(bits)


def round_to_f32(fr: fractions.Fraction) -> np.float32:
    """Correctly rounded (half to even) fp32 of an exact rational, without double rounding."""
    if fr == 0:
        return np.float32(0.0)
    guess = np.float32(float(fr))
    cands = {guess, np.nextafter(guess, np.float32(np.inf)), np.nextafter(guess, np.float32(-np.inf))}
    best = None
    for c in cands:
        err = abs(fractions.Fraction(float(c)) - fr)
        even = (int(np.float32(c).view(np.uint32)) & 1) == 0
        key = (err, 0 if even else 1)
        if best is None or key < best[0]:
            best = (key, c)
    return np.float32(best[1])


def fma_chain_exact(a_bits, b_bits):
    """acc <- round_fp32(a_t * b_t + acc) over ascending t, in exact rational arithmetic."""
    acc = np.float32(0.0)
    for x, y in zip(f32(a_bits), f32(b_bits)):
        acc = round_to_f32(fractions.Fraction(float(x)) * fractions.Fraction(float(y))
                           + fractions.Fraction(float(acc)))
    return acc


def random_tables(rng, n_rows, L, n_pre, F, qmax, fill=None):
    """Rows of distinct key indices with grid scores, sorted (score desc, idx asc)."""
    idx = np.full((n_rows, L), -1, np.int32)
    score = np.zeros((n_rows, L), np.float32)
    for r in range(n_rows):
        n = min(L, n_pre) if fill is None else fill
        ids = rng.choice(n_pre, size=n, replace=False).astype(np.int32)
        q = rng.integers(-qmax, qmax + 1, size=n)
        order = np.lexsort((ids, -q))
        idx[r, :n] = ids[order]
        score[r, :n] = (q[order] * 2.0 ** -F).astype(np.float32)
    return idx, score


def brute_select(idx, score, rows, k, F):
    """Dictionary accumulation in exact integers, then a full sort by (-sum, index)."""
    acc = {}
    for r in rows:
        for i, s in zip(idx[r], score[r]):
            if i < 0:
                continue
            q = fractions.Fraction(float(s)) * 2 ** F
            assert q.denominator == 1
            acc[int(i)] = acc.get(int(i), 0) + int(q)
    ranked = sorted(acc.items(), key=lambda kv: (-kv[1], kv[0]))
    return sorted(i for i, _ in ranked[:k]), acc


def softmax_attention_np(q_bits, K_bits, V_bits, ids):
    q, K, V = f32(q_bits).astype(np.float64), f32(K_bits).astype(np.float64), f32(V_bits).astype(np.float64)
    lg = K[ids] @ q / math.sqrt(q.shape[0])
    p = np.exp(lg - lg.max())
    return (p / p.sum()) @ V[ids]


# ------------------------------------------------------------------ dense attention (Sec. 2.1)

def test_dense_two_keys_closed_form():
    """d = 16 so sqrt(d) = 4: logits 4/4 = 1 and 0 -> weights e/(1+e), 1/(1+e).
    Catches a missing or wrong 1/sqrt(d), a transposed operand, a missing max subtraction."""
    d = 16
    q = to_bits(np.ones(d))
    K = to_bits(np.stack([np.r_[np.ones(4), np.zeros(12)], np.zeros(d)]))
    V = to_bits(np.stack([np.r_[2.0, np.zeros(15)], np.r_[0.0, -4.0, np.zeros(14)]]))
    o = oracle.dense_attention(q, K, V, 2)
    w = math.e / (1 + math.e)
    assert o[0] == pytest.approx(2 * w, rel=1e-6)
    assert o[1] == pytest.approx(-4 * (1 - w), rel=1e-6)
    assert np.all(o[2:] == 0)


def test_dense_equal_keys_is_mean_and_large_logits_do_not_overflow():
    rng = np.random.default_rng(1)
    d, n = 128, 37
    q = rand_bf16(rng, d, 30.0)                       # logits of order 1e3: exp overflows
    K = np.tile(rand_bf16(rng, d, 30.0), (n, 1))      # without the max subtraction
    V = rand_bf16(rng, (n, d))
    o = oracle.dense_attention(q, K, V, n)
    np.testing.assert_allclose(o, f32(V).astype(np.float64).mean(0), rtol=1e-6, atol=1e-6)


def test_dense_prefix_only():
    """Only rows [0, n) may contribute (catches an off-by-one in the context length)."""
    rng = np.random.default_rng(2)
    d = 128
    q, K, V = rand_bf16(rng, d), rand_bf16(rng, (50, d)), rand_bf16(rng, (50, d))
    o = oracle.dense_attention(q, K, V, 31)
    np.testing.assert_allclose(o, softmax_attention_np(q, K, V, np.arange(31)), rtol=1e-5, atol=1e-6)
    assert np.all(oracle.dense_attention(q, K, V, 1) == f32(V[0]))


# ------------------------------------------------------------------ step 1: centroid ranking

def test_centroid_scores_follow_the_fma_chain():
    """Values with heavy cancellation make the result depend on the order and on the fusing;
    the exact-rational emulation pins ascending order, start at +0, one rounding per step."""
    rng = np.random.default_rng(3)
    d, n_c = 128, 6
    q = rand_bf16(rng, d, 50.0)
    cent = rand_bf16(rng, (n_c, d), 50.0)
    # plant cancellations: consecutive dimensions with opposite huge products
    qf, cf = f32(q).copy(), f32(cent).copy()
    qf[10], qf[11] = 3.0e4, -3.0e4
    cf[:, 10] = 2.0e4
    cf[:, 11] = 2.0e4
    q, cent = to_bits(rand_round(qf)), to_bits(rand_round(cf))
    _, z = oracle.top_centroids(q, cent, 1)
    ref = np.array([fma_chain_exact(q, cent[j]) for j in range(n_c)], np.float32)
    assert np.array_equal(z.view(np.uint32), ref.view(np.uint32))
    # and the order matters on this input: the reversed chain differs somewhere
    rev = np.array([fma_chain_exact(q[::-1], cent[j][::-1]) for j in range(n_c)], np.float32)
    assert not np.array_equal(rev.view(np.uint32), ref.view(np.uint32))


def rand_round(x):
    """fp32 -> nearest bf16-representable fp32."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.view(np.float32)


def test_top_centroids_against_full_sort_with_ties():
    """Small-integer data: every inner product is exact, many ties; expected ranking from
    integer arithmetic and Python's sort.  Catches ascending/descending and tie-rule slips."""
    rng = np.random.default_rng(4)
    d, n_c = 128, 40
    qv = rng.integers(-2, 3, d).astype(np.float32)
    cv = rng.integers(-1, 2, (n_c, d)).astype(np.float32)
    cv[7] = cv[3]; cv[21] = cv[3]                       # exact ties
    z_int = (cv.astype(np.int64) @ qv.astype(np.int64))
    order = sorted(range(n_c), key=lambda j: (-z_int[j], j))
    for m in (1, 4, 17, n_c):
        rows, z = oracle.top_centroids(to_bits(qv), to_bits(cv), m)
        assert list(rows) == order[:m]
        assert np.array_equal(z, z_int.astype(np.float32))


def test_query_scale_does_not_change_the_ranking():
    """Sec. 3.3 step 1 normalises q; a positive power-of-two factor (exact in bf16) must give
    the same rows, which is why the normalisation is skipped."""
    rng = np.random.default_rng(5)
    q = rand_bf16(rng, 128)
    cent = rand_bf16(rng, (64, 128), 0.1)
    r1, _ = oracle.top_centroids(q, cent, 8)
    r2, _ = oracle.top_centroids(to_bits(f32(q) * 0.25), cent, 8)
    assert np.array_equal(r1, r2)


# ------------------------------------------------------------------ subspaces (Sec. 3.1, 3.3 (1))

def test_subspace_scores_are_partial_inner_products_of_the_matching_slices():
    """S = 4: z^(b)_j must be the fma chain over dimensions [32b, 32b+32) of q against centroid
    (b, j) - pinned with the exact-rational emulation - and the subspace partials of one vector
    add up to the full inner product (Sec. 3.1).  Catches a wrong slice offset or stride."""
    rng = np.random.default_rng(30)
    S, n_c, d = 4, 5, 128
    db = d // S
    q = rand_bf16(rng, d, 3.0)
    cent = rand_bf16(rng, (S, n_c, db), 3.0)
    _, z = oracle.top_centroids(q, cent, 1)
    z = z.reshape(S, n_c)
    for b in range(S):
        ref = np.array([fma_chain_exact(q[b * db:(b + 1) * db], cent[b, j]) for j in range(n_c)], np.float32)
        assert np.array_equal(z[b].view(np.uint32), ref.view(np.uint32))
    # decomposition: a "centroid" made of the slices of one vector c gives sum_b z^(b) = q . c
    c_full = rand_bf16(rng, d, 3.0)
    _, zc = oracle.top_centroids(q, np.ascontiguousarray(c_full.reshape(S, 1, db)), 1)
    full = float(f32(q).astype(np.float64) @ f32(c_full).astype(np.float64))
    assert float(zc.astype(np.float64).sum()) == pytest.approx(full, rel=1e-5, abs=1e-4)


def test_subspace_probes_are_the_best_tau_of_every_subspace():
    """Small-integer data (exact products, many ties): rows = for every subspace the tau best
    centroids by (score desc, j asc), as table rows b*C + j, subspace-major."""
    rng = np.random.default_rng(31)
    S, n_c, d = 8, 12, 128
    db = d // S
    qv = rng.integers(-2, 3, d).astype(np.float32)
    cv = rng.integers(-1, 2, (S, n_c, db)).astype(np.float32)
    cv[2, 5] = cv[2, 1]; cv[2, 9] = cv[2, 1]           # exact ties inside a subspace
    for tau in (1, 2, 3, n_c):
        rows, _ = oracle.top_centroids(to_bits(qv), to_bits(cv), tau)
        want = []
        for b in range(S):
            zi = cv[b].astype(np.int64) @ qv[b * db:(b + 1) * db].astype(np.int64)
            want += [b * n_c + j for j in sorted(range(n_c), key=lambda j: (-zi[j], j))[:tau]]
        assert list(rows) == want


def test_subspace_rows_score_the_matching_key_slice():
    """Keys that vanish outside subspace 2: every row of another subspace scores 0 for every key
    (its Top-L is then the L lowest indices), and row (2, j) is the sorted Top-L of
    c^(2)_j . k^(2)_i.  Catches scoring a key slice against the wrong subspace's centroid."""
    rng = np.random.default_rng(32)
    S, n_c, d, n, L, F = 4, 3, 128, 200, 16, 2
    db = d // S
    Kv = np.zeros((n, d), np.float32)
    Kv[:, 2 * db:3 * db] = rng.integers(-3, 4, (n, db))
    cv = rng.integers(-2, 3, (S, n_c, db)).astype(np.float32)
    idx, score, _ = oracle.build_tables(to_bits(Kv), n, to_bits(cv), L, F)
    for b in range(S):
        for j in range(n_c):
            r = b * n_c + j
            if b != 2:
                assert idx[r].tolist() == list(range(L)) and np.all(score[r] == 0)
            else:
                sc = Kv[:, 2 * db:3 * db].astype(np.int64) @ cv[2, j].astype(np.int64)
                order = sorted(range(n), key=lambda i: (-sc[i], i))[:L]
                assert idx[r].tolist() == order
                assert np.array_equal(score[r], sc[order].astype(np.float32))


@pytest.mark.parametrize("S", [2, 8, 16])
def test_subspace_sums_retrieve_the_true_top_k_when_centroids_equal_the_query(S):
    """Sec. 3.1 / App. C.2: q.k = sum_b q^(b).k^(b).  With one centroid per subspace equal to the
    query's own slice, every key in every row (L = N) and integer data (all products exact, on any
    grid), the accumulated score of key i IS q.k_i, so the selection must be the brute-force
    Top-k of q.K with ties to the lower index."""
    rng = np.random.default_rng(33 + S)
    d, n, k, F = 128, 150, 20, 1
    db = d // S
    qv = rng.integers(-2, 3, d).astype(np.float32)
    Kv = rng.integers(-2, 3, (n, d)).astype(np.float32)
    Kv[40] = Kv[7]; Kv[90] = Kv[7]                       # exact score ties
    cent = to_bits(np.ascontiguousarray(qv.reshape(S, 1, db)))
    K, V = to_bits(Kv), rand_bf16(rng, (n, d))
    idx, score, _ = oracle.build_tables(K, n, cent, n, F)
    rows, sel, cnt, out = oracle.decode_head(to_bits(qv), cent, idx, score, 1, k, K, V, n, n)
    assert list(rows) == list(range(S))
    full = Kv.astype(np.int64) @ qv.astype(np.int64)
    want = sorted(sorted(range(n), key=lambda i: (-full[i], i))[:k])
    assert cnt == k and sel.tolist() == want
    np.testing.assert_allclose(out, softmax_attention_np(to_bits(qv), K, V, np.array(want)), atol=1e-6)


def test_one_subspace_given_as_3d_equals_the_2d_form():
    rng = np.random.default_rng(34)
    d, n, n_c, L = 128, 120, 6, 24
    q, cent = rand_bf16(rng, d), rand_bf16(rng, (n_c, d), 0.1)
    K, V = rand_bf16(rng, (n, d)), rand_bf16(rng, (n, d))
    i2, s2, _ = oracle.build_tables(K, n, cent, L, 10)
    i3, s3, _ = oracle.build_tables(K, n, cent.reshape(1, n_c, d), L, 10)
    assert np.array_equal(i2, i3) and np.array_equal(s2, s3)
    a = oracle.decode_head(q, cent, i2, s2, 3, 30, K, V, n, n)
    b = oracle.decode_head(q, cent.reshape(1, n_c, d), i2, s2, 3, 30, K, V, n, n)
    for x, y in zip(a, b):
        assert np.array_equal(np.asarray(x), np.asarray(y))


# ------------------------------------------------------------------ offline rows (Sec. 3.2 (2))

def test_build_rows_single_centroid_is_the_sorted_top_L():
    """C = 1 on exact (small-integer) data: the row must be the library-sorted Top-L of c.k,
    ties to the lower index.  Catches key/centroid transposition, wrong sort direction."""
    rng = np.random.default_rng(6)
    d, n, L, F = 128, 300, 32, 3
    Kv = rng.integers(-3, 4, (n, d)).astype(np.float32)
    c = (rng.integers(-4, 5, (1, d)) / 8.0).astype(np.float32)      # multiples of 1/8: F = 3 is exact
    s = (Kv.astype(np.float64) @ c[0].astype(np.float64))
    order = np.lexsort((np.arange(n), -s))[:L]
    idx, score, mx = oracle.build_rows(to_bits(Kv), n, to_bits(c), [0], L, F)
    assert np.array_equal(idx[0], order)
    assert np.array_equal(score[0], s[order].astype(np.float32))
    assert mx == np.abs(s * 8).max()


def test_build_rows_grid_rounding_half_to_even():
    """One-dimensional products landing exactly on half grid steps."""
    d, F = 128, 1                                  # grid 0.5
    Kv = np.zeros((6, d), np.float32)
    Kv[:, 0] = [0.25, 0.75, 1.25, -0.25, -0.75, 0.5]   # x 2 -> .5 1.5 2.5 -.5 -1.5 1
    c = np.zeros((1, d), np.float32); c[0, 0] = 1.0
    idx, score, _ = oracle.build_rows(to_bits(Kv), 6, to_bits(c), [0], 6, F)
    got = dict(zip(idx[0].tolist(), score[0].tolist()))
    assert got == {0: 0.0, 1: 1.0, 2: 1.0, 3: -0.0, 4: -1.0, 5: 0.5}
    # ranking: 1.0 (keys 1, 2), 0.5 (5), 0 (0, 3), -1 (4)
    assert idx[0].tolist() == [1, 2, 5, 0, 3, 4]


def test_build_rows_invariants_on_the_synthetic_mixture():
    """Sec. 3.1 (iii): L distinct indices, sorted by score, nothing outside the row beats the
    row's minimum; scores sit on the grid; padding when n_pre < L."""
    rng = np.random.default_rng(7)
    d, n, n_c, L, F = 128, 700, 5, 64, 14
    K = rand_bf16(rng, (n, d))
    cent = rand_bf16(rng, (n_c, d), 1 / math.sqrt(d))
    idx, score, mx = oracle.build_tables(K, n, cent, L, F)
    s64 = f32(K).astype(np.float64) @ f32(cent).astype(np.float64).T
    for j in range(n_c):
        assert len(set(idx[j].tolist())) == L and idx[j].min() >= 0 and idx[j].max() < n
        assert np.all(np.diff(score[j]) <= 0)
        ties = np.diff(score[j]) == 0
        assert np.all(np.diff(idx[j])[ties] > 0)
        assert np.all(score[j] * 2.0 ** F == np.rint(score[j] * 2.0 ** F))
        np.testing.assert_allclose(score[j], s64[idx[j], j], atol=2.0 ** -F + 1e-4)
        outside = np.setdiff1d(np.arange(n), idx[j])
        assert s64[outside, j].max() <= score[j, -1] + 2.0 ** -F + 1e-4
    assert mx == pytest.approx(np.abs(np.rint(s64 * 2 ** F)).max(), rel=1e-3)
    idx2, score2, _ = oracle.build_rows(K, 10, cent, [2], 16, F)
    assert sorted(idx2[0, :10].tolist()) == list(range(10))
    assert np.all(idx2[0, 10:] == -1) and np.all(score2[0, 10:] == 0)


def test_build_rows_subset_equals_full():
    rng = np.random.default_rng(8)
    K, cent = rand_bf16(rng, (200, 128)), rand_bf16(rng, (9, 128), 0.1)
    full_i, full_s, _ = oracle.build_tables(K, 200, cent, 16, 12)
    sub_i, sub_s, _ = oracle.build_rows(K, 200, cent, [5, 1], 16, 12)
    assert np.array_equal(sub_i, full_i[[5, 1]]) and np.array_equal(sub_s, full_s[[5, 1]])


# ------------------------------------------------------------------ steps 2-4: select_keys

@pytest.mark.parametrize("seed", range(6))
def test_select_brute_force_tiny(seed):
    """Dictionary accumulation + full sort on tiny inputs with many ties (qmax small).
    Catches: dropped rows, wrong tie rule, output order, padding, count."""
    rng = np.random.default_rng(100 + seed)
    n_pre, n_c, L, m, F = 64, 8, 16, 4, 4
    idx, score = random_tables(rng, n_c, L, n_pre, F, qmax=3, fill=int(rng.integers(5, L + 1)))
    rows = rng.choice(n_c, m, replace=False).astype(np.int32)
    for k in (1, 7, 20, 64):
        sel, cnt, nU, acc = oracle.select_keys(idx, score, rows, n_pre, k)
        want, acc_ref = brute_select(idx, score, rows, k, F)
        assert nU == len(acc_ref) <= m * L                   # |U| <= mL (App. C.2)
        assert cnt == min(k, nU) == len(want)
        assert sel[:cnt].tolist() == want
        assert np.all(sel[cnt:] == -1)
        for i in range(n_pre):
            if i in acc_ref:
                assert acc[i] == acc_ref[i] * 2.0 ** -F
            else:
                assert np.isnan(acc[i])                       # absent keys are not in U


def test_select_order_invariance_and_exact_sums():
    """Permuting entries inside rows and the order of the probed rows leaves the selection
    bit-identical, and the fp32 sums equal the exact integer sums scaled back (grid rule:
    m * max|q| < 2^24)."""
    rng = np.random.default_rng(9)
    n_pre, n_c, L, m, F = 5000, 12, 512, 8, 14
    qmax = (1 << 24) // m - 1
    idx, score = random_tables(rng, n_c, L, n_pre, F, qmax)
    rows = rng.choice(n_c, m, replace=False).astype(np.int32)
    sel0, cnt0, nU0, acc0 = oracle.select_keys(idx, score, rows, n_pre, 300)
    _, acc_ref = brute_select(idx, score, rows, 300, F)
    seen = ~np.isnan(acc0)
    assert seen.sum() == len(acc_ref)
    for i, v in acc_ref.items():
        assert float(acc0[i]) == v * 2.0 ** -F
    for trial in range(4):
        idx2, score2 = idx.copy(), score.copy()
        for r in range(n_c):
            p = rng.permutation(L)
            idx2[r], score2[r] = idx[r, p], score[r, p]
        rows2 = rng.permutation(rows).astype(np.int32)
        sel, cnt, nU, acc = oracle.select_keys(idx2, score2, rows2, n_pre, 300)
        assert cnt == cnt0 and nU == nU0 and np.array_equal(sel, sel0)
        assert np.array_equal(acc.view(np.uint32), acc0.view(np.uint32))


def test_select_single_row_is_the_row_prefix():
    """m = 1: score(i) is that row's score, so the selection is the first k entries of the
    (score desc, idx asc) row, re-sorted by index."""
    rng = np.random.default_rng(10)
    idx, score = random_tables(rng, 3, 128, 1000, 10, qmax=20)        # heavy ties
    for k in (1, 50, 128, 200):
        sel, cnt, nU, _ = oracle.select_keys(idx, score, np.array([1], np.int32), 1000, k)
        assert nU == 128 and cnt == min(k, 128)
        assert sel[:cnt].tolist() == sorted(idx[1, :cnt].tolist())


def test_select_budget_at_least_union_returns_union():
    rng = np.random.default_rng(11)
    idx, score = random_tables(rng, 6, 40, 300, 8, qmax=1000, fill=33)
    rows = np.array([0, 2, 5], np.int32)
    sel, cnt, nU, _ = oracle.select_keys(idx, score, rows, 300, 250)
    U = sorted(set(idx[rows].ravel().tolist()) - {-1})
    assert nU == len(U) == cnt and sel[:cnt].tolist() == U and np.all(sel[cnt:] == -1)


def test_select_negative_sums_and_zero_sum_members():
    """A key whose scores cancel to 0 is still in U and outranks negative sums; keys never
    listed are not selectable even when every listed sum is negative."""
    idx = np.array([[0, 1, 2, -1], [1, 3, 0, -1]], np.int32)
    score = np.array([[1.0, 0.5, -2.0, 0], [-0.5, -1.0, -3.0, 0]], np.float32)
    # sums: key0 = -2, key1 = 0, key2 = -2, key3 = -1 ; keys 4.. never listed
    sel, cnt, nU, acc = oracle.select_keys(idx, score, np.array([0, 1], np.int32), 8, 3)
    assert nU == 4 and cnt == 3 and sel.tolist() == [0, 1, 3]       # tie -2: key 0 beats key 2
    sel, cnt, _, _ = oracle.select_keys(idx, score, np.array([0, 1], np.int32), 8, 6)
    assert cnt == 4 and sel.tolist() == [0, 1, 2, 3, -1, -1]


# ------------------------------------------------------------------ whole step

def _dense_tables(n_pre, n_c, rng, F=10):
    """Every key in every row (L = n_pre), arbitrary grid scores."""
    idx = np.empty((n_c, n_pre), np.int32)
    score = np.empty((n_c, n_pre), np.float32)
    for j in range(n_c):
        q = rng.integers(-500, 500, n_pre)
        order = np.lexsort((np.arange(n_pre), -q))
        idx[j], score[j] = order, q[order] * 2.0 ** -F
    return idx, score


@pytest.mark.parametrize("m", [1, 3])
def test_decode_with_nothing_pruned_is_dense_attention(m):
    """L = N_pre and k = N_pre: sel = all prefill keys and the output equals Sec. 2.1's dense
    attention over [0, n) (appended keys included)."""
    rng = np.random.default_rng(12)
    d, n_pre, n, n_c = 128, 257, 263, 5
    q, cent = rand_bf16(rng, d), rand_bf16(rng, (n_c, d), 0.1)
    K, V = rand_bf16(rng, (n, d)), rand_bf16(rng, (n, d))
    idx, score = _dense_tables(n_pre, n_c, rng)
    rows, sel, cnt, out = oracle.decode_head(q, cent, idx, score, m, n_pre, K, V, n_pre, n)
    assert cnt == n_pre and sel.tolist() == list(range(n_pre))
    dense = oracle.dense_attention(q, K, V, n)
    np.testing.assert_allclose(out, dense, rtol=0, atol=1e-6)
    np.testing.assert_allclose(out, softmax_attention_np(q, K, V, np.arange(n)), atol=1e-6)


def test_decode_zero_budget_attends_appended_keys_only():
    rng = np.random.default_rng(13)
    d, n_pre, n = 128, 100, 109
    q, cent = rand_bf16(rng, d), rand_bf16(rng, (4, d))
    K, V = rand_bf16(rng, (n, d)), rand_bf16(rng, (n, d))
    idx, score = random_tables(rng, 4, 16, n_pre, 8, 100)
    _, sel, cnt, out = oracle.decode_head(q, cent, idx, score, 2, 0, K, V, n_pre, n)
    assert cnt == 0
    want = oracle.dense_attention(q, np.ascontiguousarray(K[n_pre:]), np.ascontiguousarray(V[n_pre:]), n - n_pre)
    np.testing.assert_allclose(out, want, atol=1e-6)
    # nothing selected and nothing appended: defined as a zero output
    _, _, cnt, out = oracle.decode_head(q, cent, idx, score, 2, 0, K, V, n_pre, n_pre)
    assert cnt == 0 and np.all(out == 0)


def test_decode_output_is_a_convex_combination_of_attended_values():
    """Softmax weights are non-negative and sum to 1 (Sec. 2.1): each output coordinate lies
    between the min and max of the attended value rows, and equals the numpy softmax over
    exactly sel + appended."""
    rng = np.random.default_rng(14)
    d, n_pre, n, n_c, L, m, k = 128, 900, 905, 10, 64, 4, 40
    q, cent = rand_bf16(rng, d), rand_bf16(rng, (n_c, d), 0.1)
    K, V = rand_bf16(rng, (n, d)), rand_bf16(rng, (n, d))
    idx, score = random_tables(rng, n_c, L, n_pre, 12, 5000)
    rows, sel, cnt, out = oracle.decode_head(q, cent, idx, score, m, k, K, V, n_pre, n)
    want_rows, _ = oracle.top_centroids(q, cent, m)
    assert np.array_equal(rows, want_rows)
    want_sel, _ = brute_select(idx, score, rows, k, 12)
    assert sel[:cnt].tolist() == want_sel
    ids = np.r_[sel[:cnt], np.arange(n_pre, n)]
    Vf = f32(V)[ids]
    assert np.all(out <= Vf.max(0) + 1e-6) and np.all(out >= Vf.min(0) - 1e-6)
    np.testing.assert_allclose(out, softmax_attention_np(q, K, V, ids), atol=1e-6)


def test_reuse_step_attends_the_given_set_plus_appended_keys():
    """A step inside a search period (complexity appendix: the index set is reused for P-1 steps):
    with every prefill key listed it is dense attention; the order of the list is irrelevant; one
    listed key and nothing appended returns that key's value row; an index at or beyond n_pre that
    is not appended yet never enters (catches attending [0, n) instead of sel + [n_pre, n))."""
    rng = np.random.default_rng(21)
    d, n_pre, n = 128, 300, 307
    q, K, V = rand_bf16(rng, d), rand_bf16(rng, (n + 5, d)), rand_bf16(rng, (n + 5, d))
    full = oracle.attend_selected(q, K, V, np.arange(n_pre), n_pre, n)
    np.testing.assert_allclose(full, oracle.dense_attention(q, K, V, n), atol=1e-6)
    sel = rng.choice(n_pre, 40, replace=False).astype(np.int32)
    a = oracle.attend_selected(q, K, V, np.sort(sel), n_pre, n)
    b = oracle.attend_selected(q, K, V, sel, n_pre, n)
    np.testing.assert_allclose(a, b, atol=1e-6)
    np.testing.assert_allclose(a, softmax_attention_np(q, K, V, np.r_[sel, np.arange(n_pre, n)]), atol=1e-6)
    one = oracle.attend_selected(q, K, V, np.array([17], np.int32), n_pre, n_pre)
    assert np.array_equal(one, f32(V[17]))
    none = oracle.attend_selected(q, K, V, np.zeros(0, np.int32), n_pre, n_pre)
    assert np.all(none == 0)


# ------------------------------------------------------------------ streaming updates (Sec. 3.3 (5))

@pytest.mark.parametrize("S,L", [(1, 40), (4, 40), (2, 400)])
def test_try_insert_stream_equals_a_build_over_all_keys(S, L):
    """Top-L of a growing set is order-independent: tables built over the first 300 keys and then
    updated with keys 300..339 one at a time must equal tables built over all 340 keys at once
    (L = 400: lists with free slots just grow).  Small-integer keys give many equal scores, so the
    rule "an equal score does not evict" is exercised.  Catches a wrong eviction test, a wrong
    insert position, scoring the wrong key slice."""
    rng = np.random.default_rng(40 + S)
    d, n0, n1, n_c, F = 128, 300, 340, 5, 2
    Kv = rng.integers(-2, 3, (n1, d)).astype(np.float32)
    cv = rng.integers(-1, 2, (S, n_c, d // S)).astype(np.float32)
    K, cent = to_bits(Kv), to_bits(cv)
    idx, score, _ = oracle.build_tables(np.ascontiguousarray(K[:n0]), n0, cent, L, F)
    for i in range(n0, n1):
        oracle.try_insert(idx, score, cent, K[i], i, F)
    want_idx, want_score, _ = oracle.build_tables(K, n1, cent, L, F)
    assert np.array_equal(idx, want_idx) and np.array_equal(score, want_score)


def test_try_insert_on_real_valued_scores_keeps_rows_sorted_and_bounded():
    rng = np.random.default_rng(44)
    d, n0, n1, n_c, L, F = 128, 500, 560, 7, 64, 10
    K, cent = rand_bf16(rng, (n1, d)), rand_bf16(rng, (n_c, d), 0.1)
    idx, score, _ = oracle.build_tables(np.ascontiguousarray(K[:n0]), n0, cent, L, F)
    for i in range(n0, n1):
        oracle.try_insert(idx, score, cent, K[i], i, F)
    want_idx, want_score, _ = oracle.build_tables(K, n1, cent, L, F)
    assert np.array_equal(idx, want_idx) and np.array_equal(score, want_score)
    assert (np.diff(score, axis=1) <= 0).all() and all(len(set(r.tolist())) == L for r in idx)


def test_decode_with_a_recent_window_excludes_it_from_the_candidates():
    """Streaming mode: keys at or after the window start are attended unconditionally and must
    not be selected as well (they would be counted twice).  Tables contain window keys."""
    rng = np.random.default_rng(45)
    d, n, n_c, L, m, k, F, win = 128, 400, 6, 80, 3, 50, 12, 32
    q, cent = rand_bf16(rng, d), rand_bf16(rng, (n_c, d), 0.1)
    K, V = rand_bf16(rng, (n, d)), rand_bf16(rng, (n, d))
    idx, score = random_tables(rng, n_c, L, n, F, 5000)     # indices anywhere in [0, n)
    ws = n - win
    rows, sel, cnt, out = oracle.decode_head(q, cent, idx, score, m, k, K, V, ws, n)
    assert (idx[rows] >= ws).any()                            # the case is exercised
    masked_idx = np.where(idx >= ws, -1, idx)
    want_sel, _ = brute_select(masked_idx, score, rows, k, F)
    assert sel[:cnt].tolist() == want_sel and all(i < ws for i in want_sel)
    ids = np.r_[sel[:cnt], np.arange(ws, n)]
    assert len(set(ids.tolist())) == len(ids)
    np.testing.assert_allclose(out, softmax_attention_np(q, K, V, ids), atol=1e-6)


def test_single_cluster_recall_is_one():
    """Query-centric argument of Sec. 2.4: if every prefill query is a positive multiple of one
    direction u and the decode query is too, one centroid (= u) with L >= k retrieves exactly
    the true top-k of q.K.  Data are small integers so all scores are exact and tie-free
    where it matters."""
    rng = np.random.default_rng(15)
    d, n, k, F = 128, 500, 25, 0
    u = np.zeros(d, np.float32); u[5] = 1.0                      # unit direction, exact in bf16
    Kv = rng.integers(-3, 4, (n, d)).astype(np.float32)
    Kv[:, 5] = rng.permutation(n).astype(np.float32) - 250       # distinct integer scores (bf16-exact: |x| <= 256)
    cent, _ = oracle.kmeans(np.outer(rng.uniform(0.5, 3, 64), u), 1, 3, np.array([0.3]))
    cent_b = oracle.round_bf16(cent)
    assert np.array_equal(f32(cent_b)[0], u)
    idx, score, _ = oracle.build_tables(to_bits(Kv), n, cent_b, 64, F)
    q = to_bits(2.0 * u)
    V = rand_bf16(rng, (n, d))
    _, sel, cnt, _ = oracle.decode_head(q, cent_b, idx, score, 1, k, to_bits(Kv), V, n, n)
    truth = np.argsort(-(Kv @ (2.0 * u)), kind="stable")[:k]
    assert cnt == k and sel.tolist() == sorted(truth.tolist())


def test_decode_items_matches_per_head_calls():
    rng = np.random.default_rng(16)
    d, n_pre, n, n_c, L, m, k = 128, 400, 403, 6, 32, 3, 20
    items, singles = [], []
    for t in range(5):
        it = dict(q=rand_bf16(rng, d), cent=rand_bf16(rng, (n_c, d), 0.1),
                  K=rand_bf16(rng, (n, d)), V=rand_bf16(rng, (n, d)))
        it["tbl_idx"], it["tbl_score"] = random_tables(rng, n_c, L, n_pre, 12, 5000)
        items.append(it)
        singles.append(oracle.decode_head(it["q"], it["cent"], it["tbl_idx"], it["tbl_score"],
                                          m, k, it["K"], it["V"], n_pre, n))
    rows, sel, cnt, out, used = oracle.decode_items(items, m, k, n_pre, n, n_threads=2)
    assert used == 2
    for t, (r, s, c, o) in enumerate(singles):
        assert np.array_equal(rows[t], r) and np.array_equal(sel[t], s) and cnt[t] == c
        assert np.array_equal(out[t], o)


# ------------------------------------------------------------------ clustering (Sec. 3.2 (1))

def test_kmeans_objective_monotone_unit_norm_and_recovers_separated_clusters():
    rng = np.random.default_rng(17)
    d, n_c = 16, 4
    dirs = np.linalg.qr(rng.standard_normal((d, d)))[0][:n_c]           # orthonormal directions
    lab = rng.integers(0, n_c, 600)
    x = (dirs[lab] + 0.05 * rng.standard_normal((600, d))) * rng.uniform(0.5, 4.0, (600, 1))
    cent, obj = oracle.kmeans(x, n_c, 10, rng.uniform(size=n_c))
    assert np.all(np.diff(obj) <= 1e-9)                                  # Lloyd never increases it
    np.testing.assert_allclose(np.linalg.norm(cent, axis=1), 1.0, atol=1e-6)
    cos = cent @ dirs.T                                                  # each direction recovered once
    assert sorted(cos.argmax(1).tolist()) == list(range(n_c)) and np.all(cos.max(1) > 0.99)
    # scale invariance: clustering sees only directions
    cent2, _ = oracle.kmeans(x * 7.0, n_c, 10, rng.uniform(size=n_c))
    assert sorted((cent2 @ dirs.T).argmax(1).tolist()) == list(range(n_c))


def test_kmeans_in_bf16_steps_seeds_are_data_points_and_a_step_is_the_mean_direction():
    """The two-part form the GPU path is checked against.  Seeds: each is a normalised data point
    (rounded to bf16); with two tight, far-apart groups and the first seed in one of them, the D^2
    draw must land in the other for any u that is not astronomically small.  Step: on four
    well-separated directions the assignment is the obvious one, the new centroid of a cluster is
    the bf16-rounded direction of the sum of its normalised members, an empty cluster keeps its
    centroid, and a second step does not lower the mean cosine."""
    rng = np.random.default_rng(50)
    d = 32
    a, b = np.eye(d, dtype=np.float32)[0], np.eye(d, dtype=np.float32)[5]
    x = np.r_[[a * s for s in rng.uniform(1, 3, 20)], [b * s for s in rng.uniform(1, 3, 20)]].astype(np.float32)
    x += 1e-3 * rng.standard_normal(x.shape).astype(np.float32)
    for u1 in (1e-4, 0.3, 0.999):
        seeds = f32(oracle.kmeans_seed(x, 2, np.array([0.1, u1])))       # first seed: a point of group a
        assert abs(seeds[0, 0]) > 0.99 and abs(seeds[1, 5]) > 0.99
    xn = x / np.linalg.norm(x, axis=1, keepdims=True)
    seeds = oracle.kmeans_seed(x, 2, np.array([0.6, 0.5]))                # first seed: a point of group b
    assert any(np.array_equal(f32(seeds[0]), rand_round(r)) for r in xn[20:])
    # one step on 4 directions + an unused fifth centroid
    dirs = np.eye(d, dtype=np.float32)[[1, 7, 12, 30]]
    pts = np.concatenate([dirs[c] * rng.uniform(0.5, 2, (25, 1)) + 0.05 * rng.standard_normal((25, d))
                          for c in range(4)]).astype(np.float32)
    cent0 = to_bits(np.r_[dirs, -np.ones((1, d), np.float32) * 0.125])
    cent1, asg, gap, mc = oracle.kmeans_step(pts, cent0)
    assert asg.tolist() == sum([[c] * 25 for c in range(4)], [])
    pn = pts.astype(np.float64) / np.linalg.norm(pts.astype(np.float64), axis=1, keepdims=True)
    for c in range(4):
        m = pn[25 * c:25 * c + 25].sum(0)
        assert np.array_equal(f32(cent1[c]), rand_round((m / np.linalg.norm(m)).astype(np.float32)))
    assert np.array_equal(cent1[4], cent0[4]) and (gap > 0).all()
    assert mc == pytest.approx(float(np.mean([pn[i] @ f32(cent0[asg[i]]) for i in range(100)])), rel=1e-9)
    _, _, _, mc2 = oracle.kmeans_step(pts, cent1)
    assert mc2 >= mc - 1e-9


def test_kmeans_single_centroid_is_the_normalised_mean_direction():
    rng = np.random.default_rng(18)
    x = rng.standard_normal((200, 8)) + 3.0
    cent, _ = oracle.kmeans(x, 1, 2, np.array([0.5]))
    xn = x / np.linalg.norm(x, axis=1, keepdims=True)
    want = xn.mean(0) / np.linalg.norm(xn.mean(0))
    np.testing.assert_allclose(cent[0], want, atol=1e-6)


def test_round_bf16_is_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -9, -(1.0 + 2 ** -8 + 2 ** -20)], np.float32)
    got = f32(oracle.round_bf16(x))
    assert got.tolist() == [1.0, 1.0, 1.0 + 2 ** -6, 1.0, -(1.0 + 2 ** -7)]


# ------------------------------------------------------------------ hand-worked example

def test_hand_worked_example():
    """tests/golden/decode_hand_example.txt: a 6-key, 3-centroid step worked by hand from
    Sec. 3.3 steps 1-4 and Sec. 2.1 (values in the file, with the derivation)."""
    ex = {}
    with open(os.path.join(GOLDEN, "decode_hand_example.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if "=" in line:
                key, val = line.split("=", 1)
                ex[key.strip()] = [float(v) for v in val.split()]
    d = 16
    def vec(pairs):
        v = np.zeros(d, np.float32)
        for t, x in zip(pairs[0::2], pairs[1::2]):
            v[int(t)] = x
        return v
    q = to_bits(vec(ex["q"]))
    cent = to_bits(np.stack([vec(ex[f"c{j}"]) for j in range(3)]))
    K = to_bits(np.stack([vec(ex[f"k{i}"]) for i in range(6)]))
    V = to_bits(np.stack([vec(ex[f"v{i}"]) for i in range(6)]))
    idx, score, _ = oracle.build_tables(np.ascontiguousarray(K[:5]), 5, cent, 3, 1)
    assert idx.ravel().tolist() == [int(v) for v in ex["table_idx"]]
    assert score.ravel().tolist() == ex["table_score"]
    rows, sel, cnt, out = oracle.decode_head(q, cent, idx, score, 2, int(ex["k"][0]), K, V, 5, 6)
    assert rows.tolist() == [int(v) for v in ex["rows"]]
    assert sel.tolist() == [int(v) for v in ex["sel"]]
    w = np.array(ex["weights_num"]) ; w = np.exp(w) / np.exp(w).sum()
    want0 = sum(wi * vi for wi, vi in zip(w, ex["attended_v0"]))
    assert out[0] == pytest.approx(want0, rel=1e-6)


def test_kmeans_draw_matches_the_hand_worked_example():
    """tests/golden/kmeans_draw_example.txt: six points, three uniforms, the picks and margins worked
    out by hand - pins the draw to the index (first point whose running sum EXCEEDS u * total)."""
    lines = [l for l in open(os.path.join(os.path.dirname(__file__), "golden", "kmeans_draw_example.txt"))
             if l.strip() and not l.startswith("#")]
    pts = np.array([[float(v) for v in l.split()] for l in lines[:6]], np.float32)
    u = np.array([float(v) for v in lines[6].split()])
    want_picks = [int(v) for v in lines[7].split()]
    want_margin = [float(v) for v in lines[8].split()]
    cent, picks, margin = oracle.kmeans_seed(pts, 3, u, with_draws=True)
    assert picks.tolist() == want_picks
    np.testing.assert_allclose(margin[1:], want_margin, atol=1e-7)
    f32 = oracle.bits_to_f32
    np.testing.assert_array_equal(f32(cent), pts[want_picks])            # exact in bf16
    # a target that lands exactly on a running sum does not take that point ("exceeds"): after seed 0
    # the running sums are 0 2 6 ...; u_1 = 2 / 8.8 puts the target on point 1's sum (up to rounding of
    # the product, so test both sides of it)
    for u1, want in ((0.22, 1), (0.2280, 2)):      # 0.22 * 8.8 = 1.936 < 2 -> point 1; 2.0064 > 2 -> point 2
        assert oracle.kmeans_seed(pts, 2, np.array([0.0, u1]), with_draws=True)[1].tolist() == [0, want]


def test_kmeans_minibatch_step_is_a_running_mean_direction():
    """The mini-batch step: with one batch and zeroed sums it is the full step; the running sums are
    the sums of every normalised point assigned so far (checked from the definition in numpy); a
    centre that has never had a member keeps its centroid; feeding the same batch twice leaves the
    centroids where the first pass put them when the assignments do not change."""
    rng = np.random.default_rng(11)
    d, n_c = 8, 5
    dirs = rng.standard_normal((4, d))
    x = (dirs[rng.integers(0, 4, 400)] + 0.2 * rng.standard_normal((400, d))).astype(np.float32)
    cent0 = oracle.round_bf16((dirs / np.linalg.norm(dirs, axis=1, keepdims=True)).astype(np.float32))
    far = -np.sum(dirs, axis=0)
    cent0 = np.concatenate([cent0, oracle.round_bf16((far / np.linalg.norm(far)).astype(np.float32)[None])])
    full, asg_f, _, mc_f = oracle.kmeans_step(x, cent0)
    rs, rc = np.zeros((n_c, d)), np.zeros(n_c, np.int64)
    one, asg_1, _, mc_1 = oracle.kmeans_minibatch_step(x, cent0, rs, rc)
    assert np.array_equal(full, one) and np.array_equal(asg_f, asg_1) and mc_f == mc_1
    assert rc.sum() == 400 and rc[4] == 0 and np.array_equal(one[4], cent0[4])   # the far centre stays put
    xn = x.astype(np.float64) / np.linalg.norm(x.astype(np.float64), axis=1, keepdims=True)
    for j in range(4):
        np.testing.assert_allclose(rs[j], xn[asg_1 == j].sum(axis=0), rtol=1e-12)
    # two batches: the second step's centroid is the direction of ALL members so far, not of the batch
    rs, rc = np.zeros((n_c, d)), np.zeros(n_c, np.int64)
    a, asg_a, _, _ = oracle.kmeans_minibatch_step(x[0::2], cent0, rs, rc)
    b, asg_b, _, _ = oracle.kmeans_minibatch_step(x[1::2], a, rs, rc)
    f32 = oracle.bits_to_f32
    for j in range(4):
        tot = xn[0::2][asg_a == j].sum(axis=0) + xn[1::2][asg_b == j].sum(axis=0)
        np.testing.assert_allclose(rs[j], tot, rtol=1e-12)
        np.testing.assert_allclose(f32(b[j]), tot / np.linalg.norm(tot), atol=2.0 ** -8)
    # the same batch again: sums double, directions stay (up to the bf16 rounding already applied)
    rs, rc = np.zeros((n_c, d)), np.zeros(n_c, np.int64)
    c1, asg1, _, _ = oracle.kmeans_minibatch_step(x, cent0, rs, rc)
    c2, asg2, _, _ = oracle.kmeans_minibatch_step(x, c1, rs, rc)
    if np.array_equal(asg1, asg2):
        assert np.array_equal(c1, c2)

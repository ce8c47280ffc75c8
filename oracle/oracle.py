"""ctypes loader for the CPU oracle (oracle/csa_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  The HIP library and its Python binding never import this module.

bf16 tensors cross this boundary as numpy uint16 arrays holding the raw bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "csa_oracle.c")
_LIB = os.path.join(_HERE, "libcsa_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no contraction: the only fused ops are explicit fmaf)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call([
            "gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
            "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_build_rows.restype = C.c_double
        _lib.oracle_select_keys.restype = C.c_int64
        _lib.oracle_decode_items.restype = C.c_int
        _lib.oracle_try_insert.restype = C.c_double
        _lib.oracle_kmeans_step.restype = C.c_double
        _lib.oracle_kmeans_minibatch_step.restype = C.c_double
    return _lib


def _p(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"], "oracle arrays must be C-contiguous"
    return a.ctypes.data_as(C.c_void_p)


def bf16_bits(t) -> np.ndarray:
    """torch bf16 tensor (any device) -> numpy uint16 bit patterns (host, contiguous)."""
    import torch
    assert t.dtype == torch.bfloat16
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


def bits_to_f32(a: np.ndarray) -> np.ndarray:
    return (a.astype(np.uint32) << 16).view(np.float32)


def dense_attention(q, K, V, n):
    d = q.shape[-1]
    out = np.empty(d, np.float32)
    lib().oracle_dense_attention(_p(q), _p(K), _p(V), C.c_int64(n), C.c_int(d), _p(out))
    return out


def kmeans(x, n_centroids, iters, u_seed):
    x = np.ascontiguousarray(x, np.float32)
    u_seed = np.ascontiguousarray(u_seed, np.float64)
    assert u_seed.shape[0] >= n_centroids
    n, d = x.shape
    cent = np.empty((n_centroids, d), np.float32)
    obj = np.empty(iters + 1, np.float64)
    lib().oracle_kmeans(_p(x), C.c_int64(n), C.c_int(d), C.c_int(n_centroids), C.c_int(iters),
                        _p(u_seed), _p(cent), _p(obj))
    return cent, obj


def kmeans_seed(x, n_centroids, u_seed, with_draws=False):
    """k-means++ seeds (bf16 bit patterns [C][d]) of the rows of x [n][d] fp32.  with_draws: also the
    picked point of every seed and every draw's margin (see oracle_kmeans_seed)."""
    x = np.ascontiguousarray(x, np.float32)
    u_seed = np.ascontiguousarray(u_seed, np.float64)
    assert u_seed.shape[0] >= n_centroids
    n, d = x.shape
    cent = np.empty((n_centroids, d), np.uint16)
    picks = np.empty(n_centroids, np.int64)
    margin = np.empty(n_centroids, np.float64)
    lib().oracle_kmeans_seed(_p(x), C.c_int64(n), C.c_int(d), C.c_int(n_centroids), _p(u_seed), _p(cent),
                             _p(picks), _p(margin))
    return (cent, picks, margin) if with_draws else cent


def kmeans_minibatch_step(x, cent, run_sum, run_cnt):
    """One mini-batch step on the batch x [n][d] from bf16 centroids; run_sum [C][d] fp64 and run_cnt [C]
    int64 are updated in place.  Returns (new bf16 centroids, assignment [n], gap [n], mean best cosine)."""
    x = np.ascontiguousarray(x, np.float32)
    n, d = x.shape
    n_c = cent.shape[0]
    assert run_sum.dtype == np.float64 and run_sum.shape == (n_c, d) and run_sum.flags["C_CONTIGUOUS"]
    assert run_cnt.dtype == np.int64 and run_cnt.shape == (n_c,)
    out = np.empty((n_c, d), np.uint16)
    asg = np.empty(n, np.int32)
    gap = np.empty(n, np.float64)
    mc = lib().oracle_kmeans_minibatch_step(_p(x), C.c_int64(n), C.c_int(d), C.c_int(n_c), _p(cent), _p(out),
                                            _p(asg), _p(gap), _p(run_sum), _p(run_cnt))
    return out, asg, gap, mc


def kmeans_step(x, cent):
    """One Lloyd step from bf16 centroids.  Returns (new bf16 centroids, assignment [n], top-2 cosine
    gap [n], mean best cosine)."""
    x = np.ascontiguousarray(x, np.float32)
    n, d = x.shape
    n_c = cent.shape[0]
    out = np.empty((n_c, d), np.uint16)
    asg = np.empty(n, np.int32)
    gap = np.empty(n, np.float64)
    mc = lib().oracle_kmeans_step(_p(x), C.c_int64(n), C.c_int(d), C.c_int(n_c), _p(cent), _p(out), _p(asg),
                                  _p(gap))
    return out, asg, gap, mc


def round_bf16(x):
    x = np.ascontiguousarray(x, np.float32)
    out = np.empty(x.shape, np.uint16)
    lib().oracle_round_bf16(_p(x), C.c_int64(x.size), _p(out))
    return out


def _geometry(cent):
    """cent: [C][d] (one subspace) or [S][C][d/S].  Returns (cent as given, S, C, d)."""
    if cent.ndim == 2:
        return 1, cent.shape[0], cent.shape[1]
    return cent.shape[0], cent.shape[1], cent.shape[0] * cent.shape[2]


def build_rows(K, n_pre, cent, row_ids, L, F):
    """Rows `row_ids` (row = subspace * C + centroid) of one KV head's table; cent [C][d] or
    [S][C][d/S].  Returns (idx [r][L] i32, score [r][L] f32, max|q|)."""
    S, n_c, d = _geometry(cent)
    assert K.shape[-1] == d
    row_ids = np.ascontiguousarray(row_ids, np.int32)
    idx = np.empty((len(row_ids), L), np.int32)
    score = np.empty((len(row_ids), L), np.float32)
    mx = lib().oracle_build_rows(_p(K), C.c_int64(n_pre), C.c_int(d), C.c_int(S), C.c_int(n_c), _p(cent),
                                 _p(row_ids), C.c_int(len(row_ids)), C.c_int(L), C.c_int(F), _p(idx),
                                 _p(score))
    return idx, score, mx


def build_tables(K, n_pre, cent, L, F):
    S, n_c, _ = _geometry(cent)
    return build_rows(K, n_pre, cent, np.arange(S * n_c, dtype=np.int32), L, F)


def top_centroids(q, cent, tau):
    """The tau best centroids of every subspace as table rows [S*tau], and z [S*C]."""
    S, n_c, d = _geometry(cent)
    rows = np.empty(S * tau, np.int32)
    z = np.empty(S * n_c, np.float32)
    lib().oracle_top_centroids(_p(q), _p(cent), C.c_int(S), C.c_int(n_c), C.c_int(d), C.c_int(tau),
                               _p(rows), _p(z))
    return rows, z


def select_keys(tbl_idx, tbl_score, rows, n_pre, k):
    """Returns (sel [k] ascending / -1 padded, count, |U|, acc [n_pre] with NaN outside U)."""
    L = tbl_idx.shape[-1]
    rows = np.ascontiguousarray(rows, np.int32)
    sel = np.empty(max(k, 1), np.int32)
    cnt = np.zeros(1, np.int32)
    acc = np.empty(max(n_pre, 1), np.float32)
    nU = lib().oracle_select_keys(_p(tbl_idx), _p(tbl_score), C.c_int(L), _p(rows),
                                  C.c_int(len(rows)), C.c_int64(n_pre), C.c_int(k), _p(sel),
                                  _p(cnt), _p(acc))
    return sel[:k], int(cnt[0]), int(nU), acc[:n_pre]


def decode_head(q, cent, tbl_idx, tbl_score, tau, k, K, V, n_pre, n):
    """One query head, tau probes per subspace.  Returns (rows [S*tau], sel [k], count, out [d])."""
    S, n_c, d = _geometry(cent)
    L = tbl_idx.shape[-1]
    rows = np.empty(S * tau, np.int32)
    sel = np.empty(max(k, 1), np.int32)
    cnt = np.zeros(1, np.int32)
    out = np.empty(d, np.float32)
    lib().oracle_decode_head(_p(q), _p(cent), C.c_int(S), C.c_int(n_c), C.c_int(d), _p(tbl_idx),
                             _p(tbl_score), C.c_int(L), C.c_int(tau), C.c_int(k), _p(K), _p(V),
                             C.c_int64(n_pre), C.c_int64(n), _p(rows), _p(sel), _p(cnt), _p(out))
    return rows, sel[:k], int(cnt[0]), out


def try_insert(tbl_idx, tbl_score, cent, k_new, idx_new, F):
    """Streaming update of one KV head's tables [S*C][L] (in place) with the key appended at index
    idx_new.  Returns the largest |q| among the new key's scores."""
    S, n_c, d = _geometry(cent)
    assert tbl_idx.flags["C_CONTIGUOUS"] and tbl_score.flags["C_CONTIGUOUS"]
    assert tbl_idx.shape[0] == S * n_c
    return lib().oracle_try_insert(_p(tbl_idx), _p(tbl_score), C.c_int(tbl_idx.shape[-1]), _p(cent),
                                   C.c_int(S), C.c_int(n_c), C.c_int(d), _p(k_new), C.c_int32(idx_new),
                                   C.c_int(F))


def attend_selected(q, K, V, sel, n_pre, n):
    """Attention of q over the prefill keys listed in `sel` plus the appended keys [n_pre, n)."""
    d = q.shape[-1]
    sel = np.ascontiguousarray(sel, np.int32)
    out = np.empty(d, np.float32)
    lib().oracle_attend_selected(_p(q), _p(K), _p(V), _p(sel), C.c_int(len(sel)), C.c_int64(n_pre),
                                 C.c_int64(n), C.c_int(d), _p(out))
    return out


def decode_items(items, tau, k, n_pre, n, n_threads=0):
    """items: list of dicts(q [d], cent [C][d] or [S][C][d/S], tbl_idx [S*C][L], tbl_score, K, V)
    whose arrays stay alive for the call.  Returns (rows [n][S*tau], sel [n][k], cnt [n],
    out [n][d], threads_used)."""
    n_it = len(items)
    S, n_c, d = _geometry(items[0]["cent"])
    L = items[0]["tbl_idx"].shape[-1]
    arr = lambda key: (C.c_void_p * n_it)(*[it[key].ctypes.data for it in items])
    for it in items:
        for key in ("q", "cent", "tbl_idx", "tbl_score", "K", "V"):
            assert it[key].flags["C_CONTIGUOUS"]
    rows = np.empty((n_it, S * tau), np.int32)
    sel = np.empty((n_it, max(k, 1)), np.int32)
    cnt = np.zeros(n_it, np.int32)
    out = np.empty((n_it, d), np.float32)
    used = lib().oracle_decode_items(
        C.c_int(n_it), arr("q"), arr("cent"), arr("tbl_idx"), arr("tbl_score"), arr("K"),
        arr("V"), C.c_int(S), C.c_int(n_c), C.c_int(d), C.c_int(L), C.c_int(tau), C.c_int(k),
        C.c_int64(n_pre), C.c_int64(n), _p(rows), _p(sel), _p(cnt), _p(out), C.c_int(n_threads))
    return rows, sel[:, :k], cnt, out, used

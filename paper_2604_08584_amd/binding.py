"""ctypes binding of libcsattn.so: the same entry points as include/csattn.h, argument
marshalling only.  Every step of the decode path runs in the library's HIP kernels; torch is
used for device memory and streams.  There is no fallback: a missing library is an error.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("CSATTN_LIB", os.path.join(_HERE, "libcsattn.so"))

CSA_OK = 0
CSA_ERR_ARG, CSA_ERR_STATE, CSA_ERR_CAPACITY = -1, -2, -3
CSA_ERR_WORKSPACE, CSA_ERR_HIP, CSA_ERR_RANGE = -4, -5, -6
CSA_N_STAGES = 10


class csa_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "batch", "n_q_heads", "n_kv_heads", "head_dim", "n_centroids", "list_len", "n_probe",
        "budget_k", "n_subspaces", "max_ctx", "page_size", "score_frac_bits", "partition_keys",
        "stream_window")]


_lib = None


def lib() -> C.CDLL:
    """Loads the library (built in-tree by paper_2604_08584_amd/build.py or __graft_entry__.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2604_08584_amd.build` "
            "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    sig = {
        "csa_create": (C.c_int, [C.POINTER(csa_config), C.POINTER(vp)]),
        "csa_destroy": (None, [vp]),
        "csa_workspace_bytes": (C.c_int, [vp, C.POINTER(sz), C.POINTER(sz)]),
        "csa_bind": (C.c_int, [vp, vp, sz, vp, sz, vp, vp, vp]),
        "csa_build_tables": (C.c_int, [vp, vp, i32, vp]),
        "csa_cluster_workspace_bytes": (C.c_int, [vp, i32, C.POINTER(sz)]),
        "csa_cluster_queries": (C.c_int, [vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]),
        "csa_cluster_queries_minibatch": (C.c_int, [vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]),
        "csa_prefill": (C.c_int, [vp, vp, i32, i32, i32, vp, vp, vp, sz, vp]),
        "csa_export_tables": (C.c_int, [vp, i32, i32, vp, vp, vp]),
        "csa_import_tables": (C.c_int, [vp, vp, vp, vp, i32, vp]),
        "csa_append_kv": (C.c_int, [vp, vp, vp, vp]),
        "csa_decode_step": (C.c_int, [vp, vp, vp, vp, vp, vp]),
        "csa_decode_step_static": (C.c_int, [vp, vp, vp, vp, vp, vp]),
        "csa_static_scratch_bytes": (C.c_int, [vp, C.POINTER(sz), C.POINTER(sz)]),
        "csa_decode_step_reuse": (C.c_int, [vp, vp, vp, vp, vp, vp]),
        "csa_decode_step_append": (C.c_int, [vp, vp, vp, vp, vp, vp, vp, i32, vp]),
        "csa_decode_step_append_replayable": (C.c_int, [vp, vp, vp, vp, vp, vp, vp, i32, vp]),
        "csa_sync_context_len": (C.c_int, [vp, vp]),
        "csa_streaming_status": (C.c_int, [vp, vp]),
        "csa_context_len": (C.c_int, [vp, C.POINTER(i32), C.POINTER(i32)]),
        "csa_set_context_len": (C.c_int, [vp, i32]),
        "csa_score_frac_bits": (C.c_int, [vp, C.POINTER(i32)]),
        "csa_last_probed_rows": (C.c_int, [vp, vp, vp]),
        "csa_profile_enable": (C.c_int, [vp, i32]),
        "csa_profile_read": (C.c_int, [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
        "csa_stage_name": (C.c_char_p, [i32]),
        "csa_strerror": (C.c_char_p, [C.c_int]),
        "csa_last_hip_error": (C.c_int, [vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    _lib = L
    return L


EXPORTED = ("csa_create", "csa_destroy", "csa_workspace_bytes", "csa_bind", "csa_build_tables",
            "csa_cluster_workspace_bytes", "csa_cluster_queries", "csa_cluster_queries_minibatch", "csa_prefill",
            "csa_export_tables", "csa_import_tables", "csa_append_kv", "csa_decode_step",
            "csa_decode_step_static", "csa_static_scratch_bytes",
            "csa_decode_step_reuse", "csa_decode_step_append", "csa_decode_step_append_replayable",
            "csa_sync_context_len", "csa_streaming_status",
            "csa_context_len", "csa_set_context_len", "csa_score_frac_bits",
            "csa_last_probed_rows", "csa_profile_enable", "csa_profile_read", "csa_stage_name",
            "csa_strerror", "csa_last_hip_error")


class CsaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib().csa_strerror(status).decode()} ({status})")


def _check(status: int, where: str):
    if status != CSA_OK:
        raise CsaError(status, where)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensor expected"
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


# ---- the C entry points, one to one -------------------------------------------------------

def csa_create(**cfg) -> C.c_void_p:
    c = csa_config(n_subspaces=1, head_dim=128, page_size=0, score_frac_bits=-1, partition_keys=0,
                   stream_window=0)
    for key, val in cfg.items():
        setattr(c, key, val)
    ctx = C.c_void_p()
    _check(lib().csa_create(C.byref(c), C.byref(ctx)), "csa_create")
    return ctx


def csa_destroy(ctx):
    lib().csa_destroy(ctx)


def csa_workspace_bytes(ctx):
    a, b = C.c_size_t(), C.c_size_t()
    _check(lib().csa_workspace_bytes(ctx, C.byref(a), C.byref(b)), "csa_workspace_bytes")
    return a.value, b.value


def csa_bind(ctx, tables, scratch, k_cache, v_cache, block_table=None):
    _check(lib().csa_bind(ctx, _ptr(tables), tables.numel() * tables.element_size(), _ptr(scratch),
                          scratch.numel() * scratch.element_size(), _ptr(k_cache), _ptr(v_cache),
                          _ptr(block_table)), "csa_bind")


def csa_build_tables(ctx, centroids, n_pre):
    _check(lib().csa_build_tables(ctx, _ptr(centroids), n_pre, _stream()), "csa_build_tables")


def csa_cluster_workspace_bytes(ctx, n_pre) -> int:
    b = C.c_size_t()
    _check(lib().csa_cluster_workspace_bytes(ctx, n_pre, C.byref(b)), "csa_cluster_workspace_bytes")
    return b.value


def _uniforms(u_seed, device):
    """The seeding's uniforms as a device fp32 tensor (a numpy array is uploaded)."""
    if u_seed is None or isinstance(u_seed, torch.Tensor):
        return u_seed
    import numpy as np
    return torch.from_numpy(np.ascontiguousarray(u_seed, np.float32)).to(device)


def csa_cluster_queries(ctx, q_pre, n_pre, iters, u_seed, init_centroids, centroids_out, mean_cos=None,
                        assign=None, work=None, n_batches=1):
    """u_seed: fp32 uniforms, a device tensor or a numpy array (uploaded here), or None when
    init_centroids is given.  n_batches > 1 calls csa_cluster_queries_minibatch."""
    if work is None:
        work = torch.empty(csa_cluster_workspace_bytes(ctx, n_pre), dtype=torch.uint8, device=q_pre.device)
    u_dev = _uniforms(u_seed, q_pre.device)
    if n_batches == 1:
        _check(lib().csa_cluster_queries(ctx, _ptr(q_pre), n_pre, iters, _ptr(u_dev), _ptr(init_centroids),
                                         _ptr(centroids_out), _ptr(mean_cos), _ptr(assign), _ptr(work),
                                         work.numel(), _stream()), "csa_cluster_queries")
    else:
        _check(lib().csa_cluster_queries_minibatch(ctx, _ptr(q_pre), n_pre, iters, n_batches, _ptr(u_dev),
                                                   _ptr(init_centroids), _ptr(centroids_out), _ptr(mean_cos),
                                                   _ptr(assign), _ptr(work), work.numel(), _stream()),
               "csa_cluster_queries_minibatch")
    torch.cuda.current_stream().synchronize()   # the uniforms and the work buffer stay alive until here


def csa_prefill(ctx, q_pre, n_pre, iters, n_batches, u_seed, centroids_out, work=None):
    """Clustering of the prefill queries, then the table build, in one call (synchronises)."""
    if work is None:
        work = torch.empty(csa_cluster_workspace_bytes(ctx, n_pre), dtype=torch.uint8, device=q_pre.device)
    u_dev = _uniforms(u_seed, q_pre.device)
    _check(lib().csa_prefill(ctx, _ptr(q_pre), n_pre, iters, n_batches, _ptr(u_dev),
                             _ptr(centroids_out), _ptr(work), work.numel(), _stream()), "csa_prefill")


def csa_export_tables(ctx, b, g, idx_out, score_out):
    _check(lib().csa_export_tables(ctx, b, g, _ptr(idx_out), _ptr(score_out), _stream()),
           "csa_export_tables")


def csa_import_tables(ctx, centroids, idx, score, n_pre):
    _check(lib().csa_import_tables(ctx, _ptr(centroids), _ptr(idx), _ptr(score), n_pre, _stream()),
           "csa_import_tables")


def csa_append_kv(ctx, k_new, v_new):
    _check(lib().csa_append_kv(ctx, _ptr(k_new), _ptr(v_new), _stream()), "csa_append_kv")


def csa_decode_step(ctx, q, out, sel_idx=None, sel_count=None):
    _check(lib().csa_decode_step(ctx, _ptr(q), _ptr(out), _ptr(sel_idx), _ptr(sel_count), _stream()),
           "csa_decode_step")


def csa_decode_step_static(ctx, q, out, sel_idx=None, sel_count=None):
    _check(lib().csa_decode_step_static(ctx, _ptr(q), _ptr(out), _ptr(sel_idx), _ptr(sel_count), _stream()),
           "csa_decode_step_static")


def csa_static_scratch_bytes(ctx):
    a, b = C.c_size_t(), C.c_size_t()
    _check(lib().csa_static_scratch_bytes(ctx, C.byref(a), C.byref(b)), "csa_static_scratch_bytes")
    return a.value, b.value


def csa_decode_step_reuse(ctx, q, out, sel_idx=None, sel_count=None):
    _check(lib().csa_decode_step_reuse(ctx, _ptr(q), _ptr(out), _ptr(sel_idx), _ptr(sel_count), _stream()),
           "csa_decode_step_reuse")


def csa_decode_step_append(ctx, q, k_new, v_new, out, sel_idx=None, sel_count=None, reuse=False):
    _check(lib().csa_decode_step_append(ctx, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), _ptr(sel_idx),
                                        _ptr(sel_count), int(bool(reuse)), _stream()),
           "csa_decode_step_append")


def csa_decode_step_append_replayable(ctx, q, k_new, v_new, out, sel_idx=None, sel_count=None, reuse=False):
    _check(lib().csa_decode_step_append_replayable(ctx, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), _ptr(sel_idx),
                                                   _ptr(sel_count), int(bool(reuse)), _stream()),
           "csa_decode_step_append_replayable")


def csa_sync_context_len(ctx):
    _check(lib().csa_sync_context_len(ctx, _stream()), "csa_sync_context_len")


def csa_streaming_status(ctx):
    _check(lib().csa_streaming_status(ctx, _stream()), "csa_streaming_status")


def csa_context_len(ctx):
    a, b = C.c_int32(), C.c_int32()
    _check(lib().csa_context_len(ctx, C.byref(a), C.byref(b)), "csa_context_len")
    return a.value, b.value


def csa_set_context_len(ctx, n):
    _check(lib().csa_set_context_len(ctx, n), "csa_set_context_len")


def csa_score_frac_bits(ctx) -> int:
    f = C.c_int32()
    _check(lib().csa_score_frac_bits(ctx, C.byref(f)), "csa_score_frac_bits")
    return f.value


def csa_last_probed_rows(ctx, rows_out):
    _check(lib().csa_last_probed_rows(ctx, _ptr(rows_out), _stream()), "csa_last_probed_rows")


def csa_profile_enable(ctx, on: bool):
    _check(lib().csa_profile_enable(ctx, int(on)), "csa_profile_enable")


def csa_profile_read(ctx):
    """{stage name: (total ms, launches)} since the last read."""
    ms = (C.c_double * CSA_N_STAGES)()
    n = (C.c_int64 * CSA_N_STAGES)()
    _check(lib().csa_profile_read(ctx, ms, n), "csa_profile_read")
    return {lib().csa_stage_name(i).decode(): (ms[i], n[i]) for i in range(CSA_N_STAGES)}


# ---- plumbing: device buffers for one context ------------------------------------------------

class Context:
    """Owns the torch buffers a csa_ctx needs and forwards to the C calls above."""

    def __init__(self, k_cache, v_cache, block_table=None, device="cuda", **cfg):
        self.cfg = dict(cfg)
        self.ctx = csa_create(**cfg)
        tb, sb = csa_workspace_bytes(self.ctx)
        self.tables = torch.empty(tb, dtype=torch.uint8, device=device)
        self.scratch = torch.empty(sb, dtype=torch.uint8, device=device)
        self.k_cache, self.v_cache, self.block_table = k_cache, v_cache, block_table
        csa_bind(self.ctx, self.tables, self.scratch, k_cache, v_cache, block_table)
        B, Hq = cfg["batch"], cfg["n_q_heads"]
        self.out = torch.empty(B, Hq, 128, dtype=torch.float32, device=device)
        self.sel = torch.empty(B, Hq, max(cfg["budget_k"], 1), dtype=torch.int32, device=device)
        self.sel_count = torch.empty(B, Hq, dtype=torch.int32, device=device)

    def build_tables(self, centroids, n_pre):
        csa_build_tables(self.ctx, centroids, n_pre)

    def import_tables(self, centroids, idx, score, n_pre):
        csa_import_tables(self.ctx, centroids, idx, score, n_pre)

    def export_tables(self, b, g):
        C_, L = self.cfg["n_centroids"] * self.cfg.get("n_subspaces", 1), self.cfg["list_len"]
        idx = torch.empty(C_, L, dtype=torch.int32, device=self.out.device)
        score = torch.empty(C_, L, dtype=torch.float32, device=self.out.device)
        csa_export_tables(self.ctx, b, g, idx, score)
        return idx, score

    def decode_step(self, q):
        csa_decode_step(self.ctx, q, self.out, self.sel, self.sel_count)
        return self.out, self.sel, self.sel_count

    def decode_step_reuse(self, q, sel=None, sel_count=None):
        csa_decode_step_reuse(self.ctx, q, self.out, sel, sel_count)
        return self.out

    def append_kv(self, k_new, v_new):
        csa_append_kv(self.ctx, k_new, v_new)

    def decode_step_append(self, q, k_new, v_new):
        """decode_step followed by append_kv, in one call."""
        csa_decode_step_append(self.ctx, q, k_new, v_new, self.out, self.sel, self.sel_count, False)
        return self.out, self.sel, self.sel_count

    def decode_step_append_replayable(self, q, k_new, v_new, reuse=False):
        """decode_step_append in the form a HIP graph can replay (position read on the device)."""
        csa_decode_step_append_replayable(self.ctx, q, k_new, v_new, self.out,
                                          None if reuse else self.sel, None if reuse else self.sel_count, reuse)
        return self.out, self.sel, self.sel_count

    def decode_step_reuse_append(self, q, k_new, v_new, sel=None, sel_count=None):
        """decode_step_reuse followed by append_kv, in one call."""
        csa_decode_step_append(self.ctx, q, k_new, v_new, self.out, sel, sel_count, True)
        return self.out

    def probed_rows(self):
        rows = torch.empty(self.cfg["batch"], self.cfg["n_q_heads"],
                           self.cfg["n_probe"] * self.cfg.get("n_subspaces", 1),
                           dtype=torch.int32, device=self.out.device)
        csa_last_probed_rows(self.ctx, rows)
        return rows

    def close(self):
        if self.ctx is not None:
            csa_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

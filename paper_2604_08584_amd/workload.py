"""Seeded synthetic inputs for the CSAttention decode path.

This module only *draws data*: mixture-of-Gaussians keys / values / queries with a fixed
query-key offset (the Q/K distribution shift the paper's Fig. 1(d) shows), the centroids that
are handed to both the HIP library and the CPU oracle, and the physical placement of K/V
(contiguous or 16-token pages in shuffled order).  Nothing here scores a query against a
centroid, touches a lookup table, selects keys or computes attention.

Both sides of every parity test receive the *same bytes*: inputs are generated once (on the
CPU for the small cases, on the GPU for the large ones) and then copied, never regenerated.

Recipe (per sequence b, KV head g), all draws from a torch.Generator seeded with
``stream_seed(seed, cfg, b, g, stream)``:

* component means   mu_c ~ N(0, I_d), c < n_comp                       (stream "k_means")
* key i             k_i = mu_{c(i)} + 0.5 * eps,  c(i) uniform         (stream "K")
* offset            u = 3 * n / ||n||, n ~ N(0, I_d)                   (stream "offset")
* prefill query     q = mu_c + 0.5 * eps + u (same means as the keys)  (stream "Qpre")
* value i           independent mixture of the same form, own means    (streams "v_means", "V")
* decode query / appended key / appended value: fresh draws of the three forms above
* centroids         NOT made here by default: the benchmark takes them from the library's own
                    clustering of the prefill queries (make_inputs(keep_q_pre=True) returns those),
                    and the tests bring a centroid synthesis of their own (`centroid_fn`).  Without
                    either, the centroids are l2-normalised prefill query sub-vectors picked at
                    random: plain sampling, enough for anything that only needs valid inputs.
"""
from __future__ import annotations

import dataclasses
import hashlib
import math
from typing import Dict, Optional

import torch


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_pre: int          # prefill length N_pre
    n_comp: int         # mixture components per KV head
    C: int              # centroids per KV head
    L: int              # list length per centroid
    m: int              # probed centroids per query
    k: int              # key budget
    steps: int          # decode steps of the run
    pre_appended: int   # keys appended before the first timed step
    page_size: int      # 0 = contiguous K/V, 16 = paged
    kmeans_iters: int = 20
    n_sub: int = 1      # subspaces S (uniform split of the head dimension); C, m are per subspace

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def max_ctx(self) -> int:
        n = self.n_pre + self.pre_appended + self.steps
        page = self.page_size if self.page_size else 16
        return (n + page - 1) // page * page


# The five benchmark configurations (0 = tiny, 1 = 8B-shaped 32K, 2 = 8B-shaped 128K batch 1,
# 3 = paged batch 16 at 64K, 4 = 70B-shaped 128K batch 8).
CONFIGS: Dict[str, Workload] = {
    "cfg0": Workload("cfg0", 1, 4, 1, 128, 4096, 32, 64, 256, 4, 205, 1, 0, 0),
    "cfg1": Workload("cfg1", 1, 32, 8, 128, 32768, 256, 1024, 2048, 16, 1638, 1, 0, 0),
    "cfg2": Workload("cfg2", 1, 32, 8, 128, 131072, 256, 2048, 4096, 32, 6554, 64, 0, 0),
    "cfg3": Workload("cfg3", 16, 32, 8, 128, 65536, 256, 1024, 4096, 16, 3277, 1, 256, 16),
    "cfg4": Workload("cfg4", 8, 64, 8, 128, 131072, 512, 4096, 4096, 32, 6554, 256, 0, 0),
    # the paper's default geometry (Table "hyperparameters": 8 subspaces, one probe each, C = 128
    # centroids per subspace, L = 0.1 N_pre, K = 0.05 N) on the 8B-shaped layer, batch 8
    "paper_s8": Workload("paper_s8", 8, 32, 8, 128, 65536, 256, 128, 6554, 1, 3277, 64, 0, 0, n_sub=8),
}

_STREAMS = ("k_means", "v_means", "offset", "K", "V", "Qpre", "kmeans_init",
            "decode_q", "append_k", "append_v", "pages")


def stream_seed(seed: int, cfg_name: str, b: int, g: int, stream: str) -> int:
    """64-bit seed for one independent random stream (hash of its coordinates)."""
    assert stream in _STREAMS, stream
    h = hashlib.blake2b(f"{seed}/{cfg_name}/{b}/{g}/{stream}".encode(), digest_size=8)
    return int.from_bytes(h.digest(), "little") & 0x7FFF_FFFF_FFFF_FFFF


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _mixture(means: torch.Tensor, n: int, gen: torch.Generator, shift=None) -> torch.Tensor:
    """n draws of mu_{c} + 0.5*eps (+ shift); fp32 [n, d]."""
    dev = means.device
    comp = torch.randint(0, means.shape[0], (n,), generator=gen, device=dev)
    x = means[comp] + 0.5 * torch.randn(n, means.shape[1], generator=gen, device=dev)
    if shift is not None:
        x = x + shift
    return x


def make_inputs(cfg: Workload, seed: int = 0, device: str = "cpu",
                kmeans_sample: Optional[int] = None, centroid_fn=None,
                keep_q_pre: bool = False) -> Dict[str, torch.Tensor]:
    """All tensors one run of `cfg` needs.

    Returns (bf16 unless noted):
      k_cache, v_cache [B][Hkv][max_ctx][d]  rows [0, n_pre) filled, the rest zero
      centroids        [B][Hkv][C][d], or [B][Hkv][S][C][d/S] when cfg.n_sub = S > 1;
                                             unit norm before the bf16 rounding.  Made by
                                             centroid_fn(x [n][d/S] fp32, C, iters, generator) ->
                                             [C][d/S] fp32 per subspace from the pooled prefill query
                                             sub-vectors of the group if given; else normalised
                                             sub-vectors of randomly picked prefill queries.  Absent
                                             with keep_q_pre (the caller clusters q_pre itself).
      q_pre            [B][Hq][n_pre][d]     the prefill queries (only with keep_q_pre)
      q_steps          [T][B][Hq][d]         one decode query per head per step
      k_new, v_new     [T][B][Hkv][d]        the pair appended at each step
    with T = pre_appended + steps.  `kmeans_sample` caps the number of pooled prefill queries
    the centroid synthesis sees (None = all G*n_pre of them).
    """
    B, Hq, Hkv, d = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    G, T = cfg.group, cfg.pre_appended + cfg.steps
    dev = torch.device(device)
    bf = torch.bfloat16
    k_cache = torch.zeros(B, Hkv, cfg.max_ctx, d, dtype=bf, device=dev)
    v_cache = torch.zeros(B, Hkv, cfg.max_ctx, d, dtype=bf, device=dev)
    S = cfg.n_sub
    db = d // S
    centroids = None if keep_q_pre else torch.empty(B, Hkv, S, cfg.C, db, dtype=bf, device=dev)
    q_pre = torch.empty(B, Hq, cfg.n_pre, d, dtype=bf, device=dev) if keep_q_pre else None
    q_steps = torch.empty(T, B, Hq, d, dtype=bf, device=dev)
    k_new = torch.empty(T, B, Hkv, d, dtype=bf, device=dev)
    v_new = torch.empty(T, B, Hkv, d, dtype=bf, device=dev)
    for b in range(B):
        for g in range(Hkv):
            def G_(stream):
                return _gen(dev, stream_seed(seed, cfg.name, b, g, stream))
            k_means = torch.randn(cfg.n_comp, d, generator=G_("k_means"), device=dev)
            v_means = torch.randn(cfg.n_comp, d, generator=G_("v_means"), device=dev)
            u = torch.randn(d, generator=G_("offset"), device=dev)
            u = 3.0 * u / u.norm()
            k_cache[b, g, :cfg.n_pre] = _mixture(k_means, cfg.n_pre, G_("K")).to(bf)
            v_cache[b, g, :cfg.n_pre] = _mixture(v_means, cfg.n_pre, G_("V")).to(bf)
            n_pool = G * cfg.n_pre
            if kmeans_sample is not None and not keep_q_pre:
                n_pool = min(n_pool, kmeans_sample)
            # prefill queries are bf16 tensors in a model; round before clustering
            qpre = _mixture(k_means, n_pool, G_("Qpre"), shift=u).to(bf)
            if keep_q_pre:
                q_pre[b, g * G:(g + 1) * G] = qpre.view(G, cfg.n_pre, d)
            else:
                g_init = G_("kmeans_init")
                qf = qpre.float()
                for sub in range(S):
                    x = qf[:, sub * db:(sub + 1) * db].contiguous()
                    if centroid_fn is not None:
                        cent = centroid_fn(x, cfg.C, cfg.kmeans_iters, g_init)
                    else:
                        pick = torch.randint(0, x.shape[0], (cfg.C,), generator=g_init, device=dev)
                        cent = x[pick] / x[pick].norm(dim=1, keepdim=True).clamp_min(1e-20)
                    centroids[b, g, sub] = cent.to(bf)
                del qf
            del qpre
            q_steps[:, b, g * G:(g + 1) * G] = _mixture(
                k_means, T * G, G_("decode_q"), shift=u).to(bf).view(T, G, d)
            k_new[:, b, g] = _mixture(k_means, T, G_("append_k")).to(bf)
            v_new[:, b, g] = _mixture(v_means, T, G_("append_v")).to(bf)
    out = dict(k_cache=k_cache, v_cache=v_cache, q_steps=q_steps, k_new=k_new, v_new=v_new)
    if keep_q_pre:
        out["q_pre"] = q_pre
    else:
        out["centroids"] = centroids.view(B, Hkv, cfg.C, d) if S == 1 else centroids
    return out


def paginate(cache: torch.Tensor, page_size: int, seed: int, cfg_name: str,
             block_table: Optional[torch.Tensor] = None):
    """Scatter a contiguous cache [B][Hkv][max_ctx][d] into a page pool.

    Returns (pool [n_pages][Hkv][page_size][d], block_table [B][max_ctx/page_size] int32).
    The physical page order is one seeded random permutation of the whole pool; pass the
    block table of the K pool to place V identically.
    """
    B, Hkv, n, d = cache.shape
    assert n % page_size == 0
    ppb = n // page_size
    if block_table is None:
        gen = _gen(cache.device, stream_seed(seed, cfg_name, 0, 0, "pages"))
        block_table = torch.randperm(B * ppb, generator=gen, device=cache.device) \
            .to(torch.int32).view(B, ppb)
    pool = torch.empty(B * ppb, Hkv, page_size, d, dtype=cache.dtype, device=cache.device)
    src = cache.view(B, Hkv, ppb, page_size, d).permute(0, 2, 1, 3, 4).reshape(
        B * ppb, Hkv, page_size, d)
    pool[block_table.view(-1).long()] = src
    return pool, block_table


def algorithmic_bytes_per_head(cfg: Workload, t: float) -> Dict[str, float]:
    """HBM bytes the method itself must move per (sequence, query head) per decode step with
    t appended keys: centroids (shared by the G heads of a group), m table rows of L
    8-byte entries, 2*(k+t) K/V rows, and q / out / sel."""
    d = cfg.head_dim
    return dict(
        centroids=cfg.C * d * 2 / cfg.group,             # S subspaces x C centroids x d/S dimensions
        table_rows=cfg.n_sub * cfg.m * cfg.L * 8,
        kv_rows=2 * (cfg.k + t) * d * 2,
        io=d * 2 + d * 4 + cfg.k * 4,
    )

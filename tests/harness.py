"""Glue shared by the GPU parity tests: runs the HIP library (through the C ABI binding) and the
CPU oracle on the same bytes and compares them.  Holds no arithmetic of the method.

Nothing the oracle consumes comes from the GPU: its tables are the ones it builds itself from
the same K and centroids (only the rows a step probes, at full size), or arrays a test made up
and handed to both sides; tables exported from the GPU are only ever compared."""
from __future__ import annotations

import numpy as np
import torch

from oracle import oracle
from paper_2604_08584_amd import binding
from paper_2604_08584_amd.workload import Workload, make_inputs, paginate

TOL_OUT = 2e-2   # max-abs tolerance on attention outputs (bf16 inputs, fp32 accumulation)


def synth_centroids(x: torch.Tensor, C: int, iters: int, gen: torch.Generator, chunk: int = 1 << 16) -> torch.Tensor:
    """Centroids for the parity tests (inputs handed identically to the library and to the oracle;
    test infrastructure, not the library's clustering): Lloyd iterations with cosine assignment on
    unit vectors from a random sample.  x: [n, d] fp32; returns unit-norm fp32 [C, d]."""
    x = x / x.norm(dim=1, keepdim=True).clamp_min(1e-20)
    n, d = x.shape
    if n >= C:
        init = torch.randperm(n, generator=gen, device=x.device)[:C]
    else:
        init = torch.randint(0, n, (C,), generator=gen, device=x.device)
    cent = x[init].clone()
    for _ in range(iters):
        sums = torch.zeros(C, d, dtype=torch.float32, device=x.device)
        cnts = torch.zeros(C, dtype=torch.float32, device=x.device)
        for s in range(0, n, chunk):
            xs = x[s:s + chunk]
            a = (xs @ cent.t()).argmax(dim=1)
            sums.index_add_(0, a, xs)
            cnts.index_add_(0, a, torch.ones_like(a, dtype=torch.float32))
        norm = sums.norm(dim=1, keepdim=True)
        ok = (cnts > 0).unsqueeze(1) & (norm > 1e-12)
        cent = torch.where(ok, sums / norm.clamp_min(1e-12), cent)
    return cent


def cfg_kwargs(w: Workload, F: int, partition_keys: int = 0, stream_window: int = 0):
    return dict(stream_window=stream_window, batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, n_centroids=w.C,
                list_len=w.L, n_probe=w.m, budget_k=w.k, max_ctx=w.max_ctx, page_size=w.page_size,
                score_frac_bits=F, partition_keys=partition_keys, n_subspaces=w.n_sub)


class Case:
    """One workload instantiated on the GPU, with host copies for the oracle."""

    def __init__(self, w: Workload, seed=0, F=14, partition_keys=0, gen_device="cpu",
                 kmeans_sample=None, stream_window=0):
        self.w, self.F = w, F
        self.stream_window = stream_window   # > 0: appended keys are try-inserted into the tables
        inp = make_inputs(w, seed=seed, device=gen_device, kmeans_sample=kmeans_sample, centroid_fn=synth_centroids)
        self.inp = {k: v.cuda() for k, v in inp.items()}
        # logical (contiguous) host copies for the oracle; appended rows are filled in as we go
        self.K_host = oracle.bf16_bits(inp["k_cache"])
        self.V_host = oracle.bf16_bits(inp["v_cache"])
        self.cent_host = oracle.bf16_bits(inp["centroids"])
        if w.page_size:
            self.k_store, self.block_table = paginate(self.inp["k_cache"], w.page_size, seed, w.name)
            self.v_store, _ = paginate(self.inp["v_cache"], w.page_size, seed, w.name, self.block_table)
        else:
            self.k_store, self.v_store, self.block_table = self.inp["k_cache"], self.inp["v_cache"], None
        self.ctx = binding.Context(self.k_store, self.v_store, self.block_table,
                                   **cfg_kwargs(w, F, partition_keys, stream_window))
        # the oracle's own tables: (b, g) -> [idx [S*C][L], score [S*C][L], row-is-filled [S*C]]
        self.otab = {}
        self.t = 0         # appended so far

    # ---- tables
    def build_on_gpu(self):
        self.ctx.build_tables(self.inp["centroids"], self.w.n_pre)
        self.F = binding.csa_score_frac_bits(self.ctx.ctx)

    def export(self, b, g):
        """The GPU's tables of KV head (b, g), canonical layout (for comparison only)."""
        idx, score = self.ctx.export_tables(b, g)
        return idx.cpu().numpy(), score.cpu().numpy()

    def oracle_rows(self, b, g, rows=None):
        """The oracle's tables of KV head (b, g) with (at least) `rows` filled in by the oracle's own
        build over the prefill keys (None = every row).  Returns (idx, score) [S*C][L]."""
        w = self.w
        n_rows = w.n_sub * w.C
        if (b, g) not in self.otab:
            self.otab[(b, g)] = [np.full((n_rows, w.L), -1, np.int32), np.zeros((n_rows, w.L), np.float32),
                                 np.zeros(n_rows, bool)]
        idx, score, have = self.otab[(b, g)]
        want = np.arange(n_rows) if rows is None else np.unique(np.asarray(rows))
        todo = want[~have[want]]
        if len(todo):
            i, s, _ = self.oracle_tables(b, g, todo)
            idx[todo], score[todo] = i, s
            have[todo] = True
        return idx, score

    def oracle_tables(self, b, g, rows=None):
        K = np.ascontiguousarray(self.K_host[b, g, :self.w.n_pre])
        if rows is None:
            return oracle.build_tables(K, self.w.n_pre, self.cent_host[b, g], self.w.L, self.F)
        return oracle.build_rows(K, self.w.n_pre, self.cent_host[b, g], rows, self.w.L, self.F)

    def import_tables(self, idx, score):
        """idx/score: numpy [B][Hkv][C][L] canonical."""
        w = self.w
        for b in range(w.batch):
            for g in range(w.n_kv_heads):
                self.otab[(b, g)] = [np.ascontiguousarray(idx[b, g]), np.ascontiguousarray(score[b, g]),
                                     np.ones(idx.shape[2], bool)]
        self.ctx.import_tables(self.inp["centroids"], torch.from_numpy(idx).cuda(),
                               torch.from_numpy(score).cuda(), w.n_pre)

    def import_oracle_tables(self):
        w = self.w
        idx = np.empty((w.batch, w.n_kv_heads, w.n_sub * w.C, w.L), np.int32)
        score = np.empty((w.batch, w.n_kv_heads, w.n_sub * w.C, w.L), np.float32)
        for b in range(w.batch):
            for g in range(w.n_kv_heads):
                idx[b, g], score[b, g], _ = self.oracle_tables(b, g)
        self.import_tables(idx, score)

    # ---- steps
    def append(self, count=1, groups=None):
        """Appends on the GPU and mirrors it on the host; with streaming updates the oracle's
        try-insert is applied to the oracle's tables of `groups` (default: all (b, g)), which are
        built in full first."""
        w = self.w
        for _ in range(count):
            kn, vn = self.inp["k_new"][self.t], self.inp["v_new"][self.t]
            self.ctx.append_kv(kn, vn)
            self._mirror_append(groups)

    def _mirror_append(self, groups=None):
        """The host side of one append: K/V rows, and the oracle's try-insert with streaming updates."""
        w = self.w
        kn, vn = self.inp["k_new"][self.t], self.inp["v_new"][self.t]
        pos = w.n_pre + self.t
        kb = oracle.bf16_bits(kn)
        self.K_host[:, :, pos] = kb
        self.V_host[:, :, pos] = oracle.bf16_bits(vn)
        if self.stream_window:
            for (b, g) in (groups if groups is not None else
                           [(b, g) for b in range(w.batch) for g in range(w.n_kv_heads)]):
                idx, score = self.oracle_rows(b, g)
                oracle.try_insert(idx, score, self.cent_host[b, g], np.ascontiguousarray(kb[b, g]), pos, self.F)
        self.t += 1

    def check_tables(self, b, g):
        """The GPU's tables (exported now) against the oracle's (built, and kept up to date, by it)."""
        idx, score = self.export(b, g)
        want_idx, want_score = self.oracle_rows(b, g)
        assert np.array_equal(idx, want_idx), f"table indices of ({b},{g}) differ"
        assert np.array_equal(score, want_score), f"table scores of ({b},{g}) differ"

    def window_start(self):
        n = self.w.n_pre + self.t
        return max(0, n - self.stream_window) if self.stream_window else self.w.n_pre

    def decode(self, step, static=False):
        """static: through csa_decode_step_static (the step's temporaries in the library's own array)."""
        q = self.inp["q_steps"][step]
        if static:
            binding.csa_decode_step_static(self.ctx.ctx, q, self.ctx.out, self.ctx.sel, self.ctx.sel_count)
            out, sel, cnt = self.ctx.out, self.ctx.sel, self.ctx.sel_count
        else:
            out, sel, cnt = self.ctx.decode_step(q)
        rows = self.ctx.probed_rows()
        torch.cuda.synchronize()
        return out.cpu().numpy(), sel.cpu().numpy(), cnt.cpu().numpy(), rows.cpu().numpy()

    def decode_append(self, step, replayable=False):
        """The fused call: decode step `step`, then the append of the next K/V row (one call);
        replayable: its form with the context length read on the device."""
        q = self.inp["q_steps"][step]
        call = self.ctx.decode_step_append_replayable if replayable else self.ctx.decode_step_append
        out, sel, cnt = call(q, self.inp["k_new"][self.t], self.inp["v_new"][self.t])
        rows = self.ctx.probed_rows()
        torch.cuda.synchronize()
        return out.cpu().numpy(), sel.cpu().numpy(), cnt.cpu().numpy(), rows.cpu().numpy()

    def oracle_decode(self, step, heads):
        """heads: list of (b, h).  The oracle probes its own centroids and reads its own tables: the
        rows a head probes are built by the oracle on demand (all rows once streaming updates or an
        import have made the tables complete)."""
        w = self.w
        qh = oracle.bf16_bits(self.inp["q_steps"][step])
        n = w.n_pre + self.t
        items = []
        for b, h in heads:
            g = h // w.group
            probed, _ = oracle.top_centroids(np.ascontiguousarray(qh[b, h]), self.cent_host[b, g], w.m)
            idx, score = self.oracle_rows(b, g, probed)
            items.append(dict(q=np.ascontiguousarray(qh[b, h]), cent=self.cent_host[b, g], tbl_idx=idx,
                              tbl_score=score, K=self.K_host[b, g], V=self.V_host[b, g]))
        rows, sel, cnt, out, _ = oracle.decode_items(items, w.m, w.k, self.window_start(), n)
        return rows, sel, cnt, out

    def oracle_index_set(self, step):
        """The oracle's index set of every head for `step` as the arrays decode_step returns:
        sel [B][Hq][k] int32 (ascending, -1 padded) and cnt [B][Hq] int32."""
        w = self.w
        heads = [(b, h) for b in range(w.batch) for h in range(w.n_q_heads)]
        _, o_sel, o_cnt, _ = self.oracle_decode(step, heads)
        sel = np.full((w.batch, w.n_q_heads, w.k), -1, np.int32)
        cnt = np.zeros((w.batch, w.n_q_heads), np.int32)
        for t, (b, h) in enumerate(heads):
            cnt[b, h] = o_cnt[t]
            sel[b, h, :o_cnt[t]] = np.asarray(o_sel[t])[:o_cnt[t]]
        return sel, cnt

    def check_step(self, step, heads=None, fused_append=False, groups=None, static=False, replayable=False):
        """Decode on both sides, compare; returns the max-abs output error.  fused_append: the GPU
        side uses the one-call form that also appends the next K/V row (the oracle decodes on the
        context before that append, then the host mirrors it)."""
        w = self.w
        if heads is None:
            heads = [(b, h) for b in range(w.batch) for h in range(w.n_q_heads)]
        o_rows, o_sel, o_cnt, o_out = self.oracle_decode(step, heads)
        if fused_append:
            out, sel, cnt, rows = self.decode_append(step, replayable=replayable)
            self._mirror_append(groups)
        else:
            out, sel, cnt, rows = self.decode(step, static=static)
        worst = 0.0
        for t, (b, h) in enumerate(heads):
            tag = f"{w.name} step {step} head ({b},{h})"
            assert sorted(rows[b, h].tolist()) == sorted(o_rows[t].tolist()), f"{tag}: probed rows differ"
            assert cnt[b, h] == o_cnt[t], f"{tag}: count {cnt[b, h]} != {o_cnt[t]}"
            if w.k:
                assert np.array_equal(sel[b, h][:w.k], o_sel[t]), f"{tag}: selected indices differ"
            err = float(np.abs(out[b, h] - o_out[t]).max())
            assert np.isfinite(out[b, h]).all() and err <= TOL_OUT, f"{tag}: |out - oracle| = {err}"
            worst = max(worst, err)
        return worst


    def check_reuse_step(self, step, sel, cnt, heads=None, pass_buffers=False, fused_append=False, replayable=False):
        """A search-period step: attention of step `step`'s query over the index set (sel, cnt) of
        an earlier searching step plus everything appended so far; compared with the oracle.
        fused_append: the GPU side uses the one-call form that also appends the next K/V row."""
        w = self.w
        if heads is None:
            heads = [(b, h) for b in range(w.batch) for h in range(w.n_q_heads)]
        q = self.inp["q_steps"][step]
        bufs = (torch.from_numpy(sel).cuda(), torch.from_numpy(cnt).cuda()) if pass_buffers else ()
        n = w.n_pre + self.t                      # the context this step attends to
        start = self.window_start()
        if fused_append and replayable:     # (the library's copy of the index set)
            out = self.ctx.decode_step_append_replayable(q, self.inp["k_new"][self.t], self.inp["v_new"][self.t],
                                                         reuse=True)[0]
        elif fused_append:
            out = self.ctx.decode_step_reuse_append(q, self.inp["k_new"][self.t], self.inp["v_new"][self.t], *bufs)
        else:
            out = self.ctx.decode_step_reuse(q, *bufs)
        torch.cuda.synchronize()
        out = out.cpu().numpy()
        if fused_append:
            self._mirror_append()
        qh = oracle.bf16_bits(q)
        worst = 0.0
        for b, h in heads:
            g = h // w.group
            want = oracle.attend_selected(np.ascontiguousarray(qh[b, h]), self.K_host[b, g], self.V_host[b, g],
                                          sel[b, h][:cnt[b, h]], start, n)
            err = float(np.abs(out[b, h] - want).max())
            assert np.isfinite(out[b, h]).all() and err <= TOL_OUT, f"{w.name} reuse step {step} head ({b},{h}): {err}"
            worst = max(worst, err)
        return worst


def small(name="small", **kw) -> Workload:
    base = dict(name=name, batch=1, n_q_heads=4, n_kv_heads=1, head_dim=128, n_pre=3000, n_comp=16,
                C=48, L=200, m=5, k=150, steps=2, pre_appended=0, page_size=0, kmeans_iters=3)
    base.update(kw)
    return Workload(**base)

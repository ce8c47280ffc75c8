"""csa_decode_step_append_replayable: the whole decode iteration with the context length kept on
the device.  Called eagerly it must give what csa_decode_step_append gives (which the oracle checks
here step by step); captured into a HIP graph and replayed, every replay - with eager work and
synchronisations between the replays - must give what the eager twin gives at the same position,
rows must land in the K/V cache at the right positions, and a replay on a full context must append
nothing and be reported."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2604_08584_amd import binding

from harness import Case, small

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(300)]


def _twin(**kw):
    base = dict(n_q_heads=8, n_kv_heads=2, n_pre=9000, C=64, L=400, m=4, k=600, steps=8)
    base.update(kw)
    a = Case(small("replay", **base), seed=5, F=13, partition_keys=4096)
    b = Case(small("replay", **base), seed=5, F=13, partition_keys=4096)
    a.build_on_gpu()
    b.build_on_gpu()
    return a, b


def _same(tag, a, b):
    assert torch.equal(a.ctx.sel_count, b.ctx.sel_count), f"{tag}: counts differ"
    assert torch.equal(a.ctx.sel, b.ctx.sel), f"{tag}: index sets differ"
    assert torch.equal(a.ctx.out, b.ctx.out), f"{tag}: outputs differ"      # same kernels, same order
    assert torch.equal(a.k_store, b.k_store) and torch.equal(a.v_store, b.v_store), f"{tag}: caches differ"


def test_replayable_iteration_called_eagerly_matches_the_plain_one():
    a, b = _twin()
    for step in range(6):
        err = a.check_step(step, fused_append=True)                  # plain call, against the oracle
        b.ctx.decode_step_append_replayable(b.inp["q_steps"][step], b.inp["k_new"][step], b.inp["v_new"][step])
        torch.cuda.synchronize()
        _same(f"step {step}", a, b)
    binding.csa_sync_context_len(b.ctx.ctx)
    assert binding.csa_context_len(b.ctx.ctx) == binding.csa_context_len(a.ctx.ctx) == (a.w.n_pre, a.w.n_pre + 6)
    print("replayable form, eager: last err vs oracle", err)


@pytest.mark.parametrize("paged", [False, True])
def test_captured_iteration_replays_correctly(paged):
    kw = dict(page_size=16) if paged else {}
    a, b = _twin(steps=7, **kw)
    w = a.w
    q, kn, vn = (torch.empty_like(b.inp[x][0]) for x in ("q_steps", "k_new", "v_new"))
    # one eager iteration first (step 0), so that the capture does not see a first-use path
    for c in (a, b):
        c.ctx.decode_step_append(c.inp["q_steps"][0], c.inp["k_new"][0], c.inp["v_new"][0])
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(g, stream=side):
        b.ctx.decode_step_append_replayable(q, kn, vn)
    binding.csa_sync_context_len(b.ctx.ctx)        # the capture ran nothing: the count is still n_pre + 1
    assert binding.csa_context_len(b.ctx.ctx)[1] == w.n_pre + 1
    for step in range(1, w.steps):                 # up to the last row of the cache
        a.ctx.decode_step_append(a.inp["q_steps"][step], a.inp["k_new"][step], a.inp["v_new"][step])
        q.copy_(b.inp["q_steps"][step]); kn.copy_(b.inp["k_new"][step]); vn.copy_(b.inp["v_new"][step])
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        junk = (torch.randn(1 << 16, device="cuda") * 2).sum().item()      # unrelated eager work between replays
        assert np.isfinite(junk)
        _same(f"replay at step {step}", a, b)
    binding.csa_sync_context_len(b.ctx.ctx)
    n_full = binding.csa_context_len(b.ctx.ctx)[1]
    assert n_full == binding.csa_context_len(a.ctx.ctx)[1] == w.n_pre + w.steps
    # the oracle on the eager twin's last position (the replayed one equals it bit for bit)
    a.t = w.steps - 1
    for t in range(w.steps - 1):                   # mirror the appends the loop above made on the GPU
        a.K_host[:, :, w.n_pre + t] = oracle.bf16_bits(a.inp["k_new"][t])
        a.V_host[:, :, w.n_pre + t] = oracle.bf16_bits(a.inp["v_new"][t])
    heads = [(0, h) for h in range(w.n_q_heads)]
    o_rows, o_sel, o_cnt, o_out = a.oracle_decode(w.steps - 1, heads)
    out, sel, cnt = b.ctx.out.cpu().numpy(), b.ctx.sel.cpu().numpy(), b.ctx.sel_count.cpu().numpy()
    for t, (b_, h) in enumerate(heads):
        assert cnt[b_, h] == o_cnt[t] and np.array_equal(sel[b_, h][:w.k], o_sel[t])
        assert float(np.abs(out[b_, h] - o_out[t]).max()) <= 2e-2
    # fill the cache to the brim, then one replay too many: nothing is written, the count stays
    while n_full < w.max_ctx:
        g.replay()
        n_full += 1
    torch.cuda.synchronize()
    binding.csa_sync_context_len(b.ctx.ctx)
    assert binding.csa_context_len(b.ctx.ctx)[1] == w.max_ctx
    k_before = b.k_store.clone()
    g.replay()
    torch.cuda.synchronize()
    with pytest.raises(binding.CsaError) as e:
        binding.csa_sync_context_len(b.ctx.ctx)
    assert e.value.status == binding.CSA_ERR_CAPACITY
    assert binding.csa_context_len(b.ctx.ctx)[1] == w.max_ctx and torch.equal(k_before, b.k_store)
    assert torch.isfinite(b.ctx.out).all()


def test_replayed_search_period_schedule():
    """A schedule with search period 2 as two captured graphs - a searching iteration and a reusing
    one (index set of the last search, left in the caller's buffers) - replayed in turn; every step
    equals the eager twin's csa_decode_step_append with the same reuse flag."""
    a, b = _twin(steps=8)
    w = a.w
    q, kn, vn = (torch.empty_like(b.inp[x][0]) for x in ("q_steps", "k_new", "v_new"))
    for c in (a, b):                               # step 0 eagerly (a search)
        c.ctx.decode_step_append(c.inp["q_steps"][0], c.inp["k_new"][0], c.inp["v_new"][0])
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g_search, g_reuse = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
    with torch.cuda.graph(g_reuse, stream=side):
        b.ctx.decode_step_append_replayable(q, kn, vn, reuse=True)
    with torch.cuda.graph(g_search, stream=side):
        b.ctx.decode_step_append_replayable(q, kn, vn)
    binding.csa_sync_context_len(b.ctx.ctx)
    for step in range(1, w.steps):
        reuse = step % 2 == 1
        if reuse:
            a.ctx.decode_step_reuse_append(a.inp["q_steps"][step], a.inp["k_new"][step], a.inp["v_new"][step])
        else:
            a.ctx.decode_step_append(a.inp["q_steps"][step], a.inp["k_new"][step], a.inp["v_new"][step])
        q.copy_(b.inp["q_steps"][step]); kn.copy_(b.inp["k_new"][step]); vn.copy_(b.inp["v_new"][step])
        torch.cuda.synchronize()
        (g_reuse if reuse else g_search).replay()
        torch.cuda.synchronize()
        _same(f"{'reuse' if reuse else 'search'} replay at step {step}", a, b)
    binding.csa_sync_context_len(b.ctx.ctx)
    assert binding.csa_context_len(b.ctx.ctx)[1] == w.n_pre + w.steps


def test_replayable_form_is_refused_with_streaming_updates():
    c = Case(small("replay_stream", steps=2), seed=2, F=13, stream_window=8)
    c.build_on_gpu()
    with pytest.raises(binding.CsaError) as e:
        c.ctx.decode_step_append_replayable(c.inp["q_steps"][0], c.inp["k_new"][0], c.inp["v_new"][0])
    assert e.value.status == binding.CSA_ERR_ARG

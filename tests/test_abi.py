"""CPU-side checks of the C-ABI library: it loads, exports every symbol include/csattn.h
declares, and validates arguments on the host (no compute, no GPU)."""
import ctypes as C
import os
import re

import pytest

from paper_2604_08584_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "csattn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(csa_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = C.CDLL(binding.LIB_PATH)
    names = declared_symbols()
    assert len(names) >= 18
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTED) == names


GOOD = dict(batch=1, n_q_heads=4, n_kv_heads=1, n_centroids=64, list_len=256, n_probe=4,
            budget_k=205, max_ctx=4096)


def test_create_validates_configuration():
    ctx = binding.csa_create(**GOOD)
    tb, sb = binding.csa_workspace_bytes(ctx)
    assert tb >= 64 * 256 * 4 + 64 * 128 * 2 and sb > 0     # 4-byte packed entries + bf16 centroids
    binding.csa_destroy(ctx)
    binding.csa_destroy(binding.csa_create(**{**GOOD, 'n_subspaces': 8, 'n_probe': 2}))   # the paper's geometry
    for bad in (dict(head_dim=64), dict(n_probe=0), dict(n_probe=64), dict(n_probe=65, n_centroids=100),
                dict(n_q_heads=3, n_kv_heads=2), dict(n_q_heads=17), dict(n_subspaces=3), dict(n_subspaces=32), dict(n_subspaces=16, n_probe=4),
                dict(list_len=0), dict(list_len=10000),
                dict(page_size=8), dict(page_size=16, max_ctx=4100), dict(budget_k=-1),
                dict(partition_keys=3000), dict(max_ctx=0), dict(batch=0)):
        with pytest.raises(binding.CsaError) as e:
            binding.csa_create(**{**GOOD, **bad})
        assert e.value.status == binding.CSA_ERR_ARG, bad


def test_workspace_stays_proportionate_for_the_longest_context():
    """max_ctx = 2^24 with the smallest requested key ranges: the ranges are widened until a head has
    at most 2048 of them, and the per-range buffers are sized for that, not for max_ctx / 1024."""
    cfg = dict(batch=1, n_q_heads=8, n_kv_heads=1, n_centroids=64, list_len=1024, n_probe=4, budget_k=1000,
               max_ctx=1 << 24, partition_keys=1024)
    ctx = binding.csa_create(**cfg)
    tb, sb = binding.csa_workspace_bytes(ctx)
    binding.csa_destroy(ctx)
    per_head_candidates = (1 << 24) * 4                     # one 32-bit word per key index
    per_head_ranges = 2048 * (512 * 2 + 4 + 8 + 8)          # bin offsets, count, two small records per range
    build_scratch = 64 * (1 << 24) * 4                      # integer scores of a chunk of centroid rows
    assert sb < 8 * (per_head_candidates + per_head_ranges) * 1.2 + build_scratch * 1.1 + (1 << 24)
    assert tb < (64 * 1024 * 4 + 64 * 2053 * 4 + 64 * 128 * 2) * 1.1 + (1 << 20)
    # streaming updates bound the queue segments per KV head
    with pytest.raises(binding.CsaError) as e:
        binding.csa_create(**{**GOOD, 'n_centroids': 70000, 'n_probe': 4, 'stream_window': 8})
    assert e.value.status == binding.CSA_ERR_ARG


def test_calls_out_of_order_are_refused_on_the_host():
    lib = binding.lib()
    ctx = binding.csa_create(**GOOD)
    assert lib.csa_decode_step(ctx, C.c_void_p(256), C.c_void_p(256), None, None, None) == binding.CSA_ERR_STATE
    assert lib.csa_append_kv(ctx, C.c_void_p(256), C.c_void_p(256), None) == binding.CSA_ERR_STATE
    assert lib.csa_build_tables(ctx, C.c_void_p(256), 4096, None) == binding.CSA_ERR_STATE
    assert lib.csa_context_len(ctx, None, None) == binding.CSA_ERR_STATE
    # bind: misaligned / missing / too-small buffers
    assert lib.csa_bind(ctx, C.c_void_p(256), 1 << 40, C.c_void_p(256), 1 << 40, C.c_void_p(256),
                        C.c_void_p(8), None) == binding.CSA_ERR_ARG
    assert lib.csa_bind(ctx, C.c_void_p(256), 16, C.c_void_p(256), 1 << 40, C.c_void_p(256),
                        C.c_void_p(256), None) == binding.CSA_ERR_WORKSPACE
    assert lib.csa_bind(ctx, C.c_void_p(256), 1 << 40, C.c_void_p(256), 1 << 40, C.c_void_p(256),
                        C.c_void_p(256), C.c_void_p(256)) == binding.CSA_ERR_ARG  # block table without paging
    assert lib.csa_decode_step(None, None, None, None, None, None) == binding.CSA_ERR_ARG
    binding.csa_destroy(ctx)
    assert lib.csa_strerror(binding.CSA_ERR_RANGE).decode().startswith("table score")
    assert lib.csa_stage_name(0).decode() == "score_centroids" and lib.csa_stage_name(99) is None


def test_product_and_oracle_do_not_reach_into_each_other():
    """The library, its binding and the input generator never import, load or call the oracle, and
    the oracle never imports the package: parity compares two independent implementations, and a
    missing HIP library cannot be papered over by the CPU code."""
    import re
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    pkg = os.path.join(root, "paper_2604_08584_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp", ".c")):
                text = open(os.path.join(dirpath, f), errors="replace").read()
                assert not re.search(r"import\s+oracle|from\s+oracle|oracle\.|oracle/|csa_oracle", text), \
                    f"{f} reaches into the oracle"
    for f in os.listdir(os.path.join(root, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(root, "oracle", f), errors="replace").read()
            assert "paper_2604_08584_amd" not in text and "csattn" not in text, f"oracle/{f} names the product"
    # the binding refuses to work without the built library instead of falling back
    src = open(os.path.join(pkg, "binding.py")).read()
    assert "raise" in src[src.index("def lib("):src.index("def lib(") + 1500]


def test_new_entry_points_validate_on_the_host():
    """The static-scratch step, the replayable iteration, the count sync and the one-call prefill
    refuse bad arguments and calls out of order before anything touches the GPU."""
    lib = binding.lib()
    ctx = binding.csa_create(**GOOD)
    p = C.c_void_p(256)
    # nothing bound yet
    assert lib.csa_decode_step_static(ctx, p, p, None, None, None) == binding.CSA_ERR_STATE
    assert lib.csa_decode_step_append_replayable(ctx, p, p, p, p, None, None, 0, None) == binding.CSA_ERR_STATE
    assert lib.csa_decode_step_append_replayable(ctx, p, None, p, p, None, None, 0, None) == binding.CSA_ERR_ARG
    assert lib.csa_sync_context_len(ctx, None) == binding.CSA_ERR_STATE
    assert lib.csa_sync_context_len(None, None) == binding.CSA_ERR_ARG
    assert lib.csa_prefill(ctx, p, 100, 2, 1, p, p, p, 1 << 40, None) == binding.CSA_ERR_STATE
    assert lib.csa_prefill(None, p, 100, 2, 1, p, p, p, 1 << 40, None) == binding.CSA_ERR_ARG
    # the clustering calls need no bound buffers, but sane arguments
    assert lib.csa_cluster_queries_minibatch(ctx, p, 100, 2, 0, p, None, p, None, None, p, 1 << 40, None) == binding.CSA_ERR_ARG
    assert lib.csa_cluster_queries_minibatch(ctx, p, 100, 2, 401, p, None, p, None, None, p, 1 << 40, None) == binding.CSA_ERR_ARG
    assert lib.csa_cluster_queries_minibatch(ctx, p, 100, 2, 2, None, None, p, None, None, p, 1 << 40, None) == binding.CSA_ERR_ARG
    assert lib.csa_cluster_queries_minibatch(ctx, p, 100, 2, 2, p, None, p, None, None, p, 16, None) == binding.CSA_ERR_WORKSPACE
    assert lib.csa_cluster_queries(ctx, p, 100, -1, p, None, p, None, None, p, 1 << 40, None) == binding.CSA_ERR_ARG
    need, cap = binding.csa_static_scratch_bytes(ctx)
    assert 0 < need < cap == 32 << 20
    binding.csa_destroy(ctx)
    # a configuration whose step does not fit the static array is refused before anything else
    big = binding.csa_create(**{**GOOD, 'batch': 8, 'n_q_heads': 64, 'n_kv_heads': 8, 'max_ctx': 131072 + 256,
                                'n_centroids': 4096, 'list_len': 4096, 'n_probe': 32, 'budget_k': 6554})
    assert lib.csa_decode_step_static(big, p, p, None, None, None) == binding.CSA_ERR_WORKSPACE
    binding.csa_destroy(big)

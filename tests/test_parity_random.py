"""GPU parity on seeded random configurations: shapes, grids, key-range sizes, paging, streaming
updates and call schedules are drawn at random (from a fixed seed) and every step of every case is
compared with the CPU oracle exactly as in the hand-picked parity tests - probed rows, counts and
selected indices bit for bit, attention outputs within 2e-2, and the tables entry by entry
wherever streaming updates change them."""
import random

import pytest

from harness import Case, small

pytestmark = pytest.mark.gpu


def _check_all_tables(case):
    for b in range(case.w.batch):
        for g in range(case.w.n_kv_heads):
            case.check_tables(b, g)


def _steps_with_random_call_forms(case, rng, steps):
    """Each step through one of the forms of the call: the plain step (its temporaries in the bound
    scratch buffer or in the library's static array) followed by an append, or the one-call iteration
    (plain, or - without streaming updates - the replayable form with the position on the device)."""
    for step in range(steps):
        form = rng.choice(["plain", "static", "fused", "fused", "replayable"])
        if form == "replayable" and case.stream_window:
            form = "fused"
        if form in ("plain", "static"):
            case.check_step(step, static=(form == "static"))
            case.append(1)
        else:
            case.check_step(step, fused_append=True, replayable=(form == "replayable"))


@pytest.mark.parametrize("seed", [11, 12])
def test_random_shapes(seed):
    """Odd group sizes, one to eight subspaces, centroid counts around and below the probe count,
    coarse grids (many equal sums), every key-range size, K from 0 to beyond the candidates; tables
    built by the library or imported from the oracle."""
    rng = random.Random(seed)
    for ci in range(24):
        S = rng.choice([1, 1, 1, 2, 4, 8])
        tau = rng.choice([1, 2, 3, 5]) if S > 1 else rng.choice([1, 2, 4, 7, 16, 32])
        tau = min(tau, 63 // S)
        C = max(rng.choice([tau, tau + 1, 17, 40, 64, 130, 300]), tau)
        G, Hkv, B = rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 12, 16]), rng.choice([1, 2, 3]), rng.choice([1, 1, 2])
        w = small(f"rnd{seed}_{ci}", batch=B, n_q_heads=G * Hkv, n_kv_heads=Hkv,
                  n_pre=rng.choice([300, 1000, 3000, 5003, 9000, 20000]), n_comp=rng.choice([2, 8, 32]), C=C,
                  L=rng.choice([16, 64, 200, 700, 1500]), m=tau, k=rng.choice([0, 1, 10, 100, 333, 1000, 4000]),
                  steps=4, page_size=rng.choice([0, 16]), n_sub=S)
        stream = rng.choice([0, 0, 5])
        case = Case(w, seed=seed * 1000 + ci, F=rng.choice([3, 8, 12]),
                    partition_keys=rng.choice([0, 1024, 2048, 4096, 8192, 16384]), stream_window=stream)
        imported = rng.random() < 0.5
        print(ci, w, "stream", stream, "imported" if imported else "built", flush=True)
        if imported:
            case.import_oracle_tables()     # the oracle's tables through csa_import_tables
        else:
            case.build_on_gpu()
        _check_all_tables(case)
        _steps_with_random_call_forms(case, rng, 4)
        if stream:
            _check_all_tables(case)
        case.ctx.close()


@pytest.mark.parametrize("seed", [21, 22])
def test_random_tiny_shapes(seed):
    """Degenerate sizes: contexts of 1 to 1025 keys, 1 to 64 centroids, lists of 1 to 2000 entries
    (longer than the context), K of 0 to more than there are keys, windows of 1 and 3 keys."""
    rng = random.Random(seed)
    for ci in range(24):
        S = rng.choice([1, 1, 2, 8, 16])
        C = rng.choice([1, 2, 5, 64])
        tau = min(rng.choice([1, 2, 3]), C, 63 // S)
        G, Hkv, B = rng.choice([1, 3, 8]), rng.choice([1, 2]), rng.choice([1, 2])
        w = small(f"tiny{seed}_{ci}", batch=B, n_q_heads=G * Hkv, n_kv_heads=Hkv,
                  n_pre=rng.choice([1, 2, 3, 17, 63, 64, 65, 255, 1023, 1024, 1025]), n_comp=2, C=C,
                  L=rng.choice([1, 2, 16, 300, 2000]), m=tau, k=rng.choice([0, 1, 2, 50, 2000]), steps=5,
                  page_size=rng.choice([0, 16]), n_sub=S)
        stream = rng.choice([0, 1, 3])
        case = Case(w, seed=seed * 1000 + ci, F=rng.choice([2, 10]),
                    partition_keys=rng.choice([0, 1024, 8192, 16384]), stream_window=stream)
        print(ci, w, "stream", stream, flush=True)
        case.build_on_gpu()
        _check_all_tables(case)
        _steps_with_random_call_forms(case, rng, 5)
        _check_all_tables(case)
        case.ctx.close()


@pytest.mark.parametrize("seed", [31, 32])
def test_random_schedules(seed):
    """Searching steps (also through the static-scratch form), search-period steps (the library's copy of
    the index set or the caller's, with or without the append in the same call, also in the replayable
    form) and appends of one or two rows in random order."""
    rng = random.Random(seed)
    for ci in range(20):
        S = rng.choice([1, 1, 2, 8])
        tau = rng.choice([1, 2, 3]) if S > 1 else rng.choice([2, 4, 16])
        C = max(rng.choice([17, 64, 130, 300]), tau)
        G, Hkv, B = rng.choice([1, 2, 4, 8, 12]), rng.choice([1, 2]), rng.choice([1, 2])
        steps = 14
        w = small(f"sched{seed}_{ci}", batch=B, n_q_heads=G * Hkv, n_kv_heads=Hkv,
                  n_pre=rng.choice([40, 300, 3000, 9000, 17000]), n_comp=rng.choice([2, 8]), C=C,
                  L=rng.choice([16, 200, 700]), m=tau, k=rng.choice([1, 10, 100, 1000]), steps=steps,
                  page_size=rng.choice([0, 16]), n_sub=S)
        stream = rng.choice([0, 3, 16])
        case = Case(w, seed=seed * 1000 + ci, F=rng.choice([3, 8, 12]),
                    partition_keys=rng.choice([0, 1024, 4096, 8192]), stream_window=stream)
        case.build_on_gpu()
        sel = cnt = None
        ops = []
        for step in range(steps - 2):
            if case.t >= steps - 2:
                break
            op = rng.choice(["search", "search static", "search+append", "search+append replayable", "reuse",
                             "reuse given", "reuse+append", "reuse+append replayable", "append"])
            if sel is None and op.startswith("reuse"):
                op = "search"
            if stream and op.endswith("replayable"):
                op = op[:-len(" replayable")]
            ops.append(op)
            print(ci, w, "stream", stream, ops, flush=True)
            if op.startswith("search"):
                sel, cnt = case.oracle_index_set(step)
                case.check_step(step, fused_append="+append" in op, static=op.endswith("static"),
                                replayable=op.endswith("replayable"))
            elif op.startswith("reuse"):
                case.check_reuse_step(step, sel, cnt, pass_buffers=(op == "reuse given"),
                                      fused_append="+append" in op, replayable=op.endswith("replayable"))
            else:
                case.append(rng.choice([1, 2]))
        if stream:
            _check_all_tables(case)
        case.ctx.close()

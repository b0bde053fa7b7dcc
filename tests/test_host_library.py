"""Host-side checks of libchunkft (no GPU): exported symbols, the planner
bit for bit against the oracle's planner, and argument validation (every call
made here is rejected before anything could reach a device)."""

import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import chunkft_oracle as O
from paper_2605_21177_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    inc = os.path.join(ROOT, "include")
    header = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    declared = set(re.findall(r"\b(chunkft_[a-z_0-9]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    lib = B.lib()
    for name in declared:
        assert getattr(lib, name) is not None
    assert B.version() >= 100
    assert B.status_string(0) == "ok"
    assert "workspace" in B.status_string(B.ERR_WORKSPACE)


def _oracle_plan(tensors, budget, flags):
    chunks = O.plan_cycle([(r, c, d) for r, c, d, _ in tensors], budget,
                          training_cost=bool(flags & B.PLAN_TRAINING_COST),
                          balanced=bool(flags & B.PLAN_BALANCED), rows8=bool(flags & B.PLAN_ROWS8))
    segs, cks = [], []
    for ch in chunks:
        s0 = len(segs)
        segs += [(s.tensor, s.begin, s.end, s.chunk_off) for s in ch]
        numel = sum(s.end - s.begin for s in ch)
        cost = O.chunk_cost_bytes(ch, [(r, c, d) for r, c, d, _ in tensors],
                                  bool(flags & B.PLAN_TRAINING_COST))
        cks.append((s0, len(segs), numel, cost))
    return cks, segs


def test_planner_matches_oracle_block_configs():
    h, kv, ff = 4096, 1024, 14336
    tensors = [(h, h, 1, 0), (kv, h, 1, 0), (kv, h, 1, 0), (h, h, 1, 0), (ff, h, 1, 0), (ff, h, 1, 0),
               (h, ff, 1, 0), (1, h, 1, 1), (1, h, 1, 1)]
    for budget in (256 << 20, 64 << 20, (100 << 20) + 2, 1 << 20, 12345678):
        for flags in (0, 1, 2, 3, 4, 5, 6, 7):
            if (flags & 6) == 6 and budget < (64 << 20):
                continue        # balanced search in whole groups of rows: many passes of the plain-Python planner
            if flags & 1:
                budget_f = budget * 9
            else:
                budget_f = budget
            st, ck, sg = B.chunkft_plan_cycle(tensors, budget_f, flags)
            assert st == B.OK
            want_ck, want_sg = _oracle_plan(tensors, budget_f, flags)
            assert sg == want_sg
            assert ck == want_ck


def test_planner_matches_oracle_random():
    rng = np.random.default_rng(99)
    for _ in range(300):
        n = int(rng.integers(0, 8))
        tensors = [(int(rng.integers(0, 40)), int(rng.integers(0, 40)), int(rng.integers(0, 2)),
                    int(rng.integers(0, 2))) for _ in range(n)]
        flags = int(rng.integers(0, 8))
        budget = int(rng.integers(20 if flags & 1 else 4, 4000))
        st, ck, sg = B.chunkft_plan_cycle(tensors, budget, flags)
        assert st == B.OK
        want_ck, want_sg = _oracle_plan(tensors, budget, flags)
        assert (ck, sg) == (want_ck, want_sg)


def test_plan_stats_match_the_oracle_and_the_hand_worked_case():
    """chunkft_plan_stats against the oracle's imbalance / jitter / bound (appendix "Analysis of
    Memory Jitter") on planner output, and on the three-chunk case worked by hand under
    tests/golden/.  Floating point on both sides: compared to 1e-12 relative."""
    rng = np.random.default_rng(5)
    for _ in range(200):
        n = int(rng.integers(1, 7))
        tensors = [(int(rng.integers(1, 40)), int(rng.integers(1, 40)), int(rng.integers(0, 2)), 0) for _ in range(n)]
        flags = int(rng.integers(0, 8))
        tc = bool(flags & B.PLAN_TRAINING_COST)
        budget = int(rng.integers(20 if tc else 4, 4000))
        _, ck, _ = B.chunkft_plan_cycle(tensors, budget, flags)
        t3 = [(r, c, d) for r, c, d, _ in tensors]
        want = O.plan_cycle(t3, budget, training_cost=tc, balanced=bool(flags & 2), rows8=bool(flags & 4))
        resident = int(rng.integers(0, 10000))
        got = B.chunkft_plan_stats(ck, resident)
        costs = [O.chunk_cost_bytes(c, t3, tc) for c in want]
        assert got["n_chunks"] == len(want) and got["min_cost_bytes"] == min(costs) and got["max_cost_bytes"] == max(costs)
        np.testing.assert_allclose(got["mean_cost_bytes"], sum(costs) / len(costs), rtol=1e-12)
        np.testing.assert_allclose(got["imbalance_bytes"], O.imbalance(want, t3, tc), rtol=1e-12, atol=1e-9)
        np.testing.assert_allclose(got["jitter"], O.jitter(O.step_memory(want, t3, resident, tc)), rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(got["jitter_bound"], O.jitter_bound(want, t3, resident, tc), rtol=1e-12, atol=1e-15)
        assert got["jitter"] <= got["jitter_bound"] * (1 + 1e-12)
    for row in open(os.path.join(ROOT, "tests", "golden", "jitter_three_chunks_hand_worked.txt")):
        if row.startswith("#") or not row.strip():
            continue
        f = [int(x) for x in row.split()]
        got = B.chunkft_plan_stats([(0, 1, 0, f[1]), (1, 2, 0, f[2]), (2, 3, 0, f[3])], 90)
        assert got["mean_cost_bytes"] == f[4] and got["imbalance_bytes"] == f[5]
        assert got["jitter"] == f[6] / f[7] and got["jitter_bound"] == f[8] / f[9]
    assert B.chunkft_plan_stats([], 0, check=False) == B.ERR_INVALID_ARG
    assert B.chunkft_plan_stats([(0, 1, 1, 2)], -1, check=False) == B.ERR_INVALID_ARG
    assert B.chunkft_plan_stats([(0, 1, 1, -2)], 0, check=False) == B.ERR_INVALID_ARG
    lib = B.lib()
    assert lib.chunkft_plan_stats(None, 1, 0, C.byref(B.PlanSummary())) == B.ERR_INVALID_ARG
    assert lib.chunkft_plan_stats((B.Chunk * 1)(), 1, 0, None) == B.ERR_INVALID_ARG


def test_bench_plan_sweep_reports_the_oracle_numbers():
    """bench.py --plan-sweep on a small tensor list: every row's chunk count, imbalance, jitter and
    bound equal what the oracle's planner and its jitter functions give for the same budget."""
    import bench
    tensors = [(50, 16, B.BF16, B.EMBEDDING), (1, 16, B.BF16, B.RMSNORM), (16, 16, B.BF16, B.LINEAR),
               (40, 16, B.F32, B.LINEAR), (16, 40, B.BF16, B.LINEAR), (1, 16, B.BF16, B.RMSNORM), (50, 16, B.BF16, B.LINEAR)]
    groups = [[0], [1, 2, 3, 4], [5, 6]]
    budgets = [("a", 9000), ("b", 20001), ("c", 3 * 18 * 128)]
    out = bench.plan_sweep(B, tensors, groups, budgets)
    t3 = [(r, c, d) for r, c, d, _ in tensors]
    resident = sum(r * c * (4 if d == B.F32 else 2) for r, c, d in t3)
    rows = iter(out["rows"])
    for _, budget in budgets:
        for kw in (dict(), dict(balanced=True), dict(rows8=True)):
            want = O.plan_cycle(t3, budget, training_cost=True, **kw)
            row = next(rows)
            assert row["chunks"] == len(want)
            assert row["max_cost_bytes"] == max(O.chunk_cost_bytes(c, t3, True) for c in want)
            np.testing.assert_allclose(row["imbalance_bytes"], O.imbalance(want, t3, True), rtol=1e-12, atol=1e-9)
            np.testing.assert_allclose(row["jitter"], O.jitter(O.step_memory(want, t3, resident, True)), rtol=1e-12, atol=1e-15)
            np.testing.assert_allclose(row["jitter_bound"], O.jitter_bound(want, t3, resident, True), rtol=1e-12, atol=1e-15)
    # the layer-wise partition: one "chunk" per group of tensors, whole tensors only
    by_layer = [[O.Segment(t, 0, t3[t][0] * t3[t][1], 0) for t in grp] for grp in groups]
    row = next(rows)
    assert row["chunks"] == 3
    np.testing.assert_allclose(row["imbalance_bytes"], O.imbalance(by_layer, t3, True), rtol=1e-12)
    np.testing.assert_allclose(row["jitter"], O.jitter(O.step_memory(by_layer, t3, resident, True)), rtol=1e-12)


def test_balanced_search_is_quick_where_cuts_fall_between_row_groups():
    """Balanced + row groups on the Llama-3-8B block: two candidate capacities can lie a whole group of
    rows (megabytes) apart; the search skips the capacities that cannot change the plan instead of
    trying each multiple of 4 bytes.  The result is still the first capacity (in steps of 4 bytes from
    ceil(total / K)) that needs no more than K chunks: checked against a direct scan of the last
    kilobyte before it."""
    import time
    h, kv, ff = 4096, 1024, 14336
    tensors = [(h, h, 1, 0), (kv, h, 1, 0), (kv, h, 1, 0), (h, h, 1, 0), (ff, h, 1, 0), (ff, h, 1, 0),
               (h, ff, 1, 0), (1, h, 1, 1), (1, h, 1, 1)]
    for budget in (12345678, (100 << 20) + 2, 9 * 12345678):
        flags = B.PLAN_BALANCED | B.PLAN_ROWS8 | (B.PLAN_TRAINING_COST if budget > (1 << 27) else 0)
        t0 = time.perf_counter()
        _, ck, sg = B.chunkft_plan_cycle(tensors, budget, flags)
        assert time.perf_counter() - t0 < 2.0
        _, ck0, _ = B.chunkft_plan_cycle(tensors, budget, flags & ~B.PLAN_BALANCED)
        assert len(ck) <= len(ck0) and all(c[3] <= budget for c in ck)
        cap = max(c[3] for c in ck)
        # the plan is the greedy plan of some capacity b >= cap; no capacity in the kilobyte below cap
        # (same residue mod 4 as the search's candidates or not) manages with as few chunks
        for b in range(max(cap - 1024, 20), cap):
            _, ckb, _ = B.chunkft_plan_cycle(tensors, b, flags & ~B.PLAN_BALANCED)
            assert len(ckb) > len(ck0) or max(c[3] for c in ckb) >= cap or len(ckb) > len(ck)


def test_planner_count_then_fill_and_errors():
    lib = B.lib()
    arr = (B.TensorDesc * 2)(B.TensorDesc(10, 10, 1, 0), B.TensorDesc(1, 7, 0, 1))
    nc, ns = C.c_int64(-1), C.c_int64(-1)
    # size query
    st = lib.chunkft_plan_cycle(arr, 2, 64, 0, None, 0, C.byref(nc), None, 0, C.byref(ns))
    assert st == B.ERR_BUFFER_TOO_SMALL
    want = O.plan_cycle([(10, 10, 1), (1, 7, 0)], 64)
    assert nc.value == len(want) and ns.value == sum(len(c) for c in want)
    # short arrays are left untouched
    chunks = (B.Chunk * 1)()
    chunks[0].numel = -77
    segs = (B.Segment * 1)()
    st = lib.chunkft_plan_cycle(arr, 2, 64, 0, chunks, 1, C.byref(nc), segs, 1, C.byref(ns))
    assert st == B.ERR_BUFFER_TOO_SMALL and chunks[0].numel == -77
    # errors
    assert lib.chunkft_plan_cycle(arr, 2, 64, 0, None, 0, None, None, 0, C.byref(ns)) == B.ERR_INVALID_ARG
    assert lib.chunkft_plan_cycle(arr, 2, 0, 0, None, 0, C.byref(nc), None, 0, C.byref(ns)) == B.ERR_INVALID_ARG
    assert lib.chunkft_plan_cycle(arr, 2, 3, 0, None, 0, C.byref(nc), None, 0, C.byref(ns)) == B.ERR_INVALID_ARG  # < 4 B fp32
    assert lib.chunkft_plan_cycle(arr, 2, 64, 8, None, 0, C.byref(nc), None, 0, C.byref(ns)) == B.ERR_INVALID_ARG  # unknown flag
    assert lib.chunkft_plan_cycle(arr, 2, 64, 16, None, 0, C.byref(nc), None, 0, C.byref(ns)) == B.ERR_INVALID_ARG
    assert lib.chunkft_plan_cycle(None, 2, 64, 0, None, 0, C.byref(nc), None, 0, C.byref(ns)) == B.ERR_INVALID_ARG
    bad = (B.TensorDesc * 1)(B.TensorDesc(10, 10, 5, 0))
    assert lib.chunkft_plan_cycle(bad, 1, 64, 0, None, 0, C.byref(nc), None, 0, C.byref(ns)) == B.ERR_DTYPE
    neg = (B.TensorDesc * 1)(B.TensorDesc(-1, 10, 1, 0))
    assert lib.chunkft_plan_cycle(neg, 1, 64, 0, None, 0, C.byref(nc), None, 0, C.byref(ns)) == B.ERR_INVALID_ARG
    big = (B.TensorDesc * 1)(B.TensorDesc(1 << 40, 1 << 40, 1, 0))
    assert lib.chunkft_plan_cycle(big, 1, 64, 0, None, 0, C.byref(nc), None, 0, C.byref(ns)) == B.ERR_OVERFLOW
    # empty list and zero-sized tensors
    assert lib.chunkft_plan_cycle(None, 0, 64, 0, None, 0, C.byref(nc), None, 0, C.byref(ns)) == B.OK
    assert nc.value == 0 and ns.value == 0
    st, ck, sg = B.chunkft_plan_cycle([(0, 5, 1, 0), (3, 0, 0, 0)], 64)
    assert (st, ck, sg) == (B.OK, [], [])


def test_planner_rows8_block_boundaries_fall_on_rows_that_are_multiples_of_8():
    """The Llama-3-8B block under budgets that force mid-tensor cuts: with the option every segment of a
    matrix begins and ends on a row that is a multiple of 8 (or at an end of the tensor)."""
    h, kv, ff = 4096, 1024, 14336
    tensors = [(h, h, 1, 0), (kv, h, 1, 0), (kv, h, 1, 0), (h, h, 1, 0), (ff, h, 1, 0), (ff, h, 1, 0),
               (h, ff, 1, 0), (1, h, 1, 1), (1, h, 1, 1)]
    for budget in ((100 << 20) + 2, 12345678, 64 << 20):
        st, ck, sg = B.chunkft_plan_cycle(tensors, budget, B.PLAN_ROWS8)
        assert st == B.OK
        st0, ck0, sg0 = B.chunkft_plan_cycle(tensors, budget, 0)
        assert len(ck) in (len(ck0), len(ck0) + 1)        # at most one group per chunk is given up
        for t, b, e, _ in sg:
            r, c = tensors[t][0], tensors[t][1]
            assert b % (8 * c) == 0 and (e % (8 * c) == 0 or e == r * c)
        for _, _, numel, cost in ck:
            assert cost <= budget and cost == 2 * numel
    # a size query with astronomically many chunks is counted in one step with the option too:
    # 2^40 rows x 1024 bf16 under 1 MiB + 100 B: 64 groups of 8 rows = 2^19 elements per chunk
    lib = B.lib()
    t = (B.TensorDesc * 1)(B.TensorDesc(1 << 40, 1 << 10, B.BF16, B.LINEAR))
    nc, ns = C.c_int64(-1), C.c_int64(-1)
    st = lib.chunkft_plan_cycle(t, 1, (1 << 20) + 100, B.PLAN_ROWS8, None, 0, C.byref(nc), None, 0, C.byref(ns))
    assert st == B.ERR_BUFFER_TOO_SMALL and nc.value == ns.value == (1 << 50) >> 19


def test_planner_large_counts_near_int64():
    # 2^31 x 2^31 bf16 = 2^63 bytes does not fit; 2^30 x 2^31 does (2^62 bytes)
    st, ck, sg = B.chunkft_plan_cycle([(1 << 30, 1 << 31, 1, 0)], 1 << 61)
    assert st == B.OK and len(ck) == 2 and ck[0][2] == 1 << 60
    st, _, _ = B.chunkft_plan_cycle([(1 << 31, 1 << 31, 1, 0)], 1 << 61, check=False)
    assert st == B.ERR_OVERFLOW


# fake non-null addresses: every call below must be rejected by validation
P = 0x1000


def _layer(**kw):
    d = dict(kind=B.LINEAR, dtype=B.BF16, out=64, n_in=32, T=16, X=P, ldx=32, dY=P, lddy=64, split_k=0,
             reserved=0, norm_eps=0.0)
    d.update(kw)
    return B.Layer(**d)


def test_device_calls_reject_bad_arguments_without_launching():
    lib = B.lib()
    hp = B.hparams(1e-4, 0.9, 0.999, 1e-8, 0.01, 1)
    cases = [
        (_layer(X=None), 0, 10, B.ERR_INVALID_ARG),
        (_layer(T=0), 0, 10, B.ERR_INVALID_ARG),
        (_layer(T=(1 << 30) + 1), 0, 10, B.ERR_INVALID_ARG),
        (_layer(ldx=31), 0, 10, B.ERR_INVALID_ARG),
        (_layer(lddy=63), 0, 10, B.ERR_INVALID_ARG),
        (_layer(dtype=7), 0, 10, B.ERR_DTYPE),
        (_layer(kind=5), 0, 10, B.ERR_DTYPE),
        (_layer(kind=-1), 0, 10, B.ERR_DTYPE),
        (_layer(kind=B.EMBEDDING, X=P + 4, lddy=32), 0, 10, B.ERR_INVALID_ARG),     # ids are int64
        (_layer(kind=B.EMBEDDING, lddy=31), 0, 10, B.ERR_INVALID_ARG),
        (_layer(kind=B.EMBEDDING, lddy=32, split_k=2), 0, 10, B.ERR_INVALID_ARG),
        (_layer(kind=B.EMBEDDING, lddy=32, T=8193), 0, 10, B.ERR_INVALID_ARG),            # too many tokens per call
        (_layer(kind=B.RMSNORM, out=2, lddy=32), 0, 10, B.ERR_INVALID_ARG),
        (_layer(kind=B.RMSNORM, out=1, lddy=32, norm_eps=-1e-6), 0, 10, B.ERR_INVALID_ARG),
        (_layer(kind=B.LAYERNORM, out=1, lddy=32, norm_eps=float("nan")), 0, 10, B.ERR_INVALID_ARG),
        (_layer(split_k=65), 0, 10, B.ERR_INVALID_ARG),
        (_layer(reserved=1), 0, 10, B.ERR_INVALID_ARG),
        (_layer(kind=B.VECTOR, out=2), 0, 10, B.ERR_INVALID_ARG),
        (_layer(X=P + 1), 0, 10, B.ERR_INVALID_ARG),
        (_layer(), 10, 10, B.ERR_RANGE),
        (_layer(), -1, 10, B.ERR_RANGE),
        (_layer(), 0, 64 * 32 + 1, B.ERR_RANGE),
        (_layer(out=1 << 40, n_in=1 << 40, ldx=1 << 40, lddy=1 << 40), 0, 10, B.ERR_OVERFLOW),
    ]
    for layer, b, e, want in cases:
        assert lib.chunkft_chunk_wgrad(C.byref(layer), b, e, P, 0, None, 0, None) == want
        assert lib.chunkft_wgrad_adamw_fused(C.byref(layer), b, e, P, P, P, P, C.byref(hp), None, 0, None) == want
        assert lib.chunkft_split_k(C.byref(layer), b, e) == want
        assert lib.chunkft_workspace_bytes(C.byref(layer), b, e) == 0
    ok = _layer()
    assert lib.chunkft_chunk_wgrad(C.byref(ok), 0, 10, None, 0, None, 0, None) == B.ERR_INVALID_ARG
    assert lib.chunkft_chunk_wgrad(C.byref(ok), 0, 10, P, 2, None, 0, None) == B.ERR_INVALID_ARG
    assert lib.chunkft_wgrad_adamw_fused(C.byref(ok), 0, 10, P, None, P, P, C.byref(hp), None, 0, None) == B.ERR_INVALID_ARG
    assert lib.chunkft_wgrad_adamw_fused(C.byref(ok), 0, 10, P, P, P, P, None, None, 0, None) == B.ERR_INVALID_ARG
    # forced split without (enough) workspace
    sp = _layer(T=64, split_k=2)
    assert lib.chunkft_split_k(C.byref(sp), 0, 100) == 2
    assert lib.chunkft_workspace_bytes(C.byref(sp), 0, 100) == (2 * 128 + 32) * 4     # slabs of 100 -> 128 elements
    assert lib.chunkft_chunk_wgrad(C.byref(sp), 0, 100, P, 0, None, 0, None) == B.ERR_WORKSPACE
    assert lib.chunkft_chunk_wgrad(C.byref(sp), 0, 100, P, 0, P, 1151, None) == B.ERR_WORKSPACE
    assert lib.chunkft_chunk_wgrad(C.byref(sp), 0, 100, P, 0, P + 4, 1152, None) == B.ERR_WORKSPACE
    assert lib.chunkft_wgrad_adamw_fused(C.byref(sp), 0, 100, P, P, P, P, C.byref(hp), None, 0, None) == B.ERR_WORKSPACE
    # the self-normalising kinds need 8 bytes per token for the statistics
    nm = _layer(kind=B.RMSNORM, out=1, lddy=32, norm_eps=1e-6)
    assert lib.chunkft_workspace_bytes(C.byref(nm), 0, 32) == 16 * 8
    assert lib.chunkft_chunk_wgrad(C.byref(nm), 0, 32, P, 0, None, 0, None) == B.ERR_WORKSPACE
    assert lib.chunkft_chunk_wgrad(C.byref(nm), 0, 32, P, 0, P, 127, None) == B.ERR_WORKSPACE
    assert lib.chunkft_wgrad_adamw_fused(C.byref(nm), 0, 32, P, P, P, P, C.byref(hp), None, 0, None) == B.ERR_WORKSPACE
    # AdamW hyper-parameters and sizes
    for bad in (B.hparams(1e-4, 0.9, 0.999, 1e-8, 0.01, 0), B.hparams(1e-4, 1.0, 0.999, 1e-8, 0.01, 1),
                B.hparams(1e-4, 0.9, -0.1, 1e-8, 0.01, 1), B.hparams(-1.0, 0.9, 0.999, 1e-8, 0.01, 1),
                B.hparams(float("nan"), 0.9, 0.999, 1e-8, 0.01, 1)):
        assert lib.chunkft_adamw_chunk(P, P, P, P, P, B.BF16, 10, C.byref(bad), None) == B.ERR_INVALID_ARG
    assert lib.chunkft_adamw_chunk(None, P, P, P, P, B.BF16, 10, C.byref(hp), None) == B.ERR_INVALID_ARG
    assert lib.chunkft_adamw_chunk(P, P, P, P, P, B.BF16, 0, C.byref(hp), None) == B.ERR_INVALID_ARG
    assert lib.chunkft_adamw_chunk(P, P, P, P, P, 9, 10, C.byref(hp), None) == B.ERR_DTYPE
    assert lib.chunkft_adamw_chunk(P + 2, P, P, P, P, B.BF16, 10, C.byref(hp), None) == B.ERR_INVALID_ARG
    assert lib.chunkft_adamw_chunk(P, P, P, P, P + 1, B.BF16, 10, C.byref(hp), None) == B.ERR_INVALID_ARG


def test_grouped_call_rejects_bad_arguments_without_launching():
    lib = B.lib()
    hp = B.hparams(1e-4, 0.9, 0.999, 1e-8, 0.01, 1)

    def seg(layer, b, e, W=P, master=P, m=P, v=P):
        return B.GroupSegment(layer, b, e, W, master, m, v)

    good = seg(_layer(), 0, 100)
    cases = [
        ([seg(_layer(T=0), 0, 10)], B.ERR_INVALID_ARG),
        ([good, seg(_layer(dtype=7), 0, 10)], B.ERR_DTYPE),
        ([good, seg(_layer(), 10, 10)], B.ERR_RANGE),
        ([good, seg(_layer(), 0, 10, master=None)], B.ERR_INVALID_ARG),
        ([good, seg(_layer(), 0, 10, m=P + 2)], B.ERR_INVALID_ARG),
        ([seg(_layer(T=64, split_k=2), 0, 100)], B.ERR_WORKSPACE),         # a forced split needs a workspace
        ([seg(_layer(kind=B.RMSNORM, out=1, lddy=32, norm_eps=1e-6), 0, 32)], B.ERR_WORKSPACE),
    ]
    for segs, want in cases:
        arr = (B.GroupSegment * len(segs))(*segs)
        assert lib.chunkft_wgrad_adamw_fused_group(arr, len(segs), C.byref(hp), None, 0, None) == want
    arr = (B.GroupSegment * 1)(good)
    assert lib.chunkft_wgrad_adamw_fused_group(None, 1, C.byref(hp), None, 0, None) == B.ERR_INVALID_ARG
    assert lib.chunkft_wgrad_adamw_fused_group(arr, 0, C.byref(hp), None, 0, None) == B.ERR_INVALID_ARG
    assert lib.chunkft_wgrad_adamw_fused_group(arr, 4097, C.byref(hp), None, 0, None) == B.ERR_INVALID_ARG
    assert lib.chunkft_wgrad_adamw_fused_group(arr, 1, None, None, 0, None) == B.ERR_INVALID_ARG
    bad = B.hparams(1e-4, 0.9, 0.999, 1e-8, 0.01, 0)
    assert lib.chunkft_wgrad_adamw_fused_group(arr, 1, C.byref(bad), None, 0, None) == B.ERR_INVALID_ARG
    # workspace: the largest need among the segments that run by themselves; none when the kernel takes all
    forced = seg(_layer(T=64, split_k=2), 0, 100)
    norm = seg(_layer(kind=B.RMSNORM, out=1, lddy=32, norm_eps=1e-6), 0, 32)
    assert lib.chunkft_group_workspace_bytes((B.GroupSegment * 1)(forced), 1) == (2 * 128 + 32) * 4
    assert lib.chunkft_group_workspace_bytes((B.GroupSegment * 2)(forced, norm), 2) == (2 * 128 + 32) * 4
    assert lib.chunkft_group_workspace_bytes((B.GroupSegment * 1)(norm), 1) == 16 * 8
    big = _layer(out=14336, n_in=4096, T=1024, ldx=4096, lddy=14336)
    vec = _layer(kind=B.VECTOR, out=1, n_in=4096, T=1024, ldx=4096, lddy=4096)
    kv = _layer(out=1024, n_in=4096, T=8192, ldx=4096, lddy=1024)
    whole = (B.GroupSegment * 3)(seg(big, 4097, 4097 + (32 << 20)), seg(vec, 0, 4096), seg(kv, 0, 1024 * 4096))
    assert lib.chunkft_group_workspace_bytes(whole, 3) == 0
    # by itself the k projection at 8192 tokens is split into three slabs and needs their workspace
    alone = (B.GroupSegment * 1)(seg(kv, 0, 1024 * 4096))
    assert lib.chunkft_group_workspace_bytes(alone, 1) == (3 * 1024 * 4096 + 32) * 4
    assert lib.chunkft_group_workspace_bytes(None, 1) == 0


def test_split_is_a_pure_function_of_shape():
    lib = B.lib()
    # 8B up_proj chunk: many tiles, no split
    big = _layer(out=14336, n_in=4096, T=1024, ldx=4096, lddy=14336)
    assert lib.chunkft_split_k(C.byref(big), 4097, 4097 + (32 << 20)) == 1
    # a 2 Mi-element chunk of the lm_head shape at T = 4096: few tiles, split over tokens
    small = _layer(out=128256, n_in=4096, T=4096, ldx=4096, lddy=128256)
    s = lib.chunkft_split_k(C.byref(small), 12345, 12345 + (2 << 20))
    assert 2 <= s <= 64
    assert lib.chunkft_split_k(C.byref(small), 12345, 12345 + (2 << 20)) == s
    assert lib.chunkft_workspace_bytes(C.byref(small), 12345, 12345 + (2 << 20)) == (s * (2 << 20) + 32) * 4
    # a whole k / v projection at T = 1024: 64 tiles, but too few tokens for a split to pay
    kv = _layer(out=1024, n_in=4096, T=1024, ldx=4096, lddy=1024)
    assert lib.chunkft_split_k(C.byref(kv), 0, 1024 * 4096) == 1
    kv8 = _layer(out=1024, n_in=4096, T=8192, ldx=4096, lddy=1024)
    assert lib.chunkft_split_k(C.byref(kv8), 0, 1024 * 4096) == 3       # floor(sqrt(8192 / (12 * 64)))
    # no slab is empty: forcing more slabs than tokens allow is reduced
    tiny = _layer(T=40, split_k=8)
    assert lib.chunkft_split_k(C.byref(tiny), 0, 100) == 2      # slabs are whole 32-token tiles: 32 + 8


def test_autograd_segment_argument_checks():
    """The host side of the autograd wrapper: a segment names either a gradient buffer or a
    complete chunk state, and an empty segment needs neither."""
    from paper_2605_21177_amd import autograd as A
    import torch
    buf = torch.zeros(8)
    hp = B.hparams(1e-4, 0.9, 0.999, 1e-8, 0.01, 1)
    assert A.ChunkSegment(0, 0).fused is False                     # tensor not in the active chunk
    assert A.ChunkSegment(2, 10, buf).fused is False
    assert A.ChunkSegment(2, 10, master=buf, m=buf, v=buf, hp=hp).fused is True
    for bad in (dict(begin=5, end=3), dict(begin=-1, end=3), dict(begin=0, end=8),
                dict(begin=0, end=8, master=buf), dict(begin=0, end=8, g=buf, master=buf, m=buf, v=buf, hp=hp)):
        with pytest.raises(ValueError):
            A.ChunkSegment(bad.pop("begin"), bad.pop("end"), bad.pop("g", None), **bad)
    seg = A.ChunkSegment(2, 10, buf)
    seg.micro_batches = 3
    seg.reset()
    assert seg.micro_batches == 0
    with pytest.raises(ValueError):
        A.chunk_linear(torch.zeros(2, 4), torch.zeros(3, 4, requires_grad=True), None)


def test_bench_refuses_more_than_one_gpu():
    """The path has no collective: bench.py --gpus N with N > 1 exits with a message, before any GPU work."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2605_21177_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.replace("no fallback", ""), f


def test_calibration_call_validates_before_touching_the_device():
    import ctypes as C
    lib = B.lib()
    tf, mhz = C.c_double(0.0), C.c_double(0.0)
    bad = [(1, 0), (1, 6), (1, -4), (0, (1 << 20) + 4)]
    for rnd, steps in bad:
        assert lib.chunkft_calib_mfma_bf16(rnd, steps, P, 4096, C.byref(tf), C.byref(mhz), None) == B.ERR_INVALID_ARG
    assert lib.chunkft_calib_mfma_bf16(1, 8, P, 4096, None, C.byref(mhz), None) == B.ERR_INVALID_ARG
    for shape in (0, 8, 64, -16):        # only the two bf16 MFMA shapes exist
        assert lib.chunkft_calib_mfma_bf16_shape(shape, 1, 8, P, 4096, C.byref(tf), C.byref(mhz), None) == B.ERR_INVALID_ARG
    for shape in (16, 32):
        assert lib.chunkft_calib_mfma_bf16_shape(shape, 1, 6, P, 4096, C.byref(tf), C.byref(mhz), None) == B.ERR_INVALID_ARG
        assert lib.chunkft_calib_mfma_bf16_shape(shape, 1, 8, P, 4096, C.byref(tf), None, None) == B.ERR_INVALID_ARG
        # the scratch is the caller's: missing, short or misaligned is refused (nothing is allocated here)
        assert lib.chunkft_calib_mfma_bf16_shape(shape, 1, 8, None, 4096, C.byref(tf), C.byref(mhz), None) == B.ERR_WORKSPACE
        assert lib.chunkft_calib_mfma_bf16_shape(shape, 1, 8, P, 4095, C.byref(tf), C.byref(mhz), None) == B.ERR_WORKSPACE
        assert lib.chunkft_calib_mfma_bf16_shape(shape, 1, 8, P + 8, 4096, C.byref(tf), C.byref(mhz), None) == B.ERR_WORKSPACE


def test_no_source_of_the_library_allocates_device_memory():
    """Ownership rule of include/chunkft.h: every device buffer is the caller's."""
    csrc = os.path.join(ROOT, "paper_2605_21177_amd", "csrc")
    for f in os.listdir(csrc):
        text = open(os.path.join(csrc, f)).read()
        for call in ("hipMalloc", "hipFree", "hipMallocAsync", "hipExtMallocWithFlags", "hipHostMalloc", "hipMallocManaged"):
            assert call + "(" not in text, (f, call)


def test_schedule_matches_the_simulated_algorithm():
    for K, H in ((1, 1), (1, 4), (2, 1), (3, 2), (5, 3), (7, 10)):
        ref = O.rotating_schedule(4 * K * H + 3, K, H)
        for t, want in enumerate(ref):
            assert B.chunkft_schedule_at(t, K, H) == want
    # far into training, values stay exact
    big = 10 ** 15
    k, load, off, n = B.chunkft_schedule_at(big, 7, 1000)
    assert k == (big // 1000) % 7 and n == (big // 7000) * 1000 + big % 1000 + 1
    assert B.chunkft_schedule_at((1 << 62), 3, (1 << 62))[3] == 1
    for bad in ((-1, 3, 2), (0, 0, 2), (0, 3, 0)):
        assert B.chunkft_schedule_at(*bad, check=False) == B.ERR_INVALID_ARG


def test_mover_null_handling_without_a_device():
    lib = B.lib()
    lib.chunkft_mover_destroy(None)                                   # allowed
    assert lib.chunkft_mover_create(None) == B.ERR_INVALID_ARG
    assert lib.chunkft_mover_sync(None) == B.ERR_INVALID_ARG
    assert lib.chunkft_mover_await_load(None, None) == B.ERR_INVALID_ARG
    assert lib.chunkft_mover_load(None, P, P, P, P, P, P, 4, None) == B.ERR_INVALID_ARG
    assert lib.chunkft_mover_offload(None, P, P, P, P, P, P, 4, None) == B.ERR_INVALID_ARG


def test_plan_counts_astronomic_chunk_numbers_at_once():
    """A size query for a 2^60-element tensor under a 100-byte budget returns the count
    (the closed form for one dtype) instead of walking 2^55 chunks."""
    import ctypes as C
    lib = B.lib()
    t = (B.TensorDesc * 2)(B.TensorDesc(1 << 40, 1 << 20, B.BF16, B.LINEAR), B.TensorDesc(3, 7, B.BF16, B.LINEAR))
    nc, ns = C.c_int64(-1), C.c_int64(-1)
    st = lib.chunkft_plan_cycle(t, 2, 100, 0, None, 0, C.byref(nc), None, 0, C.byref(ns))
    assert st == B.ERR_BUFFER_TOO_SMALL
    total = (1 << 60) + 21
    assert nc.value == -(-total // 50)
    # the first tensor ends a chunk exactly (2^60 is not a multiple of 50: 2^60 % 50 = 26 elements in
    # its last chunk, which the 21 elements of the second tensor join)
    assert ns.value == -(-(1 << 60) // 50) + 1


def test_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """plan.cpp, api.cpp and shape.cpp built for the CPU with -fsanitize=address,undefined and driven
    by tests/host_sanitize.cpp: random plans (count-then-fill, coverage, budgets near int64), plan
    summaries, schedules, and a few hundred thousand device-call argument sets whose launches are
    replaced by host-side checks of what the kernels would have been given."""
    import shutil
    import subprocess
    gxx = shutil.which("g++")
    assert gxx, "g++ is part of the image"
    csrc = os.path.join(ROOT, "paper_2605_21177_amd", "csrc")
    exe = str(tmp_path / "host_sanitize")
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-I", os.path.join(ROOT, "include"), "-I", csrc,
           os.path.join(ROOT, "tests", "host_sanitize.cpp")]
    cmd += [os.path.join(csrc, f) for f in ("plan.cpp", "api.cpp", "shape.cpp")] + ["-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0 and r.stdout.startswith("ok:"), (r.stdout[-1000:], r.stderr[-3000:])

"""Pins of the CPU oracle against things other than itself (no GPU).

Each block states what fixes the expected value: brute force, a closed form
derived from the paper's equations, a special case with a textbook answer, a
library routine, or a hand-worked fixture under tests/golden/.
"""

import itertools
import os

import numpy as np
import pytest
import torch

from oracle import chunkft_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    out = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                out.append(line.split())
    return out


# ------------------------------------------------------------------ planner
def _check_partition(tensors, chunks):
    """Section 3.2: the chunks are a disjoint partition of all elements."""
    per_tensor = {}
    for ch in chunks:
        off = 0
        for s in ch:
            assert s.begin < s.end
            assert s.chunk_off == off
            off += s.end - s.begin
            per_tensor.setdefault(s.tensor, []).append((s.begin, s.end))
    for t, (r, c, _) in enumerate(tensors):
        segs = per_tensor.get(t, [])
        # emitted in order, so no sort: order itself is part of the contract
        pos = 0
        for b, e in segs:
            assert b == pos
            pos = e
        assert pos == r * c


def test_plan_block_golden():
    h, kv, ff = 4096, 1024, 14336
    tensors = [(h, h, O.BF16), (kv, h, O.BF16), (kv, h, O.BF16), (h, h, O.BF16),
               (ff, h, O.BF16), (ff, h, O.BF16), (h, ff, O.BF16), (1, h, O.BF16), (1, h, O.BF16)]
    chunks = O.plan_cycle(tensors, 256 << 20)
    got = [(k, s.tensor, s.begin, s.end, s.chunk_off) for k, ch in enumerate(chunks) for s in ch]
    want = [tuple(int(x) for x in row) for row in _rows("plan_block_256MiB.txt")]
    assert got == want
    _check_partition(tensors, chunks)


def test_plan_mixed_dtype_golden():
    tensors = [(1, 3, O.BF16), (1, 2, O.F32)]
    chunks = O.plan_cycle(tensors, 7)
    got = [(k, s.tensor, s.begin, s.end, s.chunk_off) for k, ch in enumerate(chunks) for s in ch]
    want = [tuple(int(x) for x in row) for row in _rows("plan_mixed_dtype.txt")]
    assert got == want


def test_plan_uniform_closed_form_all_budgets():
    """Uniform dtype, budget a multiple of the element size: element with global
    index G (tensors concatenated in order) lies in chunk G // (budget / size)."""
    tensors = [(3, 5, O.BF16), (1, 7, O.BF16), (4, 2, O.BF16)]
    total = sum(r * c for r, c, _ in tensors)
    starts = np.cumsum([0] + [r * c for r, c, _ in tensors])
    for cap in range(1, total + 3):
        for slack in (0, 1):   # an odd byte left over changes nothing for 2-byte elements
            chunks = O.plan_cycle(tensors, 2 * cap + slack)
            _check_partition(tensors, chunks)
            assert len(chunks) == -(-total // cap)
            for k, ch in enumerate(chunks):
                for s in ch:
                    G = starts[s.tensor] + np.arange(s.begin, s.end)
                    assert np.all(G // cap == k)
                    assert s.chunk_off == G[0] - k * cap


def test_plan_random_invariants():
    rng = np.random.default_rng(7)
    for _ in range(200):
        n = int(rng.integers(1, 7))
        tensors = [(int(rng.integers(0, 9)), int(rng.integers(0, 9)), int(rng.integers(0, 2)))
                   for _ in range(n)]
        budget = int(rng.integers(4, 120))
        for tc in (False, True):
            if tc and budget < 20:
                continue
            chunks = O.plan_cycle(tensors, budget, training_cost=tc)
            _check_partition(tensors, chunks)
            for ch in chunks:
                assert 0 < O.chunk_cost_bytes(ch, tensors, tc) <= budget
            # greedy: a chunk is closed only when the next element does not fit
            for k in range(len(chunks) - 1):
                nxt = chunks[k + 1][0]
                s = 4 if tensors[nxt.tensor][2] == O.F32 else 2
                s += 16 if tc else 0
                assert O.chunk_cost_bytes(chunks[k], tensors, tc) + s > budget


def test_plan_training_cost_scales_budget():
    """bf16 only: charging 18 B/element with budget 9*B gives the same split as
    charging 2 B/element with budget B (Section 3.1 vs Section 3 cost)."""
    tensors = [(5, 6, O.BF16), (2, 9, O.BF16), (7, 3, O.BF16)]
    for cap in range(1, 40):
        a = O.plan_cycle(tensors, 2 * cap)
        b = O.plan_cycle(tensors, 18 * cap, training_cost=True)
        assert a == b


def test_imbalance_and_jitter_hand_worked():
    """Appendix "Analysis of Memory Jitter": eps_B, the step memory 2M + B(C_k), the jitter
    ratio and its bound on a three-chunk plan whose numbers are worked by hand in the fixture.
    max - min (50) or the deviation from the median (40) instead of eps_B = 30 fail here."""
    tensors = [(1, 45, O.BF16)]
    chunks = [[O.Segment(0, 0, 5, 0)], [O.Segment(0, 5, 15, 0)], [O.Segment(0, 15, 45, 0)]]
    _check_partition(tensors, chunks)
    resident = 2 * 45
    for row in _rows("jitter_three_chunks_hand_worked.txt"):
        tc = bool(int(row[0]))
        b = [int(x) for x in row[1:4]]
        mean, eps, jn, jd, bn, bd = (int(x) for x in row[4:10])
        assert [O.chunk_cost_bytes(c, tensors, tc) for c in chunks] == b
        assert O.imbalance(chunks, tensors, tc) == float(eps)
        mem = O.step_memory(chunks, tensors, resident, tc)
        assert mem == [float(resident + x) for x in b] and sum(mem) / 3 == jd
        assert O.jitter(mem) == jn / jd
        assert O.jitter_bound(chunks, tensors, resident, tc) == bn / bd
    # a single chunk and equal chunks have no imbalance
    assert O.imbalance(chunks[:1], tensors) == 0.0
    assert O.imbalance([[O.Segment(0, 0, 15, 0)], [O.Segment(0, 15, 30, 0)], [O.Segment(0, 30, 45, 0)]], tensors) == 0.0


def test_jitter_never_exceeds_the_appendix_bound_on_planner_output():
    """max_k M_k - min_k M_k <= 2 eps_B for M_k = 2M + B(C_k), so the jitter of a plan stays
    below 2 eps_B / (2M + mean B) (last equation of the appendix); equality when the largest
    and the smallest chunk lie equally far from the mean."""
    rng = np.random.default_rng(23)
    for _ in range(200):
        n = int(rng.integers(1, 6))
        tensors = [(int(rng.integers(1, 30)), int(rng.integers(1, 9)), int(rng.integers(0, 2))) for _ in range(n)]
        budget = int(rng.integers(20, 600))
        for balanced in (False, True):
            chunks = O.plan_cycle(tensors, budget, training_cost=True, balanced=balanced)
            resident = sum(r * c * (4 if d == O.F32 else 2) for r, c, d in tensors)
            j = O.jitter(O.step_memory(chunks, tensors, resident, True))
            bound = O.jitter_bound(chunks, tensors, resident, True)
            assert j <= bound * (1 + 1e-12)
            costs = [O.chunk_cost_bytes(c, tensors, True) for c in chunks]
            mean = sum(costs) / len(costs)
            if abs((max(costs) - mean) - (mean - min(costs))) < 1e-9:
                assert abs(j - bound) <= 1e-12 * max(bound, 1.0)
    # two chunks always lie equally far from their mean: the bound is attained
    tensors = [(7, 9, O.BF16)]
    chunks = O.plan_cycle(tensors, 2 * 40)
    assert len(chunks) == 2
    assert O.jitter(O.step_memory(chunks, tensors, 126, False)) == O.jitter_bound(chunks, tensors, 126, False)


def test_plan_balanced_random_invariants():
    """The balanced plan, alone and with each other option: an exact partition, no chunk above
    the caller's budget (Section 3 "Method": a predefined byte budget), no more chunks than the
    greedy plan (exactly as many when tensors are cut anywhere), never a larger imbalance than greedy's capacity search started from, and for one
    dtype without row groups an imbalance below one element's cost plus the rounding of the
    capacity to 4 bytes."""
    rng = np.random.default_rng(29)
    tried = 0
    for _ in range(400):
        n = int(rng.integers(1, 6))
        uniform = bool(rng.integers(0, 2))
        d0 = int(rng.integers(0, 2))
        tensors = [(int(rng.integers(0, 40)), int(rng.integers(0, 7)), d0 if uniform else int(rng.integers(0, 2)))
                   for _ in range(n)]
        for tc, rows8 in itertools.product((False, True), (False, True)):
            budget = int(rng.integers(20 if tc else 4, 500))
            greedy = O.plan_cycle(tensors, budget, training_cost=tc, rows8=rows8)
            bal = O.plan_cycle(tensors, budget, training_cost=tc, rows8=rows8, balanced=True)
            _check_partition(tensors, bal)
            # the chunk count of a plan cut anywhere never rises with the budget, so the smallest capacity
            # that needs no more than K chunks needs exactly K; with cuts between row groups a capacity
            # too small for a group falls back to cuts anywhere and can need fewer
            assert len(bal) == len(greedy) if not rows8 else len(bal) <= len(greedy)
            costs = [O.chunk_cost_bytes(c, tensors, tc) for c in bal]
            assert all(0 < c <= budget for c in costs)
            if len(bal) < 2:
                assert bal == greedy
                continue
            tried += 1
            # the capacity actually used is the largest chunk: it is the smallest one (in steps of
            # 4 bytes from ceil(total / K)) that still gives K chunks, so one step less must not
            cap = max(costs)
            total = sum(costs)
            lowest = max(-(-(-(-total // len(bal))) // 4) * 4, max((4 if d == O.F32 else 2) + (16 if tc else 0)
                                                                   for r, c, d in tensors if r * c))
            assert cap <= budget
            if bal != greedy:
                # found below the caller's budget: some candidate b in [lowest, budget) gave K chunks and
                # every earlier candidate gave more
                b = lowest
                while len(O._greedy([r * c for r, c, _ in tensors],
                                    [(4 if d == O.F32 else 2) + (16 if tc else 0) for _, _, d in tensors], b,
                                    [8 * c for _, c, _ in tensors] if rows8 else None)) > len(greedy):
                    b += 4
                assert cap <= b < budget
                assert len(bal) == len(O.plan_cycle(tensors, b, training_cost=tc, rows8=rows8))
            if uniform and not rows8:
                s = (4 if d0 == O.F32 else 2) + (16 if tc else 0)
                # every chunk but the last is full to within one element; the last holds the rest
                assert max(costs[:-1]) - min(costs[:-1]) == 0
                assert cap - costs[-1] < len(bal) * (s + 4)
                assert O.imbalance(bal, tensors, tc) <= O.imbalance(greedy, tensors, tc) + 1e-9
    assert tried > 300


def test_plan_balanced():
    tensors = [(100, 64, O.BF16), (30, 64, O.BF16), (1, 64, O.BF16), (64, 200, O.BF16)]
    total = sum(r * c for r, c, _ in tensors) * 2
    budget = int(total / 3.1)          # greedy: three full chunks and a short tail
    g = O.plan_cycle(tensors, budget)
    b = O.plan_cycle(tensors, budget, balanced=True)
    _check_partition(tensors, b)
    assert len(b) == len(g) == 4
    assert O.imbalance(b, tensors) <= 4.0          # within one rounding step of the mean
    assert O.imbalance(g, tensors) > 1000.0
    # flops of the cycle equal the dense backward's (Section 3.2: sum_k C_k = C)
    T = 11
    assert sum(2 * T * (s.end - s.begin) for ch in b for s in ch) == 2 * T * total // 2


def test_plan_rows8_golden():
    tensors = [(20, 4, O.BF16), (3, 4, O.BF16), (10, 5, O.F32)]
    chunks = O.plan_cycle(tensors, 150, rows8=True)
    got = [(k, s.tensor, s.begin, s.end, s.chunk_off) for k, ch in enumerate(chunks) for s in ch]
    want = [tuple(int(x) for x in row) for row in _rows("plan_rows8_hand_worked.txt")]
    assert got == want
    _check_partition(tensors, chunks)


def test_plan_rows8_single_matrix_closed_form():
    """One R x c matrix, any budget that holds a group of 8 rows: every chunk but the last holds
    floor(floor(budget / size) / 8c) groups, so row r lies in chunk (r // 8) // groups_per_chunk."""
    for R, c in ((40, 3), (64, 5), (23, 2)):
        tensors = [(R, c, O.BF16)]
        for budget in range(2 * 8 * c, 2 * R * c + 5):
            chunks = O.plan_cycle(tensors, budget, rows8=True)
            _check_partition(tensors, chunks)
            gpc = (budget // 2) // (8 * c)
            n_groups = -(-R // 8)
            if budget // 2 >= R * c:
                assert len(chunks) == 1
                continue
            # a tail of fewer than 8 rows counts as a group unless it still fits behind the last whole ones
            for k, ch in enumerate(chunks):
                assert len(ch) == 1
                s = ch[0]
                assert s.begin == k * gpc * 8 * c
                assert s.begin % (8 * c) == 0 and (s.end % (8 * c) == 0 or s.end == R * c)
                assert 2 * (s.end - s.begin) <= budget
            assert len(chunks) in (-(-n_groups // gpc), -(-n_groups // gpc) - 1 if R % 8 else -(-n_groups // gpc))


def test_plan_rows8_random_invariants():
    rng = np.random.default_rng(17)
    for _ in range(300):
        n = int(rng.integers(1, 6))
        tensors = [(int(rng.integers(0, 40)), int(rng.integers(0, 6)), int(rng.integers(0, 2))) for _ in range(n)]
        budget = int(rng.integers(4, 400))
        for tc in (False, True):
            if tc and budget < 20:
                continue
            chunks = O.plan_cycle(tensors, budget, training_cost=tc, rows8=True)
            _check_partition(tensors, chunks)
            size = [(4 if d == O.F32 else 2) + (16 if tc else 0) for _, _, d in tensors]
            for ch in chunks:
                assert 0 < O.chunk_cost_bytes(ch, tensors, tc) <= budget
                for sg in ch:
                    r, c, _ = tensors[sg.tensor]
                    if 8 * c * size[sg.tensor] <= budget:      # a group fits: only whole groups, or the ends
                        assert sg.begin % (8 * c) == 0
                        assert sg.end % (8 * c) == 0 or sg.end == r * c
            # a chunk is closed only when not one more group (element, for tensors cut anywhere) fits
            for k in range(len(chunks) - 1):
                nxt = chunks[k + 1][0]
                r, c, _ = tensors[nxt.tensor]
                s = size[nxt.tensor]
                step = 8 * c if 8 * c * s <= budget else 1
                step = min(step, r * c - nxt.begin)            # a short rest may go in whole
                assert O.chunk_cost_bytes(chunks[k], tensors, tc) + step * s > budget
            # without the option nothing changes for tensors that are never cut
            if all(r * c * s <= budget for (r, c, _), s in zip(tensors, size)) and len(chunks) == 1:
                assert chunks == O.plan_cycle(tensors, budget, training_cost=tc)


def test_plan_rows8_equals_plain_when_the_budget_is_a_whole_number_of_groups():
    """Uniform matrices of one width, budget a multiple of a group's bytes: the plain planner's cuts
    already fall on group boundaries, so the option changes nothing."""
    tensors = [(32, 4, O.BF16), (16, 4, O.BF16), (48, 4, O.BF16)]
    for groups in range(1, 14):
        budget = groups * 8 * 4 * 2
        assert O.plan_cycle(tensors, budget, rows8=True) == O.plan_cycle(tensors, budget)


def test_plan_errors():
    with pytest.raises(ValueError):
        O.plan_cycle([(2, 2, O.F32)], 3)
    with pytest.raises(ValueError):
        O.plan_cycle([(2, 2, O.F32)], 0)
    assert O.plan_cycle([], 8) == []
    assert O.plan_cycle([(0, 5, O.F32), (3, 0, O.BF16)], 8) == []


def test_jitter_definition():
    # (max - min) / mean of 1, 2, 3 = 2 / 2
    assert O.jitter([1.0, 2.0, 3.0]) == 1.0
    assert O.jitter([5.0, 5.0]) == 0.0


# -------------------------------------------------------------------- wgrad
def _brute_dense(X, dY):
    T, n_in, n_out = len(X), len(X[0]), len(dY[0])
    dW = [[0.0] * n_in for _ in range(n_out)]
    for r in range(n_out):
        for c in range(n_in):
            acc = 0.0
            for t in range(T):
                acc += float(dY[t][r]) * float(X[t][c])
            dW[r][c] = acc
    return dW


def test_wgrad_bruteforce_every_range():
    rng = np.random.default_rng(11)
    for (n_out, n_in, T) in ((4, 3, 5), (5, 7, 2)):
        X = rng.integers(-4, 5, size=(T, n_in)).astype(np.float64)     # integers: sums are exact
        dY = rng.integers(-4, 5, size=(T, n_out)).astype(np.float64)
        flat = [v for row in _brute_dense(X.tolist(), dY.tolist()) for v in row]
        N = n_out * n_in
        for b, e in itertools.combinations(range(N + 1), 2):
            for dense in (True, False):
                got = O.chunk_wgrad(X, dY, b, e, dense=dense)
                assert got.shape == (e - b,)
                assert got.tolist() == flat[b:e]
        idx = np.arange(N)[::-1].copy()
        assert O.wgrad_elements(X, dY, idx).tolist() == [flat[i] for i in idx]


def test_wgrad_special_cases():
    rng = np.random.default_rng(12)
    n_out, n_in = 6, 4
    # one token: outer product dY[0, r] * X[0, c]
    x = rng.standard_normal((1, n_in))
    dy = rng.standard_normal((1, n_out))
    assert np.array_equal(O.dense_wgrad(x, dy), np.outer(dy[0], x[0]))
    # X = identity (T = in): dW = dY^T -- catches a transposed operand
    dY = rng.standard_normal((n_in, n_out))
    assert np.array_equal(O.dense_wgrad(np.eye(n_in), dY), dY.T)
    # dY = identity (T = out): dW = X
    X = rng.standard_normal((n_out, n_in))
    assert np.array_equal(O.dense_wgrad(X, np.eye(n_out)), X)
    # all ones: every element counts the tokens
    assert np.array_equal(O.dense_wgrad(np.ones((9, n_in)), np.ones((9, n_out))), np.full((n_out, n_in), 9.0))
    # only one (t, r) and one (t, c) entry non-zero: a single non-zero element, at [r, c]
    X = np.zeros((3, n_in)); dY = np.zeros((3, n_out))
    X[2, 1] = 3.0; dY[2, 5] = 5.0
    dW = O.dense_wgrad(X, dY)
    assert dW[5, 1] == 15.0 and np.count_nonzero(dW) == 1
    assert O.chunk_wgrad(X, dY, 5 * n_in + 1, 5 * n_in + 2).tolist() == [15.0]


def test_wgrad_linearity_and_token_concatenation():
    rng = np.random.default_rng(13)
    T, n_out, n_in = 16, 5, 6
    X = rng.integers(-3, 4, (T, n_in)).astype(np.float64)
    A = rng.integers(-3, 4, (T, n_out)).astype(np.float64)
    B = rng.integers(-3, 4, (T, n_out)).astype(np.float64)
    b, e = 7, 23
    assert np.array_equal(O.chunk_wgrad(X, A + 2 * B, b, e),
                          O.chunk_wgrad(X, A, b, e) + 2 * O.chunk_wgrad(X, B, b, e))
    # two micro-batches accumulate to the gradient of their concatenation
    assert np.array_equal(O.chunk_wgrad(X, A, b, e),
                          O.chunk_wgrad(X[:9], A[:9], b, e) + O.chunk_wgrad(X[9:], A[9:], b, e))


def test_wgrad_against_fp32_library_matmul():
    # a second library routine (torch, other BLAS call path, float64)
    rng = np.random.default_rng(14)
    X = rng.standard_normal((33, 20)); dY = rng.standard_normal((33, 17))
    ref = (torch.from_numpy(dY).T @ torch.from_numpy(X)).numpy().reshape(-1)
    got = O.chunk_wgrad(X, dY, 5, 300)
    np.testing.assert_allclose(got, ref[5:300], rtol=1e-13, atol=1e-13)


def test_vector_wgrad_bruteforce():
    rng = np.random.default_rng(15)
    T, n = 6, 9
    X = rng.integers(-4, 5, (T, n)).astype(np.float64)
    dY = rng.integers(-4, 5, (T, n)).astype(np.float64)
    full = [sum(dY[t, j] * X[t, j] for t in range(T)) for j in range(n)]
    for b, e in itertools.combinations(range(n + 1), 2):
        assert O.vector_wgrad(X, dY, b, e).tolist() == full[b:e]
    # xhat = 1 everywhere: a bias gradient, the column sum of dY
    assert O.vector_wgrad(np.ones((T, n)), dY, 0, n).tolist() == dY.sum(axis=0).tolist()


# -------------------------------------------------------------------- AdamW
HP = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)


def test_adamw_golden_two_steps():
    for wd in (0.0, 0.5):
        rows = [r for r in _rows("adamw_two_steps.txt") if float(r[0]) == wd]
        th, m, v = np.array([1.0]), np.array([0.0]), np.array([0.0])
        for r in rows:
            step, g = int(r[1]), float(r[2])
            th, m, v = O.adamw_step(np.array([g]), th, m, v, lr=0.1, beta1=0.5, beta2=0.5,
                                    eps=0.0, weight_decay=wd, step=step)
            assert abs(th[0] - float(r[3])) < 2e-16 * 4
            assert m[0] == float(r[4]) and v[0] == float(r[5])


def test_adamw_first_step_closed_form():
    """From m = v = 0: m1 = (1-b1) g, v1 = (1-b2) g^2, mhat = g, vhat = g^2, hence
    theta1 = theta0 (1 - lr wd) - lr g / (|g| + eps)."""
    rng = np.random.default_rng(21)
    g = rng.standard_normal(1000) * 10.0 ** rng.uniform(-9, 1, 1000)
    g[:5] = 0.0
    th0 = rng.standard_normal(1000) * 0.02
    z = np.zeros(1000)
    th, m, v = O.adamw_step(g, th0, z, z, step=1, **HP)
    np.testing.assert_allclose(m, 0.1 * g, rtol=1e-14)
    np.testing.assert_allclose(v, 0.001 * g * g, rtol=1e-12)
    want = th0 * (1 - HP["lr"] * HP["weight_decay"]) - HP["lr"] * g / (np.abs(g) + HP["eps"])
    np.testing.assert_allclose(th, want, rtol=1e-12, atol=1e-18)
    # zero gradient: only the decay acts, moments stay zero
    assert np.array_equal(th[:5], th0[:5] - HP["lr"] * HP["weight_decay"] * th0[:5])
    assert not m[:5].any() and not v[:5].any()


def test_adamw_constant_gradient_bias_correction():
    """With the same g at every step, m_n = (1 - b1^n) g and v_n = (1 - b2^n) g^2,
    so the corrected moments are g and g^2 at every n and each step moves theta
    by theta*(-lr wd) - lr g/(|g| + eps).  A wrong counter or a missing
    correction breaks this from n = 2 on."""
    g = np.array([0.3, -2.0, 1e-3])
    th = np.array([0.5, -0.25, 1.0])
    m = np.zeros(3); v = np.zeros(3)
    for n in range(1, 8):
        want = th * (1 - HP["lr"] * HP["weight_decay"]) - HP["lr"] * g / (np.abs(g) + HP["eps"])
        th, m, v = O.adamw_step(g, th, m, v, step=n, **HP)
        np.testing.assert_allclose(th, want, rtol=1e-12)
        np.testing.assert_allclose(m, (1 - 0.9 ** n) * g, rtol=1e-12)
        np.testing.assert_allclose(v, (1 - 0.999 ** n) * g * g, rtol=1e-12)


def test_adamw_no_memory_is_sign_descent():
    # b1 = b2 = 0, wd = 0: theta - lr g / (|g| + eps)
    g = np.array([2.0, -0.5, 0.0, 1e-8])
    th = np.ones(4)
    out, m, v = O.adamw_step(g, th, np.full(4, 9.0), np.full(4, 9.0), lr=0.1, beta1=0.0, beta2=0.0,
                             eps=1e-8, weight_decay=0.0, step=3)
    np.testing.assert_allclose(out, th - 0.1 * g / (np.abs(g) + 1e-8), rtol=1e-15)
    assert np.array_equal(m, g) and np.array_equal(v, g * g)


def test_adamw_against_torch_float64():
    """torch.optim.AdamW (decoupled decay, eps outside the square root) on
    float64 tensors, five steps with fresh gradients."""
    rng = np.random.default_rng(22)
    n = 257
    th0 = rng.standard_normal(n) * 0.02
    p = torch.nn.Parameter(torch.from_numpy(th0.copy()))
    opt = torch.optim.AdamW([p], lr=HP["lr"], betas=(HP["beta1"], HP["beta2"]), eps=HP["eps"],
                            weight_decay=HP["weight_decay"], amsgrad=False)
    th, m, v = th0, np.zeros(n), np.zeros(n)
    for step in range(1, 6):
        g = rng.standard_normal(n) * 10.0 ** rng.uniform(-4, 0, n)
        p.grad = torch.from_numpy(g.copy())
        opt.step()
        th, m, v = O.adamw_step(g, th, m, v, step=step, **HP)
        np.testing.assert_allclose(th, p.detach().numpy(), rtol=1e-11, atol=1e-15)
        st = opt.state[p]
        np.testing.assert_allclose(m, st["exp_avg"].numpy(), rtol=1e-12, atol=1e-300)
        np.testing.assert_allclose(v, st["exp_avg_sq"].numpy(), rtol=1e-12, atol=1e-300)


def test_adamw_rejects_step_zero():
    with pytest.raises(ValueError):
        O.adamw_step(np.ones(1), np.ones(1), np.zeros(1), np.zeros(1), step=0, **HP)


# --------------------------------------------------------------------- bf16
def _all_bf16_values():
    bits = np.arange(65536, dtype=np.uint32)
    vals = (bits << np.uint32(16)).view(np.float32)
    return bits.astype(np.uint16), vals


def test_bf16_grid_fixed_points_and_bits():
    bits, vals = _all_bf16_values()
    fin = np.isfinite(vals)
    r = O.round_to_bf16(vals[fin].astype(np.float64))
    assert np.array_equal(r, vals[fin].astype(np.float64))
    got = O.bf16_bits(vals[fin].astype(np.float64))
    # +0 and -0 keep their sign bit through the float32 cast
    assert np.array_equal(got, bits[fin])
    assert np.array_equal(O.bf16_from_bits(bits[fin]), vals[fin].astype(np.float64))


def test_bf16_midpoints_tie_to_even_everywhere():
    bits, vals = _all_bf16_values()
    pos = (bits < 0x7F80)                      # positive finite, including subnormals and zero
    lo = vals[pos][:-1].astype(np.float64)
    hi = vals[pos][1:].astype(np.float64)
    lo_bits = bits[pos][:-1]
    mid = (lo + hi) / 2                        # exact in fp64
    even = np.where(lo_bits % 2 == 0, lo, hi)
    assert np.array_equal(O.round_to_bf16(mid), even)
    assert np.array_equal(O.round_to_bf16(-mid), -even)
    below = mid - (hi - lo) / 1024             # strictly nearer the lower neighbour
    above = mid + (hi - lo) / 1024
    assert np.array_equal(O.round_to_bf16(below), lo)
    assert np.array_equal(O.round_to_bf16(above), hi)
    assert np.isinf(O.round_to_bf16(np.array([3.4e38]))[0])   # beyond the largest bf16 (3.3895e38)


def test_bf16_matches_library_conversion():
    rng = np.random.default_rng(31)
    x = (rng.standard_normal(200000) * 10.0 ** rng.uniform(-30, 30, 200000)).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(O.bf16_bits(x.astype(np.float64)), want)


# -------------------------------------------------------------------- cycle
def test_cycle_equals_one_dense_update():
    """Section 3.2 / Appendix G notation: chunks are disjoint and the update is
    element-wise, so stepping every chunk once equals one dense AdamW step on
    the dense gradient; elements of other chunks are untouched by a chunk's step."""
    rng = np.random.default_rng(41)
    T = 8
    tensors = [(6, 5, O.BF16), (1, 7, O.BF16), (3, 4, O.BF16)]
    kinds = [O.LINEAR, O.VECTOR, O.LINEAR]
    inputs, params = [], []
    for (r, c, _), kind in zip(tensors, kinds):
        X = rng.standard_normal((T, c))
        dY = rng.standard_normal((T, r if kind == O.LINEAR else c))
        inputs.append((kind, X, dY))
        params.append(rng.standard_normal(r * c) * 0.02)
    for budget in (2 * 9, 2 * 30, 2 * 1000):
        chunks = O.plan_cycle(tensors, budget)
        states = [{"m": np.zeros(sum(s.end - s.begin for s in ch)),
                   "v": np.zeros(sum(s.end - s.begin for s in ch))} for ch in chunks]
        newp, news = O.cycle_step(tensors, inputs, params, states, chunks, HP, [1] * len(chunks))
        for t, (kind, X, dY) in enumerate(inputs):
            g = O.dense_wgrad(X, dY).reshape(-1) if kind == O.LINEAR else (dY * X).sum(axis=0)
            z = np.zeros_like(g)
            want, _, _ = O.adamw_step(g, params[t], z, z, step=1, **HP)
            np.testing.assert_allclose(newp[t], want, rtol=1e-13, atol=1e-16)
        # stepping only chunk 0 leaves every element of the other chunks bit-identical
        only0, _ = O.cycle_step(tensors, inputs, params, states[:1], chunks[:1], HP, [1])
        touched = [np.zeros(r * c, dtype=bool) for r, c, _ in tensors]
        for s in chunks[0]:
            touched[s.tensor][s.begin:s.end] = True
        for t in range(len(tensors)):
            assert np.array_equal(only0[t][~touched[t]], params[t][~touched[t]])
            assert np.all(only0[t][touched[t]] != params[t][touched[t]])


# ---------------------------------------------------------------- embedding / norms
def test_embedding_wgrad_bruteforce_and_one_hot_identity():
    rng = np.random.default_rng(31)
    vocab, dim, T = 7, 5, 19
    ids = rng.integers(0, vocab, size=T)
    dY = rng.standard_normal((T, dim))
    # brute force: one element at a time
    dense = np.zeros((vocab, dim))
    for r in range(vocab):
        for c in range(dim):
            for t in range(T):
                if ids[t] == r:
                    dense[r, c] += dY[t, c]
    flat = dense.reshape(-1)
    for begin, end in ((0, vocab * dim), (3, 4), (6, 23), (5, 10), (30, 35)):
        np.testing.assert_allclose(O.embedding_wgrad(ids, dY, vocab, begin, end), flat[begin:end], rtol=0, atol=1e-13)
    # an embedding lookup is a linear layer on one-hot inputs: dW = onehot^T dY
    onehot = np.zeros((T, vocab))
    onehot[np.arange(T), ids] = 1.0
    np.testing.assert_allclose(O.dense_wgrad(dY, onehot), dense, rtol=0, atol=1e-13)
    # rows that no token names stay zero; a table hit once returns that token's row
    ids2 = np.array([4, 1])
    out = O.embedding_wgrad(ids2, dY[:2], vocab, 0, vocab * dim).reshape(vocab, dim)
    assert np.array_equal(out[4], dY[0]) and np.array_equal(out[1], dY[1]) and not out[[0, 2, 3, 5, 6]].any()
    # every token names the same row: that row is the column sum
    out = O.embedding_wgrad(np.full(T, 2), dY, vocab, 2 * dim, 3 * dim)
    np.testing.assert_allclose(out, dY.sum(axis=0), rtol=0, atol=1e-13)
    with pytest.raises(ValueError):
        O.embedding_wgrad(np.array([7]), dY[:1], vocab, 0, 1)


def test_embedding_wgrad_against_library_autograd():
    rng = np.random.default_rng(32)
    vocab, dim, T = 11, 6, 40
    ids = rng.integers(0, vocab, size=T)
    dY = rng.standard_normal((T, dim))
    W = torch.zeros(vocab, dim, dtype=torch.float64, requires_grad=True)
    y = torch.nn.functional.embedding(torch.from_numpy(ids), W)
    (y * torch.from_numpy(dY)).sum().backward()
    ref = W.grad.numpy().reshape(-1)
    np.testing.assert_allclose(O.embedding_wgrad(ids, dY, vocab, 0, vocab * dim), ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(O.embedding_wgrad(ids, dY, vocab, 13, 47), ref[13:47], rtol=0, atol=1e-12)


@pytest.mark.parametrize("subtract_mean", [False, True])
def test_norm_weight_wgrad_against_library_autograd_and_closed_forms(subtract_mean):
    rng = np.random.default_rng(33)
    T, n, eps = 9, 12, 1e-5
    x = rng.standard_normal((T, n)) * 3.0 + (1.5 if subtract_mean else 0.0)
    dY = rng.standard_normal((T, n))
    w = torch.ones(n, dtype=torch.float64, requires_grad=True)
    xt = torch.from_numpy(x)
    if subtract_mean:
        y = torch.nn.functional.layer_norm(xt, (n,), weight=w, bias=None, eps=eps)
    else:
        y = xt * torch.rsqrt((xt * xt).mean(dim=1, keepdim=True) + eps) * w
    (y * torch.from_numpy(dY)).sum().backward()
    ref = w.grad.numpy()
    np.testing.assert_allclose(O.norm_weight_wgrad(x, dY, eps, subtract_mean, 0, n), ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(O.norm_weight_wgrad(x, dY, eps, subtract_mean, 3, 8), ref[3:8], rtol=1e-12, atol=1e-13)
    # brute force of the definition for one element
    j = 5
    acc = 0.0
    for t in range(T):
        row = x[t] - (x[t].mean() if subtract_mean else 0.0)
        acc += dY[t, j] * row[j] / np.sqrt(np.mean(row * row) + eps)
    assert abs(O.norm_weight_wgrad(x, dY, eps, subtract_mean, j, j + 1)[0] - acc) < 1e-12
    # scale invariance: with eps = 0 the normalised input does not change when x is scaled
    a = O.norm_xhat(x, 0.0, subtract_mean)
    b = O.norm_xhat(7.0 * x, 0.0, subtract_mean)
    np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)
    # its rows have unit mean square (and zero mean for LayerNorm)
    np.testing.assert_allclose((a * a).mean(axis=1), 1.0, rtol=1e-12)
    if subtract_mean:
        np.testing.assert_allclose(a.mean(axis=1), 0.0, atol=1e-13)


# ---------------------------------------------------------------- rotating schedule
def test_rotating_schedule_hand_worked_and_invariants():
    # K = 3 chunks, interval 2: chunks 0 0 1 1 2 2 0 0 ..., counters 1 2 1 2 1 2 3 4 ...
    got = O.rotating_schedule(8, 3, 2)
    assert [g[0] for g in got] == [0, 0, 1, 1, 2, 2, 0, 0]
    assert [g[3] for g in got] == [1, 2, 1, 2, 1, 2, 3, 4]
    assert [g[1] for g in got] == [True, False] * 4
    assert [g[2] for g in got] == [False, True] * 4
    # interval 1: plain round robin, every step loads and offloads
    got = O.rotating_schedule(7, 4, 1)
    assert [g[0] for g in got] == [0, 1, 2, 3, 0, 1, 2]
    assert all(g[1] and g[2] for g in got)
    assert [g[3] for g in got] == [1, 1, 1, 1, 2, 2, 2]
    # one chunk: always active, the counter is the step count
    assert [g[3] for g in O.rotating_schedule(5, 1, 3)] == [1, 2, 3, 4, 5]
    for K, H in itertools.product((1, 2, 5), (1, 3, 4)):
        n = 3 * K * H + 2
        got = O.rotating_schedule(n, K, H)
        # over whole cycles every chunk is active exactly H steps per cycle
        cyc = got[:3 * K * H]
        for k in range(K):
            assert sum(1 for g in cyc if g[0] == k) == 3 * H
        # the counters of all chunks add up to the number of steps taken
        last = {}
        for g in got:
            last[g[0]] = g[3]
        assert sum(last.values()) == n
        # a chunk's counter rises by exactly one each step it is active
        seen = {}
        for g in got:
            assert g[3] == seen.get(g[0], 0) + 1
            seen[g[0]] = g[3]
    with pytest.raises(ValueError):
        O.rotating_schedule(3, 0, 1)

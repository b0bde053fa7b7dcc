"""CPU oracle for the ChunkFT hot path -- TEST INFRASTRUCTURE, not product code.

This file is the plain, slow, fp64 statement of what the hot path computes.
It is written from the paper (Algorithm 1; Section 3 "Method"; Section 3.1
"Algorithm Description"; Section 3.2 "BP Time Analysis"; Appendix F "Analysis
of Memory Jitter") and shares no code, header, table or helper with the HIP
library.  Only tests, the smoke check and the bench's `cpu_baseline` leg may
import it; the product path never does.

What each function follows:

* plan_cycle            -- Section 3 "Method", first paragraph (size of a tensor
                           is numel x element_size; tensors are accumulated in
                           model order until a byte budget is reached; a tensor
                           may span several chunks) and Algorithm 1 lines 1-2.
                           Section 3.1 lists a second cost (parameter + gradient
                           + fp32 master + optimizer state); `training_cost`
                           selects it.  `balanced` follows the byte-balance
                           condition of Appendix F (every chunk close to the
                           mean chunk cost).
* chunk_wgrad / dense_wgrad / wgrad_elements
                        -- Section 3.1, equation g^(k) = grad of the loss w.r.t.
                           the active slices only: the chunk gradient is the
                           restriction of the dense gradient.  For a linear
                           layer y = x W^T the dense weight gradient is
                           dW = dY^T X (textbook), so the oracle forms dW in
                           fp64 and slices the flattened row-major range.
* vector_wgrad          -- same equation for a 1-D scale vector (LayerNorm /
                           RMSNorm weight, Algorithm 1 line 8): y = xhat * w
                           gives dw[j] = sum_t dY[t, j] * xhat[t, j].
* embedding_wgrad       -- same equation for an embedding table (Algorithm 1 line 8
                           names Embedding among the chunk-aware operators;
                           Appendix "Limitations" lists the set): y[t] = W[id[t]]
                           gives dW[r, :] = sum over the tokens with id[t] = r
                           of dY[t, :] (textbook), restricted to the range.
* norm_weight_wgrad     -- same equation for the scale vector of RMSNorm /
                           LayerNorm when the operator normalises its input
                           itself: y = w * xhat(x), xhat = x * rstd (RMSNorm) or
                           (x - mean) * rstd (LayerNorm), so
                           dw[j] = sum_t dY[t, j] * xhat[t, j] (textbook; the
                           paper names the operators without formulas).
* adamw_step            -- Algorithm 1 lines 19-21 (the AdamW update), in that order, fp64.
* round_to_bf16         -- round-to-nearest-even onto the bfloat16 grid (the
                           paper keeps low-precision parameters beside fp32
                           master weights, Section 3.3; the rounding mode is
                           this build's reading: nearest-even).
* cycle_step            -- Section 3.2: chunks are a disjoint partition, so one
                           cycle applies the chunk update to every element once.
* rotating_schedule     -- Algorithm 1, the loop over training steps: the active
                           index, the load / offload steps and the per-chunk
                           update counters n^(k), simulated step by step.
* jitter / imbalance / step_memory / jitter_bound
                        -- appendix "Analysis of Memory Jitter": the jitter ratio of
                           a sequence of step memories, the chunking imbalance
                           epsilon_B, the step memory 2M + B(C_k) of a chunk
                           (activations and temporary buffers left out) and the
                           bound 2 epsilon_B / (2M + mean B) on the jitter.

Pins (tests/test_oracle_pins.py): brute-force loops on tiny layers, closed
forms of the first AdamW step, hand-worked two-step values, torch.optim.AdamW
in float64, partition invariants and a closed form for the uniform-dtype
planner, exhaustive bf16 grid checks.  Nothing in the paper prints a worked
numeric example for these operations, so the pins are mathematical.
"""

from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence, Tuple

import numpy as np

F32 = 0
BF16 = 1
_ELEMENT_SIZE = {F32: 4, BF16: 2}

LINEAR = 0
VECTOR = 1
EMBEDDING = 2
RMSNORM = 3
LAYERNORM = 4

# bytes of training state per element besides the parameter itself:
# fp32 gradient + fp32 master + fp32 m + fp32 v (Section 3.3: 4+4+4+4).
STATE_BYTES_PER_ELEMENT = 16


# --------------------------------------------------------------------------
# planner
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Segment:
    tensor: int      # index into the caller's tensor list
    begin: int       # first flat element of the tensor in this segment
    end: int         # one past the last flat element
    chunk_off: int   # position of `begin` inside the chunk's state arrays


def _cost_per_element(dtype: int, training_cost: bool) -> int:
    s = _ELEMENT_SIZE[dtype]
    return s + STATE_BYTES_PER_ELEMENT if training_cost else s


def _greedy(numels: Sequence[int], costs: Sequence[int], budget: int,
            groups: Sequence[int] = None) -> List[List[Segment]]:
    """groups[t] > 1: tensor t may only be cut at multiples of groups[t] elements (whole
    groups of rows), provided an empty chunk has room for one such group; otherwise, and
    with groups = None, it is cut at any element."""
    chunks: List[List[Segment]] = []
    cur: List[Segment] = []
    room = budget
    filled = 0  # elements already in the open chunk
    for t, (n, s) in enumerate(zip(numels, costs)):
        p = 0
        group = groups[t] if groups is not None and groups[t] * s <= budget else 1
        while p < n:
            fits = room // s
            if fits >= n - p:
                take = n - p            # the rest of the tensor goes in whole
            else:
                take = fits - fits % group   # p is a multiple of group: so is the cut
            if take == 0:
                # the open chunk cannot hold one more element of this tensor
                chunks.append(cur)
                cur, room, filled = [], budget, 0
                continue
            cur.append(Segment(t, p, p + take, filled))
            p += take
            filled += take
            room -= take * s
    if cur:
        chunks.append(cur)
    return chunks


def plan_cycle(tensors: Sequence[Tuple[int, int, int]], budget_bytes: int,
               training_cost: bool = False, balanced: bool = False,
               rows8: bool = False) -> List[List[Segment]]:
    """tensors: (rows, cols, dtype) in model order.  Returns chunks in cycle
    order; each chunk is its ordered list of segments.

    rows8: a tensor is split along its row dimension only (Section 3 "Method",
    first paragraph), between groups of 8 rows: the open chunk takes as many whole groups as fit, and is
    closed if not one fits.  A tensor so wide that an empty chunk cannot hold one
    group is cut at any element.

    Greedy: walk the tensors in order, put as many elements as still fit the
    budget into the open chunk, close the chunk when not even one element of
    the current tensor fits.  Balanced: keep the greedy chunk count K but
    shrink the budget to the smallest multiple of 4 bytes, not below
    ceil(total/K) and below the caller's budget, for which greedy still needs
    only K chunks; if there is none the caller's budget stands (no chunk may
    exceed the predefined budget).
    """
    if budget_bytes <= 0:
        raise ValueError("budget must be positive")
    numels = [int(r) * int(c) for r, c, _ in tensors]
    if any(r < 0 or c < 0 for r, c, _ in tensors):
        raise ValueError("negative shape")
    costs = [_cost_per_element(d, training_cost) for _, _, d in tensors]
    for n, s in zip(numels, costs):
        if n > 0 and s > budget_bytes:
            raise ValueError("budget smaller than one element")
    groups = [8 * int(c) for _, c, _ in tensors] if rows8 else None
    chunks = _greedy(numels, costs, budget_bytes, groups)
    if balanced and len(chunks) > 1:
        k = len(chunks)
        total = sum(n * s for n, s in zip(numels, costs))
        b = -(-total // k)          # ceil
        b = -(-b // 4) * 4          # round up to a multiple of 4 bytes
        b = max(b, max(s for n, s in zip(numels, costs) if n > 0))
        while b < budget_bytes:
            cand = _greedy(numels, costs, b, groups)
            if len(cand) <= k:
                return cand
            b += 4
        # no smaller budget keeps K chunks: the caller's budget is the cap
    return chunks


def chunk_cost_bytes(chunk: Sequence[Segment], tensors, training_cost: bool = False) -> int:
    return sum((s.end - s.begin) * _cost_per_element(tensors[s.tensor][2], training_cost)
               for s in chunk)


def imbalance(chunks, tensors, training_cost: bool = False) -> float:
    """epsilon_B of Appendix F: max_k | B(C_k) - mean_j B(C_j) |."""
    b = np.array([chunk_cost_bytes(c, tensors, training_cost) for c in chunks], dtype=np.float64)
    return float(np.max(np.abs(b - b.mean())))


def jitter(step_memory: Sequence[float]) -> float:
    """Appendix F: (max_t M_t - min_t M_t) / mean_t M_t."""
    m = np.asarray(step_memory, dtype=np.float64)
    return float((m.max() - m.min()) / m.mean())


def step_memory(chunks, tensors, resident_bytes: int, training_cost: bool = True) -> List[float]:
    """Appendix F: M_k = 2M + B(C_k) + A_k + Delta_k with the activation and temporary
    terms left out; `resident_bytes` is the 2M of the formula (the low-precision
    parameters of the whole model, resident at every step)."""
    return [float(resident_bytes + chunk_cost_bytes(c, tensors, training_cost)) for c in chunks]


def jitter_bound(chunks, tensors, resident_bytes: int, training_cost: bool = True) -> float:
    """Appendix F, last equation: 2 epsilon_B / (2M + (1/K) sum_j B(C_j))."""
    b = np.array([chunk_cost_bytes(c, tensors, training_cost) for c in chunks], dtype=np.float64)
    return float(2.0 * imbalance(chunks, tensors, training_cost) / (resident_bytes + b.mean()))


# --------------------------------------------------------------------------
# rotating schedule
# --------------------------------------------------------------------------
def rotating_schedule(n_steps: int, n_chunks: int, interval: int):
    """Algorithm 1's outer loop, run for training steps t = 0 .. n_steps - 1.

    Returns one tuple per step: (active chunk k, load_before, offload_after,
    n^(k) after its increment).  Written as the algorithm states it: an active
    index that advances after every `interval` steps, a chunk selected as
    index mod K when t mod interval = 0, one counter per chunk.
    """
    if n_chunks < 1 or interval < 1 or n_steps < 0:
        raise ValueError("need at least one chunk, a positive interval and a non-negative step count")
    counters = [0] * n_chunks
    index = 0
    k = 0
    out = []
    for t in range(n_steps):
        load = t % interval == 0
        if load:
            k = index % n_chunks
        counters[k] += 1
        offload = t % interval == interval - 1
        out.append((k, load, offload, counters[k]))
        if offload:
            index += 1
    return out


# --------------------------------------------------------------------------
# weight gradient
# --------------------------------------------------------------------------
def dense_wgrad(X: np.ndarray, dY: np.ndarray) -> np.ndarray:
    """dW[r, c] = sum_t dY[t, r] * X[t, c], all of it, in fp64."""
    X64 = np.asarray(X, dtype=np.float64)
    dY64 = np.asarray(dY, dtype=np.float64)
    if X64.ndim != 2 or dY64.ndim != 2 or X64.shape[0] != dY64.shape[0]:
        raise ValueError("X must be [T, in] and dY [T, out]")
    return dY64.T @ X64


def chunk_wgrad(X: np.ndarray, dY: np.ndarray, begin: int, end: int,
                dense: bool = True) -> np.ndarray:
    """Gradient of flat row-major elements [begin, end) of W [out, in].

    dense=True forms the whole dW and slices it (the definition).  dense=False
    forms only the rows of dW that the range touches, every one of them over
    all columns, and slices that: each element's formula is unchanged, only
    rows that cannot appear in the slice are not computed (for layers whose
    dense fp64 dW would take minutes on the host).
    """
    T, n_in = X.shape
    n_out = dY.shape[1]
    if not (0 <= begin < end <= n_out * n_in):
        raise ValueError("range outside the tensor")
    if dense:
        return dense_wgrad(X, dY).reshape(-1)[begin:end].copy()
    r0 = begin // n_in
    r1 = (end - 1) // n_in
    rows = dense_wgrad(X, dY[:, r0:r1 + 1]).reshape(-1)
    return rows[begin - r0 * n_in:end - r0 * n_in].copy()


def wgrad_elements(X: np.ndarray, dY: np.ndarray, flat_index: np.ndarray) -> np.ndarray:
    """dW.flat[i] for each listed flat index, one dot product over tokens each."""
    n_in = X.shape[1]
    idx = np.asarray(flat_index, dtype=np.int64)
    out = np.empty(idx.shape[0], dtype=np.float64)
    step = 4096
    for s in range(0, idx.shape[0], step):
        part = idx[s:s + step]
        r = part // n_in
        c = part % n_in
        a = np.asarray(dY[:, r], dtype=np.float64)
        b = np.asarray(X[:, c], dtype=np.float64)
        out[s:s + step] = np.einsum("tn,tn->n", a, b)
    return out


def vector_wgrad(Xhat: np.ndarray, dY: np.ndarray, begin: int, end: int) -> np.ndarray:
    """Scale-vector gradient g[j] = sum_t dY[t, j] * Xhat[t, j], j in [begin, end)."""
    if Xhat.shape != dY.shape:
        raise ValueError("Xhat and dY must have the same [T, n] shape")
    if not (0 <= begin < end <= Xhat.shape[1]):
        raise ValueError("range outside the vector")
    full = np.sum(np.asarray(dY, dtype=np.float64) * np.asarray(Xhat, dtype=np.float64), axis=0)
    return full[begin:end].copy()


def embedding_wgrad(ids: np.ndarray, dY: np.ndarray, vocab: int, begin: int, end: int) -> np.ndarray:
    """Gradient of flat elements [begin, end) of an embedding table W [vocab, dim]
    whose forward is y[t] = W[ids[t]]: the dense table gradient, formed row by
    row in token order, then the slice."""
    ids = np.asarray(ids, dtype=np.int64)
    dY64 = np.asarray(dY, dtype=np.float64)
    if dY64.ndim != 2 or ids.shape != (dY64.shape[0],):
        raise ValueError("ids must be [T] and dY [T, dim]")
    if ids.size and (ids.min() < 0 or ids.max() >= vocab):
        raise ValueError("token id outside the table")
    dim = dY64.shape[1]
    if not (0 <= begin < end <= vocab * dim):
        raise ValueError("range outside the tensor")
    dW = np.zeros((vocab, dim), dtype=np.float64)
    for t in range(ids.shape[0]):
        dW[ids[t]] += dY64[t]
    return dW.reshape(-1)[begin:end].copy()


def norm_xhat(x: np.ndarray, eps: float, subtract_mean: bool) -> np.ndarray:
    """Normalised input of RMSNorm (subtract_mean=False: x / sqrt(mean(x^2) + eps))
    or LayerNorm (True: (x - mean) / sqrt(var + eps), biased variance), per token."""
    x64 = np.asarray(x, dtype=np.float64)
    if subtract_mean:
        x64 = x64 - x64.mean(axis=1, keepdims=True)
    return x64 / np.sqrt((x64 * x64).mean(axis=1, keepdims=True) + eps)


def norm_weight_wgrad(x: np.ndarray, dY: np.ndarray, eps: float, subtract_mean: bool,
                      begin: int, end: int) -> np.ndarray:
    """dw[j] = sum_t dY[t, j] * xhat[t, j] for j in [begin, end), xhat formed from x itself."""
    return vector_wgrad(norm_xhat(x, eps, subtract_mean), dY, begin, end)


# --------------------------------------------------------------------------
# AdamW on a chunk
# --------------------------------------------------------------------------
def adamw_step(g, theta, m, v, *, lr: float, beta1: float, beta2: float, eps: float,
               weight_decay: float, step: int):
    """One update of Algorithm 1 lines 19-21.  `step` is the chunk's own
    counter n AFTER its increment (first update: 1).  Returns new
    (theta, m, v) as fp64 arrays; the inputs are not modified.
    """
    if step < 1:
        raise ValueError("step counts from 1")
    g = np.asarray(g, dtype=np.float64)
    theta = np.asarray(theta, dtype=np.float64)
    m = np.asarray(m, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    m_new = beta1 * m + (1.0 - beta1) * g
    v_new = beta2 * v + (1.0 - beta2) * (g * g)
    m_hat = m_new / (1.0 - beta1 ** step)
    v_hat = v_new / (1.0 - beta2 ** step)
    theta_new = theta - lr * (m_hat / (np.sqrt(v_hat) + eps) + weight_decay * theta)
    return theta_new, m_new, v_new


# --------------------------------------------------------------------------
# bfloat16 grid
# --------------------------------------------------------------------------
def round_to_bf16(x) -> np.ndarray:
    """Nearest bfloat16 value (ties to even), returned as fp64.

    bfloat16 has 8 significand bits (7 stored) and fp32's exponent range:
    a value with binary exponent e lies on a grid of spacing 2^(e-7), with
    e clamped below at -126 (subnormals).  Scaling by a power of two is exact
    in fp64, and numpy's rint rounds halves to even.
    """
    x = np.asarray(x, dtype=np.float64)
    out = np.array(x, dtype=np.float64, copy=True)
    finite = np.isfinite(x) & (x != 0.0)
    xf = x[finite]
    _, e = np.frexp(xf)              # xf = f * 2^e, 0.5 <= |f| < 1
    e = e - 1                        # now 1 <= |xf| / 2^e < 2
    e = np.maximum(e, -126)
    q = np.ldexp(1.0, e - 7)
    y = np.rint(xf / q) * q
    y = np.where(np.abs(y) >= 2.0 ** 128, np.copysign(np.inf, y), y)
    out[finite] = y
    return out


def bf16_bits(x) -> np.ndarray:
    """uint16 bit patterns of round_to_bf16(x)."""
    y = round_to_bf16(x).astype(np.float32)  # exact: the bf16 grid is a subset of fp32
    return (y.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bf16_from_bits(bits) -> np.ndarray:
    b = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------
# one full-parameter cycle (every chunk stepped once)
# --------------------------------------------------------------------------
def cycle_step(tensors, layer_inputs, params, states, chunks, hp: dict, steps: Sequence[int]):
    """Apply one chunk update per chunk of `chunks`, in order.

    tensors       (rows, cols, dtype) list
    layer_inputs  per tensor (kind, X, dY): LINEAR -> X [T, cols], dY [T, rows];
                  VECTOR -> Xhat [T, cols], dY [T, cols]
    params        per tensor flat fp64 array (the fp32 master values)
    states        per chunk dict(m=..., v=...) fp64 arrays of the chunk length
    steps         per chunk counter n (after increment)
    Returns (new_params, new_states); inputs are not modified.
    """
    new_params = [np.array(p, dtype=np.float64, copy=True) for p in params]
    new_states = []
    for k, chunk in enumerate(chunks):
        m = np.array(states[k]["m"], dtype=np.float64, copy=True)
        v = np.array(states[k]["v"], dtype=np.float64, copy=True)
        for seg in chunk:
            kind, X, dY = layer_inputs[seg.tensor]
            if kind == LINEAR:
                g = chunk_wgrad(X, dY, seg.begin, seg.end, dense=False)
            else:
                g = vector_wgrad(X, dY, seg.begin, seg.end)
            lo, hi = seg.chunk_off, seg.chunk_off + (seg.end - seg.begin)
            th, mm, vv = adamw_step(g, params[seg.tensor][seg.begin:seg.end], m[lo:hi], v[lo:hi],
                                    step=steps[k], **hp)
            new_params[seg.tensor][seg.begin:seg.end] = th
            m[lo:hi] = mm
            v[lo:hi] = vv
        new_states.append({"m": m, "v": v})
    return new_params, new_states

"""Shared plumbing of the GPU parity tests: move a seeded case to the device,
call libchunkft through its ctypes binding, bring results back, and the
comparison rules.  Not a test module itself.

Comparison rules (the tolerances the build is held to):

* gradient: relative Frobenius error over the chunk, 3e-3 for bf16 inputs with
  fp32 accumulation, 1e-5 for the fp32 configuration;
* AdamW state fed the SAME fp32 gradient on both sides: element-wise
  |a - b| <= 1e-5 * max(|b|, floor), floor = 1e-2 * rms(b) for theta and m
  (their update is a difference and may cancel), none for v (a sum of
  non-negative terms); the elements under the floor are counted, printed and
  held to at most 2 % of the array;
* fused path against the full oracle: max|a - b| / max|b| <= 1e-5 for m and v;
  the same for theta, except that on a cold start (m = v = 0) the step is
  lr * g / (|g| + eps), a sign function where g is tiny, which no
  finite-precision gradient can reproduce: elements with |g| < 1e-4 rms(g)
  are then only required to move by at most 2 lr (+ 1e-5 |theta|);
* low-precision copy: bit-exact round-to-nearest-even of the GPU's own fp32
  master, and within one bf16 step of the oracle's rounded value where a bf16
  step is at least the 1e-5 of the largest parameter that the two masters may
  differ by (|theta| >= 2.56e-3 max|theta|); closer to zero the rounded value is
  within that difference plus one step of the oracle's master;
* anything outside the chunk: bit-identical to before the call.
"""

from __future__ import annotations

import numpy as np
import torch

from oracle import chunkft_oracle as O
from paper_2605_21177_amd import binding as B
from paper_2605_21177_amd import workloads as WL

DEV = "cuda:0"
GUARD = 64          # canary elements on both sides of every chunk-local array
CANARY = 12345.678


def require_gpu():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    B.lib()  # fails loudly if the library was not built


class DeviceLayer:
    def __init__(self, case: WL.LayerCase, split_k: int = 0):
        self.case = case
        self.X = case.X.to(DEV)
        self.dY = case.dY.to(DEV)
        self.split_k = split_k

    def layer(self, split_k=None) -> B.Layer:
        sk = self.split_k if split_k is None else split_k
        return B.make_layer(self.case.kind, self.X, self.dY, self.case.out, self.case.n_in, sk,
                            norm_eps=self.case.eps)


# When set to a tensor element index, guarded() places element 0 of the fp32 arrays it makes at
# the 128-byte phase of that element (the layout include/chunkft.h recommends); otherwise the
# arrays start GUARD elements into a fresh allocation.
PHASE_OF = None


class phase_aligned:
    """with phase_aligned(begin): chunk arrays are laid out at the phase of tensor element begin."""

    def __init__(self, begin: int):
        self.begin = begin

    def __enter__(self):
        global PHASE_OF
        self.prev, PHASE_OF = PHASE_OF, self.begin

    def __exit__(self, *exc):
        global PHASE_OF
        PHASE_OF = self.prev


def guarded(n: int, fill=None, dtype=torch.float32):
    """Device array of n elements inside canary bands; returns (full, view)."""
    lead = GUARD
    full = torch.full((n + 2 * GUARD + 32,), CANARY, dtype=dtype, device=DEV)
    if PHASE_OF is not None and dtype == torch.float32:
        lead += (PHASE_OF - (full.data_ptr() // 4 + GUARD)) % 32
    view = full[lead:lead + n]
    if fill is not None:
        view.copy_(fill if torch.is_tensor(fill) else torch.as_tensor(fill, dtype=dtype))
    full._lead, full._n = lead, n
    return full, view


def guards_intact(full: torch.Tensor) -> bool:
    c = torch.tensor(CANARY, dtype=full.dtype).item()
    lead, n = full._lead, full._n
    return bool((full[:lead] == c).all().item() and (full[lead + n:] == c).all().item())


_WS_FULL = {}


def workspace_for(layer: B.Layer, begin: int, end: int):
    """Exactly chunkft_workspace_bytes() of workspace, between canary bands (see workspace_intact)."""
    nbytes = B.chunkft_workspace_bytes(layer, begin, end)
    if nbytes == 0:
        return None
    assert nbytes % 4 == 0
    full = torch.full((nbytes // 4 + 2 * GUARD,), CANARY, dtype=torch.float32, device=DEV)
    view = full[GUARD:GUARD + nbytes // 4]
    _WS_FULL[view.data_ptr()] = full
    return view


def workspace_intact(ws) -> bool:
    """Nothing was written outside the workspace handed out by workspace_for()."""
    if ws is None:
        return True
    full = _WS_FULL.pop(ws.data_ptr())
    c = torch.tensor(CANARY, dtype=torch.float32).item()
    return bool((full[:GUARD] == c).all().item() and (full[-GUARD:] == c).all().item())


def gpu_wgrad(dl: DeviceLayer, begin, end, split_k=None, accumulate_into=None):
    layer = dl.layer(split_k)
    n = end - begin
    init = accumulate_into if accumulate_into is not None else None
    full, g = guarded(n, init)
    ws = workspace_for(layer, begin, end)
    B.chunkft_chunk_wgrad(layer, begin, end, g, accumulate=accumulate_into is not None, ws=ws)
    torch.cuda.synchronize()
    assert guards_intact(full), "chunk gradient wrote outside [0, end - begin)"
    assert workspace_intact(ws), "wrote outside the workspace"
    return g.cpu().numpy().astype(np.float64)


def gpu_fused(dl: DeviceLayer, begin, end, W0, master0, m0, v0, hp: dict, step: int, split_k=None):
    """Returns (W_bits or None, master, m, v) after one fused call."""
    layer = dl.layer(split_k)
    n = end - begin
    fm, master = guarded(n, master0)
    fmm, m = guarded(n, m0)
    fv, v = guarded(n, v0)
    W = None if W0 is None else W0.clone().to(DEV)
    ws = workspace_for(layer, begin, end)
    B.chunkft_wgrad_adamw_fused(layer, begin, end, W, master, m, v, B.hparams(step=step, **hp), ws=ws)
    torch.cuda.synchronize()
    assert guards_intact(fm) and guards_intact(fmm) and guards_intact(fv), "state written outside the chunk"
    assert workspace_intact(ws), "wrote outside the workspace"
    Wc = None if W is None else W.cpu()
    return Wc, master.cpu().numpy(), m.cpu().numpy(), v.cpu().numpy()


def gpu_adamw(g, master0, m0, v0, W_slice, hp: dict, step: int, w_dtype=B.BF16):
    n = g.numel()
    fm, master = guarded(n, master0)
    fmm, m = guarded(n, m0)
    fv, v = guarded(n, v0)
    B.chunkft_adamw_chunk(g, master, m, v, W_slice, n, B.hparams(step=step, **hp), w_dtype=w_dtype)
    torch.cuda.synchronize()
    assert guards_intact(fm) and guards_intact(fmm) and guards_intact(fv)
    return master.cpu().numpy(), m.cpu().numpy(), v.cpu().numpy()


# ------------------------------------------------------------- comparisons
def rel_frobenius(a, b) -> float:
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    nb = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / nb) if nb > 0 else float(np.linalg.norm(a - b))


def assert_elementwise(a, b, floor_frac, what, rtol=1e-5, max_floored=0.02):
    """|a - b| <= rtol * max(|b|, floor), floor = floor_frac * rms(b).  With a floor the number of
    elements it protects (0 < |b| < floor) is printed and must stay a small share of the array:
    about 0.8 % of a Gaussian lies below a hundredth of its rms."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    floor = floor_frac * float(np.sqrt(np.mean(b * b))) if floor_frac > 0 else 0.0
    denom = np.maximum(np.abs(b), max(floor, 1e-300))
    err = np.abs(a - b) / denom
    bad = ~(err <= rtol)
    # exact zeros on both sides (never-touched moments) are fine
    bad &= ~((a == 0) & (b == 0))
    assert not bad.any(), f"{what}: max relative error {np.nanmax(err):.3e} at {int(np.nanargmax(err))}"
    if floor > 0:
        under = int(np.count_nonzero((np.abs(b) < floor) & (b != 0)))
        beyond = int(np.count_nonzero((np.abs(a - b) > rtol * np.abs(b)) & (np.abs(b) < floor) & (b != 0)))
        print(f"[floor] {what}: {under} of {b.size} elements below {floor_frac:g} rms "
              f"({100.0 * under / max(b.size, 1):.3f} %), {beyond} of them beyond {rtol:g} of their own size", flush=True)
        assert under <= 3 + max_floored * b.size, f"{what}: {under} of {b.size} elements sit under the floor"


def assert_scale_relative(a, b, what, rtol=1e-5, mask=None):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    scale = float(np.max(np.abs(b)))
    d = np.abs(a - b)
    if mask is not None:
        d = d[mask]
    worst = float(d.max()) if d.size else 0.0
    assert worst <= rtol * scale, f"{what}: max |a-b| / max|b| = {worst / scale:.3e}"


def check_fused_against_oracle(g_ref, th0, m0, v0, hp, step, master, m, v, W_bits=None):
    """Fused-path outputs against the full fp64 oracle (rules in the module docstring)."""
    th_ref, m_ref, v_ref = O.adamw_step(g_ref, th0, m0, v0, step=step, **hp)
    assert_scale_relative(m, m_ref, "m")
    assert_scale_relative(v, v_ref, "v")
    rms = float(np.sqrt(np.mean(g_ref * g_ref)))
    cold = not (np.any(m0) or np.any(v0))
    if cold:
        # from m = v = 0 the step is lr * g / (|g| + eps): a sign function where g is tiny
        # (an exactly zero gradient -- an embedding row that no token names -- is exact on both sides)
        well = (np.abs(g_ref) >= 1e-4 * rms) | (g_ref == 0)
    else:
        # warm moments dominate a tiny gradient: every element is well-conditioned
        well = np.ones(g_ref.shape, dtype=bool)
    assert_scale_relative(master, th_ref, "theta (well-conditioned elements)", mask=well)
    ill = ~well
    # a Gaussian gradient has about 8e-5 of its elements below 1e-4 rms
    assert ill.sum() <= 3 + 5e-4 * ill.size, f"too many tiny-gradient elements: {int(ill.sum())} of {ill.size}"
    if ill.any():
        moved = np.abs(np.asarray(master, np.float64)[ill] - np.asarray(th0, np.float64)[ill])
        assert np.all(moved <= 2 * hp["lr"] + 1e-5 * np.abs(np.asarray(th0, np.float64)[ill]) + 1e-12), \
            "an element with a tiny gradient moved by more than two learning rates"
    if W_bits is not None:
        # bit-exact rounding of the GPU's own master, and one grid step from the oracle's
        assert np.array_equal(W_bits, O.bf16_bits(np.asarray(master, dtype=np.float64))), \
            "low-precision copy is not the round-to-nearest-even of the GPU's own master"
        ref_bits = O.bf16_bits(th_ref).astype(np.int64)
        ulp = np.abs(W_bits.astype(np.int64) - ref_bits)
        # The two masters may differ by 1e-5 of the largest parameter (checked above).  Where a bf16 step
        # (2^-8 of the value) is at least that large the two roundings are the same or neighbouring grid
        # points (bit patterns of same-sign neighbours differ by 1); for the few parameters closer to zero
        # the difference spans several of their much finer steps, and the rounded value itself is compared.
        scale = float(np.max(np.abs(th_ref)))
        coarse = well & (np.abs(th_ref) >= 256 * 1e-5 * scale)
        if coarse.any():
            assert ulp[coarse].max() <= 1, \
                f"low-precision copy {int(ulp[coarse].max())} steps from the oracle's at element {int(np.argmax(ulp * coarse))}"
        fine = well & ~coarse
        if fine.any():
            val = (W_bits[fine].astype(np.uint32) << 16).view(np.float32).astype(np.float64)
            assert np.all(np.abs(val - th_ref[fine]) <= 1e-5 * scale + np.abs(th_ref[fine]) / 256), \
                "low-precision copy of a parameter near zero is off by more than the masters may differ"
    return th_ref, m_ref, v_ref

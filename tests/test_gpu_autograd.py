"""GPU tests of the autograd wrapper: a two-layer block whose backward calls
libchunkft for the active chunk (Algorithm 1 line 8, Section 3.2).

The operands each layer's backward saw (X from the forward pass, dY captured by a
tensor hook) are torch's; the expected gradient is the fp64 oracle's on exactly
those operands, restricted to the chunk's segment on each weight.
"""

import numpy as np
import pytest
import torch

from oracle import chunkft_oracle as O
from paper_2605_21177_amd import autograd as A
from paper_2605_21177_amd import binding as B
from paper_2605_21177_amd import workloads as WL

import gpu_harness as H

pytestmark = pytest.mark.gpu

HP = WL.HPARAMS


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    H.require_gpu()


def _block(seed, T=(3, 70), d0=264, d1=520, d2=136):
    """x [3, 70, d0] -> W1 [d1, d0] -> relu -> W2 [d2, d1]; loss = sum(y * R)."""
    gen = torch.Generator().manual_seed(seed)
    x = torch.randn(*T, d0, generator=gen).to(torch.bfloat16)
    W1 = (0.05 * torch.randn(d1, d0, generator=gen)).to(torch.bfloat16)
    W2 = (0.05 * torch.randn(d2, d1, generator=gen)).to(torch.bfloat16)
    R = (1e-3 * torch.randn(*T, d2, generator=gen)).to(torch.bfloat16)
    return x, W1, W2, R


def _run_backward(x, W1, W2, R, seg1, seg2, x_requires_grad=False):
    """One forward + backward on the GPU; returns what each layer's backward consumed."""
    xd = x.to(H.DEV).requires_grad_(x_requires_grad)
    seen = {}
    h = torch.relu(A.chunk_linear(xd, W1, seg1))
    h.register_hook(lambda gr: seen.__setitem__("dh", gr.detach().clone()))
    y = A.chunk_linear(h, W2, seg2)
    y.register_hook(lambda gr: seen.__setitem__("dy", gr.detach().clone()))
    loss = (y.float() * R.to(H.DEV).float()).sum()
    loss.backward()
    torch.cuda.synchronize()
    pre = A.chunk_linear(xd.detach(), W1, None)          # pre-activation again, for relu's mask
    dy1 = seen["dh"] * (pre > 0).to(seen["dh"].dtype)
    ops = {
        1: (xd.detach().reshape(-1, W1.shape[1]).cpu(), dy1.reshape(-1, W1.shape[0]).cpu()),
        2: (h.detach().reshape(-1, W2.shape[1]).cpu(), seen["dy"].reshape(-1, W2.shape[0]).cpu()),
    }
    return ops, xd.grad


def _oracle_grad(ops, which, begin, end):
    X, dY = ops[which]
    return O.chunk_wgrad(WL.as_f64(X), WL.as_f64(dY), begin, end)


def test_backward_fills_the_chunk_gradient_and_accumulates_micro_batches():
    x, W1, W2, R = _block(5)
    W1d, W2d = W1.to(H.DEV), W2.to(H.DEV)
    # one chunk: the tail of W1 from mid-row and the head of W2 to mid-row
    b1, e1 = 300 * 264 + 17, W1.numel()
    b2, e2 = 0, 57 * 520 + 333
    full1, g1 = H.guarded(e1 - b1)
    full2, g2 = H.guarded(e2 - b2)
    seg1, seg2 = A.ChunkSegment(b1, e1, g1), A.ChunkSegment(b2, e2, g2)

    ops_a, xgrad = _run_backward(x, W1d, W2d, R, seg1, seg2, x_requires_grad=True)
    assert seg1.micro_batches == 1 and seg2.micro_batches == 1
    assert H.guards_intact(full1) and H.guards_intact(full2)
    ref1, ref2 = _oracle_grad(ops_a, 1, b1, e1), _oracle_grad(ops_a, 2, b2, e2)
    assert H.rel_frobenius(g1.cpu().numpy(), ref1) <= 3e-3
    assert H.rel_frobenius(g2.cpu().numpy(), ref2) <= 3e-3
    # the input gradient is passed on: dX = dY1 W1
    dx_ref = WL.as_f64(ops_a[1][1]) @ WL.as_f64(W1)
    assert H.rel_frobenius(xgrad.float().cpu().numpy().reshape(dx_ref.shape), dx_ref) <= 1e-2

    # a second micro-batch adds to the first
    x_b, _, _, R_b = _block(6)
    ops_b, _ = _run_backward(x_b, W1d, W2d, R_b, seg1, seg2)
    assert seg1.micro_batches == 2
    assert H.guards_intact(full1) and H.guards_intact(full2)
    assert H.rel_frobenius(g1.cpu().numpy(), ref1 + _oracle_grad(ops_b, 1, b1, e1)) <= 3e-3
    assert H.rel_frobenius(g2.cpu().numpy(), ref2 + _oracle_grad(ops_b, 2, b2, e2)) <= 3e-3

    # after reset() the next backward overwrites
    seg1.reset()
    seg2.reset()
    _run_backward(x, W1d, W2d, R, seg1, seg2)
    assert H.rel_frobenius(g1.cpu().numpy(), ref1) <= 3e-3
    assert H.rel_frobenius(g2.cpu().numpy(), ref2) <= 3e-3


def test_first_layer_backward_runs_without_input_gradient_and_inactive_tensors_are_skipped():
    x, W1, W2, R = _block(8)
    W1d, W2d = W1.to(H.DEV), W2.to(H.DEV)
    b1, e1 = 1000, 90000
    full1, g1 = H.guarded(e1 - b1)
    seg1 = A.ChunkSegment(b1, e1, g1)
    idle = A.ChunkSegment(0, 0)
    ops, xgrad = _run_backward(x, W1d, W2d, R, seg1, idle)
    assert xgrad is None and seg1.micro_batches == 1 and idle.micro_batches == 0
    assert H.guards_intact(full1)
    assert H.rel_frobenius(g1.cpu().numpy(), _oracle_grad(ops, 1, b1, e1)) <= 3e-3


def test_fused_mode_updates_the_segment_in_backward():
    x, W1, W2, R = _block(9)
    W1d, W2d = W1.to(H.DEV), W2.clone().to(H.DEV)
    b2, e2 = 11 * 520 + 5, 120 * 520 + 519
    n = e2 - b2
    th0 = W2.reshape(-1)[b2:e2].float()
    fm, master = H.guarded(n, th0)
    fmm, m = H.guarded(n)
    fv, v = H.guarded(n)
    m.zero_()
    v.zero_()
    seg2 = A.ChunkSegment(b2, e2, master=master, m=m, v=v, hp=B.hparams(step=1, **HP))
    ops, xgrad = _run_backward(x, W1d, W2d, R, None, seg2, x_requires_grad=True)
    assert H.guards_intact(fm) and H.guards_intact(fmm) and H.guards_intact(fv)
    # X of layer 2 and the gradients passed down were computed with W2 as it was before the update
    g_ref = O.chunk_wgrad(WL.as_f64(ops[2][0]), WL.as_f64(ops[2][1]), b2, e2)
    zero = np.zeros(n)
    H.check_fused_against_oracle(g_ref, th0.numpy().astype(np.float64), zero, zero, HP, 1,
                                 master.cpu().numpy(), m.cpu().numpy(), v.cpu().numpy(),
                                 W_bits=WL.bits_u16(W2d.reshape(-1)[b2:e2].cpu()))
    # outside the segment W2 is untouched
    W2f, W2df = W2.reshape(-1), W2d.reshape(-1).cpu()
    assert torch.equal(W2df[:b2].view(torch.int16), W2f[:b2].view(torch.int16))
    assert torch.equal(W2df[e2:].view(torch.int16), W2f[e2:].view(torch.int16))
    dh_ref = WL.as_f64(ops[2][1]) @ WL.as_f64(W2)
    # a second backward in the same optimizer step is refused in fused mode
    with pytest.raises(RuntimeError):
        _run_backward(x, W1d, W2d, R, None, seg2)
    assert np.isfinite(dh_ref).all() and xgrad is not None


def test_argument_checks():
    W = torch.zeros(8, 8, dtype=torch.bfloat16, device=H.DEV, requires_grad=True)
    x = torch.zeros(4, 8, dtype=torch.bfloat16, device=H.DEV)
    with pytest.raises(ValueError):
        A.chunk_linear(x, W, None)
    with pytest.raises(ValueError):
        A.ChunkSegment(5, 3)
    with pytest.raises(ValueError):
        A.ChunkSegment(0, 8)                      # neither g nor state
    with pytest.raises(ValueError):
        A.ChunkSegment(0, 8, master=x)            # incomplete state

"""GPU tests of the autograd wrapper: a two-layer block whose backward calls
libchunkft for the active chunk (Algorithm 1 line 18, Section 3.1).

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


def _block(seed, T=(3, 70), d0=264, d1=520, d2=136, dtype=torch.bfloat16):
    """x [3, 70, d0] -> W1 [d1, d0] -> relu -> W2 [d2, d1]; loss = sum(y * R)."""
    gen = torch.Generator().manual_seed(seed)
    x = torch.randn(*T, d0, generator=gen).to(dtype)
    W1 = (0.05 * torch.randn(d1, d0, generator=gen)).to(dtype)
    W2 = (0.05 * torch.randn(d2, d1, generator=gen)).to(dtype)
    R = (1e-3 * torch.randn(*T, d2, generator=gen)).to(dtype)
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
    ops["dh"] = seen["dh"].reshape(-1, W2.shape[1]).cpu()     # gradient w.r.t. the hidden activations
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
    # a large step (the first one moves every element by about lr): W2 after the update gives a
    # visibly different input gradient than W2 before it
    hp = dict(HP, lr=1e-2)
    seg2 = A.ChunkSegment(b2, e2, master=master, m=m, v=v, hp=B.hparams(step=1, **hp))
    ops, xgrad = _run_backward(x, W1d, W2d, R, None, seg2, x_requires_grad=True)
    assert H.guards_intact(fm) and H.guards_intact(fmm) and H.guards_intact(fv)
    g_ref = O.chunk_wgrad(WL.as_f64(ops[2][0]), WL.as_f64(ops[2][1]), b2, e2)
    zero = np.zeros(n)
    H.check_fused_against_oracle(g_ref, th0.numpy().astype(np.float64), zero, zero, hp, 1,
                                 master.cpu().numpy(), m.cpu().numpy(), v.cpu().numpy(),
                                 W_bits=WL.bits_u16(W2d.reshape(-1)[b2:e2].cpu()))
    # outside the segment W2 is untouched
    W2f, W2df = W2.reshape(-1), W2d.reshape(-1).cpu()
    assert torch.equal(W2df[:b2].view(torch.int16), W2f[:b2].view(torch.int16))
    assert torch.equal(W2df[e2:].view(torch.int16), W2f[e2:].view(torch.int16))
    # the gradient passed down to the hidden activations was computed with W2 as it was in the
    # forward pass, before the in-place update that the same backward makes
    dh = WL.as_f64(ops["dh"])
    dh_before = WL.as_f64(ops[2][1]) @ WL.as_f64(W2)
    dh_after = WL.as_f64(ops[2][1]) @ WL.as_f64(W2d.cpu())
    assert H.rel_frobenius(dh, dh_before) <= 1e-2
    assert H.rel_frobenius(dh_after, dh_before) >= 5e-2 and H.rel_frobenius(dh, dh_after) >= 5e-2
    assert xgrad is not None
    # a second backward in the same optimizer step is refused in fused mode
    with pytest.raises(RuntimeError):
        _run_backward(x, W1d, W2d, R, None, seg2)


@pytest.mark.parametrize("master_is_the_parameter", [False, True])
def test_fused_mode_fp32_weights_follow_the_update(master_is_the_parameter):
    """fp32 training: the weight the next forward multiplies with must carry the update, whether
    the chunk's master array is separate from the fp32 parameter or is the parameter's own range.
    Two optimizer steps; after each the segment of W equals the master bit for bit, the state
    matches the oracle, and the second forward runs on the updated weights."""
    x, W1, W2, R = _block(12, T=(2, 40), dtype=torch.float32)
    W1d, W2d = W1.to(H.DEV), W2.clone().to(H.DEV)
    b2, e2 = 7 * 520 + 3, 101 * 520 + 77
    n = e2 - b2
    if master_is_the_parameter:
        master = W2d.view(-1)[b2:e2]
    else:
        master = W2d.view(-1)[b2:e2].clone()
    m = torch.zeros(n, dtype=torch.float32, device=H.DEV)
    v = torch.zeros(n, dtype=torch.float32, device=H.DEV)
    th = W2.reshape(-1)[b2:e2].numpy().astype(np.float64)
    mm, vv = np.zeros(n), np.zeros(n)
    y_prev = None
    for step in (1, 2):
        W2_before = W2d.cpu().clone()
        seg2 = A.ChunkSegment(b2, e2, master=master, m=m, v=v, hp=B.hparams(step=step, **HP))
        ops, _ = _run_backward(x, W1d, W2d, R, None, seg2)
        X2, dY2 = ops[2]
        # the forward of this step used the weights as the previous step left them
        y = X2.double() @ W2_before.double().t()
        if y_prev is not None:
            assert H.rel_frobenius(y.numpy(), y_prev) > 1e-6      # the update reached the forward pass
        y_prev = y.numpy()
        g_ref = O.chunk_wgrad(X2.numpy().astype(np.float64), dY2.numpy().astype(np.float64), b2, e2)
        th_ref, m_ref, v_ref = O.adamw_step(g_ref, th, mm, vv, step=step, **HP)
        H.assert_scale_relative(m.cpu().numpy(), m_ref, "m")
        H.assert_scale_relative(v.cpu().numpy(), v_ref, "v")
        well = np.abs(g_ref) >= 1e-4 * np.sqrt(np.mean(g_ref ** 2))
        H.assert_scale_relative(master.cpu().numpy(), th_ref, "theta", mask=well)
        # the segment of W is the master, everything else is as before
        Wc = W2d.cpu().view(-1)
        assert torch.equal(Wc[b2:e2].view(torch.int32), master.cpu().view(torch.int32))
        assert not torch.equal(Wc[b2:e2], W2_before.view(-1)[b2:e2])
        assert torch.equal(Wc[:b2], W2_before.view(-1)[:b2]) and torch.equal(Wc[e2:], W2_before.view(-1)[e2:])
        # carry on from the GPU's own state, so that a sign flip at a tiny gradient does not compound
        th = master.cpu().numpy().astype(np.float64)
        mm, vv = m.cpu().numpy().astype(np.float64), v.cpu().numpy().astype(np.float64)


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

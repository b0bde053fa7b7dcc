"""Chunk-aware linear operator for torch autograd (Section 3.1, gradient of the active
slices only; Algorithm 1 line 18, the chunk-aware backward).

`chunk_linear(x, W, seg)` is `x @ W^T` whose backward passes the input gradient
on as usual but never forms the dense weight gradient: it hands the layer's
`X` and `dY` to libchunkft for the active segment `[begin, end)` of `W` only,
either into a gradient buffer (summed over micro-batches, the optimizer step is
then `chunkft_adamw_chunk`) or straight into the fused gradient + AdamW call.
`W` itself does not require grad.  The forward product and the input gradient
are torch's; every step of the chunk path runs in the library's kernels.
"""

from __future__ import annotations

from typing import Optional

import torch

from . import binding as B


class ChunkSegment:
    """The active chunk's segment on one weight tensor and where its gradient goes.

    Plain mode (`g` given): backward writes the segment's fp32 gradient to `g`
    (`end - begin` elements) on the first micro-batch after `reset()` and adds to
    it on the following ones.
    Fused mode (`master`, `m`, `v`, `hp` given): backward updates the chunk state
    and the segment of `W` in place (a bf16 `W` receives the rounded master, an fp32
    `W` a copy of it; `master` may also be the segment of an fp32 `W` itself, the
    parameter then being its own master); one micro-batch per step.
    A segment with `begin == end` (tensor not in the active chunk) makes backward
    skip the weight gradient altogether.
    """

    def __init__(self, begin: int, end: int, g=None, *, master=None, m=None, v=None,
                 hp: Optional[B.AdamWHparams] = None, split_k: int = 0):
        if not 0 <= begin <= end:
            raise ValueError("need 0 <= begin <= end")
        fused = master is not None
        if fused and (m is None or v is None or hp is None):
            raise ValueError("fused mode needs master, m, v and hp")
        if fused == (g is not None) and end > begin:
            raise ValueError("give either g (plain mode) or master/m/v/hp (fused mode)")
        self.begin, self.end = int(begin), int(end)
        self.g, self.master, self.m, self.v, self.hp = g, master, m, v, hp
        self.split_k = split_k
        self.micro_batches = 0
        self._ws = None

    @property
    def fused(self) -> bool:
        return self.master is not None

    def reset(self) -> None:
        """Start a new optimizer step: the next backward overwrites `g`."""
        self.micro_batches = 0

    def workspace(self, layer: B.Layer):
        need = B.chunkft_workspace_bytes(layer, self.begin, self.end)
        if need == 0:
            return None
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        return self._ws


class _ChunkLinear(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, W, anchor, seg):
        ctx.save_for_backward(x, W)
        ctx.seg = seg
        return x.matmul(W.t())

    @staticmethod
    def backward(ctx, dy):
        x, W = ctx.saved_tensors
        seg: Optional[ChunkSegment] = ctx.seg
        # the input gradient uses W as it was in the forward pass: enqueue it before any update
        dx = dy.matmul(W) if ctx.needs_input_grad[0] else None
        if seg is not None and seg.end > seg.begin:
            out, n_in = W.shape
            x2 = x.reshape(-1, n_in)
            dy2 = dy.reshape(-1, out)
            if x2.stride(1) != 1:
                x2 = x2.contiguous()
            if dy2.stride(1) != 1:
                dy2 = dy2.contiguous()
            layer = B.make_layer(B.LINEAR, x2, dy2, out, n_in, split_k=seg.split_k)
            ws = seg.workspace(layer)
            if seg.fused:
                if seg.micro_batches:
                    raise RuntimeError("fused mode takes one micro-batch per optimizer step")
                # W is what the next forward multiplies with: it always receives the update
                B.chunkft_wgrad_adamw_fused(layer, seg.begin, seg.end, W, seg.master, seg.m, seg.v, seg.hp, ws=ws)
            else:
                B.chunkft_chunk_wgrad(layer, seg.begin, seg.end, seg.g, accumulate=seg.micro_batches > 0, ws=ws)
            seg.micro_batches += 1
        return dx, None, None, None


_anchor = None


def chunk_linear(x: torch.Tensor, W: torch.Tensor, seg: Optional[ChunkSegment]) -> torch.Tensor:
    """`x @ W^T` with the chunk-restricted weight gradient in backward.  `W` is
    `[out, in]` row-major on the GPU, bf16 or fp32, and must not require grad."""
    if W.requires_grad:
        raise ValueError("W must not require grad: the dense weight gradient is never formed")
    if not W.is_contiguous():
        raise ValueError("W must be contiguous (the chunk is a range of its flattened elements)")
    global _anchor
    if _anchor is None or _anchor.device != x.device:
        # makes autograd run backward also for a first layer whose input needs no gradient
        _anchor = torch.zeros((), device=x.device, requires_grad=True)
    return _ChunkLinear.apply(x, W, _anchor, seg)

"""GPU test of chunkft_wgrad_adamw_fused_static: the fused call whose workspace is the library's
own static device array (for callers that cannot allocate).  It runs the kernels of
chunkft_wgrad_adamw_fused, so its outputs must equal that call's bit for bit -- on two calls in
a row, the second on a smaller input (the array keeps the first call's contents), for the
token-split path (slab partials) and for a normalising kind (per-token statistics)."""

import ctypes as C

import numpy as np
import pytest
import torch

from paper_2605_21177_amd import binding as B
from paper_2605_21177_amd import workloads as WL

import gpu_harness as H

pytestmark = pytest.mark.gpu

HP = WL.HPARAMS


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    H.require_gpu()


def _state(n, W_flat, begin, seed):
    rng = np.random.default_rng(seed)
    th = W_flat[begin:begin + n].float().clone()
    m = torch.from_numpy((rng.standard_normal(n) * 1e-3).astype(np.float32)).to(H.DEV)
    v = torch.from_numpy(((0.25 + rng.standard_normal(n) ** 2) * 1e-6).astype(np.float32)).to(H.DEV)
    return th, m, v


def _both_ways(layer, begin, end, W0, step, seed):
    """The existing entry point with a caller workspace, then the static one, on equal inputs."""
    n = end - begin
    hp = B.hparams(step=step, **HP)
    ws = H.workspace_for(layer, begin, end)
    assert ws is not None, "the case must need a workspace, or the static array is not exercised"
    ref = [t.clone() for t in _state(n, W0, begin, seed)]
    Wr = W0.clone()
    B.chunkft_wgrad_adamw_fused(layer, begin, end, Wr, ref[0], ref[1], ref[2], hp, ws=ws)
    torch.cuda.synchronize()
    assert H.workspace_intact(ws)
    guarded = [H.guarded(n, t) for t in _state(n, W0, begin, seed)]
    Ws = W0.clone()
    st = B.lib().chunkft_wgrad_adamw_fused_static(C.byref(layer), begin, end, Ws.data_ptr(),
                                                  guarded[0][1].data_ptr(), guarded[1][1].data_ptr(),
                                                  guarded[2][1].data_ptr(), C.byref(hp),
                                                  torch.cuda.current_stream().cuda_stream)
    assert st == B.OK, B.status_string(st)
    torch.cuda.synchronize()
    for (full, view), want, name in zip(guarded, ref, ("master", "m", "v")):
        assert H.guards_intact(full), name
        assert torch.equal(view.view(torch.int32), want.view(torch.int32)), name
    assert torch.equal(Ws.view(torch.int16), Wr.view(torch.int16))
    # and the update did something
    assert not torch.equal(guarded[0][1], _state(n, W0, begin, seed)[0])


def test_static_workspace_call_equals_the_workspace_call_twice_in_a_row():
    rng = np.random.default_rng(WL.SEED_BASE + 70)
    big = WL.linear_case(rng, "static-big", 776, 520, 300, WL.BF16, 1e-3)
    small = WL.linear_case(rng, "static-small", 264, 136, 96, WL.BF16, 1e-3)
    for case, (begin, end), split, seed in ((big, (520 * 3 + 17, 520 * 770 + 201), 4, 1),
                                            (small, (136 * 2 + 5, 136 * 200 + 77), 3, 2)):
        dl = H.DeviceLayer(case, split_k=split)
        layer = dl.layer()
        assert B.chunkft_split_k(layer, begin, end) == split
        W0 = case.W0.reshape(-1).clone().to(H.DEV)
        _both_ways(layer, begin, end, W0, step=2, seed=seed)


def test_static_workspace_holds_the_statistics_of_a_normalising_kind():
    rng = np.random.default_rng(WL.SEED_BASE + 71)
    for n_in, T in ((1032, 200), (264, 77)):
        X = torch.from_numpy(rng.standard_normal((T, n_in)).astype(np.float32)).to(torch.bfloat16).to(H.DEV)
        dY = torch.from_numpy((rng.standard_normal((T, n_in)) * 1e-3).astype(np.float32)).to(torch.bfloat16).to(H.DEV)
        layer = B.make_layer(B.RMSNORM, X, dY, 1, n_in, norm_eps=1e-5)
        W0 = torch.ones(n_in, dtype=torch.bfloat16, device=H.DEV)
        _both_ways(layer, 3, n_in - 5, W0, step=1, seed=3)


def test_static_workspace_refuses_what_does_not_fit_and_bad_arguments():
    """A forced split of a chunk whose slab partials exceed the static array is refused with its
    own status and nothing is written; argument errors are those of the workspace call."""
    T, out, n_in = 64, 4096, 4096
    X = torch.zeros(T, n_in, dtype=torch.bfloat16, device=H.DEV)
    dY = torch.zeros(T, out, dtype=torch.bfloat16, device=H.DEV)
    layer = B.make_layer(B.LINEAR, X, dY, out, n_in, split_k=2)
    begin, end = 0, out * n_in                        # 16 Mi elements x 2 slabs x 4 B = 128 MiB
    assert B.chunkft_workspace_bytes(layer, begin, end) > B.STATIC_WORKSPACE_BYTES
    n = end - begin
    full, master = H.guarded(n, torch.ones(n, device=H.DEV))
    m = torch.zeros(n, device=H.DEV)
    v = torch.zeros(n, device=H.DEV)
    st = B.chunkft_wgrad_adamw_fused_static(layer, begin, end, None, master, m, v, B.hparams(step=1, **HP), check=False)
    torch.cuda.synchronize()
    assert st == B.ERR_STATIC_WORKSPACE and "static" in B.status_string(st)
    assert H.guards_intact(full) and bool((master == 1).all().item()) and not bool(m.any().item())
    # the same argument errors as the workspace call
    assert B.chunkft_wgrad_adamw_fused_static(layer, 5, 5, None, master, m, v, B.hparams(step=1, **HP), check=False) == B.ERR_RANGE
    assert B.chunkft_wgrad_adamw_fused_static(layer, 0, 64, None, master, m, v, B.hparams(step=0, **HP), check=False) == B.ERR_INVALID_ARG

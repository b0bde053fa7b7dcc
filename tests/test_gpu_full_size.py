"""GPU parity at the full sizes of configurations 2-5, in the launch
configuration the benchmark times (default split, fused and un-fused calls).

At these sizes the fp64 oracle cannot produce every element in seconds, so each
case is checked on
  * sampled elements (the chunk's first and last ones, the elements around row
    boundaries, a few thousand random ones) and sampled complete rows, each
    computed by the oracle one by one;
  * a property that holds at any size: for sign vectors u (rows) and z
    (columns), u^T dW z = (dY u) . (X z), evaluated over the complete rows of the
    chunk -- one wrong tile, row or element anywhere changes it;
  * AdamW over sampled windows of the chunk against the oracle fed the GPU's own
    fp32 gradient (element-wise 1e-5), and over the sampled rows against the full
    oracle (the scale-relative rule of the small tests);
  * bit-identity of everything outside the chunk.
"""

import numpy as np
import pytest
import torch

from oracle import chunkft_oracle as O
from paper_2605_21177_amd import binding as B
from paper_2605_21177_amd import workloads as WL

import gpu_harness as H

pytestmark = pytest.mark.gpu

HP = WL.HPARAMS
MiB = 1 << 20


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    H.require_gpu()


def _say(msg):
    print(f"[full-size] {msg}", flush=True)


def _f32(t: torch.Tensor) -> np.ndarray:
    return t.float().numpy()


def _sample_rows(rng, r_first, r_last, k):
    """k distinct complete rows in [r_first, r_last], always with both ends."""
    rows = {r_first, r_last}
    while len(rows) < min(k, r_last - r_first + 1):
        rows.add(int(rng.integers(r_first, r_last + 1)))
    return np.array(sorted(rows), dtype=np.int64)


def _oracle_rows(case, rows):
    """fp64 gradient of whole rows: the oracle on the sub-layer made of those rows."""
    X64 = WL.as_f64(case.X)
    dY64 = WL.as_f64(case.dY[:, torch.from_numpy(rows)])
    return O.chunk_wgrad(X64, dY64, 0, rows.size * case.n_in, dense=True).reshape(rows.size, case.n_in)


def _oracle_elements(case, flat):
    """fp64 gradient of single elements (operands restricted to the rows in use)."""
    rows, inv = np.unique(flat // case.n_in, return_inverse=True)
    dY_sub = _f32(case.dY[:, torch.from_numpy(rows)])
    return O.wgrad_elements(_f32(case.X), dY_sub, inv * case.n_in + flat % case.n_in)


def _bilinear_reference(case, r_lo, r_hi, u, z):
    """(dY[:, r_lo:r_hi] u) . (X z) in fp64."""
    a = np.zeros(case.T)
    step = 4096
    for s in range(r_lo, r_hi, step):
        e = min(s + step, r_hi)
        a += WL.as_f64(case.dY[:, s:e]) @ u[s - r_lo:e - r_lo]
    b = WL.as_f64(case.X) @ z
    return float(a @ b)


def _bilinear_of(g_rows_cpu: torch.Tensor, u, z):
    """u^T G z for G [rows, in] fp32 on the CPU, accumulated in fp64, block by block."""
    total = 0.0
    step = 2048
    for s in range(0, g_rows_cpu.shape[0], step):
        blk = g_rows_cpu[s:s + step].numpy().astype(np.float64)
        total += float(u[s:s + step] @ (blk @ z))
    return total


def check_segment(case, dl, begin, end, *, split_k=None, fused=True, n_rows=8, n_elems=2000, seed=0):
    """One chunk segment of one tensor at full size; returns the gradient (device tensor)."""
    n_in = case.n_in
    E = end - begin
    rng = np.random.default_rng([9917, seed])
    layer = dl.layer(split_k)
    ws = H.workspace_for(layer, begin, end)
    _say(f"{case.name} {case.out}x{n_in} T={case.T} [{begin},{end}) split={B.chunkft_split_k(layer, begin, end)}")

    full_g, g = H.guarded(E)
    B.chunkft_chunk_wgrad(layer, begin, end, g, ws=ws)
    torch.cuda.synchronize()
    assert H.guards_intact(full_g)
    g_cpu = g.cpu()
    assert bool(torch.isfinite(g_cpu).all())

    # --- accumulate = 1 adds exactly this gradient to what the array holds (one fp32 addition per element)
    prefill = torch.randn(E, dtype=torch.float32, device=H.DEV, generator=torch.Generator(device=H.DEV).manual_seed(seed + 5)) * 1e-3
    full_a, ga = H.guarded(E, prefill)
    B.chunkft_chunk_wgrad(layer, begin, end, ga, accumulate=True, ws=ws)
    torch.cuda.synchronize()
    assert H.guards_intact(full_a)
    assert torch.equal(ga, prefill + g), "accumulated gradient differs from prefill + gradient"
    del full_a, ga, prefill

    # --- sampled elements
    r0, r1 = begin // n_in, (end - 1) // n_in
    picks = [np.arange(begin, min(begin + 128, end)), np.arange(max(end - 128, begin), end),
             rng.integers(begin, end, size=n_elems)]
    for r in rng.integers(r0, r1 + 1, size=6):
        lo, hi = max(begin, r * n_in - 4), min(end, r * n_in + 4)
        if lo < hi:
            picks.append(np.arange(lo, hi))
    flat = np.unique(np.concatenate(picks))
    ref_e = _oracle_elements(case, flat)
    got_e = g_cpu[torch.from_numpy(flat - begin)].numpy().astype(np.float64)
    assert H.rel_frobenius(got_e, ref_e) <= 3e-3, "sampled elements"
    rms = float(np.sqrt(np.mean(ref_e ** 2)))
    assert np.max(np.abs(got_e - ref_e)) <= 3e-3 * 8 * rms, "one sampled element is far off"

    # --- sampled complete rows
    rc0 = r0 + (1 if begin % n_in else 0)
    rc1 = r1 - (1 if end % n_in else 0)
    rows = None
    if rc1 >= rc0:
        rows = _sample_rows(rng, rc0, rc1, n_rows)
        ref_rows = _oracle_rows(case, rows)
        idx = (torch.from_numpy(rows * n_in - begin)[:, None] + torch.arange(n_in)[None, :]).reshape(-1)
        got_rows = g_cpu[idx].numpy().astype(np.float64).reshape(rows.size, n_in)
        assert H.rel_frobenius(got_rows, ref_rows) <= 3e-3, "sampled rows"

        # --- bilinear property over all complete rows
        u = rng.choice([-1.0, 1.0], size=rc1 - rc0 + 1)
        z = rng.choice([-1.0, 1.0], size=n_in)
        body = g_cpu[rc0 * n_in - begin:(rc1 + 1) * n_in - begin].view(rc1 - rc0 + 1, n_in)
        s_got = _bilinear_of(body, u, z)
        s_ref = _bilinear_reference(case, rc0, rc1 + 1, u, z)
        scale = float(np.sqrt(body.numel())) * rms
        assert abs(s_got - s_ref) <= 1e-4 * scale, f"bilinear property: {s_got} vs {s_ref} (scale {scale})"

    if not fused:
        assert H.workspace_intact(ws)
        return g

    # --- fused call on the same range
    W0 = case.W0.reshape(-1)
    Wd = W0.clone().to(H.DEV)
    th0_dev = Wd[begin:end].float()
    fm, master = H.guarded(E, th0_dev)
    fmm, m = H.guarded(E)
    fv, v = H.guarded(E)
    m.zero_()
    v.zero_()
    is_bf16 = case.dtype == WL.BF16
    B.chunkft_wgrad_adamw_fused(layer, begin, end, Wd if is_bf16 else None, master, m, v,
                                B.hparams(step=1, **HP), ws=ws)
    torch.cuda.synchronize()
    assert H.guards_intact(fm) and H.guards_intact(fmm) and H.guards_intact(fv)
    W0d = W0.to(H.DEV)
    assert torch.equal(Wd[:begin].view(torch.int16), W0d[:begin].view(torch.int16))
    assert torch.equal(Wd[end:].view(torch.int16), W0d[end:].view(torch.int16))
    # every element of the chunk was updated once: m = (1 - beta1) g is non-zero wherever g is
    assert int((m != 0).sum().item()) == int((g != 0).sum().item())

    # windows: AdamW of the oracle on the GPU's own gradient, element-wise
    wins = [(0, min(E, 1 << 16)), (max(0, E - (1 << 16)), E)]
    for s in rng.integers(0, max(1, E - (1 << 18)), size=4):
        wins.append((int(s), int(min(E, s + (1 << 18)))))
    for (a, b) in wins:
        gw = g_cpu[a:b].numpy()
        th0 = th0_dev[a:b].cpu().numpy()
        zero = np.zeros_like(th0)
        ref = O.adamw_step(gw, th0, zero, zero, step=1, **HP)
        H.assert_elementwise(master[a:b].cpu().numpy(), ref[0], 1e-2, "theta (window)")
        H.assert_elementwise(m[a:b].cpu().numpy(), ref[1], 1e-2, "m (window)")
        H.assert_elementwise(v[a:b].cpu().numpy(), ref[2], 0.0, "v (window)")
        if is_bf16:
            assert np.array_equal(WL.bits_u16(Wd[begin + a:begin + b].cpu()),
                                  O.bf16_bits(master[a:b].cpu().numpy().astype(np.float64)))

    # sampled rows: the full oracle (gradient and update)
    if rows is not None:
        idx_d = idx.to(H.DEV)
        th0_r = th0_dev[idx_d].cpu().numpy()
        zero = np.zeros_like(th0_r)
        bits = WL.bits_u16(Wd[idx_d + begin].cpu()) if is_bf16 else None
        H.check_fused_against_oracle(ref_rows.reshape(-1), th0_r, zero, zero, HP, 1,
                                     master[idx_d].cpu().numpy(), m[idx_d].cpu().numpy(),
                                     v[idx_d].cpu().numpy(), bits)

    # --- every element, two steps: the fused call equals the plain gradient followed by the AdamW call bit
    # for bit (the second step starts from warm moments, where an element updated twice or not at all shows)
    master_u, m_u, v_u = th0_dev.clone(), torch.zeros_like(th0_dev), torch.zeros_like(th0_dev)
    Wu = W0.clone().to(H.DEV) if is_bf16 else None
    for step in (1, 2):
        if step == 2:
            B.chunkft_wgrad_adamw_fused(layer, begin, end, Wd if is_bf16 else None, master, m, v,
                                        B.hparams(step=2, **HP), ws=ws)
        B.chunkft_adamw_chunk(g, master_u, m_u, v_u, Wu[begin:end] if is_bf16 else None, E, B.hparams(step=step, **HP),
                              w_dtype=B.BF16 if is_bf16 else B.F32)
        torch.cuda.synchronize()
        assert torch.equal(master, master_u) and torch.equal(m, m_u) and torch.equal(v, v_u), \
            f"step {step}: fused call and un-fused pair differ"
        if is_bf16:
            assert torch.equal(Wd.view(torch.int16), Wu.view(torch.int16)), f"step {step}: low-precision copies differ"
    assert H.guards_intact(fm) and H.guards_intact(fmm) and H.guards_intact(fv) and H.workspace_intact(ws)
    return g


# ------------------------------------------------------------ configuration 2
def test_config2_full_size_as_benchmarked():
    case, begin, end = WL.config2()
    assert end - begin == 32 * MiB
    dl = H.DeviceLayer(case)
    check_segment(case, dl, begin, end, seed=2)
    # row-aligned special case of the same size
    b0 = (begin // case.n_in) * case.n_in
    check_segment(case, dl, b0, b0 + 32 * MiB, fused=False, seed=22)


# ------------------------------------------------------------ configuration 3
def test_config3_full_size_cycle():
    layers = WL.config3()
    tensors = [(c.out, c.n_in, c.dtype, c.kind) for c in layers]
    budget = 256 * MiB
    st, chunks, segs = B.chunkft_plan_cycle(tensors, budget)
    oc = O.plan_cycle([c.desc() for c in layers], budget)
    assert [(s.tensor, s.begin, s.end, s.chunk_off) for ch in oc for s in ch] == segs
    assert len(chunks) == 2 and sum(c[2] for c in chunks) == sum(c.numel for c in layers)
    covered = {t: 0 for t in range(len(layers))}
    dls = {}
    for k, (s0, s1, numel, _) in enumerate(chunks):
        for (t, b, e, off) in segs[s0:s1]:
            case = layers[t]
            covered[t] += e - b
            if case.kind == WL.VECTOR:
                continue                      # the scale vectors are checked element by element below
            if t not in dls:
                dls[t] = H.DeviceLayer(case)
            check_segment(case, dls[t], b, e, n_rows=4, n_elems=500, seed=30 + t)
            if len(dls) > 2:                  # keep at most two layers' operands on the device
                dls.pop(next(iter(dls)))
    assert all(covered[t] == layers[t].numel for t in covered)
    for case in layers:
        if case.kind == WL.VECTOR:
            dl = H.DeviceLayer(case)
            layer = dl.layer()
            _, g = H.guarded(case.n_in)
            B.chunkft_chunk_wgrad(layer, 0, case.n_in, g)
            torch.cuda.synchronize()
            ref = O.vector_wgrad(WL.as_f64(case.X), WL.as_f64(case.dY), 0, case.n_in)
            assert H.rel_frobenius(g.cpu().numpy(), ref) <= 3e-3


def test_config3_full_size_cycle_in_one_launch_per_chunk():
    """The transformer block at full size in the benchmark's launch shape: each of the planner's two chunks
    (6 and 4 segments, 4096 and 2688 work items) through chunkft_wgrad_adamw_fused_group, with the chunk's state in
    one set of arrays cut at the planner's chunk_off.  Every segment's state and every tensor's bf16 copy must equal,
    bit for bit, what one chunkft_wgrad_adamw_fused call per segment gives (whose values the test above holds
    against the oracle); nothing outside the chunks' state arrays is written."""
    layers = WL.config3()
    tensors = [(c.out, c.n_in, c.dtype, c.kind) for c in layers]
    st, chunks, segs = B.chunkft_plan_cycle(tensors, 256 * MiB)
    dls = [H.DeviceLayer(c) for c in layers]
    hp = B.hparams(step=1, **HP)
    results = []
    for grouped in (False, True):
        Wd = [c.W0.reshape(-1).clone().to(H.DEV) for c in layers]
        states = []
        for (s0, s1, numel, _) in chunks:
            fm, master = H.guarded(numel)
            for (t, b, e, off) in segs[s0:s1]:
                master[off:off + (e - b)] = Wd[t][b:e].float()
            fmm, m = H.guarded(numel, torch.zeros(1).expand(numel))
            fv, v = H.guarded(numel, torch.zeros(1).expand(numel))
            if grouped:
                call = B.GroupCall([(dls[t].layer(), b, e, Wd[t], master[off:off + e - b], m[off:off + e - b],
                                     v[off:off + e - b]) for (t, b, e, off) in segs[s0:s1]], device=H.DEV)
                assert call.ws_bytes == 0                  # the kernel takes every segment of these chunks
                call(hp)
            else:
                for (t, b, e, off) in segs[s0:s1]:
                    n = e - b
                    B.chunkft_wgrad_adamw_fused(dls[t].layer(), b, e, Wd[t], master[off:off + n], m[off:off + n],
                                                v[off:off + n], hp)
            torch.cuda.synchronize()
            assert H.guards_intact(fm) and H.guards_intact(fmm) and H.guards_intact(fv)
            states.append((master, m, v))
        results.append((Wd, states))
    (Wa, sa), (Wb, sb) = results
    for k in range(len(chunks)):
        for x, y, name in zip(sa[k], sb[k], ("master", "m", "v")):
            assert torch.equal(x.view(torch.int32), y.view(torch.int32)), f"{name} of chunk {k}"
            del x, y
    for t in range(len(layers)):
        assert torch.equal(Wa[t].view(torch.int16), Wb[t].view(torch.int16)), f"W of tensor {t}"
    # every master value moved: one update per element of the block
    for k, (s0, s1, numel, _) in enumerate(chunks):
        for (t, b, e, off) in segs[s0:s1]:
            assert not bool((sb[k][0][off:off + e - b] == layers[t].W0.reshape(-1)[b:e].float().to(H.DEV)).any().item()) \
                or layers[t].kind == WL.VECTOR


# ------------------------------------------------------------ configuration 4
@pytest.fixture(scope="module")
def config4_layers():
    _say("drawing configuration 4 (about 10^9 values)")
    layers = WL.config4()
    yield layers
    del layers


def _config4_offsets(gate):
    length = 64 * MiB                                   # 128 MiB of bf16
    # seeded offset in the concatenated [gate | down] space, and one straddling the boundary
    chunks = WL.config4_chunks(gate.numel, gate.n_in, gate.numel, length)

    def start(segs):
        t, b, _ = segs[0]
        return b + (gate.numel if t == 1 else 0)

    off, straddle = start(chunks["seeded"]), start(chunks["straddling"])
    assert straddle == gate.numel - length // 3 - 17
    return length, off, straddle


def test_config4_full_size_gate(config4_layers):
    gate, _ = config4_layers
    length, off, straddle = _config4_offsets(gate)
    dl = H.DeviceLayer(gate)
    for o in (off, straddle):
        if o < gate.numel:
            check_segment(gate, dl, o, min(o + length, gate.numel), n_rows=4, n_elems=500, seed=40)
    # forced token splits at full size (gradient only)
    b = straddle - 5 * gate.n_in
    for s in (1, 2, 4, 8):
        check_segment(gate, dl, b, b + (8 * MiB), split_k=s, fused=False, n_rows=3, n_elems=300, seed=41 + s)
    # 1 GiB budget: more than both tensors together, so the chunk takes each tensor whole
    check_segment(gate, dl, 0, gate.numel, n_rows=4, n_elems=500, seed=46)


def test_config4_full_size_down(config4_layers):
    gate, down = config4_layers
    length, off, straddle = _config4_offsets(gate)
    dl = H.DeviceLayer(down)
    for o in (off, straddle):
        lo, hi = max(o, gate.numel) - gate.numel, o + length - gate.numel
        if hi > lo:
            check_segment(down, dl, lo, min(hi, down.numel), n_rows=4, n_elems=500, seed=47)
    check_segment(down, dl, 0, down.numel, n_rows=4, n_elems=500, seed=48)


def test_config4_full_size_straddling_chunk_in_one_launch(config4_layers):
    """The 128 MiB chunk that ends the gate projection and begins the down projection (two segments, both
    on the 256 x 256 tile at this token count) through chunkft_wgrad_adamw_fused_group, two steps (the second
    from warm moments): state and bf16 copies equal, bit for bit, one chunkft_wgrad_adamw_fused call per segment
    (whose values the two tests above hold against the oracle)."""
    gate, down = config4_layers
    length, _, straddle = _config4_offsets(gate)
    parts = [(gate, straddle, gate.numel, 0), (down, 0, straddle + length - gate.numel, gate.numel - straddle)]
    dls = [H.DeviceLayer(gate), H.DeviceLayer(down)]
    results = []
    for grouped in (False, True):
        Wd = [c.W0.reshape(-1).clone().to(H.DEV) for c, _, _, _ in parts]
        fm, master = H.guarded(length)
        for i, (c, b, e, off) in enumerate(parts):
            master[off:off + (e - b)] = Wd[i][b:e].float()
        fmm, m = H.guarded(length, torch.zeros(1).expand(length))
        fv, v = H.guarded(length, torch.zeros(1).expand(length))
        calls = [(dls[i].layer(), b, e, Wd[i], master[off:off + e - b], m[off:off + e - b], v[off:off + e - b])
                 for i, (c, b, e, off) in enumerate(parts)]
        group = B.GroupCall(calls, device=H.DEV) if grouped else None
        if grouped:
            assert group.ws_bytes == 0                     # the kernel takes both segments
        for step in (1, 2):
            hp = B.hparams(step=step, **HP)
            if grouped:
                group(hp)
            else:
                for (layer, b, e, W, ma, mm, vv) in calls:
                    B.chunkft_wgrad_adamw_fused(layer, b, e, W, ma, mm, vv, hp)
            torch.cuda.synchronize()
        assert H.guards_intact(fm) and H.guards_intact(fmm) and H.guards_intact(fv)
        results.append((Wd, (master, m, v)))
    (Wa, sa), (Wb, sb) = results
    for x, y, name in zip(sa, sb, ("master", "m", "v")):
        assert torch.equal(x.view(torch.int32), y.view(torch.int32)), name
    for i in range(2):
        assert torch.equal(Wa[i].view(torch.int16), Wb[i].view(torch.int16)), f"W of tensor {i}"
    # every element of the chunk was updated: no moment is left at zero where the gradient is not
    assert int((sb[1] == 0).sum().item()) <= 8


# ------------------------------------------------------------ configuration 5
def test_config5_full_size_chunk_sweep():
    case = WL.config5()
    dl = H.DeviceLayer(case)
    for i, (begin, end) in enumerate(WL.config5_ranges(case)):
        check_segment(case, dl, begin, end, n_rows=4, n_elems=500, seed=50 + i)


# ------------------------------------------------------------ flat indices past 32 bits
def test_flat_element_indices_beyond_32_bits():
    """A tensor of more than 2^31 elements (270000 x 8192) and a range that starts past element 2^31, mid-row:
    the plain gradient and the fused call (warm moments) of a linear layer on the MFMA path, and the same
    range of an embedding table, against the oracle; nothing outside the range changes.  The embedding's
    reference is the oracle on the rows the range touches (token ids re-based to the first of them; tokens
    that name other rows add nothing to the range)."""
    out, n_in, T = 270000, 8192, 72
    assert out * n_in > (1 << 31)
    rng = np.random.default_rng([9917, 77])
    begin = (1 << 31) + 4099
    end = begin + 3 * MiB + 5
    r0, r1 = begin // n_in, (end - 1) // n_in
    gen = torch.Generator(device=H.DEV).manual_seed(771)
    W = torch.zeros(out * n_in, dtype=torch.bfloat16, device=H.DEV)
    W[begin - 4096:end + 4096] = (torch.randn(end - begin + 8192, device=H.DEV, generator=gen) * 0.02).to(torch.bfloat16)
    W_before = W.clone()
    hp = dict(HP)

    def run(kind, Xh, dYh, g_ref, what):
        _say(f"{what}: {out}x{n_in} [{begin},{end})")
        Xd, dYd = Xh.to(H.DEV), dYh.to(H.DEV)
        layer = B.make_layer(kind, Xd, dYd, out, n_in)
        full_g, g = H.guarded(end - begin)
        ws = H.workspace_for(layer, begin, end)
        B.chunkft_chunk_wgrad(layer, begin, end, g, ws=ws)
        torch.cuda.synchronize()
        assert H.guards_intact(full_g)
        assert H.rel_frobenius(g.cpu().numpy(), g_ref) <= 3e-3, what
        th0 = W_before[begin:end].float().cpu().numpy()
        m0 = (rng.standard_normal(end - begin) * 1e-3).astype(np.float32)
        v0 = ((0.25 + rng.standard_normal(end - begin) ** 2) * 1e-6).astype(np.float32)
        fm, master = H.guarded(end - begin, th0)
        fmm, m = H.guarded(end - begin, m0)
        fv, v = H.guarded(end - begin, v0)
        W.copy_(W_before)
        B.chunkft_wgrad_adamw_fused(layer, begin, end, W, master, m, v, B.hparams(step=2, **hp), ws=ws)
        torch.cuda.synchronize()
        assert H.guards_intact(fm) and H.guards_intact(fmm) and H.guards_intact(fv) and H.workspace_intact(ws)
        assert torch.equal(W[:begin].view(torch.int16), W_before[:begin].view(torch.int16)), what
        assert torch.equal(W[end:].view(torch.int16), W_before[end:].view(torch.int16)), what
        H.check_fused_against_oracle(g_ref, th0, m0, v0, hp, 2, master.cpu().numpy(), m.cpu().numpy(),
                                     v.cpu().numpy(), WL.bits_u16(W[begin:end].cpu()))

    X = WL.normal(rng, (T, n_in), 1.0, WL.BF16)
    dY = WL.normal(rng, (T, out), 1e-3, WL.BF16)
    run(B.LINEAR, X, dY, O.chunk_wgrad(WL.as_f64(X), WL.as_f64(dY), begin, end, dense=False), "linear layer")
    del X, dY

    T_e = 600
    ids = rng.integers(0, out, size=T_e)
    inside = rng.random(T_e) < 0.6                      # most tokens name rows of the range, some of them the same row
    ids[inside] = rng.integers(r0, r1 + 1, size=int(inside.sum()))
    ids[:7] = r0 + 3
    dYe = WL.normal(rng, (T_e, n_in), 1e-3, WL.BF16)
    hit = (ids >= r0) & (ids <= r1)
    g_ref = O.embedding_wgrad(ids[hit] - r0, WL.as_f64(dYe)[hit], r1 - r0 + 1, begin - r0 * n_in, end - r0 * n_in)
    run(B.EMBEDDING, torch.from_numpy(ids.astype(np.int64)), dYe, g_ref, "embedding table")

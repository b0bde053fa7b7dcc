"""GPU parity: libchunkft (through its C ABI) against the CPU oracle, element by
element on the same seeded inputs.  Sizes here are ones the oracle finishes in
seconds while still spanning several tiles, ragged tails and both code paths
(MFMA body + FMA edge rows, FMA fallback, split over tokens)."""

import numpy as np
import pytest
import torch

from oracle import chunkft_oracle as O
from paper_2605_21177_amd import binding as B
from paper_2605_21177_amd import workloads as WL

import gpu_harness as H

pytestmark = pytest.mark.gpu

HP = WL.HPARAMS
TOL_G = {WL.BF16: 3e-3, WL.F32: 1e-5}


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    H.require_gpu()


def _state_for(case, begin, end, rng, warm):
    th0 = WL.as_f64(case.W0).reshape(-1)[begin:end].astype(np.float32)
    n = end - begin
    if warm:
        m0 = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        v0 = ((0.25 + rng.standard_normal(n) ** 2) * 1e-6).astype(np.float32)
    else:
        m0 = np.zeros(n, np.float32)
        v0 = np.zeros(n, np.float32)
    return th0, m0, v0


def _full_check(case, begin, end, split_k=None, warm=False, step=1, check_accum=True):
    """wgrad, accumulate, fused (+ fused == un-fused + AdamW bit for bit), W untouched outside."""
    dl = H.DeviceLayer(case)
    dY64 = WL.as_f64(case.dY)
    if case.kind == WL.EMBEDDING:
        g_ref = O.embedding_wgrad(case.X.numpy(), dY64, case.out, begin, end)
    elif case.kind == WL.LINEAR:
        g_ref = O.chunk_wgrad(WL.as_f64(case.X), dY64, begin, end, dense=(case.numel <= (1 << 22)))
    elif case.kind == WL.VECTOR:
        g_ref = O.vector_wgrad(WL.as_f64(case.X), dY64, begin, end)
    else:
        g_ref = O.norm_weight_wgrad(WL.as_f64(case.X), dY64, case.eps, case.kind == WL.LAYERNORM, begin, end)
    n = end - begin

    g = H.gpu_wgrad(dl, begin, end, split_k)
    err = H.rel_frobenius(g, g_ref)
    assert err <= TOL_G[case.dtype], f"gradient relative Frobenius error {err:.3e}"
    # determinism: the same call again gives the same bits
    g2 = H.gpu_wgrad(dl, begin, end, split_k)
    assert np.array_equal(g, g2)

    if check_accum:
        rng = np.random.default_rng(5)
        base = rng.standard_normal(n).astype(np.float32)
        ga = H.gpu_wgrad(dl, begin, end, split_k, accumulate_into=torch.from_numpy(base))
        assert np.array_equal(ga.astype(np.float32), (base + g.astype(np.float32)))

    rng = np.random.default_rng(6)
    th0, m0, v0 = _state_for(case, begin, end, rng, warm)
    is_bf16 = case.dtype == WL.BF16
    W0 = case.W0.reshape(-1) if is_bf16 else None
    Wd, master, m, v = H.gpu_fused(dl, begin, end, W0, th0, m0, v0, HP, step, split_k)
    W_bits = None
    if is_bf16:
        allbits = WL.bits_u16(Wd)
        before = WL.bits_u16(case.W0.reshape(-1))
        assert np.array_equal(allbits[:begin], before[:begin]) and np.array_equal(allbits[end:], before[end:]), \
            "low-precision parameters outside the chunk changed"
        W_bits = allbits[begin:end]
    H.check_fused_against_oracle(g_ref, th0, m0, v0, HP, step, master, m, v, W_bits)

    # the fused call equals the un-fused pair bit for bit
    gdev = torch.from_numpy(g.astype(np.float32)).to(H.DEV)
    Wslice = None
    if is_bf16:
        Wfull = case.W0.reshape(-1).clone().to(H.DEV)
        Wslice = Wfull[begin:end]
    master2, m2, v2 = H.gpu_adamw(gdev, th0, m0, v0, Wslice, HP, step)
    assert np.array_equal(master, master2) and np.array_equal(m, m2) and np.array_equal(v, v2)
    if is_bf16:
        assert np.array_equal(WL.bits_u16(Wfull.cpu()), allbits)
    return g, g_ref


# ------------------------------------------------------------ configuration 1
def test_config1_fp32_layer():
    case, begin, end = WL.config1()
    _full_check(case, begin, end)


def test_config1_standalone_adamw_elementwise():
    """The AdamW entry point alone, both sides fed the same fp32 gradient."""
    case, begin, end = WL.config1()
    g64 = O.chunk_wgrad(WL.as_f64(case.X), WL.as_f64(case.dY), begin, end)
    g32 = g64.astype(np.float32)
    th0 = WL.as_f64(case.W0).reshape(-1)[begin:end].astype(np.float32)
    z = np.zeros_like(th0)
    th, m, v = th0, z, z
    gdev = torch.from_numpy(g32).to(H.DEV)
    for step in (1, 2, 3):
        ref = O.adamw_step(g32, th, m, v, step=step, **HP)
        th, m, v = H.gpu_adamw(gdev, th, m, v, None, HP, step, w_dtype=B.F32)
        H.assert_elementwise(th, ref[0], 1e-2, f"theta step {step}")
        H.assert_elementwise(m, ref[1], 1e-2, f"m step {step}")
        H.assert_elementwise(v, ref[2], 0.0, f"v step {step}")


def test_chunk_array_has_the_phase_of_the_tensor_element():
    for begin in (0, 1, 3, 31, 32, 13233635, 4096 * 77 + 5):
        for n in (1, 7, 1000):
            a = B.chunk_array(n, begin, H.DEV, fill=torch.arange(n, dtype=torch.float32))
            assert a.numel() == n and a.dtype == torch.float32 and a.is_cuda
            assert (a.data_ptr() // 4 - begin) % 32 == 0
            assert torch.equal(a.cpu(), torch.arange(n, dtype=torch.float32))


def test_chunk_state_arrays_share_the_phase_and_keep_their_pitch():
    mib = 1 << 20
    for begin, n, count in ((0, 1, 3), (13233635, 1000, 3), (4096 * 77 + 5, (1 << 18) + 3, 4), (31, 3 << 18, 2)):
        arrs = B.chunk_state(n, begin, H.DEV, count)
        assert len(arrs) == count
        for a in arrs:
            assert a.numel() == n and a.dtype == torch.float32 and a.is_cuda
            assert (a.data_ptr() // 4 - begin) % 32 == 0
        for a, b in zip(arrs, arrs[1:]):
            d = b.data_ptr() - a.data_ptr()
            assert d >= 4 * n and d % mib == mib // 4          # a whole number of MiB plus 256 KiB, no overlap
        for i, a in enumerate(arrs):                            # disjoint: each keeps its own values
            a.fill_(float(i + 1))
        for i, a in enumerate(arrs):
            assert bool((a == float(i + 1)).all().item())


@pytest.mark.parametrize("phase", [0, 1, 3, 4, 17, 31])
def test_standalone_adamw_at_every_array_phase(phase):
    """The element-wise pass peels up to 31 leading elements so that its 16-byte groups start on a
    128-byte line: arrays at several phases inside a line, lengths that leave 0-3 trailing elements."""
    rng = np.random.default_rng([41, phase])
    for n in (1, 5, 30, 33, 1000, 4099 + phase):
        g32 = rng.standard_normal(n).astype(np.float32) * 1e-3
        th0 = rng.standard_normal(n).astype(np.float32) * 0.02
        # warm moments that do not cancel against the gradient, so every element is well-conditioned
        m0 = (g32 * rng.uniform(0.1, 0.9, n)).astype(np.float32)
        v0 = (g32 * g32 * rng.uniform(0.1, 0.9, n)).astype(np.float32)
        ref = O.adamw_step(g32, th0, m0, v0, step=3, **HP)
        with H.phase_aligned(phase):
            fg, gdev = H.guarded(n, torch.from_numpy(g32))
            th, m, v = H.gpu_adamw(gdev, th0, m0, v0, None, HP, 3, w_dtype=B.F32)
        assert H.guards_intact(fg)
        H.assert_elementwise(th, ref[0], 0.0, f"theta n={n}")
        H.assert_elementwise(m, ref[1], 0.0, f"m n={n}")
        H.assert_elementwise(v, ref[2], 0.0, f"v n={n}")


# -------------------------------------------------- adversarial ranges, bf16
def _small_bf16(out=520, n_in=264, T=100, seed=77, sigma_dy=1e-3):
    rng = np.random.default_rng(seed)
    return WL.linear_case(rng, "small", out, n_in, T, WL.BF16, sigma_dy)


RANGES_520x264 = [
    (0, 520 * 264),                 # the whole tensor
    (264 * 7 + 5, 264 * 7 + 6),     # a single element
    (264 * 9 + 10, 264 * 9 + 200),  # inside one row
    (264 * 16, 264 * 17),           # exactly one row, 8-aligned row index
    (264 * 3, 264 * 4),             # exactly one row, unaligned row index
    (264 * 8, 264 * 300 + 100),     # begin on a row boundary, end mid-row
    (264 * 5 + 77, 264 * 400),      # begin mid-row, end on a row boundary
    (264 * 2 + 33, 264 * 519 + 1),  # odd begin: 2-byte-aligned bf16 stores
    (264 * 6 + 1, 264 * 9 + 263),   # few rows: one body row between edge rows
    (264 * 1 + 1, 264 * 6 + 5),     # six rows, none of them in the 8-aligned body
    (264 * 259 + 263, 264 * 519),   # starts on the last element of a row
    (0, 264 * 4 + 100),             # from the tensor's first row: four complete rows, the partial one in the same 8-row group
    (0, 264 * 100 + 77),            # from the first row: a body of at most 128 rows and a partial last row
    (264 * 8, 264 * 11 + 5),        # begin on an 8-aligned row boundary, three complete rows, a partial one
    (264 * 16, 264 * 120 + 9),      # the same with a longer body that still leaves the edge rows to their own kernel
]


@pytest.mark.parametrize("begin,end", RANGES_520x264)
def test_bf16_ranges(begin, end):
    _full_check(_small_bf16(), begin, end)


@pytest.mark.parametrize("begin,end", [(0, 520 * 288), (288 * 2 + 33, 288 * 519 + 1), (288 * 8, 288 * 300 + 100),
                                       (288 * 5 + 77, 288 * 400), (288 * 259 + 287, 288 * 519)])
def test_bf16_ranges_with_chunk_arrays_at_the_tensor_phase(begin, end):
    """g, master, m, v laid out so that element i has the 128-byte phase of tensor element begin + i
    (the recommended layout: whole 16-byte groups per row, no left-over columns)."""
    with H.phase_aligned(begin):
        _full_check(_small_bf16(n_in=288), begin, end)


@pytest.mark.parametrize("T", [70, 96, 161, 2070, 2080])
def test_bf16_many_tiles_at_short_and_long_token_counts(T):
    """More than 128 tiles of 256 x 256 and a range with edge rows.  At the short token counts the plain
    gradient runs on the small tile (two workgroups per compute unit, 32x32x16 MFMAs), at the long ones on
    the large one (16x16x32 MFMAs) while the fused call stays on the small tile: the bit-identity of
    fused and un-fused results then holds across the two tiles and MFMA shapes.  Token counts that leave
    a ragged last slab (70, 161, 2070) or none (96, 2080)."""
    rng = np.random.default_rng([83, T])
    case = WL.linear_case(rng, "many tiles", 2400, 4096, T, WL.BF16, 1e-3)
    _full_check(case, 4096 * 3 + 77, 4096 * 2397 + 5, check_accum=True)


@pytest.mark.parametrize("begin,end", [(10928 * 3 + 40, 10928 * 779 + 9000), (10928 * 8, 10928 * 776)])
def test_bf16_long_token_count_takes_the_large_tile_in_the_fused_call(begin, end):
    """Many tokens and enough tiles send the fused call to the 256 x 256 tile with the AdamW epilogue (6144
    tokens; 4 tile rows x 43 tile columns = 172 large tiles, more than half the compute units, in rounds
    filled alike by both tiles: the rule of csrc/shape.cpp then compares 0.55 + 2600 / 6144 = 0.97 with 0.99):
    whole oracle comparison on a layer of four tile rows (the last of 8 - 11 rows) and a ragged last column
    tile, with and without edge rows, and the bit-identity of the fused call with the un-fused pair."""
    rng = np.random.default_rng(WL.SEED_BASE + 45)
    case = WL.linear_case(rng, "long-wide", 784, 10928, 6144, WL.BF16, 1e-3)
    _full_check(case, begin, end, check_accum=False)


@pytest.mark.parametrize("split_k", [2, 3, 4])
def test_bf16_forced_token_split(split_k):
    case = _small_bf16(T=200)
    begin, end = 264 * 2 + 33, 264 * 519 + 1
    g, _ = _full_check(case, begin, end, split_k=split_k, warm=True, step=2)
    layer = H.DeviceLayer(case).layer(split_k)
    assert B.chunkft_split_k(layer, begin, end) == split_k


@pytest.mark.parametrize("begin", [288 * 2 + 33, 288 * 8 + 5, 288 * 3 + 31])
def test_bf16_forced_token_split_with_arrays_at_the_tensor_phase(begin):
    """The slab partials are placed in the workspace at the line phase of the array they are summed
    into: with chunk arrays at the tensor's phase that placement starts at a non-zero offset."""
    case = _small_bf16(n_in=288, T=200)
    with H.phase_aligned(begin):
        _full_check(case, begin, 288 * 519 + 1, split_k=3, warm=True, step=2)


def test_bf16_random_shapes_and_ranges():
    """Seeded random layers (sizes that are multiples of 8, so the MFMA path takes them), token
    counts with ragged last slabs, ranges from one element to the whole tensor, with and without
    a forced token split: every branch of the tile kernel (partial tiles in both directions, edge
    rows folded or not, body-less chunks) against the oracle."""
    rng = np.random.default_rng(20250521)
    for case_no in range(28):
        out = 8 * int(rng.integers(1, 90))
        n_in = 8 * int(rng.integers(1, 75))
        T = int(rng.integers(1, 330))
        case = WL.linear_case(rng, f"rand{case_no}", out, n_in, T, WL.BF16, 1e-3)
        numel = out * n_in
        kind = case_no % 4
        if kind == 0:
            begin, end = 0, numel
        elif kind == 1:
            begin = int(rng.integers(0, numel))
            end = begin + 1 + int(rng.integers(0, min(numel - begin, 3 * n_in)))
        else:
            begin = int(rng.integers(0, numel - 1))
            end = int(rng.integers(begin + 1, numel + 1))
        split = None if case_no % 3 else int(rng.integers(2, 5))
        print(f"[random-case] {case_no}: {out}x{n_in} T={T} [{begin},{end}) split={split}", flush=True)
        _full_check(case, begin, end, split_k=split, check_accum=(case_no % 5 == 0), warm=(case_no % 2 == 1),
                    step=1 + case_no % 3)


def test_bf16_unaligned_shape_takes_fma_path():
    rng = np.random.default_rng(78)
    case = WL.linear_case(rng, "odd", 137, 100, 53, WL.BF16, 1e-3)   # in, out not multiples of 8
    for begin, end in ((0, 13700), (101, 9999), (5, 6)):
        _full_check(case, begin, end)
    _full_check(case, 101, 9999, split_k=2)


def test_bf16_strided_operands():
    """Row strides larger than the row length (views into wider buffers)."""
    rng = np.random.default_rng(79)
    out, n_in, T = 264, 136, 70
    case = WL.linear_case(rng, "strided", out, n_in, T, WL.BF16, 1e-3)
    Xw = torch.zeros(T, n_in + 24, dtype=torch.bfloat16, device=H.DEV)
    dYw = torch.zeros(T, out + 40, dtype=torch.bfloat16, device=H.DEV)
    Xw[:, :n_in] = case.X.to(H.DEV)
    dYw[:, :out] = case.dY.to(H.DEV)
    Xw[:, n_in:] = 99.0
    dYw[:, out:] = 99.0             # must never be read into a result
    layer = B.make_layer(B.LINEAR, Xw[:, :n_in], dYw[:, :out], out, n_in)
    begin, end = 136 * 3 + 7, 136 * 260 + 3
    full, g = H.guarded(end - begin)
    B.chunkft_chunk_wgrad(layer, begin, end, g)
    torch.cuda.synchronize()
    g_ref = O.chunk_wgrad(WL.as_f64(case.X), WL.as_f64(case.dY), begin, end)
    assert H.rel_frobenius(g.cpu().numpy(), g_ref) <= 3e-3 and H.guards_intact(full)


@pytest.mark.parametrize("log2_stride", [24, 25])
def test_bf16_very_large_row_strides(log2_stride):
    """The global->LDS loads address a lane's data as a 32-bit byte offset from a per-slab base: a dY row
    stride of 2^24 elements (offsets up to 2^30 bytes) stays on the MFMA path, one of 2^25 is beyond what
    the library accepts for it and takes the FMA kernel; both must give the gradient."""
    rng = np.random.default_rng(83 + log2_stride)
    out, n_in, T = 264, 136, 40 if log2_stride == 24 else 3
    case = WL.linear_case(rng, "wide-stride", out, n_in, T, WL.BF16, 1e-3)
    ld = (1 << log2_stride) + 8
    dYw = torch.zeros(T, ld, dtype=torch.bfloat16, device=H.DEV)
    dYw[:, :out] = case.dY.to(H.DEV)
    dYw[:, out:out + 64] = 99.0          # must never be read into a result
    X = case.X.to(H.DEV)
    layer = B.make_layer(B.LINEAR, X, dYw[:, :out], out, n_in)
    assert layer.lddy == ld
    begin, end = 136 * 3 + 7, 136 * 260 + 3
    full, g = H.guarded(end - begin)
    B.chunkft_chunk_wgrad(layer, begin, end, g)
    torch.cuda.synchronize()
    g_ref = O.chunk_wgrad(WL.as_f64(case.X), WL.as_f64(case.dY), begin, end)
    assert H.rel_frobenius(g.cpu().numpy(), g_ref) <= 3e-3 and H.guards_intact(full)
    del dYw


@pytest.mark.parametrize("seed", [101, 102])
def test_bf16_random_shapes_strides_ranges_and_splits(seed):
    """Seeded random bf16 layers: shape, row strides, token count, range (a third begin or end on a row
    boundary) and forced token split all drawn; the plain gradient on strided operands between canaries,
    the fused call against the full oracle, parameters outside the range untouched."""
    rng = np.random.default_rng(seed)
    for it in range(25):
        out, n_in, T = int(rng.integers(1, 90)) * 8, int(rng.integers(1, 90)) * 8, int(rng.integers(1, 300))
        case = WL.linear_case(rng, "random", out, n_in, T, WL.BF16, 1e-3)
        padx, pady = int(rng.integers(0, 4)) * 8, int(rng.integers(0, 4)) * 8
        Xw = torch.full((T, n_in + padx), 99.0, dtype=torch.bfloat16, device=H.DEV)
        dYw = torch.full((T, out + pady), 99.0, dtype=torch.bfloat16, device=H.DEV)
        Xw[:, :n_in] = case.X.to(H.DEV)
        dYw[:, :out] = case.dY.to(H.DEV)
        N = out * n_in
        b = int(rng.integers(0, N))
        e = int(rng.integers(b + 1, N + 1))
        if rng.random() < 0.3:
            b = (b // n_in) * n_in
        if rng.random() < 0.3:
            e = max(b + 1, (e // n_in) * n_in)
        sk = int(rng.choice([0, 0, 1, 2, 3, 5]))
        if sk > T:
            sk = 0
        what = f"case {it}: {out} x {n_in}, T {T}, strides +{padx} +{pady}, [{b}, {e}), split {sk}"
        layer = B.make_layer(B.LINEAR, Xw[:, :n_in], dYw[:, :out], out, n_in, sk)
        ws = H.workspace_for(layer, b, e)
        full, g = H.guarded(e - b)
        B.chunkft_chunk_wgrad(layer, b, e, g, ws=ws)
        torch.cuda.synchronize()
        g_ref = O.chunk_wgrad(WL.as_f64(case.X), WL.as_f64(case.dY), b, e)
        assert H.rel_frobenius(g.cpu().numpy(), g_ref) <= 3e-3, what
        assert H.guards_intact(full) and H.workspace_intact(ws), what
        th0 = WL.as_f64(case.W0).reshape(-1)[b:e].astype(np.float32)
        z = np.zeros_like(th0)
        Wd, master, m, v = H.gpu_fused(H.DeviceLayer(case), b, e, case.W0.reshape(-1), th0, z, z, HP, 1,
                                       sk if sk else None)
        bits, before = WL.bits_u16(Wd), WL.bits_u16(case.W0.reshape(-1))
        assert np.array_equal(bits[:b], before[:b]) and np.array_equal(bits[e:], before[e:]), what
        H.check_fused_against_oracle(g_ref, th0, z, z, HP, 1, master, m, v, bits[b:e])


@pytest.mark.parametrize("seed", [201, 202])
def test_random_cases_of_every_kind_cold_and_warm(seed):
    """Seeded random layers of every kind and dtype (fp32 and odd-shaped bf16 matrices on the plain-FMA
    path, bf16 matrices on the MFMA path with forced splits, scale vectors, embedding tables, the two
    self-normalising vectors), ranges that often start at the tensor's first element or on a row boundary
    and are often only a few rows long, half of them with warm moments: everything _full_check checks."""
    rng = np.random.default_rng(seed)
    for it in range(40):
        kind = rng.choice(["lin_f32", "lin_bf16_odd", "lin_bf16", "vec", "emb", "rms", "ln"])
        dtype = WL.BF16 if rng.random() < 0.6 else WL.F32
        T = int(rng.integers(1, 400))
        sk = None
        if kind == "lin_f32":
            case = WL.linear_case(rng, "f", int(rng.integers(1, 300)), int(rng.integers(1, 300)), T, WL.F32, 1e-3)
            sk = [None, None, 2, 3][int(rng.integers(0, 4))]
        elif kind == "lin_bf16_odd":
            case = WL.linear_case(rng, "o", int(rng.integers(1, 300)), int(rng.integers(1, 300)), T, WL.BF16, 1e-3)
            sk = [None, None, 2][int(rng.integers(0, 3))]
        elif kind == "lin_bf16":
            case = WL.linear_case(rng, "b", int(rng.integers(1, 120)) * 8, int(rng.integers(1, 120)) * 8, T, WL.BF16, 1e-3)
            sk = [None, 1, 2, 3][int(rng.integers(0, 4))]
        elif kind == "vec":
            case = WL.vector_case(rng, "v", int(rng.integers(1, 5000)), T, dtype, 1e-3)
        elif kind == "emb":
            case = WL.embedding_case(rng, "e", int(rng.integers(1, 400)), int(rng.integers(1, 2200)), T, dtype, 1e-3)
        else:
            case = WL.norm_case(rng, "n", int(rng.integers(2, 5000)), T, dtype, 1e-3,
                                WL.RMSNORM if kind == "rms" else WL.LAYERNORM)
        if sk is not None and sk > T:
            sk = None
        N = case.numel
        b = int(rng.integers(0, N))
        e = int(rng.integers(b + 1, N + 1))
        r = rng.random()
        if r < 0.25:
            b = 0
        elif r < 0.5:
            b = (b // case.n_in) * case.n_in
        if rng.random() < 0.3:
            e = min(N, b + int(rng.integers(1, 12 * case.n_in + 1)))
        e = max(e, b + 1)
        warm = bool(rng.random() < 0.5)
        print(f"[case {it}] {kind} dtype {case.dtype} {case.out} x {case.n_in}, T {T}, [{b}, {e}), split {sk}, warm {warm}",
              flush=True)
        _full_check(case, b, e, split_k=sk, warm=warm, step=3 if warm else 1)


def test_vector_kind():
    rng = np.random.default_rng(80)
    for dtype in (WL.BF16, WL.F32):
        case = WL.vector_case(rng, "norm", 1000, 77, dtype, 1e-3)
        for begin, end in ((0, 1000), (3, 997), (500, 501)):
            _full_check(case, begin, end)


@pytest.mark.parametrize("dtype", [WL.BF16, WL.F32])
def test_embedding_kind(dtype):
    """Table rows hit by many tokens, by one and by none; ranges that start and end mid-row;
    a width that is not a multiple of 4 (element-wise path) and one wider than a column block."""
    rng = np.random.default_rng(82)
    case = WL.embedding_case(rng, "embed", 300, 264, 500, dtype, 1e-3)
    for begin, end in ((0, 300 * 264), (264 * 7 + 33, 264 * 251 + 5), (264 * 40, 264 * 41), (17, 18)):
        _full_check(case, begin, end)
    odd = WL.embedding_case(rng, "embed_odd", 50, 2051, 90, dtype, 1e-3)      # 2051 columns: two blocks, ragged
    _full_check(odd, 2051 * 3 + 1, 2051 * 44 + 2050)
    same = WL.embedding_case(rng, "embed_same", 40, 64, 200, dtype, 1e-3)
    same.X[:] = 11                                                            # every token names row 11
    _full_check(same, 0, 40 * 64)


@pytest.mark.parametrize("kind", [WL.RMSNORM, WL.LAYERNORM])
def test_self_normalising_scale_vectors(kind):
    rng = np.random.default_rng(83)
    for dtype in (WL.BF16, WL.F32):
        case = WL.norm_case(rng, "norm", 1000, 77, dtype, 1e-3, kind)
        for begin, end in ((0, 1000), (3, 997), (500, 501)):
            _full_check(case, begin, end)
    wide = WL.norm_case(rng, "norm_wide", 4096, 300, WL.BF16, 1e-3, kind, eps=1e-6)
    _full_check(wide, 0, 4096)


def test_warm_state_second_step():
    _full_check(_small_bf16(seed=81), 264 * 2 + 33, 264 * 519 + 1, warm=True, step=2)


@pytest.mark.parametrize("begin,end", [(0, 264 * 4 + 100), (0, 264 * 100 + 77), (264 * 8, 264 * 11 + 5),
                                       (264 * 16, 264 * 120 + 9), (264 * 1 + 1, 264 * 6 + 5), (0, 264 * 300 + 100)])
@pytest.mark.parametrize("split_k", [None, 2])
def test_warm_state_on_ranges_with_separate_edge_rows(begin, end, split_k):
    """Warm moments make a second update of an element visible (from m = v = 0 an update with a zero
    gradient changes nothing but the weight decay): ranges whose edge rows go to their own kernel, with
    and without leading rows, fused against the oracle and against the un-fused pair bit for bit."""
    _full_check(_small_bf16(seed=83), begin, end, split_k=split_k, warm=True, step=3)


# ------------------------------------------- scaled-down configurations 2-5
def test_config2_scaled():
    case, begin, end = WL.config2(scale=4)          # 3584 x 1024, 2 Mi-element chunk
    _full_check(case, begin, end)


def test_config4_scaled_token_splits():
    layers = WL.config4(scale=16, T=512)            # 1792 x 512 and 512 x 1792
    rng = WL.rng_for(4, 2)
    for case in layers:
        length = case.numel // 3
        begin = WL.draw_offset(rng, case.numel, length, case.n_in)
        ref = None
        for s in (1, 2, 4, 8):
            g, g_ref = _full_check(case, begin, begin + length, split_k=s, check_accum=(s == 2))
            ref = g_ref


def test_config5_scaled_chunk_sizes():
    case = WL.config5(scale=8, T=512)               # 16032 x 512
    for begin, end in WL.config5_ranges(case, scale=8):
        _full_check(case, begin, end, check_accum=False)


def _run_cycle(layers, budget, flags=0, grouped=False, split_k=0):
    """One full-parameter cycle on the GPU: plan, then one fused call per segment, or (grouped)
    one chunkft_wgrad_adamw_fused_group call per chunk."""
    tensors = [(c.out, c.n_in, c.dtype, c.kind) for c in layers]
    st, chunks, segs = B.chunkft_plan_cycle(tensors, budget, flags)
    dls = [H.DeviceLayer(c, split_k=split_k) for c in layers]
    Wd = [c.W0.reshape(-1).clone().to(H.DEV) for c in layers]
    masters, ms, vs = [], [], []
    for (s0, s1, numel, _) in chunks:
        fm, master = H.guarded(numel)
        for (t, b, e, off) in segs[s0:s1]:
            master[off:off + (e - b)] = Wd[t][b:e].float()
        fmm, m = H.guarded(numel, torch.zeros(numel))
        fv, v = H.guarded(numel, torch.zeros(numel))
        if grouped:
            group = B.GroupCall([(dls[t].layer(), b, e, Wd[t], master[off:off + e - b], m[off:off + e - b],
                                  v[off:off + e - b]) for (t, b, e, off) in segs[s0:s1]], device=H.DEV)
            group(B.hparams(step=1, **HP))
        else:
            for (t, b, e, off) in segs[s0:s1]:
                layer = dls[t].layer()
                ws = H.workspace_for(layer, b, e)
                n = e - b
                B.chunkft_wgrad_adamw_fused(layer, b, e, Wd[t], master[off:off + n], m[off:off + n],
                                            v[off:off + n], B.hparams(step=1, **HP), ws=ws)
        torch.cuda.synchronize()
        assert H.guards_intact(fm) and H.guards_intact(fmm) and H.guards_intact(fv)
        masters.append(master); ms.append(m); vs.append(v)
    return chunks, segs, Wd, masters, ms, vs


@pytest.mark.parametrize("budget_mib_x16,rows8", [(256, False), (100, False), (100, True), (20, False)])
def test_grouped_call_equals_one_call_per_segment(budget_mib_x16, rows8):
    """chunkft_wgrad_adamw_fused_group on every chunk of the scaled transformer block (matrix
    segments with and without edge rows, the two scale vectors, cuts in mid-row) against one
    chunkft_wgrad_adamw_fused call per segment: master, m, v of every chunk and every tensor's bf16
    copy bit for bit (the per-segment results are checked against the oracle in
    test_config3_scaled_cycle)."""
    layers = WL.config3(scale=4, T=256)
    budget = budget_mib_x16 * (1 << 20) // 16 + (2 if budget_mib_x16 != 256 else 0)
    flags = B.PLAN_ROWS8 if rows8 else 0
    # the 256 MiB plan's chunks fill the device and are grouped as they are; the smaller ones would each be
    # handed to the single call's own split rule, so one slab is asked for (in both runs) to group them
    split_k = 0 if budget_mib_x16 == 256 else 1
    a = _run_cycle(layers, budget, flags, split_k=split_k)
    b = _run_cycle(layers, budget, flags, grouped=True, split_k=split_k)
    assert a[0] == b[0] and a[1] == b[1] and len(a[0]) >= 2
    for k in range(len(a[0])):
        for x, y, name in ((a[3][k], b[3][k], "master"), (a[4][k], b[4][k], "m"), (a[5][k], b[5][k], "v")):
            assert torch.equal(x.view(torch.int32), y.view(torch.int32)), f"{name} of chunk {k}"
    for t in range(len(layers)):
        assert torch.equal(a[2][t].view(torch.int16), b[2][t].view(torch.int16)), f"W of tensor {t}"
    for k, (s0, s1, numel, _) in enumerate(a[0]):                 # and the grouped call did update every segment
        for (t, lo, hi, off) in a[1][s0:s1]:
            assert not torch.equal(b[3][k][off:off + hi - lo], layers[t].W0.reshape(-1)[lo:hi].float().to(H.DEV))


@pytest.mark.parametrize("seed", [301, 302])
def test_grouped_call_on_random_groups_of_every_kind(seed):
    """Seeded random groups of one to eight segments (bf16 matrices with a forced token split of 1 - 3, bf16
    scale vectors, embedding tables, self-normalising vectors, fp32 and odd-shaped matrices), the first
    segment starting and the last one ending anywhere, warm moments: the grouped call equals one fused
    call per segment bit for bit, and nothing is written outside a segment's arrays."""
    rng = np.random.default_rng(seed)
    for it in range(25):
        nseg = int(rng.integers(1, 9))
        T = int(rng.integers(1, 700))
        segs, desc = [], []
        for s in range(nseg):
            kind = rng.choice(["lin", "lin", "lin", "vec", "emb", "norm", "f32", "odd"])
            if kind == "emb":
                case = WL.embedding_case(rng, "e", int(rng.integers(1, 300)), int(rng.integers(1, 600)), T,
                                         WL.BF16 if rng.random() < 0.5 else WL.F32, 1e-3)
            elif kind == "norm":
                case = WL.norm_case(rng, "n", int(rng.integers(2, 3000)), T, WL.BF16, 1e-3,
                                    WL.RMSNORM if rng.random() < 0.5 else WL.LAYERNORM)
            elif kind == "f32":
                case = WL.linear_case(rng, "f", int(rng.integers(1, 200)), int(rng.integers(1, 200)), T, WL.F32, 1e-3)
            elif kind == "odd":
                case = WL.linear_case(rng, "o", int(rng.integers(1, 200)), int(rng.integers(1, 200)), T, WL.BF16, 1e-3)
            elif kind == "vec":
                case = WL.vector_case(rng, "v", int(rng.integers(1, 200)) * 8, T, WL.BF16, 1e-3)
            else:
                case = WL.linear_case(rng, "m", int(rng.integers(1, 200)) * 8, int(rng.integers(1, 200)) * 8, T, WL.BF16, 1e-3)
            N = case.numel
            b = 0 if s > 0 else int(rng.integers(0, N))
            e = N if s < nseg - 1 else int(rng.integers(b + 1, N + 1))
            sk = int(rng.choice([1, 1, 1, 1, 2, 3]))      # a forced split: the grouped call obeys it as the single call does
            if sk > T or kind in ("vec", "emb", "norm"):
                sk = 0
            segs.append((H.DeviceLayer(case, sk), b, e, case))
            desc.append(f"{kind} {case.out} x {case.n_in} [{b}, {e}) split {sk}")
        print(f"[case {it}] T {T}: " + " | ".join(desc), flush=True)

        def run(grouped):
            outs, calls, fulls = [], [], []
            for si, (dl, b, e, case) in enumerate(segs):
                n = e - b
                gen = torch.Generator().manual_seed(1000 * it + si)
                fm, master = H.guarded(n, case.W0.reshape(-1)[b:e].float())
                fmm, m = H.guarded(n, torch.randn(n, generator=gen) * 1e-3)
                fv, v = H.guarded(n, (0.25 + torch.randn(n, generator=gen) ** 2) * 1e-6)
                W = case.W0.reshape(-1).clone().to(H.DEV)
                outs.append((W, master, m, v))
                fulls += [fm, fmm, fv]
                calls.append((dl.layer(), b, e, W, master, m, v))
            hp = B.hparams(step=3, **HP)
            if grouped:
                B.GroupCall(calls, device=H.DEV)(hp)
            else:
                for layer, b, e, W, master, m, v in calls:
                    ws = H.workspace_for(layer, b, e)
                    B.chunkft_wgrad_adamw_fused(layer, b, e, W, master, m, v, hp, ws=ws)
                    torch.cuda.synchronize()
                    assert H.workspace_intact(ws)
            torch.cuda.synchronize()
            assert all(H.guards_intact(f) for f in fulls), "state written outside a segment"
            return outs

        single, group = run(False), run(True)
        for si, (a, g) in enumerate(zip(single, group)):
            for name, x, y in zip(("W", "master", "m", "v"), a, g):
                assert torch.equal(x, y), f"case {it} segment {si} ({desc[si]}): {name} differs"


def test_grouped_call_runs_what_its_kernel_cannot_take_by_itself():
    """A group that mixes segments for the one-launch kernel (bf16 matrices, a bf16 scale vector) with
    ones it cannot take -- an fp32 matrix, a forced token split, a chunk of three rows, an embedding
    table, a self-normalising scale vector -- and more than twelve segments in all, so that the table
    is cut into several launches.  Every segment's state against the single call's, bit for bit."""
    rng = np.random.default_rng(WL.SEED_BASE + 80)
    cases = []

    def add(case, begin, end, split_k=0):
        cases.append((case, begin, end, split_k))

    big = WL.linear_case(rng, "a", 776, 520, 200, WL.BF16, 1e-3)
    add(big, 520 * 3 + 17, 520 * 400 + 9, 1)                       # edge rows on both sides
    add(big, 520 * 408, 520 * 776, 1)                              # row aligned, another range of the same tensor
    add(WL.linear_case(rng, "b", 264, 136, 200, WL.F32, 1e-3), 77, 136 * 200 + 3)      # fp32: by itself
    add(WL.linear_case(rng, "c", 520, 264, 200, WL.BF16, 1e-3), 264 * 5 + 1, 264 * 519 + 100, 3)   # forced split
    add(WL.linear_case(rng, "d", 520, 264, 200, WL.BF16, 1e-3), 264 * 10 + 7, 264 * 13 + 5)        # three rows
    add(WL.vector_case(rng, "e", 1032, 200, WL.BF16, 1e-3), 5, 1000)
    add(WL.embedding_case(rng, "f", 300, 264, 150, WL.BF16, 1e-3), 264 * 3 + 9, 264 * 290)
    add(WL.norm_case(rng, "g", 520, 200, WL.BF16, 1e-3, WL.RMSNORM), 0, 520)
    for i in range(8):                                             # fills the table past twelve segments
        c = WL.linear_case(rng, f"h{i}", 264 + 8 * i, 136, 200, WL.BF16, 1e-3)
        add(c, 136 * i + i, 136 * (200 + i) + 3 * i, 1)             # one slab asked for: the kernel takes them
    assert len(cases) == 16
    hp = B.hparams(step=2, **HP)

    def run(grouped):
        out, keep, segs = [], [], []
        for case, begin, end, split_k in cases:
            dl = H.DeviceLayer(case, split_k=split_k)
            layer = dl.layer()
            n = end - begin
            is_bf16 = case.dtype == WL.BF16
            W = case.W0.reshape(-1).clone().to(H.DEV)
            th0, m0, v0 = _state_for(case, begin, end, np.random.default_rng(7), warm=True)
            st = [H.guarded(n, torch.from_numpy(x)) for x in (th0, m0, v0)]
            keep.append((dl, layer, W, st))
            segs.append((layer, begin, end, W if is_bf16 else None, st[0][1], st[1][1], st[2][1]))
        if grouped:
            call = B.GroupCall(segs, device=H.DEV)
            assert call.ws_bytes > 0                                # the forced split and the norm need some
            call(hp)
        else:
            for (layer, begin, end, W, master, m, v) in segs:
                ws = H.workspace_for(layer, begin, end)
                B.chunkft_wgrad_adamw_fused(layer, begin, end, W, master, m, v, hp, ws=ws)
                torch.cuda.synchronize()
                assert H.workspace_intact(ws)
        torch.cuda.synchronize()
        for (dl, layer, W, st) in keep:
            assert all(H.guards_intact(f) for f, _ in st)
            out.append((W.cpu(), [x.cpu() for _, x in st]))
        return out

    single, grouped = run(False), run(True)
    for i, ((Wa, sa), (Wb, sb)) in enumerate(zip(single, grouped)):
        for x, y in zip(sa, sb):
            assert torch.equal(x.view(torch.int32), y.view(torch.int32)), f"state of segment {i}"
        assert torch.equal(Wa.view(torch.uint8), Wb.view(torch.uint8)), f"W of segment {i}"
        assert not torch.equal(sa[0], torch.from_numpy(_state_for(cases[i][0], cases[i][1], cases[i][2],
                                                                  np.random.default_rng(7), warm=True)[0]))


@pytest.mark.parametrize("budget_mib_x16,rows8", [(256, False), (64, False), (100, False), (100, True)])
def test_config3_scaled_cycle(budget_mib_x16, rows8):
    """The transformer block at 1/4 linear scale (1/16 of the elements), budgets
    scaled alike (+2 bytes on the 100 MiB one to force mid-row cuts; the same budget once more
    with cuts between groups of 8 rows only)."""
    layers = WL.config3(scale=4, T=256)
    budget = budget_mib_x16 * (1 << 20) // 16 + (2 if budget_mib_x16 == 100 else 0)
    chunks, segs, Wd, masters, ms, vs = _run_cycle(layers, budget, B.PLAN_ROWS8 if rows8 else 0)
    # the library's plan is the oracle's plan
    oc = O.plan_cycle([c.desc() for c in layers], budget, rows8=rows8)
    assert [(s.tensor, s.begin, s.end, s.chunk_off) for ch in oc for s in ch] == segs
    if rows8:
        for (t, b, e, _) in segs:
            assert b % (8 * layers[t].n_in) == 0 and (e % (8 * layers[t].n_in) == 0 or e == layers[t].numel)
    # every element updated exactly once: compare with one dense AdamW step per tensor
    for t, case in enumerate(layers):
        X64, dY64 = WL.as_f64(case.X), WL.as_f64(case.dY)
        g_ref = (O.dense_wgrad(X64, dY64).reshape(-1) if case.kind == WL.LINEAR
                 else O.vector_wgrad(X64, dY64, 0, case.n_in))
        th0 = WL.as_f64(case.W0).reshape(-1)
        z = np.zeros_like(th0)
        got_master = np.empty(case.numel, np.float32)
        got_m = np.empty(case.numel, np.float32)
        got_v = np.empty(case.numel, np.float32)
        for k, (s0, s1, _, _) in enumerate(chunks):
            for (tt, b, e, off) in segs[s0:s1]:
                if tt == t:
                    got_master[b:e] = masters[k][off:off + e - b].cpu().numpy()
                    got_m[b:e] = ms[k][off:off + e - b].cpu().numpy()
                    got_v[b:e] = vs[k][off:off + e - b].cpu().numpy()
        bits = WL.bits_u16(Wd[t].cpu())
        H.check_fused_against_oracle(g_ref, th0, z, z, HP, 1, got_master, got_m, got_v, bits)
        # with a non-zero gradient every master value moved (update counter = 1 everywhere)
        assert np.all(got_master != th0.astype(np.float32))


def test_rotating_schedule_trajectory():
    """Algorithm 1 end to end on a small block: chunks rotate with interval 2 for two and a half
    cycles, every step has its own output gradients, the active chunk's segments are updated
    with the chunk's own counter.  Checked step by step with the single-step rules, so that no
    tolerance has to grow with the number of steps:
      * the gradient of every segment (the un-fused call on the same operands, whose bits the
        fused call's internal gradient equals) against the oracle's, relative Frobenius 3e-3;
      * the state after the fused call against the oracle's AdamW applied to the GPU's own
        gradient and the GPU's own state before the step, element-wise 1e-5;
      * the bf16 copy bit-exact against the rounded GPU master;
    and at the end the whole trajectory: the oracle's schedule, counters and AdamW run from the
    initial state on the GPU's gradients must land on the GPU's final state, element-wise 1e-5
    (per-step differences are fp32 rounding, about 1e-7, and do not pass through a sign)."""
    layers = WL.config3(scale=16, T=64)
    tensors = [(c.out, c.n_in, c.dtype, c.kind) for c in layers]
    budget = sum(c.numel for c in layers) * 2 // 3 + 2              # three chunks, mid-row cuts
    st, chunks, segs = B.chunkft_plan_cycle(tensors, budget)
    K, interval = len(chunks), 2
    assert K == 3
    n_steps = 2 * K * interval + K * interval // 2
    rng = np.random.default_rng(91)
    scales = 1.0 + rng.random(n_steps)                              # the batch changes from step to step
    dls = [H.DeviceLayer(c) for c in layers]
    Wd = [c.W0.reshape(-1).clone().to(H.DEV) for c in layers]
    state = []
    for (s0, s1, numel, _) in chunks:
        master = torch.empty(numel, dtype=torch.float32, device=H.DEV)
        for (t, b, e, off) in segs[s0:s1]:
            master[off:off + (e - b)] = Wd[t][b:e].float()
        state.append((master, torch.zeros_like(master), torch.zeros_like(master)))
    # oracle side
    params = [WL.as_f64(c.W0).reshape(-1).copy() for c in layers]
    ostate = [dict(m=np.zeros(ch[2]), v=np.zeros(ch[2])) for ch in chunks]
    sched = O.rotating_schedule(n_steps, K, interval)
    visits = [0] * K
    for t in range(n_steps):
        k, load, off, n = B.chunkft_schedule_at(t, K, interval)
        assert (k, load, off, n) == sched[t]
        visits[k] += 1
        s0, s1, numel, _ = chunks[k]
        master, m, v = state[k]
        for (ti, b, e, o) in segs[s0:s1]:
            case = layers[ti]
            dY_t = (case.dY.float() * float(scales[t])).to(case.dY.dtype)
            dY_dev = dY_t.to(H.DEV)              # the layer descriptor holds its address only: keep it alive
            layer = B.make_layer(case.kind, dls[ti].X, dY_dev, case.out, case.n_in)
            ws = H.workspace_for(layer, b, e)
            cnt = e - b
            before = tuple(x[o:o + cnt].cpu().numpy().astype(np.float64) for x in (master, m, v))
            g_gpu = torch.empty(cnt, dtype=torch.float32, device=H.DEV)
            B.chunkft_chunk_wgrad(layer, b, e, g_gpu, ws=ws)
            B.chunkft_wgrad_adamw_fused(layer, b, e, Wd[ti], master[o:o + cnt], m[o:o + cnt], v[o:o + cnt],
                                        B.hparams(step=n, **HP), ws=ws)
            torch.cuda.synchronize()
            assert H.workspace_intact(ws)
            g64 = g_gpu.cpu().numpy().astype(np.float64)
            X64, dY64 = WL.as_f64(case.X), WL.as_f64(dY_t)
            g_ref = (O.chunk_wgrad(X64, dY64, b, e, dense=False) if case.kind == WL.LINEAR
                     else O.vector_wgrad(X64, dY64, b, e))
            assert H.rel_frobenius(g64, g_ref) <= 3e-3
            # this step alone: the oracle's update of the GPU's state by the GPU's gradient
            ref = O.adamw_step(g64, *before, step=n, **HP)
            tag = f"step {t} chunk {k} tensor {ti}"
            H.assert_elementwise(master[o:o + cnt].cpu().numpy(), ref[0], 1e-2, "theta " + tag)
            H.assert_elementwise(m[o:o + cnt].cpu().numpy(), ref[1], 1e-2, "m " + tag)
            H.assert_elementwise(v[o:o + cnt].cpu().numpy(), ref[2], 0.0, "v " + tag)
            bits = WL.bits_u16(Wd[ti][b:e].cpu())
            assert np.array_equal(bits, O.bf16_bits(master[o:o + cnt].cpu().numpy().astype(np.float64)))
            # the whole trajectory on the oracle's own state
            th, mm, vv = O.adamw_step(g64, params[ti][b:e], ostate[k]["m"][o:o + cnt], ostate[k]["v"][o:o + cnt],
                                      step=n, **HP)
            params[ti][b:e] = th
            ostate[k]["m"][o:o + cnt] = mm
            ostate[k]["v"][o:o + cnt] = vv
    assert min(visits) >= 2 * interval                      # every chunk came round at least twice
    for k, (s0, s1, numel, _) in enumerate(chunks):
        master, m, v = (x.cpu().numpy() for x in state[k])
        H.assert_elementwise(m, ostate[k]["m"], 1e-2, f"m of chunk {k} after {n_steps} steps")
        H.assert_elementwise(v, ostate[k]["v"], 0.0, f"v of chunk {k} after {n_steps} steps")
        for (ti, b, e, o) in segs[s0:s1]:
            H.assert_elementwise(master[o:o + e - b], params[ti][b:e], 1e-2, f"theta of chunk {k} tensor {ti} after {n_steps} steps")
    for ti, case in enumerate(layers):
        # the oracle's bf16 copy of its own trajectory: the GPU's may differ by one grid step where a
        # 1e-7 difference of the masters falls on a rounding boundary
        bits = WL.bits_u16(Wd[ti].cpu()).astype(np.int64)
        ref = O.bf16_bits(params[ti]).astype(np.int64)
        assert np.abs(bits - ref).max() <= 1


def test_calls_replay_from_a_captured_graph():
    """The device entry points only enqueue kernels on the caller's stream, so a caller may
    capture them into a HIP graph.  Each replay (with fresh inputs written in place and eager
    work in between) must give the bits of the same calls made eagerly."""
    case = _small_bf16(T=96, seed=93)
    begin, end = 264 * 2 + 33, 264 * 519 + 1
    n = end - begin
    dl = H.DeviceLayer(case)
    layer = dl.layer()
    hp = B.hparams(step=3, **HP)
    W0 = case.W0.reshape(-1).to(H.DEV)

    def fresh_state(seed):
        rng = np.random.default_rng(seed)
        th = W0[begin:end].float()
        m = torch.from_numpy((rng.standard_normal(n) * 1e-3).astype(np.float32)).to(H.DEV)
        v = torch.from_numpy(((0.25 + rng.standard_normal(n) ** 2) * 1e-6).astype(np.float32)).to(H.DEV)
        return th, m, v

    g = torch.empty(n, dtype=torch.float32, device=H.DEV)
    st_a = [t.clone() for t in fresh_state(0)]       # un-fused pair works on these
    st_b = [t.clone() for t in fresh_state(0)]       # fused call on these
    Wa, Wb = W0.clone(), W0.clone()

    def calls():
        B.chunkft_chunk_wgrad(layer, begin, end, g)
        B.chunkft_adamw_chunk(g, st_a[0], st_a[1], st_a[2], Wa[begin:end], n, hp)
        B.chunkft_wgrad_adamw_fused(layer, begin, end, Wb, st_b[0], st_b[1], st_b[2], hp)

    calls()                                           # first use outside the capture (sets kernel attributes)
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            calls()
    torch.cuda.synchronize()

    for rep in range(3):
        new_dY = torch.from_numpy((np.random.default_rng(100 + rep).standard_normal(tuple(dl.dY.shape)) * 1e-3)
                                  .astype(np.float32)).to(torch.bfloat16).to(H.DEV)
        dl.dY.copy_(new_dY)                           # same buffers, new contents
        init = fresh_state(10 + rep)
        # eager reference
        for dst, src in zip(st_a + st_b, list(init) + list(init)):
            dst.copy_(src)
        Wa.copy_(W0); Wb.copy_(W0)
        calls()
        torch.cuda.synchronize()
        want = [t.clone() for t in [g] + st_a + st_b + [Wa, Wb]]
        # some unrelated eager work, then the replay on re-initialised state
        _ = (torch.randn(1 << 20, device=H.DEV) * 2).sum().item()
        for dst, src in zip(st_a + st_b, list(init) + list(init)):
            dst.copy_(src)
        Wa.copy_(W0); Wb.copy_(W0)
        g.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [g] + st_a + st_b + [Wa, Wb]
        for a, b in zip(got, want):
            assert torch.equal(a.view(torch.int32) if a.dtype == torch.float32 else a.view(torch.int16),
                               b.view(torch.int32) if b.dtype == torch.float32 else b.view(torch.int16))
        # and the fused state equals the un-fused pair's, replay after replay
        assert torch.equal(st_a[0], st_b[0]) and torch.equal(st_a[1], st_b[1]) and torch.equal(st_a[2], st_b[2])


def test_grouped_and_static_workspace_calls_replay_from_a_captured_graph():
    """The two calls meant for callers that cannot allocate or launch much: a chunk of three segments (two
    matrices and a scale vector) through chunkft_wgrad_adamw_fused_group, and a forced token split through
    chunkft_wgrad_adamw_fused_static (its slab partials live in the library's static device array), captured
    into one HIP graph after an eager first call.  Three replays with fresh inputs and state, eager work in
    between, each against the same calls made eagerly."""
    rng = np.random.default_rng(WL.SEED_BASE + 95)
    a = WL.linear_case(rng, "a", 520, 264, 96, WL.BF16, 1e-3)
    b = WL.linear_case(rng, "b", 264, 520, 96, WL.BF16, 1e-3)
    c = WL.vector_case(rng, "c", 520, 96, WL.BF16, 1e-3)
    ranges = [(264 * 3 + 7, 264 * 500 + 100), (0, 520 * 200 + 33), (5, 500)]
    dls = [H.DeviceLayer(a, split_k=1), H.DeviceLayer(b, split_k=1), H.DeviceLayer(c)]
    split = H.DeviceLayer(a, split_k=3)
    W0 = [x.W0.reshape(-1).to(H.DEV) for x in (a, b, c)]
    W = [w.clone() for w in W0]
    Ws = W0[0].clone()
    hp = B.hparams(step=2, **HP)

    def fresh(seed):
        r = np.random.default_rng(seed)
        out = []
        for (lo, hi), w0 in list(zip(ranges, W0)) + [(ranges[0], W0[0])]:
            n = hi - lo
            out.append([w0[lo:hi].float(),
                        torch.from_numpy((r.standard_normal(n) * 1e-3).astype(np.float32)).to(H.DEV),
                        torch.from_numpy(((0.25 + r.standard_normal(n) ** 2) * 1e-6).astype(np.float32)).to(H.DEV)])
        out[3] = [t.clone() for t in out[0]]              # the static call starts from the first segment's state
        return out

    state = [[t.clone() for t in trio] for trio in fresh(0)]        # three group segments + the static call's
    group = B.GroupCall([(dls[i].layer(), ranges[i][0], ranges[i][1], W[i], *state[i]) for i in range(3)], device=H.DEV)
    assert group.ws_bytes == 0
    layer_s = split.layer()

    def calls():
        group(hp)
        B.chunkft_wgrad_adamw_fused_static(layer_s, ranges[0][0], ranges[0][1], Ws, *state[3], hp)

    def reset(seed):
        for dst, src in zip(state, fresh(seed)):
            for d, s_ in zip(dst, src):
                d.copy_(s_)
        for w, w0 in zip(W + [Ws], W0 + [W0[0]]):
            w.copy_(w0)

    calls()                                            # eager first use: kernel attributes, the static array's address
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            calls()
    torch.cuda.synchronize()
    for rep in range(3):
        for dl in dls + [split]:
            dl.dY.copy_((torch.randn(tuple(dl.dY.shape), generator=torch.Generator().manual_seed(200 + rep)) * 1e-3)
                        .to(torch.bfloat16).to(H.DEV))
        split.dY.copy_(dls[0].dY)
        reset(20 + rep)
        calls()
        torch.cuda.synchronize()
        want = [t.clone() for trio in state for t in trio] + [w.clone() for w in W + [Ws]]
        _ = (torch.randn(1 << 20, device=H.DEV) * 2).sum().item()       # unrelated eager work
        reset(20 + rep)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [t for trio in state for t in trio] + W + [Ws]
        for x, y in zip(got, want):
            assert torch.equal(x.view(torch.int32) if x.dtype == torch.float32 else x.view(torch.int16),
                               y.view(torch.int32) if y.dtype == torch.float32 else y.view(torch.int16))
        # the split call sums its slabs in another order than the single slab of the grouped call: close, not equal
        assert H.rel_frobenius(state[3][1].cpu().numpy(), state[0][1].cpu().numpy()) <= 1e-5


def test_streamed_state_gives_the_resident_trajectory():
    """Algorithm 1 with the chunk state kept in (pinned) host memory: the next chunk's state is
    prefetched into the second device buffer set while the active chunk computes, the previous
    one is offloaded behind it.  After several visits per chunk the host copies must hold,
    bit for bit, what a run with everything resident on the device produces."""
    layers = WL.config3(scale=16, T=64)
    tensors = [(c.out, c.n_in, c.dtype, c.kind) for c in layers]
    budget = sum(c.numel for c in layers) * 2 // 3 + 2
    st, chunks, segs = B.chunkft_plan_cycle(tensors, budget)
    K, interval = len(chunks), 2
    n_steps = 3 * K * interval
    dls = [H.DeviceLayer(c) for c in layers]
    cap = max(ch[2] for ch in chunks)

    def init_state(k):
        s0, s1, numel, _ = chunks[k]
        master = torch.empty(numel, dtype=torch.float32)
        for (t, b, e, off) in segs[s0:s1]:
            master[off:off + (e - b)] = layers[t].W0.reshape(-1)[b:e].float()
        return master, torch.zeros(numel), torch.zeros(numel)

    def run_steps(step_fn):
        Wd = [c.W0.reshape(-1).clone().to(H.DEV) for c in layers]
        for t in range(n_steps):
            k, load, off, n = B.chunkft_schedule_at(t, K, interval)
            master, m, v = step_fn(t, k, load)
            s0, s1, numel, _ = chunks[k]
            for (ti, b, e, o) in segs[s0:s1]:
                layer = dls[ti].layer()
                cnt = e - b
                B.chunkft_wgrad_adamw_fused(layer, b, e, Wd[ti], master[o:o + cnt], m[o:o + cnt], v[o:o + cnt],
                                            B.hparams(step=n, **HP), ws=H.workspace_for(layer, b, e))
            yield t, k, off
        torch.cuda.synchronize()
        yield Wd

    # --- resident run
    resident = [tuple(x.to(H.DEV) for x in init_state(k)) for k in range(K)]
    *_, W_res = run_steps(lambda t, k, load: resident[k])

    # --- streamed run: host state pinned, two device sets, prefetch of the next chunk
    host = [tuple(x.pin_memory() for x in init_state(k)) for k in range(K)]
    sets = [tuple(torch.empty(cap, dtype=torch.float32, device=H.DEV) for _ in range(3)) for _ in range(2)]
    mover = B.Mover()
    visit = {"n": -1}

    def numel_of(k):
        return chunks[k][2]

    def step_fn(t, k, load):
        if load:
            visit["n"] += 1
            cur = sets[visit["n"] % 2]
            if visit["n"] == 0:                       # nothing was prefetched for the very first visit
                mover.load(cur, host[k], numel_of(k))
            mover.await_load()
            nxt_k = (k + 1) % K                       # prefetch the next chunk into the other set; its
            mover.load(sets[(visit["n"] + 1) % 2], host[nxt_k], numel_of(nxt_k))   # old occupant's offload is ahead on the copy stream
        return sets[visit["n"] % 2]

    gen = run_steps(step_fn)
    for item in gen:
        if isinstance(item, list):
            W_str = item
            break
        t, k, off = item
        if off:
            # BEFORE the prefetch of the chunk after next can overwrite this set, its offload is enqueued:
            # the prefetch into this set is only issued at the next visit's first step, after this line
            mover.offload(host[k], sets[visit["n"] % 2], numel_of(k))
    mover.sync()
    mover.close()
    for k in range(K):
        for a, b in zip(host[k], resident[k]):
            assert torch.equal(a, b.cpu()), f"state of chunk {k} differs between streamed and resident run"
    for a, b in zip(W_str, W_res):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_matrix_core_rate_measurement_runs_for_both_shapes():
    """The measurement aid: each bf16 MFMA shape reports a rate below the part's 2.5 PFLOP/s and a clock
    below its 2.4 GHz, and a rate that is consistent with that clock (256 CUs x 4096 flop per cycle; the
    clock is one workgroup's sample of the last launch and moves with the power management, the rate is
    the mean over five launches: hence the wide margin)."""
    for shape in (32, 16):
        for rnd in (False, True):
            tf, mhz = B.chunkft_calib_mfma_bf16_shape(shape, rnd, steps=2000)
            assert 200.0 < tf < 2600.0, (shape, rnd, tf)
            assert 500.0 < mhz < 2500.0, (shape, rnd, mhz)
            at_clock = 256 * 4096 * mhz * 1e6 / 1e12
            assert tf < 1.3 * at_clock, (shape, rnd, tf, at_clock)
    tf32, _ = B.chunkft_calib_mfma_bf16(True, steps=2000)
    assert 200.0 < tf32 < 2600.0

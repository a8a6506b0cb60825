"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.

Bar: integer results (codes, packed bytes, zero points, int32 accumulators) bit-exact, fp32 scales bit-exact;
16-bit outputs within relative Frobenius error 1e-3 and |err| <= 1e-2 * max|ref| per element."""
import numpy as np
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu

FRO_TOL = 1e-3
ELT_TOL = 1e-2
ALL_BITS = (2, 3, 4, 8)


@pytest.fixture(scope="module")
def mq():
    import paper_2405_17873_amd as m
    m.load()
    assert torch.cuda.is_available()
    yield m
    m.tune_force_tile(-1)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def assert_close16(y, ref_bits, what=""):
    y = np.asarray(y).astype(np.float64)
    ref = np.asarray(ref_bits).view(np.float16).astype(np.float64)
    assert y.shape == ref.shape, (y.shape, ref.shape)
    assert np.isfinite(y).all(), what
    fro = np.linalg.norm(y - ref) / max(np.linalg.norm(ref), 1e-30)
    elt = np.abs(y - ref).max() / max(np.abs(ref).max(), 1e-30)
    assert fro <= FRO_TOL and elt <= ELT_TOL, f"{what}: fro={fro:.3e} elt={elt:.3e}"


def sample_rows(x, n=512, seed=0):
    """A seeded sample of at least n distinct rows that always holds the first row, the last row and the rows with the
    tensor's largest and smallest value (output rows are independent given the activation parameters)."""
    M = x.shape[0]
    rng = np.random.default_rng(seed)
    fixed = [0, M - 1, int(np.argmax(x.max(1))), int(np.argmin(x.min(1)))]
    rows = np.unique(np.concatenate([fixed, rng.choice(M, size=min(M, n), replace=False)]))
    return rows.astype(np.int64)


def make_weight(mq, orc, w, bits, symmetric=False):
    """Quantise + pack on the GPU, checking both against the oracle bit for bit; returns (PackedWeight, codes...)."""
    wd = dev(w)
    c, s, z = mq.quantize_weights(wd, bits, symmetric)
    oc, os_, oz = orc.quantize_weights(w, bits, symmetric)
    assert np.array_equal(host(c), oc), "codes"
    assert np.array_equal(host(s).view(np.uint32), os_.view(np.uint32)), "scale bits"
    assert np.array_equal(host(z), oz), "zero points"
    packed, colsum = mq.pack_weights(c, bits, mq.LAYOUT_KERNEL, codes_signed=symmetric)
    assert np.array_equal(host(colsum), orc.code_rowsum(oc, signed=symmetric))
    N, K = w.shape
    return mq.PackedWeight(packed, s, z, colsum, N, K, bits, mq.LAYOUT_KERNEL, symmetric), oc, os_, oz


# ----------------------------------------------------------------------------------------------- quantiser / packers

@pytest.mark.parametrize("bits", ALL_BITS)
@pytest.mark.parametrize("symmetric", (False, True))
def test_quantize_weights_bit_exact(mq, orc, bits, symmetric):
    if symmetric and bits not in (4, 8):
        pytest.skip("symmetric scheme is used at 4 and 8 bits")
    for (N, K, std) in ((320, 320, 0.02), (37, 1000, 1.0), (5, 64, 0.02), (640, 2560, 0.02)):
        w = si.weights_f16(7, f"q/{N}x{K}", N, K, std)
        if N > 4:
            w[1] = 0
            w[2] = np.abs(w[2])
            w[3] = -np.abs(w[3])
        c, s, z = mq.quantize_weights(dev(w), bits, symmetric)
        oc, os_, oz = orc.quantize_weights(w, bits, symmetric)
        assert np.array_equal(host(c), oc)
        assert np.array_equal(host(s).view(np.uint32), os_.view(np.uint32))
        assert np.array_equal(host(z), oz)


def test_quantize_weights_bf16(mq, orc):
    w = torch.from_numpy(si.normal(8, "q/bf16", (64, 320), 0.02).astype(np.float32)).to(torch.bfloat16)
    bits16 = w.view(torch.int16).numpy().view(np.uint16)
    c, s, z = mq.quantize_weights(w.cuda(), 4)
    oc, os_, oz = orc.quantize_weights(bits16, 4, dtype=orc.BF16)
    assert np.array_equal(host(c), oc) and np.array_equal(host(s), os_) and np.array_equal(host(z), oz)


@pytest.mark.parametrize("bits", ALL_BITS)
def test_pack_canonical_bytes_bit_exact(mq, orc, bits):
    rng = np.random.default_rng(bits)
    for (N, K) in ((7, 32), (320, 320), (33, 5120), (1, 8)):
        codes = rng.integers(0, 1 << bits, (N, K)).astype(np.uint8)
        p, cs = mq.pack_weights(dev(codes), bits, mq.LAYOUT_CANONICAL)
        assert np.array_equal(host(p).reshape(N, -1), orc.pack_weights(codes, bits))
        assert np.array_equal(host(cs), codes.astype(np.int64).sum(1))
        back = mq.unpack_weights(p, N, K, bits, mq.LAYOUT_CANONICAL)
        assert np.array_equal(host(back), codes)


@pytest.mark.parametrize("bits", ALL_BITS)
def test_pack_kernel_layout_round_trip(mq, orc, bits):
    rng = np.random.default_rng(10 + bits)
    for (N, K) in ((32, 64), (320, 320), (33, 128), (4, 5120), (100, 2048)):
        codes = rng.integers(0, 1 << bits, (N, K)).astype(np.uint8)
        p, _ = mq.pack_weights(dev(codes), bits, mq.LAYOUT_KERNEL)
        assert p.numel() == mq.packed_bytes(N, K, bits, mq.LAYOUT_KERNEL) == (N + 31) // 32 * 32 * K * bits // 8
        assert np.array_equal(host(mq.unpack_weights(p, N, K, bits, mq.LAYOUT_KERNEL)), codes)
        # same multiset of bits as the canonical form (a permutation, nothing lost): compare popcounts per tile row group
        if N % 32 == 0:
            can = orc.pack_weights(codes, bits)
            assert int(np.unpackbits(host(p)).sum()) == int(np.unpackbits(can).sum())
    signed = rng.integers(-127, 128, (64, 128)).astype(np.int8).view(np.uint8)
    p, cs = mq.pack_weights(dev(signed), 8, mq.LAYOUT_KERNEL, codes_signed=True)
    assert np.array_equal(host(cs), signed.view(np.int8).astype(np.int64).sum(1))


# ----------------------------------------------------------------------------------------------- weight-only

W_ONLY_SHAPES = [
    # M, K, N
    (256, 320, 320),   # stated small configuration (b)
    (1, 64, 32),
    (77, 128, 40),     # N not a multiple of the tile, M ragged
    (608, 2048, 640),
    (300, 640, 640),
    (513, 192, 264),
]


@pytest.mark.parametrize("bits", ALL_BITS)
@pytest.mark.parametrize("tile", (-1, 0, 1, 2, 3, 4, 5, 6))
def test_w_only_small_shapes(mq, orc, bits, tile):
    mq.tune_force_tile(tile)
    for (M, K, N) in W_ONLY_SHAPES:
        if tile == 0 and M * N > 400000:
            continue
        x = si.activations_f16(11, f"wo/x{M}x{K}", M, K, outlier_prob=0.01)
        w = si.weights_f16(11, f"wo/w{N}x{K}", N, K)
        b = si.bias_f16(11, f"wo/b{N}", N)
        pw, oc, os_, oz = make_weight(mq, orc, w, bits)
        for bias in (b, None):
            y = mq.qlinear_w_only(dev(x), pw, None if bias is None else dev(bias))
            ref = orc.linear_w_only(x, oc, os_, oz, bias)
            assert_close16(host(y), ref, f"w_only b{bits} tile{tile} {M}x{K}x{N}")
    mq.tune_force_tile(-1)


def test_w_only_exact_integer_case(mq, orc):
    """Integer activations, scale 1: every product and sum is exact in fp32, so the result is exact."""
    rng = np.random.default_rng(5)
    for bits in ALL_BITS:
        M, K, N = 96, 256, 64
        x = rng.integers(-4, 5, (M, K)).astype(np.float16)
        codes = rng.integers(0, 1 << bits, (N, K)).astype(np.uint8)
        zp = rng.integers(0, 1 << bits, N).astype(np.int32)
        packed, cs = mq.pack_weights(dev(codes), bits, mq.LAYOUT_KERNEL)
        pw = mq.PackedWeight(packed, dev(np.ones(N, np.float32)), dev(zp), cs, N, K, bits, mq.LAYOUT_KERNEL, False)
        y = host(mq.qlinear_w_only(dev(x), pw))
        ref = x.astype(np.int64) @ (codes.astype(np.int64) - zp[:, None]).T
        assert np.array_equal(y.astype(np.float64), ref.astype(np.float16).astype(np.float64)), bits


def test_w_only_bf16(mq, orc):
    """bfloat16 activations, bias and output (fp32 accumulate); weights quantised from bf16 as well."""
    for (M, K, N, tile) in ((256, 320, 320, -1), (300, 640, 640, 1), (77, 128, 40, 2), (513, 2048, 264, 0), (300, 640, 264, 5)):
        mq.tune_force_tile(tile)
        xb = torch.from_numpy(si.normal(21, f"bf/x{M}", (M, K)).astype(np.float32)).to(torch.bfloat16)
        wb = torch.from_numpy(si.normal(21, f"bf/w{N}", (N, K), 0.02).astype(np.float32)).to(torch.bfloat16)
        bb = torch.from_numpy(si.normal(21, f"bf/b{N}", (N,), 0.01).astype(np.float32)).to(torch.bfloat16)
        bits16 = lambda t: t.view(torch.int16).numpy().view(np.uint16)
        for bits in ALL_BITS:
            c, s, z = mq.quantize_weights(wb.cuda(), bits)
            oc, os_, oz = orc.quantize_weights(bits16(wb), bits, dtype=orc.BF16)
            assert np.array_equal(host(c), oc) and np.array_equal(host(s), os_) and np.array_equal(host(z), oz)
            packed, cs = mq.pack_weights(c, bits, mq.LAYOUT_KERNEL)
            pw = mq.PackedWeight(packed, s, z, cs, N, K, bits, mq.LAYOUT_KERNEL, False)
            y = mq.qlinear_w_only(xb.cuda(), pw, bb.cuda())
            assert y.dtype == torch.bfloat16
            ref = orc.linear_w_only(bits16(xb), oc, os_, oz, bits16(bb), dtype=orc.BF16)
            got = host(y.float()).astype(np.float64)
            want = torch.from_numpy(ref.view(np.int16)).view(torch.bfloat16).float().numpy().astype(np.float64)
            fro = np.linalg.norm(got - want) / np.linalg.norm(want)
            elt = np.abs(got - want).max() / np.abs(want).max()
            assert fro <= FRO_TOL and elt <= ELT_TOL, f"bf16 b{bits} {M}x{K}x{N}: fro={fro:.3e} elt={elt:.3e}"
    mq.tune_force_tile(-1)


def test_w_only_strided_views(mq, orc):
    M, K, N = 130, 128, 64
    xbig = si.activations_f16(12, "wo/xs", M, K + 64)
    w = si.weights_f16(12, "wo/ws", N, K)
    pw, oc, os_, oz = make_weight(mq, orc, w, 4)
    xd = dev(xbig)[:, :K]
    out = torch.zeros((M, N + 16), dtype=torch.float16, device="cuda")
    mq.qlinear_w_only(xd, pw, out=out[:, :N])
    ref = orc.linear_w_only(np.ascontiguousarray(xbig[:, :K]), oc, os_, oz)
    assert_close16(host(out)[:, :N], ref, "strided")
    assert not host(out)[:, N:].any()


@pytest.mark.parametrize("M,K,N", [(4096, 640, 640), (4096, 640, 5120), (4096, 2560, 640)])
def test_w_only_transformer_block_shapes_sampled_rows(mq, orc, M, K, N):
    """64x64-level block linears (batch 1) at full size, in the launch configuration the benchmark uses;
    the oracle evaluates a seeded sample of rows including the first, the last and the rows of extreme values."""
    x = si.activations_f16(0, f"c2/x{K}", M, K, outlier_prob=0.01)
    w = si.weights_f16(0, f"c2/w{N}x{K}", N, K)
    b = si.bias_f16(0, f"c2/b{N}", N)
    rows = sample_rows(x, 512, M + K + N)
    for bits in (8, 4, 3):
        pw, oc, os_, oz = make_weight(mq, orc, w, bits)
        y = host(mq.qlinear_w_only(dev(x), pw, dev(b)))
        ref = orc.linear_w_only(x, oc, os_, oz, b, rows=rows)
        assert_close16(y[rows], ref, f"c2 b{bits} {M}x{K}x{N}")
        # rows the oracle did not visit: finite and of plausible magnitude
        assert np.isfinite(y).all() and np.abs(y.astype(np.float64)).max() < 4 * np.abs(
            ref.view(np.float16).astype(np.float64)).max() + 1


# ----------------------------------------------------------------------------------------------- layers kept at 16 bits

@pytest.mark.parametrize("tile", (-1, 0, 1, 2, 3, 4, 5, 6))
def test_unquantised_16bit_layer(mq, orc, tile):
    """bits = 16: the weights go through the same tile order and GEMM skeleton unquantised (fp16 and bf16)."""
    mq.tune_force_tile(tile)
    try:
        for (M, K, N) in ((256, 320, 320), (77, 128, 40), (300, 640, 264), (513, 2048, 640)):
            if tile == 0 and M * N > 400000:
                continue
            x = si.activations_f16(51, f"w16/x{M}x{K}", M, K)
            w = si.weights_f16(51, f"w16/w{N}x{K}", N, K)
            b = si.bias_f16(51, f"w16/b{N}", N)
            wd = dev(w)
            pw = mq.keep_weights_16bit(wd)
            assert pw.packed.numel() == (N + 31) // 32 * 32 * K * 2
            assert torch.equal(mq.unpack_weights(pw.packed, N, K, 16, mq.LAYOUT_KERNEL), wd)
            for bias in (b, None):
                y = mq.qlinear_w_only(dev(x), pw, None if bias is None else dev(bias))
                assert_close16(host(y), orc.linear_fp(x, w, bias), f"w16 tile{tile} {M}x{K}x{N}")
        # bf16
        M, K, N = 130, 192, 72
        xb = torch.from_numpy(si.normal(52, "w16/xb", (M, K)).astype(np.float32)).to(torch.bfloat16)
        wb = torch.from_numpy(si.normal(52, "w16/wb", (N, K), 0.02).astype(np.float32)).to(torch.bfloat16)
        pw = mq.keep_weights_16bit(wb.cuda())
        y = mq.qlinear_w_only(xb.cuda(), pw)
        assert y.dtype == torch.bfloat16
        ref = orc.linear_fp(xb.view(torch.int16).numpy().view(np.uint16), wb.view(torch.int16).numpy().view(np.uint16),
                            dtype=orc.BF16)
        got = host(y.view(torch.int16)).view(np.uint16)
        a = orc.f16_to_f64(got, orc.BF16)
        r = orc.f16_to_f64(ref, orc.BF16)
        assert np.linalg.norm(a - r) <= FRO_TOL * np.linalg.norm(r) and np.abs(a - r).max() <= ELT_TOL * np.abs(r).max()
    finally:
        mq.tune_force_tile(-1)


def test_16bit_canonical_pack_is_the_matrix(mq):
    w = dev(si.weights_f16(53, "w16/c", 40, 128))
    p, cs = mq.pack_weights(w, 16, mq.LAYOUT_CANONICAL)
    assert cs is None and torch.equal(p.view(torch.float16).view(40, 128), w)
    assert torch.equal(mq.unpack_weights(p, 40, 128, 16, mq.LAYOUT_CANONICAL), w)


# ----------------------------------------------------------------------------------------------- reduction split over workgroups

SPLIT_SHAPES = [(1, 5120, 1280), (16, 1280, 320), (77, 2048, 1280), (308, 2048, 640), (130, 640, 96), (33, 256, 40)]


@pytest.mark.parametrize("tile", (-1, 1, 2, 3, 4, 5))
@pytest.mark.parametrize("parts", (0, 2, 3, 7))
def test_split_reduction_matches_oracle(mq, orc, tile, parts):
    """Few tiles, long reduction: several workgroups per tile, partial sums through the caller's workspace.
    parts = 0 is the automatic choice; forced part counts also cover uneven splits and the k-split tiles."""
    mq.tune_force_tile(tile)
    mq.tune_force_splits(parts)
    try:
        for (M, K, N) in SPLIT_SHAPES:
            x = si.activations_f16(31, f"sp/x{M}x{K}", M, K, outlier_prob=0.01)
            w = si.weights_f16(31, f"sp/w{N}x{K}", N, K)
            b = si.bias_f16(31, f"sp/b{N}", N)
            for bits in (4, 3):
                pw, oc, os_, oz = make_weight(mq, orc, w, bits)
                y = mq.qlinear_w_only(dev(x), pw, dev(b))
                assert_close16(host(y), orc.linear_w_only(x, oc, os_, oz, b), f"split w{bits} {M}x{K}x{N} parts{parts}")
            pw, oc, os_, oz = make_weight(mq, orc, w, 4)
            y, acc, _ = mq.qlinear_w4a8(dev(x), pw, bias=dev(b), want_acc=True)
            ry, racc, _ = orc.linear_a8(x, oc, os_, oz, bias=b)
            assert np.array_equal(host(acc), racc), f"split acc {M}x{K}x{N} parts{parts}"
            assert_close16(host(y), ry, f"split a4 {M}x{K}x{N} parts{parts}")
    finally:
        mq.tune_force_splits(0)
        mq.tune_force_tile(-1)


def test_split_reduction_is_deterministic_and_reuses_its_workspace(mq, orc):
    """Many launches in a row through ONE workspace whose contents start as garbage (the counters are cleared on the
    stream before every launch): every result is bit-identical.  Without a workspace the same call does not split and
    still matches the oracle; a workspace that holds only some of the parts is used for as many as fit."""
    M, K, N = 64, 5120, 1280
    xh = si.activations_f16(32, "sp/det", M, K)
    x = dev(xh)
    pw, oc, os_, oz = make_weight(mq, orc, si.weights_f16(32, "sp/detw", N, K), 4)
    ref = orc.linear_w_only(xh, oc, os_, oz)
    mq.tune_force_splits(16)
    try:
        ws = torch.full((mq.split_workspace_bytes(M, N, K),), 0xA5, dtype=torch.uint8, device="cuda")
        y0 = mq.qlinear_w_only(x, pw, ws=ws).clone()
        assert_close16(host(y0), ref, "forced 16 parts")
        for _ in range(40):
            assert torch.equal(mq.qlinear_w_only(x, pw, ws=ws), y0)
        with pytest.raises(mq.MixdqError) as e:
            mq.qlinear_w_only(x, pw, ws=ws[:1 << 20])
        assert e.value.code == -4
    finally:
        mq.tune_force_splits(0)
    need = mq.split_workspace_bytes(M, N, K)
    assert need > 0
    full = mq.plan_qlinear_w_only(x, pw, None, torch.empty_like(y0), ws=torch.empty(need, dtype=torch.uint8, device="cuda"))
    none = mq.plan_qlinear_w_only(x, pw, None, torch.empty_like(y0), ws=None)
    some = mq.plan_qlinear_w_only(x, pw, None, torch.empty_like(y0), ws=torch.empty(need // 5 // 256 * 256, dtype=torch.uint8,
                                                                                  device="cuda"))
    for plan in (full, none, some):
        plan()
        assert_close16(host(plan.keepalive[3]), ref, "automatic split, full / no / small workspace")


def test_split_reductions_on_two_streams_with_a_workspace_each(mq, orc):
    """Split launches queued on two streams at once, each stream with its own workspace, one of them behind a long
    kernel so that the launches of the other overtake it: all results equal the single-stream result bit for bit.
    (One workspace per stream is the contract; nothing of the library is shared between the launches.)"""
    M, K, N = 64, 5120, 1280
    x = dev(si.activations_f16(33, "sp2/x", M, K))
    pw, *_ = make_weight(mq, orc, si.weights_f16(33, "sp2/w", N, K), 4)
    big_x = dev(si.activations_f16(33, "sp2/bx", 4096, 1280))
    big_w, *_ = make_weight(mq, orc, si.weights_f16(33, "sp2/bw", 5120, 1280), 4)
    mq.tune_force_splits(16)
    try:
        need = mq.split_workspace_bytes(M, N, K)
        wsa = torch.empty(need, dtype=torch.uint8, device="cuda")
        wsb = torch.empty(need, dtype=torch.uint8, device="cuda")
        ref = mq.qlinear_w_only(x, pw, ws=wsa).clone()
        torch.cuda.synchronize()
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        for it in range(6):
            with torch.cuda.stream(s1):
                for _ in range(4):
                    mq.qlinear_w_only(big_x, big_w)           # long kernels ahead of the split launch
                ya = [mq.qlinear_w_only(x, pw, ws=wsa) for _ in range(3)]
            with torch.cuda.stream(s2):
                yb = [mq.qlinear_w_only(x, pw, ws=wsb) for _ in range(12)]
            torch.cuda.synchronize()
            for y in ya + yb:
                assert torch.equal(y, ref), f"round {it}"
    finally:
        mq.tune_force_splits(0)


# ----------------------------------------------------------------------------------------------- 8-bit activations

A8_SHAPES = [(256, 320, 320), (1, 64, 32), (77, 128, 40), (608, 2048, 640), (300, 1280, 264), (130, 192, 64)]


@pytest.mark.parametrize("mode", ("w8s", "w8a", "w4", "w2"))
@pytest.mark.parametrize("tile", (-1, 0, 1, 2, 3, 4, 5, 6))
def test_a8_small_shapes(mq, orc, mode, tile):
    mq.tune_force_tile(tile)
    bits, sym = {"w8s": (8, True), "w8a": (8, False), "w4": (4, False), "w2": (2, False)}[mode]
    fn = {8: mq.qlinear_w8a8, 4: mq.qlinear_w4a8, 2: mq.qlinear_w2a8}[bits]
    for (M, K, N) in A8_SHAPES:
        x = si.activations_f16(13, f"a8/x{M}x{K}", M, K, outlier_prob=0.01)
        w = si.weights_f16(13, f"a8/w{N}x{K}", N, K)
        b = si.bias_f16(13, f"a8/b{N}", N)
        pw, oc, os_, oz = make_weight(mq, orc, w, bits, sym)
        # dynamic activation parameters
        y, acc, (s_out, z_out) = fn(dev(x), pw, bias=dev(b), want_acc=True, want_act=True)
        ry, racc, (rs, rz) = orc.linear_a8(x, oc, os_, oz, w_signed=sym, bias=b)
        assert host(s_out)[0] == rs and host(z_out)[0] == rz, "dynamic activation parameters"
        assert np.array_equal(host(acc), racc), f"acc {mode} tile{tile} {M}x{K}x{N}"
        assert_close16(host(y), ry, f"a8 {mode} tile{tile} {M}x{K}x{N}")
        # static (calibrated) parameters, narrower than the data so that codes saturate
        act = (np.float32(0.03), 117)
        y, acc, _ = fn(dev(x), pw, act=(dev(np.array([act[0]], np.float32)), dev(np.array([act[1]], np.int32))),
                       want_acc=True)
        ry, racc, _ = orc.linear_a8(x, oc, os_, oz, w_signed=sym, act=act)
        assert np.array_equal(host(acc), racc)
        assert_close16(host(y), ry, f"a8 static {mode}")
    mq.tune_force_tile(-1)


def test_a8_is_deterministic(mq, orc):
    M, K, N = 608, 2048, 640
    x = dev(si.activations_f16(14, "a8/det", M, K))
    pw, *_ = make_weight(mq, orc, si.weights_f16(14, "a8/detw", N, K), 4)
    y0, a0, _ = mq.qlinear_w4a8(x, pw, want_acc=True)
    for _ in range(3):
        y1, a1, _ = mq.qlinear_w4a8(x, pw, want_acc=True)
        assert torch.equal(a0, a1) and torch.equal(y0, y1)


@pytest.mark.parametrize("K,N", [(1280, 1280), (1280, 10240), (5120, 1280)])
def test_a8_transformer_block_shapes_sampled_rows(mq, orc, K, N):
    """32x32-level block linears (batch 4, M = 4096) at full size; oracle on sampled rows, accumulators bit-exact."""
    M = 4096
    x = si.activations_f16(0, f"c3/x{K}", M, K)
    w = si.weights_f16(0, f"c3/w{N}x{K}", N, K)
    b = si.bias_f16(0, f"c3/b{N}", N)
    rows = sample_rows(x, 512, K + N)
    for bits, sym, fn in ((4, False, mq.qlinear_w4a8), (8, True, mq.qlinear_w8a8), (2, False, mq.qlinear_w2a8)):
        pw, oc, os_, oz = make_weight(mq, orc, w, bits, sym)
        y, acc, (s_out, z_out) = fn(dev(x), pw, bias=dev(b), want_acc=True, want_act=True)
        ry, racc, (rs, rz) = orc.linear_a8(x, oc, os_, oz, w_signed=sym, bias=b, rows=rows)
        assert host(s_out)[0] == rs and host(z_out)[0] == rz
        assert np.array_equal(host(acc)[rows], racc)
        assert_close16(host(y)[rows], ry, f"c3 W{bits}A8 {K}->{N}")


def test_a8_longest_reduction_and_extreme_codes(mq, orc):
    """K = 33024 is the longest reduction the int32 accumulator is guaranteed to hold (255 * 255 * K < 2^31).  All
    activation codes and all weight codes are 0 or 255 with zero points 0; row 0 against channel 0 is 255 * 255 in
    every term, which puts that accumulator within 1e-4 of the int32 limit."""
    M, K, N = 40, 33024, 72
    rng = np.random.default_rng(33024)
    x = np.where(rng.random((M, K)) < 0.5, 0.0, 1.0)
    x[0] = 1.0
    w = np.where(rng.random((N, K)) < 0.5, 0.0, 0.02)
    w[0] = 0.02
    x, w = x.astype(np.float16), w.astype(np.float16)
    pw, oc, os_, oz = make_weight(mq, orc, w, 8)
    y, acc, _ = mq.qlinear_w8a8(dev(x), pw, want_acc=True)
    ry, racc, _ = orc.linear_a8(x, oc, os_, oz)
    assert int(racc[0, 0]) == 255 * 255 * K and 255 * 255 * K > 0.9999 * 2 ** 31
    assert np.array_equal(host(acc), racc)
    assert_close16(host(y), ry, "longest reduction")


def test_many_rows_and_smallest_problem(mq, orc):
    """70001 activation rows (a ragged multiple of every tile height) against the smallest weight the layout allows,
    and a 1 x 64 -> 8 problem."""
    for (M, K, N, bits) in ((70001, 64, 32, 2), (1, 64, 8, 3), (3, 64, 8, 8)):
        x = si.activations_f16(41, f"edge/x{M}", M, K)
        w = si.weights_f16(41, f"edge/w{N}", N, K)
        pw, oc, os_, oz = make_weight(mq, orc, w, bits)
        assert_close16(host(mq.qlinear_w_only(dev(x), pw)), orc.linear_w_only(x, oc, os_, oz), f"edge w{bits} M={M}")
        if bits == 8:
            y, acc, _ = mq.qlinear_w8a8(dev(x), pw, want_acc=True)
            ry, racc, _ = orc.linear_a8(x, oc, os_, oz)
            assert np.array_equal(host(acc), racc)
            assert_close16(host(y), ry, "edge a8")


def test_degenerate_tensors(mq, orc):
    """Constant activations (all zero: scale 1, zero point 0; all equal and positive: the range is [0, v]) and weight
    rows that are constant or zero."""
    M, K, N = 96, 128, 64
    w = si.weights_f16(42, "deg/w", N, K)
    w[0] = 0
    w[1] = np.float16(0.015)
    w[2] = np.float16(-0.015)
    b = si.bias_f16(42, "deg/b", N)
    for bits, fn in ((4, mq.qlinear_w4a8), (8, mq.qlinear_w8a8)):
        pw, oc, os_, oz = make_weight(mq, orc, w, bits)
        for fill in (0.0, 0.75, -2.0):
            x = np.full((M, K), fill, np.float16)
            y, acc, (s_out, z_out) = fn(dev(x), pw, bias=dev(b), want_acc=True, want_act=True)
            ry, racc, (rs, rz) = orc.linear_a8(x, oc, os_, oz, bias=b)
            assert host(s_out)[0] == rs and host(z_out)[0] == rz
            assert np.array_equal(host(acc), racc)
            assert_close16(host(y), ry, f"degenerate a8 fill {fill}")
            assert_close16(host(mq.qlinear_w_only(dev(x), pw, dev(b))), orc.linear_w_only(x, oc, os_, oz, b),
                           f"degenerate w_only fill {fill}")
    x = np.zeros((M, K), np.float16)
    pw, *_ = make_weight(mq, orc, w, 4)
    y, _, (s_out, z_out) = mq.qlinear_w4a8(dev(x), pw, bias=dev(b), want_act=True)
    assert host(s_out)[0] == 1.0 and host(z_out)[0] == 0
    assert np.array_equal(host(y), np.broadcast_to(b.view(np.float16), (M, N)))  # zero input: the output is the bias


# ----------------------------------------------------------------------------------------------- feed-forward pair, 8 bits in between

def a8_layout(codes):
    """Unsigned codes [M,K] -> the int8 activation layout the GEMM reads (test-side marshalling only)."""
    M, K = codes.shape
    Kp = (K + 127) // 128 * 128
    a = np.zeros((M, Kp), np.int8)
    a[:, :K] = (codes.astype(np.int16) - 128).astype(np.int8)
    perm = np.array([0, 4, 1, 5, 2, 6, 3, 7])
    return a.reshape(M, Kp // 8, 8)[:, :, perm].reshape(M, Kp)


def a8_unlayout(a8, K):
    """The inverse: int8 layout [M,Kp] -> unsigned codes [M,K] and the padding bytes."""
    M, Kp = a8.shape
    inv = np.argsort(np.array([0, 4, 1, 5, 2, 6, 3, 7]))
    lin = a8.reshape(M, Kp // 8, 8)[:, :, inv].reshape(M, Kp)
    return (lin[:, :K].astype(np.int16) + 128).astype(np.uint8), lin[:, K:]


def geglu_code_slack(u, lin, bias, H, out_scale, acc_err=None):
    """How far the kernel's fp32 evaluation of u = value * gelu(gate) / s_o may lie from the oracle's fp64 one,
    element by element.  The integer accumulators are exact on both sides; the kernel then takes, each rounded once to
    fp32: s_x * s_w[n], (float)ACC, one fma per half (<= 4 roundings of 2^-24 on |lin| + |bias|), a GELU whose error
    function is good to 3e-7 absolute (so gelu to 1.5e-7 |g| plus the slope 1.13 times the gate's error plus its own
    rounding), the product, 1 / s_o and the multiplication by it (3 more roundings).
    acc_err [R, 2H]: what the accumulation itself may be off by where it is not exact (the fp16 MFMA path)."""
    e24 = 2.0 ** -24
    v, g = lin[:, :H], lin[:, H:]
    bv, bg = np.abs(bias[:H].astype(np.float64))[None, :], np.abs(bias[H:].astype(np.float64))[None, :]
    e_v = 4 * e24 * (np.abs(v) + bv)
    e_g = 4 * e24 * (np.abs(g) + bg)
    if acc_err is not None:
        e_v = e_v + acc_err[:, :H]
        e_g = e_g + acc_err[:, H:]
    from scipy.special import erf
    gelu = 0.5 * g * (1.0 + erf(g / np.sqrt(2.0)))
    e_gelu = 1.13 * e_g + 1.5e-7 * np.maximum(np.abs(g), 1.0) + 2 * e24 * np.abs(gelu)
    e_h = np.abs(v) * e_gelu + np.abs(gelu) * e_v
    return e_h / np.float64(out_scale) + 4 * e24 * np.abs(u)


def assert_geglu_codes(codes, rq, u, slack, out_zp, what):
    """Every element: the kernel's code is the oracle's, or its neighbour where the oracle's un-rounded value lies
    within the kernel's arithmetic error of the rounding boundary between the two."""
    d = codes.astype(np.int64) - rq.astype(np.int64)
    assert np.abs(d).max() <= 1, f"{what}: a code is off by more than one"
    off = d != 0
    # boundary between the oracle's code and the kernel's: (oracle code - z_o) + d / 2, in units of s_o
    boundary = (rq.astype(np.float64) - out_zp) + 0.5 * d
    assert (np.abs(u - boundary)[off] <= slack[off]).all(), \
        f"{what}: {int((np.abs(u - boundary)[off] > slack[off]).sum())} codes differ away from a rounding boundary"
    assert off.sum() <= max(3, 1e-3 * off.size), f"{what}: {off.mean():.2e} of the codes sit on a boundary"
    return int(off.sum())


@pytest.mark.parametrize("bits,sym", [(4, False), (8, True), (8, False), (2, False)])
@pytest.mark.parametrize("tile", (-1, 0, 1))
def test_geglu_projection_codes_against_the_fp64_oracle(mq, orc, bits, sym, tile):
    """value * gelu(gate) -> 8-bit codes.  The oracle states the layer in fp64 with the library erf; the kernel
    evaluates the epilogue in fp32.  Rule, checked on every element: equal codes, or neighbours where the oracle's
    un-rounded value lies within the kernel's error bound of the boundary between them."""
    mq.tune_force_tile(tile)
    try:
        for (M, K, H) in ((256, 320, 320), (77, 128, 32), (300, 640, 96), (130, 1280, 160)):
            x = si.activations_f16(61, f"ff/x{M}x{K}", M, K, outlier_prob=0.01)
            w = si.weights_f16(61, f"ff/w{H}x{K}", 2 * H, K)
            b = si.bias_f16(61, f"ff/b{H}", 2 * H)
            pw, oc, os_, oz = make_weight(mq, orc, w, bits, sym)
            out_act = (np.float32(0.006), 28)
            d_out = (dev(np.array([out_act[0]], np.float32)), dev(np.array([out_act[1]], np.int32)))
            for act in (None, (np.float32(0.03), 117)):
                d_act = None if act is None else (dev(np.array([act[0]], np.float32)), dev(np.array([act[1]], np.int32)))
                a8, h16, got_act = mq.qlinear_a8_geglu(dev(x), pw, d_out, act=d_act, bias=dev(b), want_h16=True,
                                                       want_act=True)
                rq, rh, ract, u, lin = orc.linear_a8_geglu(x, oc, os_, oz, out_act, w_signed=sym, act=act, bias=b,
                                                           want_pre=True)
                assert host(got_act[0])[0] == ract[0] and host(got_act[1])[0] == ract[1]
                codes, pad = a8_unlayout(host(a8), H)
                assert a8.shape[1] == (H + 127) // 128 * 128 and not pad.any()
                what = f"geglu codes b{bits} tile{tile} {M}x{K}x{H}"
                assert_geglu_codes(codes, rq, u, geglu_code_slack(u, lin, b, H, out_act[0]), out_act[1], what)
                assert_close16(host(h16), rh, what + " (gated product in fp16)")
    finally:
        mq.tune_force_tile(-1)


@pytest.mark.parametrize("bits", (2, 3, 4, 8))
@pytest.mark.parametrize("tile", (-1, 0, 1))
def test_w_only_geglu_projection_with_8_bit_output(mq, orc, bits, tile):
    """The gated projection of the 16-bit-activation path emitting 8-bit codes.  Same rule as for the int8 projection
    (equal codes, or neighbours at a rounding boundary), with the error of the fp32 accumulation of the fp16 MFMA
    added to the bound: the products are exact, every MFMA adds a 16-term dot product to an fp32 accumulator, so a
    sum of K terms is off by at most (K/16 + 4) 2^-24 times the sum of their magnitudes."""
    mq.tune_force_tile(tile)
    try:
        for (M, K, H) in ((256, 320, 320), (77, 128, 32), (300, 640, 96), (130, 1280, 160)):
            x = si.activations_f16(65, f"wg/x{M}x{K}", M, K, outlier_prob=0.01)
            w = si.weights_f16(65, f"wg/w{H}x{K}", 2 * H, K)
            b = si.bias_f16(65, f"wg/b{H}", 2 * H)
            pw, oc, os_, oz = make_weight(mq, orc, w, bits)
            out_act = (np.float32(0.006), 28)
            d_out = (dev(np.array([out_act[0]], np.float32)), dev(np.array([out_act[1]], np.int32)))
            a8, h16 = mq.qlinear_w_only_geglu_a8(dev(x), pw, d_out, bias=dev(b), want_h16=True)
            rq, rh, u, lin = orc.linear_w_only_geglu(x, oc, os_, oz, bias=b, out_act=out_act, want_pre=True)
            wmag = np.abs(oc.astype(np.float64) - oz[:, None]) * os_[:, None].astype(np.float64)
            acc_err = (K / 16 + 4) * 2.0 ** -24 * (np.abs(x.astype(np.float64)) @ wmag.T)
            codes, pad = a8_unlayout(host(a8), H)
            assert a8.shape[1] == (H + 127) // 128 * 128 and not pad.any()
            what = f"w-only geglu codes b{bits} tile{tile} {M}x{K}x{H}"
            assert_geglu_codes(codes, rq, u, geglu_code_slack(u, lin, b, H, out_act[0], acc_err), out_act[1], what)
            assert_close16(host(h16), rh, what + " (gated product in fp16)")
            a8b, none = mq.qlinear_w_only_geglu_a8(dev(x), pw, d_out, bias=dev(b))   # without the fp16 product
            assert none is None and torch.equal(a8b, a8)
    finally:
        mq.tune_force_tile(-1)


@pytest.mark.parametrize("bits,sym", [(4, False), (8, True), (2, False)])
@pytest.mark.parametrize("tile", (-1, 0, 1))
def test_geglu_projection_with_dynamic_output_parameters(mq, orc, bits, sym, tile):
    """The gated product leaves as fp16 with one (min, max) pair per workgroup; the codes follow from the range of
    the whole product.  Checked in two steps: the fp16 product against the oracle's (16-bit tolerance), and, on the
    kernel's own product, parameters and codes bit for bit against the oracle's dynamic quantiser; end to end the
    scale may differ from the oracle's by one fp16 step of the extreme value at most."""
    mq.tune_force_tile(tile)
    try:
        for (M, K, H) in ((256, 320, 320), (77, 128, 32), (300, 640, 96), (130, 1280, 160), (1, 64, 32)):
            x = si.activations_f16(63, f"fd/x{M}x{K}", M, K, outlier_prob=0.01)
            w = si.weights_f16(63, f"fd/w{H}x{K}", 2 * H, K)
            b = si.bias_f16(63, f"fd/b{H}", 2 * H)
            pw, oc, os_, oz = make_weight(mq, orc, w, bits, sym)
            for act in (None, (np.float32(0.03), 117)):
                d_act = None if act is None else (dev(np.array([act[0]], np.float32)), dev(np.array([act[1]], np.int32)))
                a8, h16, (so, zo), got_act = mq.qlinear_a8_geglu_dynamic(dev(x), pw, act=d_act, bias=dev(b), want_act=True)
                rq, rh, (rso, rzo), ract = orc.linear_a8_geglu_dynamic(x, oc, os_, oz, w_signed=sym, act=act, bias=b)
                what = f"geglu dynamic b{bits} tile{tile} {M}x{K}x{H}"
                assert host(got_act[0])[0] == ract[0] and host(got_act[1])[0] == ract[1], what
                gh = host(h16)
                assert_close16(gh, rh, what + " (gated product in fp16)")
                s2, z2 = orc.act_params(gh)
                assert host(so)[0] == s2 and host(zo)[0] == z2, what + " (parameters of the kernel's own product)"
                codes, pad = a8_unlayout(host(a8), H)
                assert a8.shape[1] == (H + 127) // 128 * 128 and not pad.any()
                assert np.array_equal(codes, orc.act_quantize(gh, s2, z2)), what + " (codes)"
                assert abs(float(s2) - float(rso)) <= 2.0 ** -9 * float(rso) and abs(z2 - rzo) <= 1, what
                if s2 == rso and z2 == rzo:
                    assert np.abs(codes.astype(np.int64) - rq.astype(np.int64)).max() <= 1, what
    finally:
        mq.tune_force_tile(-1)


def test_feed_forward_pair_with_dynamic_parameters_in_between(mq, orc):
    """Gated projection with dynamic output parameters, then the output linear on its codes: against the oracle run
    on the kernel's own codes (accumulators bit for bit) and end to end within the 16-bit tolerance."""
    M, C = 200, 320
    x = si.activations_f16(64, "fp/x", M, C, outlier_prob=0.01)
    w1 = si.weights_f16(64, "fp/w1", 8 * C, C)
    b1 = si.bias_f16(64, "fp/b1", 8 * C)
    w2 = si.weights_f16(64, "fp/w2", C, 4 * C)
    b2 = si.bias_f16(64, "fp/b2", C)
    pw1, c1, s1, z1 = make_weight(mq, orc, w1, 4)
    pw2, c2, s2, z2 = make_weight(mq, orc, w2, 4)
    a8, h16, (so, zo), _ = mq.qlinear_a8_geglu_dynamic(dev(x), pw1, bias=dev(b1))
    y, acc = mq.qlinear_a8_codes(a8, 4 * C, (so, zo), pw2, bias=dev(b2), want_acc=True)
    codes, _ = a8_unlayout(host(a8), 4 * C)
    ry, racc = orc.linear_a8_codes(codes, (host(so)[0], int(host(zo)[0])), c2, s2, z2, bias=b2)
    assert np.array_equal(host(acc), racc)
    assert_close16(host(y), ry, "second linear on the kernel's codes")
    rq, _, ro, _ = orc.linear_a8_geglu_dynamic(x, c1, s1, z1, bias=b1)
    if ro[0] == host(so)[0] and ro[1] == int(host(zo)[0]):  # (the extreme product rounds the same way on both sides)
        ry2, _ = orc.linear_a8_codes(rq, ro, c2, s2, z2, bias=b2)
        assert_close16(host(y), ry2, "feed-forward pair end to end")


@pytest.mark.parametrize("bits,sym", [(4, False), (8, True), (8, False), (2, False)])
@pytest.mark.parametrize("tile", (-1, 1, 2, 5))
def test_a8_linear_on_codes(mq, orc, bits, sym, tile):
    mq.tune_force_tile(tile)
    try:
        rng = np.random.default_rng(62)
        for (M, K, N) in ((256, 320, 320), (77, 128, 40), (300, 2560, 264), (1, 64, 8)):
            qx = rng.integers(0, 256, (M, K)).astype(np.uint8)
            qx[0] = 255
            qx[-1] = 0
            act = (np.float32(0.0123), 97)
            w = si.weights_f16(62, f"cd/w{N}x{K}", N, K)
            b = si.bias_f16(62, f"cd/b{N}", N)
            pw, oc, os_, oz = make_weight(mq, orc, w, bits, sym)
            d_act = (dev(np.array([act[0]], np.float32)), dev(np.array([act[1]], np.int32)))
            y, acc = mq.qlinear_a8_codes(dev(a8_layout(qx)), K, d_act, pw, bias=dev(b), want_acc=True)
            ry, racc = orc.linear_a8_codes(qx, act, oc, os_, oz, w_signed=sym, bias=b)
            assert np.array_equal(host(acc), racc), f"codes acc b{bits} tile{tile} {M}x{K}x{N}"
            assert_close16(host(y), ry, f"codes b{bits} tile{tile} {M}x{K}x{N}")
    finally:
        mq.tune_force_tile(-1)


@pytest.mark.parametrize("bits", ALL_BITS)
@pytest.mark.parametrize("tile", (-1, 0, 1))
def test_w_only_geglu_projection(mq, orc, bits, tile):
    mq.tune_force_tile(tile)
    try:
        for (M, K, H) in ((256, 320, 320), (77, 128, 32), (300, 640, 96)):
            x = si.activations_f16(64, f"wg/x{M}x{K}", M, K)
            w = si.weights_f16(64, f"wg/w{H}x{K}", 2 * H, K)
            b = si.bias_f16(64, f"wg/b{H}", 2 * H)
            pw, oc, os_, oz = make_weight(mq, orc, w, bits)
            for bias in (b, None):
                h = mq.qlinear_w_only_geglu(dev(x), pw, None if bias is None else dev(bias))
                assert_close16(host(h), orc.linear_w_only_geglu(x, oc, os_, oz, bias), f"w_only geglu b{bits} tile{tile}")
    finally:
        mq.tune_force_tile(-1)


def test_feed_forward_pair_end_to_end(mq, orc):
    """Gated projection (C -> 8C) into the output linear (4C -> C) with the activation kept in 8 bits in between.  The
    first call's codes follow the rule above; the second call consumes exactly what the first wrote, so the oracle's
    second layer is run on those very codes and its accumulators must match bit for bit."""
    M, C_ = 200, 320
    x = si.activations_f16(63, "ffp/x", M, C_)
    w1 = si.weights_f16(63, "ffp/w1", 8 * C_, C_)
    w2 = si.weights_f16(63, "ffp/w2", C_, 4 * C_)
    b1, b2 = si.bias_f16(63, "ffp/b1", 8 * C_), si.bias_f16(63, "ffp/b2", C_)
    p1, c1, s1, z1 = make_weight(mq, orc, w1, 4)
    p2, c2, s2, z2 = make_weight(mq, orc, w2, 4)
    mid = (np.float32(0.004), 42)
    d_mid = (dev(np.array([mid[0]], np.float32)), dev(np.array([mid[1]], np.int32)))
    a8, _, _ = mq.qlinear_a8_geglu(dev(x), p1, d_mid, bias=dev(b1))
    y, acc = mq.qlinear_a8_codes(a8, 4 * C_, d_mid, p2, bias=dev(b2), want_acc=True)
    rq, _, _, u, lin = orc.linear_a8_geglu(x, c1, s1, z1, mid, bias=b1, want_h16=False, want_pre=True)
    codes, pad = a8_unlayout(host(a8), 4 * C_)
    assert not pad.any()
    assert_geglu_codes(codes, rq, u, geglu_code_slack(u, lin, b1, 4 * C_, mid[0]), mid[1], "feed-forward pair, first layer")
    ry, racc = orc.linear_a8_codes(codes, mid, c2, s2, z2, bias=b2)
    assert np.array_equal(host(acc), racc)
    assert_close16(host(y), ry, "feed-forward pair")
    # and the whole pair against the oracle run end to end: the few boundary codes move the output within tolerance
    ry0, _ = orc.linear_a8_codes(rq, mid, c2, s2, z2, bias=b2)
    assert_close16(host(y), ry0, "feed-forward pair, oracle end to end")


# ----------------------------------------------------------------------------------------------- 3x3 convolution

CONV_SHAPES = [  # B, H, W, Cin, N
    (2, 8, 8, 64, 32),
    (1, 16, 16, 128, 64),
    (2, 5, 7, 64, 40),      # ragged rows, N not a multiple of the tile
    (1, 32, 32, 320, 320),  # five 64-channel chunks per tap: an int8 stage straddles two taps, the last one is half padding
    (3, 1, 1, 64, 8),       # a single pixel: only the centre tap is inside
    (1, 1, 9, 192, 24),
    (1, 9, 1, 64, 16),
]


def conv_weight(mq, orc, seed, N, Cin, bits, sym=False):
    w = si.weights_f16(seed, f"cv/w{N}x{Cin}", N, 9 * Cin, 0.05)   # [N, (r, s, c)]
    pw, oc, os_, oz = make_weight(mq, orc, w, bits, sym)
    c, _, _ = mq.quantize_weights(dev(w), bits, sym)
    tapsum = mq.conv_tap_sums(c, Cin, bits, sym)
    q = oc.view(np.int8).astype(np.int64) if sym else oc.astype(np.int64)
    assert np.array_equal(host(tapsum), q.reshape(N, 9, Cin).sum(2).T)
    return pw, oc, os_, oz, tapsum


@pytest.mark.parametrize("bits", ALL_BITS)
@pytest.mark.parametrize("tile", (-1, 0, 1, 2, 5))
def test_conv_w_only(mq, orc, bits, tile):
    mq.tune_force_tile(tile)
    try:
        for (B, H, W, Cin, N) in CONV_SHAPES:
            if tile == 0 and B * H * W * N > 200000:
                continue
            x = si.activations_f16(71, f"cv/x{B}x{H}x{W}x{Cin}", B * H * W, Cin).reshape(B, H, W, Cin)
            b = si.bias_f16(71, f"cv/b{N}", N)
            pw, oc, os_, oz, _ = conv_weight(mq, orc, 71, N, Cin, bits)
            y = mq.conv3x3_w_only(dev(x), pw, dev(b))
            assert_close16(host(y).reshape(-1, N), orc.conv3x3_w_only(x, oc, os_, oz, b),
                           f"conv w{bits} tile{tile} {B}x{H}x{W}x{Cin}->{N}")
    finally:
        mq.tune_force_tile(-1)


@pytest.mark.parametrize("bits,sym", [(4, False), (8, True), (8, False), (2, False)])
@pytest.mark.parametrize("tile", (-1, 1, 2, 5))
def test_conv_a8(mq, orc, bits, sym, tile):
    """Integer accumulators bit-exact, also on the border pixels (taps outside the image) and with a zero point far
    from 128 (static parameters)."""
    mq.tune_force_tile(tile)
    try:
        for (B, H, W, Cin, N) in CONV_SHAPES:
            x = si.activations_f16(72, f"cv8/x{B}x{H}x{W}x{Cin}", B * H * W, Cin, outlier_prob=0.01).reshape(B, H, W, Cin)
            b = si.bias_f16(72, f"cv8/b{N}", N)
            pw, oc, os_, oz, tapsum = conv_weight(mq, orc, 72, N, Cin, bits, sym)
            for act in (None, (np.float32(0.05), 31)):
                d_act = None if act is None else (dev(np.array([act[0]], np.float32)), dev(np.array([act[1]], np.int32)))
                y, acc, got = mq.conv3x3_a8(dev(x), pw, tapsum, act=d_act, bias=dev(b), want_acc=True, want_act=True)
                ry, racc, ract = orc.conv3x3_a8(x, oc, os_, oz, w_signed=sym, act=act, bias=b)
                assert host(got[0])[0] == ract[0] and host(got[1])[0] == ract[1]
                assert np.array_equal(host(acc), racc), f"conv acc b{bits} tile{tile} {B}x{H}x{W}x{Cin}->{N}"
                assert_close16(host(y).reshape(-1, N), ry, f"conv a8 b{bits} tile{tile}")
    finally:
        mq.tune_force_tile(-1)


@pytest.mark.parametrize("tile", (-1, 0, 1, 2, 5))
def test_conv_stride_two(mq, orc, tile):
    """The downsampling convolutions (stride 2, padding 1), odd image sizes included: weight-only outputs within
    tolerance, int32 accumulators of the 8-bit-activation form bit-exact (borders included), with and without a
    residual of the output's shape."""
    mq.tune_force_tile(tile)
    try:
        for (B, H, W, Cin, N) in CONV_SHAPES:
            if tile == 0 and B * H * W * N > 800000:
                continue
            Ho, Wo = (H - 1) // 2 + 1, (W - 1) // 2 + 1
            x = si.activations_f16(73, f"cs/x{B}x{H}x{W}x{Cin}", B * H * W, Cin, outlier_prob=0.01).reshape(B, H, W, Cin)
            b = si.bias_f16(73, f"cs/b{N}", N)
            r = si.normal(73, f"cs/r{B}x{Ho}x{Wo}x{N}", (B, Ho, Wo, N)).astype(np.float16)
            what = f"tile{tile} {B}x{H}x{W}x{Cin}->{N}"
            pw, oc, os_, oz, tapsum = conv_weight(mq, orc, 73, N, Cin, 4)
            y = mq.conv3x3_w_only(dev(x), pw, dev(b), stride=2)
            assert tuple(y.shape) == (B, Ho, Wo, N)
            assert_close16(host(y).reshape(-1, N), orc.conv3x3_w_only(x, oc, os_, oz, b, stride=2), "stride 2 w4 " + what)
            y = mq.conv3x3_w_only(dev(x), pw, dev(b), residual=dev(r), stride=2)
            assert_close16(host(y).reshape(-1, N), orc.conv3x3_w_only(x, oc, os_, oz, b, stride=2, residual=r),
                           "stride 2 w4 + residual " + what)
            if tile != 0:
                for act in (None, (np.float32(0.05), 31)):
                    d_act = None if act is None else (dev(np.array([act[0]], np.float32)), dev(np.array([act[1]], np.int32)))
                    y, acc, got = mq.conv3x3_a8(dev(x), pw, tapsum, act=d_act, bias=dev(b), want_acc=True, want_act=True,
                                                residual=dev(r), stride=2)
                    ry, racc, ract = orc.conv3x3_a8(x, oc, os_, oz, act=act, bias=b, residual=r, stride=2)
                    assert host(got[0])[0] == ract[0] and host(got[1])[0] == ract[1]
                    assert np.array_equal(host(acc), racc), "stride 2 acc " + what
                    assert_close16(host(y).reshape(-1, N), ry, "stride 2 a8 " + what)
    finally:
        mq.tune_force_tile(-1)


# ----------------------------------------------------------------------------------------------- residual operand

RES_SHAPES = [(256, 320, 320), (77, 128, 40), (513, 192, 264), (300, 640, 640), (1, 64, 32)]


@pytest.mark.parametrize("tile", (-1, 0, 1, 2, 3, 4, 5, 6))
def test_residual_weight_only(mq, orc, tile):
    """y = linear(x) + residual with one rounding; the residual as its own tensor, as a strided view, and as the
    output tensor itself (in place)."""
    mq.tune_force_tile(tile)
    try:
        for bits in (4, 8):
            for (M, K, N) in RES_SHAPES:
                x = si.activations_f16(81, f"rs/x{M}x{K}", M, K)
                w = si.weights_f16(81, f"rs/w{N}x{K}", N, K)
                b = si.bias_f16(81, f"rs/b{N}", N)
                r = si.normal(81, f"rs/r{M}x{N}", (M, N)).astype(np.float16)
                pw, oc, os_, oz = make_weight(mq, orc, w, bits)
                ref = orc.linear_w_only(x, oc, os_, oz, b, residual=r)
                what = f"res w{bits} tile{tile} {M}x{K}x{N}"
                assert_close16(host(mq.qlinear_w_only(dev(x), pw, dev(b), residual=dev(r))), ref, what)
                wide = torch.zeros((M, N + 24), dtype=torch.float16, device="cuda")
                wide[:, 8:8 + N] = dev(r)
                assert_close16(host(mq.qlinear_w_only(dev(x), pw, dev(b), residual=wide[:, 8:8 + N])), ref, what + " view")
                inplace = dev(r).clone()
                mq.qlinear_w_only(dev(x), pw, dev(b), out=inplace, residual=inplace)
                assert_close16(host(inplace), ref, what + " in place")
    finally:
        mq.tune_force_tile(-1)


def test_residual_is_added_before_the_rounding(mq, orc):
    """Integers: linear part up to about 2^13 (fp16 spacing 4 to 8 there), residual in [-3, 3]; rounding the linear
    part first and adding afterwards gives other numbers, the fp32 sum rounded once is the oracle's, bit for bit."""
    rng = np.random.default_rng(9)
    M, K, N = 160, 256, 96
    x = rng.integers(0, 9, (M, K)).astype(np.float16)
    codes = rng.integers(0, 16, (N, K)).astype(np.uint8)
    zp = np.full(N, 3, np.int32)
    one = np.ones(N, np.float32)
    r = rng.integers(-3, 4, (M, N)).astype(np.float16)
    packed, cs = mq.pack_weights(dev(codes), 4, mq.LAYOUT_KERNEL)
    pw = mq.PackedWeight(packed, dev(one), dev(zp), cs, N, K, 4, mq.LAYOUT_KERNEL, False)
    ref = orc.linear_w_only(x, codes, one, zp, None, residual=r).view(np.float16)
    lin = x.astype(np.int64) @ (codes.astype(np.int64) - 3).T
    assert np.array_equal(ref, (lin + r.astype(np.int64)).astype(np.float16))
    twice = (lin.astype(np.float16) + r).astype(np.float16)
    assert (twice != ref).any()
    for tile in (-1, 0, 1, 2, 3, 4, 5):
        mq.tune_force_tile(tile)
        try:
            assert np.array_equal(host(mq.qlinear_w_only(dev(x), pw, residual=dev(r))), ref), tile
        finally:
            mq.tune_force_tile(-1)


def test_residual_bf16_and_unquantised_layer(mq, orc):
    M, K, N = 200, 256, 136
    bits16 = lambda t: t.view(torch.int16).numpy().view(np.uint16)
    f32 = lambda name, shape, std: torch.from_numpy(si.normal(82, name, shape, std).astype(np.float32))
    xb, wb = f32("rb/x", (M, K), 1.0).to(torch.bfloat16), f32("rb/w", (N, K), 0.03).to(torch.bfloat16)
    rb = f32("rb/r", (M, N), 1.0).to(torch.bfloat16)
    c, s, z = mq.quantize_weights(wb.cuda(), 4)
    oc, os_, oz = orc.quantize_weights(bits16(wb), 4, dtype=orc.BF16)
    packed, cs = mq.pack_weights(c, 4, mq.LAYOUT_KERNEL)
    pw = mq.PackedWeight(packed, s, z, cs, N, K, 4, mq.LAYOUT_KERNEL, False)
    y = mq.qlinear_w_only(xb.cuda(), pw, residual=rb.cuda())
    ref = orc.linear_w_only(bits16(xb), oc, os_, oz, None, dtype=orc.BF16, residual=bits16(rb))
    want = torch.from_numpy(ref.view(np.int16)).view(torch.bfloat16).float().numpy().astype(np.float64)
    got = host(y.float()).astype(np.float64)
    assert np.linalg.norm(got - want) / np.linalg.norm(want) <= FRO_TOL
    assert np.abs(got - want).max() <= ELT_TOL * np.abs(want).max()
    # a layer kept at 16 bits (fp16)
    x = si.activations_f16(82, "rb/x16", M, K)
    w = si.weights_f16(82, "rb/w16", N, K)
    r = si.normal(82, "rb/r16", (M, N)).astype(np.float16)
    pw16 = mq.keep_weights_16bit(dev(w))
    assert_close16(host(mq.qlinear_w_only(dev(x), pw16, residual=dev(r))), orc.linear_fp(x, w, None, residual=r),
                   "16-bit layer + residual")


@pytest.mark.parametrize("mode", ("w8s", "w4"))
@pytest.mark.parametrize("tile", (-1, 0, 1, 2, 3, 4, 5, 6))
def test_residual_a8(mq, orc, mode, tile):
    bits, sym = (8, True) if mode == "w8s" else (4, False)
    mq.tune_force_tile(tile)
    try:
        for (M, K, N) in RES_SHAPES:
            x = si.activations_f16(83, f"r8/x{M}x{K}", M, K, outlier_prob=0.01)
            w = si.weights_f16(83, f"r8/w{N}x{K}", N, K)
            b = si.bias_f16(83, f"r8/b{N}", N)
            r = si.normal(83, f"r8/r{M}x{N}", (M, N)).astype(np.float16)
            pw, oc, os_, oz = make_weight(mq, orc, w, bits, sym)
            fn = mq.qlinear_w8a8 if bits == 8 else mq.qlinear_w4a8
            y, acc, _ = fn(dev(x), pw, bias=dev(b), want_acc=True, residual=dev(r))
            ry, racc, _ = orc.linear_a8(x, oc, os_, oz, w_signed=sym, bias=b, residual=r)
            assert np.array_equal(host(acc), racc)
            assert_close16(host(y), ry, f"res a8 {mode} tile{tile} {M}x{K}x{N}")
    finally:
        mq.tune_force_tile(-1)


@pytest.mark.parametrize("parts", (0, 3))
def test_residual_with_split_reduction(mq, orc, parts):
    """The workgroup that arrives last at a split tile adds the residual once."""
    mq.tune_force_splits(parts)
    try:
        for (M, K, N) in ((16, 1280, 320), (77, 2048, 1280), (130, 640, 96)):
            x = si.activations_f16(84, f"rsp/x{M}x{K}", M, K)
            w = si.weights_f16(84, f"rsp/w{N}x{K}", N, K)
            r = si.normal(84, f"rsp/r{M}x{N}", (M, N)).astype(np.float16)
            pw, oc, os_, oz = make_weight(mq, orc, w, 4)
            assert_close16(host(mq.qlinear_w_only(dev(x), pw, residual=dev(r))),
                           orc.linear_w_only(x, oc, os_, oz, None, residual=r), f"split res {M}x{K}x{N}")
            y, acc, _ = mq.qlinear_w4a8(dev(x), pw, want_acc=True, residual=dev(r))
            ry, racc, _ = orc.linear_a8(x, oc, os_, oz, residual=r)
            assert np.array_equal(host(acc), racc)
            assert_close16(host(y), ry, f"split res a8 {M}x{K}x{N}")
    finally:
        mq.tune_force_splits(-1)


def test_feed_forward_output_linear_adds_the_skip_connection(mq, orc):
    """The linear on 8-bit codes (second half of a feed-forward) with the block's skip connection as residual."""
    M, K, N = 300, 1280, 320
    rng = np.random.default_rng(85)
    codes = rng.integers(0, 256, (M, K)).astype(np.uint8)
    act = (np.float32(0.031), 117)
    w = si.weights_f16(85, "rc/w", N, K)
    b = si.bias_f16(85, "rc/b", N)
    r = si.normal(85, "rc/r", (M, N)).astype(np.float16)
    d_act = (dev(np.array([act[0]], np.float32)), dev(np.array([act[1]], np.int32)))
    for bits, sym in ((8, True), (4, False)):
        pw, oc, os_, oz = make_weight(mq, orc, w, bits, sym)
        for tile in (-1, 1, 2):
            mq.tune_force_tile(tile)
            try:
                y, acc = mq.qlinear_a8_codes(dev(a8_layout(codes)), K, d_act, pw, bias=dev(b), want_acc=True,
                                             residual=dev(r))
            finally:
                mq.tune_force_tile(-1)
            ry, racc = orc.linear_a8_codes(codes, act, oc, os_, oz, w_signed=sym, bias=b, residual=r)
            assert np.array_equal(host(acc), racc)
            assert_close16(host(y), ry, f"codes + residual b{bits} tile{tile}")


@pytest.mark.parametrize("tile", (-1, 0, 1, 2, 5))
def test_conv_residual_and_split_shortcut(mq, orc, tile):
    """Residual block tail (conv + skip), and the first convolution of an up block whose input is the channel
    concatenation [trunk | shortcut], run as two convolutions with separate quantisation parameters (Sec. 4.1): the
    second adds the first one's output, on the weight-only and on the 8-bit-activation path."""
    mq.tune_force_tile(tile)
    try:
        for (B, H, W, C1, C2, N) in ((2, 8, 8, 128, 64, 64), (1, 16, 16, 320, 64, 320), (2, 5, 7, 64, 64, 40)):
            if tile == 0 and B * H * W * N > 200000:
                continue
            xa = si.activations_f16(86, f"sp/xa{B}x{H}x{C1}", B * H * W, C1).reshape(B, H, W, C1)
            xb = (3.0 * si.activations_f16(86, f"sp/xb{B}x{H}x{C2}", B * H * W, C2).astype(np.float32)).astype(
                np.float16).reshape(B, H, W, C2)          # the shortcut has another range than the trunk
            b = si.bias_f16(86, f"sp/b{N}", N)
            what = f"tile{tile} {B}x{H}x{W} {C1}+{C2}->{N}"
            pa, ca, sa, za, ta = conv_weight(mq, orc, 86, N, C1, 4)
            pb, cb, sb, zb, tb = conv_weight(mq, orc, 87, N, C2, 8)
            first = mq.conv3x3_w_only(dev(xa), pa, dev(b))
            second = mq.conv3x3_w_only(dev(xb), pb, None, residual=first)
            rfirst = orc.conv3x3_w_only(xa, ca, sa, za, b)
            rsecond = orc.conv3x3_w_only(xb, cb, sb, zb, None, residual=rfirst.reshape(B, H, W, N))
            assert_close16(host(second).reshape(-1, N), rsecond, "split weight-only " + what)
            mq.conv3x3_w_only(dev(xb), pb, None, out=first, residual=first)     # in place
            assert_close16(host(first).reshape(-1, N), rsecond, "split weight-only in place " + what)
            if tile != 0:
                y1, acc1, _ = mq.conv3x3_a8(dev(xa), pa, ta, bias=dev(b), want_acc=True)
                y2, acc2, _ = mq.conv3x3_a8(dev(xb), pb, tb, want_acc=True, residual=y1)
                r1, racc1, _ = orc.conv3x3_a8(xa, ca, sa, za, bias=b)
                r2, racc2, _ = orc.conv3x3_a8(xb, cb, sb, zb, residual=r1.reshape(B, H, W, N))
                assert np.array_equal(host(acc1), racc1) and np.array_equal(host(acc2), racc2)
                assert_close16(host(y2).reshape(-1, N), r2, "split a8 " + what)
    finally:
        mq.tune_force_tile(-1)


# ----------------------------------------------------------------------------------------------- BOS-aware K/V

@pytest.mark.parametrize("N", (640, 1280))
@pytest.mark.parametrize("bits,sym", [(8, True), (4, False), (2, False)])
def test_bos_aware_kv_projection(mq, orc, N, bits, sym):
    B, T, K = 8, 77, 2048
    ctx = si.bos_context_f16(0, "c4/ctx", B, T, K)
    w = si.weights_f16(0, f"c4/w{N}", N, K)
    pw, oc, os_, oz = make_weight(mq, orc, w, bits, sym)
    # run-time fp16 BOS row
    y, (s_out, z_out) = mq.bos_aware_kv_proj(dev(ctx), pw, w_f16=dev(w), want_act=True)
    ry, (rs, rz) = orc.bos_aware_kv_proj(ctx, oc, os_, oz, w_signed=sym, w_f16=w)
    assert host(s_out)[0] == rs and host(z_out)[0] == rz
    yh = host(y)
    assert_close16(yh[:, 1:], ry[:, 1:], "body rows")
    assert_close16(yh[:, 0], ry[:, 0], "BOS rows")
    # pre-computed BOS vector: copied verbatim
    bos_out = orc.linear_fp(ctx[0, 0:1], w)[0]
    y2, _ = mq.bos_aware_kv_proj(dev(ctx), pw, bos_out=dev(bos_out.view(np.float16)))
    y2h = host(y2)
    assert np.array_equal(y2h[:, 0].view(np.uint16), np.broadcast_to(bos_out, (B, N)))
    assert np.array_equal(y2h[:, 1:], yh[:, 1:])
    # comparator: all rows through the 8-bit path
    y3, (s3, _) = mq.bos_aware_kv_proj(dev(ctx), pw, naive_all_rows=True, want_act=True)
    ry3, (rs3, _) = orc.bos_aware_kv_proj(ctx, oc, os_, oz, w_signed=sym, naive_all_rows=True)
    assert host(s3)[0] == rs3 and rs3 > 5 * rs
    assert_close16(host(y3), ry3, "naive all rows")


@pytest.mark.parametrize("N", (640, 1280))
@pytest.mark.parametrize("bits,sym", [(8, True), (4, False)])
def test_bos_aware_kv_projection_static_parameters_and_bias(mq, orc, N, bits, sym):
    """Eight prompts at full size with calibrated (static) activation parameters and a bias: the parameters are the given
    ones (narrower than the data, so body codes saturate), the BOS rows stay in fp16 and carry the bias too; the naive
    comparator under the same static parameters; the pre-computed BOS vector with a bias on the body rows."""
    B, T, K = 8, 77, 2048
    ctx = si.bos_context_f16(0, "c4/ctx", B, T, K)
    w = si.weights_f16(0, f"c4/w{N}", N, K)
    b = si.bias_f16(0, f"c4/b{N}", N)
    pw, oc, os_, oz = make_weight(mq, orc, w, bits, sym)
    act = (np.float32(0.03), 120)
    d_act = (dev(np.array([act[0]], np.float32)), dev(np.array([act[1]], np.int32)))
    y, (s_out, z_out) = mq.bos_aware_kv_proj(dev(ctx), pw, w_f16=dev(w), act=d_act, bias=dev(b), want_act=True)
    ry, (rs, rz) = orc.bos_aware_kv_proj(ctx, oc, os_, oz, w_signed=sym, w_f16=w, act=act, bias=b)
    assert host(s_out)[0] == act[0] == rs and host(z_out)[0] == act[1] == rz
    yh = host(y)
    assert_close16(yh[:, 1:], ry[:, 1:], "static + bias, body rows")
    assert_close16(yh[:, 0], ry[:, 0], "static + bias, BOS rows")
    # dynamic parameters with a bias at full size
    y, (s_out, z_out) = mq.bos_aware_kv_proj(dev(ctx), pw, w_f16=dev(w), bias=dev(b), want_act=True)
    ry, (rs, rz) = orc.bos_aware_kv_proj(ctx, oc, os_, oz, w_signed=sym, w_f16=w, bias=b)
    assert host(s_out)[0] == rs and host(z_out)[0] == rz
    assert_close16(host(y)[:, 1:], ry[:, 1:], "dynamic + bias, body rows")
    assert_close16(host(y)[:, 0], ry[:, 0], "dynamic + bias, BOS rows")
    # pre-computed BOS output (it already holds its bias), static parameters, bias on the body rows
    bos_out = orc.linear_fp(ctx[0, 0:1], w, b)[0]
    y2, _ = mq.bos_aware_kv_proj(dev(ctx), pw, bos_out=dev(bos_out.view(np.float16)), act=d_act, bias=dev(b))
    ry2, _ = orc.bos_aware_kv_proj(ctx, oc, os_, oz, w_signed=sym, bos_out=bos_out, act=act, bias=b)
    assert np.array_equal(host(y2)[:, 0].view(np.uint16), np.broadcast_to(bos_out, (B, N)))
    assert_close16(host(y2)[:, 1:], ry2[:, 1:], "pre-computed + static + bias, body rows")
    # comparator under the same static parameters
    y3, _ = mq.bos_aware_kv_proj(dev(ctx), pw, act=d_act, bias=dev(b), naive_all_rows=True)
    ry3, _ = orc.bos_aware_kv_proj(ctx, oc, os_, oz, w_signed=sym, act=act, bias=b, naive_all_rows=True)
    assert_close16(host(y3), ry3, "naive all rows, static + bias")


def test_bos_distinct_rows_small_and_degenerate(mq, orc):
    for (B, T, K, N) in ((3, 9, 128, 40), (1, 2, 64, 32), (2, 1, 64, 32)):
        ctx = si.bos_context_f16(3, f"bos/{B}{T}", B, T, K, n_outlier=4, shared_bos=False)
        w = si.weights_f16(3, f"bos/w{N}", N, K)
        b = si.bias_f16(3, f"bos/b{N}", N)
        pw, oc, os_, oz = make_weight(mq, orc, w, 8, True)
        y, _ = mq.bos_aware_kv_proj(dev(ctx), pw, w_f16=dev(w), bias=dev(b))
        ry, _ = orc.bos_aware_kv_proj(ctx, oc, os_, oz, w_signed=True, w_f16=w, bias=b)
        assert_close16(host(y), ry, f"bos {B}x{T}")


# ----------------------------------------------------------------------------------------------- full-size sweep shapes

@pytest.mark.parametrize("K,N", [(640, 640), (640, 5120), (2560, 640)])
def test_sweep_640_level_shapes_sampled_rows(mq, orc, K, N):
    """M = 16384 (latent 128x128, batch 4), all three shapes of the level, in the launch configuration of the benchmark:
    weight-only at 2 and 4 bits and W4A8, oracle on 512 sampled rows."""
    M = 16384
    x = si.activations_f16(0, f"c5/x{K}", M, K, outlier_prob=0.01)
    w = si.weights_f16(0, f"c5/w{N}x{K}", N, K)
    b = si.bias_f16(0, f"c5/b{N}", N)
    rows = sample_rows(x, 512, K + N)
    xd = dev(x)
    for bits in (2, 4):
        pw, oc, os_, oz = make_weight(mq, orc, w, bits)
        y = host(mq.qlinear_w_only(xd, pw, dev(b)))
        assert_close16(y[rows], orc.linear_w_only(x, oc, os_, oz, b, rows=rows), f"c5 W{bits}A16 {K}->{N}")
        assert np.isfinite(y).all()
    y, acc, (s_out, z_out) = mq.qlinear_w4a8(xd, pw, bias=dev(b), want_acc=True, want_act=True)
    ry, racc, (rs, rz) = orc.linear_a8(x, oc, os_, oz, bias=b, rows=rows)
    assert host(s_out)[0] == rs and host(z_out)[0] == rz
    assert np.array_equal(host(acc)[rows], racc)
    assert_close16(host(y)[rows], ry, f"c5 W4A8 {K}->{N}")


@pytest.mark.parametrize("N", (640, 1280))
def test_sweep_kv_projection_four_prompts(mq, orc, N):
    """The cross-attention K/V call of the sweep as the benchmark launches it: four prompts (M = 4 * 77 = 308 rows, 304 of
    them quantised), W4A8 with the BOS rows in fp16, dynamic and static activation parameters, with a bias."""
    B, T, K = 4, 77, 2048
    ctx = si.bos_context_f16(0, "c5/ctx", B, T, K)
    w = si.weights_f16(0, f"c5/kvw{N}", N, K)
    b = si.bias_f16(0, f"c5/kvb{N}", N)
    pw, oc, os_, oz = make_weight(mq, orc, w, 4)
    y, (s_out, z_out) = mq.bos_aware_kv_proj(dev(ctx), pw, w_f16=dev(w), bias=dev(b), want_act=True)
    ry, (rs, rz) = orc.bos_aware_kv_proj(ctx, oc, os_, oz, w_f16=w, bias=b)
    assert host(s_out)[0] == rs and host(z_out)[0] == rz
    assert_close16(host(y)[:, 1:], ry[:, 1:], f"kv B=4 N={N} body rows")
    assert_close16(host(y)[:, 0], ry[:, 0], f"kv B=4 N={N} BOS rows")
    act = (np.float32(0.035), 131)
    d_act = (dev(np.array([act[0]], np.float32)), dev(np.array([act[1]], np.int32)))
    y, (s_out, z_out) = mq.bos_aware_kv_proj(dev(ctx), pw, w_f16=dev(w), bias=dev(b), act=d_act, want_act=True)
    ry, _ = orc.bos_aware_kv_proj(ctx, oc, os_, oz, w_f16=w, bias=b, act=act)
    assert host(s_out)[0] == act[0] and host(z_out)[0] == act[1]
    assert_close16(host(y)[:, 1:], ry[:, 1:], f"kv B=4 N={N} static, body rows")
    assert_close16(host(y)[:, 0], ry[:, 0], f"kv B=4 N={N} static, BOS rows")


@pytest.mark.parametrize("B,H,W,Cin,N,stride", [(4, 128, 128, 320, 320, 1), (4, 128, 128, 320, 320, 2), (4, 32, 32, 1280, 1280, 1)])
def test_conv_unet_sizes_sampled_pixels(mq, orc, B, H, W, Cin, N, stride):
    """The UNet's convolutions at latent 128x128, batch 4, in the launch configuration of the per-shape report (the
    library's own tile choice): oracle on sampled output pixels, corners and edges among them; W4A16 within tolerance,
    W4A8 accumulators bit-exact with the dynamic parameters of the whole input tensor."""
    x = si.activations_f16(90, f"cu/x{H}x{Cin}", B * H * W, Cin, outlier_prob=0.01).reshape(B, H, W, Cin)
    b = si.bias_f16(90, f"cu/b{N}", N)
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    Mo = B * Ho * Wo
    pix = np.unique(np.concatenate([[0, Wo - 1, (Ho - 1) * Wo, Ho * Wo - 1, Mo - 1, Mo - Wo, Ho * Wo, Ho * Wo + Wo - 1],
                                    np.random.default_rng(H + Cin + stride).integers(0, Mo, 40)]))
    pw, oc, os_, oz, tapsum = conv_weight(mq, orc, 90, N, Cin, 4)
    xd = dev(x)
    y = host(mq.conv3x3_w_only(xd, pw, dev(b), stride=stride)).reshape(-1, N)
    assert_close16(y[pix], orc.conv3x3_w_only(x, oc, os_, oz, b, pix=pix, stride=stride), "conv W4A16 full size")
    y, acc, got = mq.conv3x3_a8(xd, pw, tapsum, bias=dev(b), want_acc=True, want_act=True, stride=stride)
    ry, racc, ract = orc.conv3x3_a8(x, oc, os_, oz, bias=b, pix=pix, stride=stride)
    assert host(got[0])[0] == ract[0] and host(got[1])[0] == ract[1]
    assert np.array_equal(host(acc)[pix], racc)
    assert_close16(host(y).reshape(-1, N)[pix], ry, "conv W4A8 full size")


def test_stacked_layers_that_share_their_input(mq, orc):
    """q, k, v as one call: the concatenated packed buffers are the packed form of the stacked matrix (bit for bit),
    and one launch writes the three outputs side by side, equal to the three separate calls (int32 accumulators and,
    with the same dynamic activation parameters, every output bit)."""
    M, K, N = 300, 640, 320
    x = si.activations_f16(95, "st/x", M, K, outlier_prob=0.01)
    ws = [si.weights_f16(95, f"st/w{i}", N, K) for i in range(3)]
    for bits, sym in ((4, False), (8, True), (2, False), (3, False)):
        parts = [make_weight(mq, orc, w, bits, sym)[0] for w in ws]
        stacked = mq.stack_weights(parts)
        whole = make_weight(mq, orc, np.concatenate(ws, 0), bits, sym)[0]
        assert torch.equal(stacked.packed, whole.packed) and torch.equal(stacked.scale, whole.scale)
        assert torch.equal(stacked.zp, whole.zp) and torch.equal(stacked.colsum, whole.colsum)
        y = mq.qlinear_w_only(dev(x), stacked)
        for i, p in enumerate(parts):   # (the tile choice, and with it the order of the fp32 sums, may differ)
            yi = mq.qlinear_w_only(dev(x), p).float()
            assert (y[:, i * N:(i + 1) * N].float() - yi).abs().max() <= 2e-3 * yi.abs().max()
        if bits in (4, 8):
            fn = mq.qlinear_w4a8 if bits == 4 else mq.qlinear_w8a8
            y, acc, _ = fn(dev(x), stacked, want_acc=True)
            for i, p in enumerate(parts):
                yi, acci, _ = fn(dev(x), p, want_acc=True)
                assert torch.equal(acc[:, i * N:(i + 1) * N], acci) and torch.equal(y[:, i * N:(i + 1) * N], yi)


def test_side_streams_and_two_streams_at_once(mq, orc):
    """The library launches on the stream it is handed and keeps no state that two streams could trample: the results
    on a side stream, and on two streams that run different layers at the same time (each call with a workspace of its
    own), equal those of the default stream bit for bit."""
    xa = dev(si.activations_f16(96, "ss/xa", 64, 5120))
    wa, *_ = make_weight(mq, orc, si.weights_f16(96, "ss/wa", 1280, 5120), 4)
    xb = dev(si.activations_f16(96, "ss/xb", 2048, 1280, outlier_prob=0.01))
    wb, *_ = make_weight(mq, orc, si.weights_f16(96, "ss/wb", 640, 1280), 4)
    xc = dev(si.activations_f16(96, "ss/xc", 308, 2048))
    wc, *_ = make_weight(mq, orc, si.weights_f16(96, "ss/wc", 640, 2048), 8, True)

    def layer_a():
        return mq.qlinear_w_only(xa, wa)

    def layer_b():
        return mq.qlinear_w4a8(xb, wb)[0]

    def layer_c():
        return mq.qlinear_w8a8(xc, wc)[0]

    ref = [f().clone() for f in (layer_a, layer_b, layer_c)]
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    for f, r in zip((layer_a, layer_b, layer_c), ref):
        with torch.cuda.stream(s1):
            y = f()
        s1.synchronize()
        assert torch.equal(y, r), "side stream"
    for it in range(8):
        with torch.cuda.stream(s1):
            ya = [layer_a() for _ in range(3)]
            yc = layer_c()
        with torch.cuda.stream(s2):
            yb = [layer_b() for _ in range(3)]
            ya2 = layer_a()
        torch.cuda.synchronize()
        for y in ya + [ya2]:
            assert torch.equal(y, ref[0]), f"two streams, split reduction, round {it}"
        for y in yb:
            assert torch.equal(y, ref[1]), f"two streams, W4A8, round {it}"
        assert torch.equal(yc, ref[2]), f"two streams, W8A8, round {it}"


@pytest.mark.parametrize("tile", (-1, 2, 5))
def test_band_height_of_the_tile_walk_changes_no_result(mq, orc, tile):
    """The order in which workgroups take the output tiles (bands of row blocks, a ragged last band, bands higher than
    the problem) decides cache behaviour only: every output bit equals that of the row-by-row walk, and the int32
    accumulators equal the oracle's."""
    M, K, N = 1100, 320, 520            # 64-row tiles: 18 row blocks (ragged), 64x64 tiles: 9 column blocks
    x = si.activations_f16(97, "band/x", M, K, outlier_prob=0.01)
    w = si.weights_f16(97, "band/w", N, K)
    p4, oc, os_, oz = make_weight(mq, orc, w, 4)
    img = si.activations_f16(97, "band/img", 2 * 20 * 24, 64).reshape(2, 20, 24, 64)
    cw, *_, tapsum = conv_weight(mq, orc, 97, 96, 64, 4, False)
    _, racc, _ = orc.linear_a8(x, oc, os_, oz, w_signed=False)
    mq.tune_force_tile(tile)
    try:
        ref = None
        for band in (1, 2, 5, 7, 16, 1000):
            mq.tune_force_band(band)
            y = mq.qlinear_w_only(dev(x), p4)
            y8, acc, _ = mq.qlinear_w4a8(dev(x), p4, want_acc=True)
            yc = mq.conv3x3_w_only(dev(img), cw)
            yc8 = mq.conv3x3_a8(dev(img), cw, tapsum)[0]
            got = [t.clone() for t in (y, y8, acc, yc, yc8)]
            assert np.array_equal(host(acc), racc), f"band {band}"
            if ref is None:
                ref = got
            for a, b in zip(got, ref):
                assert torch.equal(a, b), f"band {band} tile {tile}"
    finally:
        mq.tune_force_band(0)
        mq.tune_force_tile(-1)


def test_one_prompt_through_many_stacked_projections(mq, orc):
    """One prompt's 77 text tokens through a stack of K/V projections wide enough for the 96-row tile that the library
    picks for a single row block of 65 to 96 rows over very many column tiles (here 257 of 256 channels; the reduction
    is kept short for the oracle's sake): weight-only, W4A8 (int32 accumulators bit-exact) and the BOS-aware call."""
    B, T, K, N = 1, 77, 128, 257 * 256
    ctx = si.bos_context_f16(98, "kvall/ctx", B, T, K, n_outlier=4)
    w = si.weights_f16(98, "kvall/w", N, K)
    b = si.bias_f16(98, "kvall/b", N)
    x = ctx.reshape(T, K)
    pw, oc, os_, oz = make_weight(mq, orc, w, 4)
    assert_close16(host(mq.qlinear_w_only(dev(x), pw, bias=dev(b))), orc.linear_w_only(x, oc, os_, oz, bias=b), "w4a16")
    y, acc, _ = mq.qlinear_w4a8(dev(x), pw, bias=dev(b), want_acc=True)
    ry, racc, _ = orc.linear_a8(x, oc, os_, oz, w_signed=False, bias=b)
    assert np.array_equal(host(acc), racc)
    assert_close16(host(y), ry, "w4a8")
    y, _ = mq.bos_aware_kv_proj(dev(ctx), pw, w_f16=dev(w), bias=dev(b))
    ry, _ = orc.bos_aware_kv_proj(ctx, oc, os_, oz, w_signed=False, w_f16=w, bias=b)
    assert_close16(host(y)[0], ry[0], "bos-aware")
    # (3 x 32 rows: the third slab holds rows 64..76 and 19 rows of padding that must not be stored)
    guard = torch.full((T + 8, N), 7.0, dtype=torch.float16, device="cuda")
    mq.qlinear_w_only(dev(x), pw, out=guard[:T])
    assert bool((guard[T:] == 7.0).all())


def test_microbenchmarks_of_the_machine_report_plausible_rates(mq):
    """The measured-peak columns of the per-shape report come from these kernels: every kind runs, and its rate lies
    between a tenth of the published peak and the published peak (int8 5.0 POP/s, fp16 2.5 PFLOP/s, HBM 8 TB/s); four
    vector instructions behind every MFMA cost less than eight."""
    buf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    pk = mq.machine_peaks(buf)
    assert 500.0 < pk["int8_TOPs"] <= 5000.0
    assert 250.0 < pk["f16_TFLOPs"] <= 2500.0
    assert 800.0 < pk["read_GBps"] <= 8000.0
    assert pk["lds_read_TBps"] > 10.0 and pk["l2_to_lds_TBps"] > 3.0
    assert 0.5 <= pk["serial_share_same_wave"] <= 1.05 and 0.5 <= pk["serial_share_two_waves"] <= 1.05
    assert pk["four_valu_per_mfma_ms"] < pk["same_wave_ms"]

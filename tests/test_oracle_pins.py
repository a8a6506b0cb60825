"""Pins for the CPU oracle: hand-worked vectors, closed forms, invariants, brute force and
independent library routines.  None of these re-type the oracle's own code: the numpy
re-derivations below use different primitives (exact rationals, float64 matmul, bit unpacking)."""
import os
from fractions import Fraction

import numpy as np
import pytest

import synth_inputs as si

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "quantizer_handworked.txt")
ALL_BITS = (2, 3, 4, 8)


def _golden_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            bits, vals, scale, zp, codes, packed = [p.strip() for p in line.split("|")]
            rows.append((int(bits), [float(v) for v in vals.split()], float(scale), int(zp),
                         [int(c) for c in codes.split()], bytes.fromhex(packed.replace(" ", ""))))
    return rows


# ----------------------------------------------------------------------------- 16-bit formats

def test_f16_decode_all_patterns(orc):
    bits = np.arange(65536, dtype=np.uint16)
    got = orc.f16_to_f64(bits)
    ref = bits.view(np.float16).astype(np.float64)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))


def test_f16_encode_matches_numpy_rne(orc):
    rng = np.random.default_rng(1)
    v = np.concatenate([
        rng.normal(0, 1, 20000), rng.normal(0, 300, 20000), rng.normal(0, 1e-5, 20000),
        rng.normal(0, 1e-7, 5000), np.array([0.0, -0.0, 65504, 65519.99, 65520, 1e9, -1e9, 2.0 ** -24, 2.0 ** -25,
                                             2.0 ** -25 * 1.0000001, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -26]),
    ])
    # exact ties between neighbouring halfs: midpoints of consecutive finite patterns
    pats = np.arange(0, 0x7BFF, dtype=np.uint16)
    lo = pats.view(np.float16).astype(np.float64)
    hi = (pats + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    v = np.concatenate([v, (lo + hi) / 2, -(lo + hi) / 2])
    got = orc.f64_to_f16(v)
    with np.errstate(over="ignore"):
        ref = v.astype(np.float16).view(np.uint16)
    assert np.array_equal(got, ref)


def test_bf16_roundtrip_and_rne(orc):
    import torch
    rng = np.random.default_rng(2)
    f = np.concatenate([rng.normal(0, 1, 20000), rng.normal(0, 1e4, 5000), rng.normal(0, 1e-30, 2000)]).astype(
        np.float32)
    got = orc.f64_to_f16(f.astype(np.float64), orc.BF16)
    ref = torch.from_numpy(f).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, ref)
    back = orc.f16_to_f64(got, orc.BF16)
    ref_back = torch.from_numpy(ref.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(back, ref_back)


# ----------------------------------------------------------------------------- quantiser

@pytest.mark.parametrize("row", _golden_rows(), ids=lambda r: f"b{r[0]}")
def test_quantizer_handworked(orc, row):
    bits, vals, scale, zp, codes, packed = row
    w = np.array([vals], np.float16)
    assert np.array_equal(w.astype(np.float64)[0], vals), "fixture values must be exact in fp16"
    c, s, z = orc.quantize_weights(w, bits)
    assert s[0] == np.float32(scale) and z[0] == zp
    assert c[0].tolist() == codes
    if (len(codes) * bits) % 8 == 0:
        assert bytes(orc.pack_weights(c, bits)[0]) == packed


def _quant_exact_reference(vals_f16, bits):
    """Independent derivation: scale and reciprocal as correctly rounded fp32 values obtained through exact
    rational arithmetic, code from the exactly rounded fp32 product.  Returns codes, scale, zp and a mask of
    inputs whose exact product sits close to a rounding tie (where the reading 'multiply by reciprocal' and
    the reading 'divide' could differ)."""
    def rnd32(fr: Fraction) -> np.float32:
        # correctly rounded fp32 of an exact rational: float(Fraction) is correctly rounded to double;
        # double->single double rounding is avoided by checking the two neighbouring singles exactly.
        d = np.float32(float(fr))
        cands = [np.nextafter(d, np.float32(-np.inf)), d, np.nextafter(d, np.float32(np.inf))]
        best = min(cands, key=lambda c: (abs(Fraction(float(c)) - fr), int(np.float32(c).view(np.uint32)) & 1))
        return np.float32(best)

    qmax = (1 << bits) - 1
    v = [Fraction(float(x)) for x in vals_f16]
    lo, hi = min(min(v), Fraction(0)), max(max(v), Fraction(0))
    if hi == lo:
        s = np.float32(1.0)
    else:
        s = rnd32(Fraction(float(rnd32(hi - lo))) / qmax)
    inv = rnd32(Fraction(1) / Fraction(float(s)))

    def rne(fr: Fraction) -> int:
        fl = fr.numerator // fr.denominator
        rem = fr - fl
        if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
            return fl + 1
        return fl

    z = min(max(rne(Fraction(float(rnd32(-lo * Fraction(float(inv)))))), 0), qmax)
    codes, near_tie = [], []
    for x in v:
        p = Fraction(float(rnd32(x * Fraction(float(inv)))))
        codes.append(min(max(rne(p) + z, 0), qmax))
        frac = (x / Fraction(float(s))) % 1
        near_tie.append(abs(frac - Fraction(1, 2)) < Fraction(1, 10 ** 6))
    return codes, s, z, near_tie


@pytest.mark.parametrize("bits", ALL_BITS)
def test_quantizer_bruteforce_exact_rational(orc, bits):
    rng = np.random.default_rng(10 + bits)
    for trial in range(12):
        K = int(rng.integers(4, 64))
        w = (rng.normal(0, 0.02 if trial % 2 else 1.0, (1, K))).astype(np.float16)
        c, s, z = orc.quantize_weights(w, bits)
        rc, rs, rz, _ = _quant_exact_reference(w[0], bits)
        assert s[0] == rs and z[0] == rz
        assert c[0].tolist() == rc


@pytest.mark.parametrize("bits", ALL_BITS)
def test_quantizer_invariants(orc, bits):
    qmax = (1 << bits) - 1
    w = si.weights_f16(3, f"pin/w{bits}", 64, 320)
    w[5] = 0  # constant-zero row
    w[6] = np.abs(w[6])  # all non-negative: lo is forced to 0
    w[7] = -np.abs(w[7])  # all non-positive
    c, s, z = orc.quantize_weights(w, bits)
    wd = w.astype(np.float64)
    assert c.max() <= qmax and z.min() >= 0 and z.max() <= qmax
    assert s[5] == 1.0 and z[5] == 0 and not c[5].any()
    assert z[6] == 0 and z[7] == qmax
    what = s[:, None].astype(np.float64) * (c.astype(np.int64) - z[:, None])
    # endpoints map to the extreme codes, every element is within half a step (plus fp32 slack)
    for n in range(64):
        if n == 5:
            continue
        lo, hi = min(wd[n].min(), 0), max(wd[n].max(), 0)
        assert c[n, np.argmin(wd[n])] == (0 if wd[n].min() <= 0 else c[n, np.argmin(wd[n])])
        assert c[n, np.argmax(wd[n])] == (qmax if wd[n].max() >= 0 else c[n, np.argmax(wd[n])])
        assert abs(float(s[n]) * qmax - (hi - lo)) <= 1e-6 * (hi - lo)
        # the zero point is rounded, so the grid is shifted by up to half a step: error <= one step at the ends,
        # and <= half a step wherever the code was not clamped
        err = np.abs(what[n] - wd[n])
        interior = (c[n] > 0) & (c[n] < qmax)
        assert err[interior].max(initial=0) <= 0.5 * s[n] * (1 + 1e-5)
        assert err.max() <= 1.0 * s[n] * (1 + 1e-5)


@pytest.mark.parametrize("bits", ALL_BITS)
def test_round_trip_of_every_code(orc, bits):
    """quantise(dequantise(q)) == q for every code, on grids that are exact in fp16 (power-of-two scales)."""
    qmax = (1 << bits) - 1
    for scale in (1.0, 0.5, 0.0625, 4.0):
        for z in sorted({0, 1, qmax // 2, qmax - 1, qmax}):
            grid = ((np.arange(qmax + 1) - z) * scale).astype(np.float16)[None]
            c, s, zz = orc.quantize_weights(grid, bits)
            assert s[0] == np.float32(scale) and zz[0] == z
            assert c[0].tolist() == list(range(qmax + 1))


@pytest.mark.parametrize("bits", (4, 8))
def test_symmetric_quantizer(orc, bits):
    Q = (1 << (bits - 1)) - 1
    w = si.weights_f16(4, f"pin/sym{bits}", 32, 320)
    w[3] = 0
    c, s, z = orc.quantize_weights(w, bits, symmetric=True)
    ci = c.view(np.int8).astype(np.int64)
    assert not z.any() and s[3] == 1.0 and not ci[3].any()
    assert ci.max() <= Q and ci.min() >= -Q
    wd = w.astype(np.float64)
    for n in range(32):
        if n == 3:
            continue
        amax = np.abs(wd[n]).max()
        assert s[n] == np.float32(np.float32(amax) / np.float32(Q))
        k = int(np.argmax(np.abs(wd[n])))
        assert ci[n, k] == (Q if wd[n, k] > 0 else -Q)
        assert np.abs(ci[n] * np.float64(s[n]) - wd[n]).max() <= 0.5 * s[n] * (1 + 1e-5)
    # antisymmetry under x -> -x
    c2, s2, _ = orc.quantize_weights((-w).astype(np.float16), bits, symmetric=True)
    assert np.array_equal(s2, s) and np.array_equal(c2.view(np.int8).astype(np.int64), -ci)
    # textbook formula through numpy fp32 primitives
    inv = np.float32(1.0) / s
    ref = np.clip(np.rint(w.astype(np.float32) * inv[:, None]), -Q, Q).astype(np.int64)
    assert np.array_equal(ci, ref)


def test_activation_quantizer_is_textbook_affine(orc):
    x = si.activations_f16(5, "pin/x", 96, 320, outlier_prob=0.01)
    s, z = orc.act_params(x)
    xf = x.astype(np.float32)
    lo, hi = min(xf.min(), np.float32(0)), max(xf.max(), np.float32(0))
    s_ref = np.float32(hi - lo) / np.float32(255)
    inv = np.float32(1) / s_ref
    z_ref = int(np.clip(np.rint(-lo * inv), 0, 255))
    assert s == s_ref and z == z_ref
    q = orc.act_quantize(x, s, z)
    q_ref = np.clip(np.rint(xf * inv).astype(np.int64) + z_ref, 0, 255)
    assert np.array_equal(q, q_ref)
    assert q.min() == 0 and q.max() == 255
    # static parameters narrower than the data: saturation, no wrap-around
    q2 = orc.act_quantize(x, np.float32(0.01), 100)
    q2_ref = np.clip(np.rint(xf * (np.float32(1) / np.float32(0.01))).astype(np.int64) + 100, 0, 255)
    assert np.array_equal(q2, q2_ref)


# ----------------------------------------------------------------------------- packing

def _pack_reference(codes, bits):
    """Independent packer: explode every code into its bits (LSB first), concatenate per row, regroup into
    bytes LSB first, all through numpy's bit unpack/pack."""
    N, K = codes.shape
    b = np.unpackbits(codes[:, :, None], axis=2, bitorder="little")[:, :, :bits]
    return np.packbits(b.reshape(N, K * bits), axis=1, bitorder="little")


@pytest.mark.parametrize("bits", ALL_BITS)
@pytest.mark.parametrize("K", (32, 64, 320, 5120))
def test_pack_roundtrip_and_layout(orc, bits, K):
    rng = np.random.default_rng(100 * bits + K)
    codes = rng.integers(0, 1 << bits, (7, K)).astype(np.uint8)
    p = orc.pack_weights(codes, bits)
    assert p.shape == (7, K * bits // 8)
    assert np.array_equal(p, _pack_reference(codes, bits))
    assert np.array_equal(orc.unpack_weights(p, K, bits), codes)


def test_pack_nibble_and_crumb_positions(orc):
    # 4 bit: even k in the low nibble; 2 bit: k mod 4 == 0 in bits 1:0
    assert orc.pack_weights(np.array([[0x3, 0xA]], np.uint8), 4)[0, 0] == 0xA3
    assert orc.pack_weights(np.array([[1, 0, 0, 0]], np.uint8), 2)[0, 0] == 0x01
    assert orc.pack_weights(np.array([[0, 0, 0, 2]], np.uint8), 2)[0, 0] == 0x80
    with pytest.raises(ValueError):
        orc.pack_weights(np.zeros((1, 5), np.uint8), 3)


# ----------------------------------------------------------------------------- weight-only linear

def _random_quantised_layer(orc, seed, M, K, N, bits, symmetric=False, outliers=0.0):
    x = si.activations_f16(seed, "pin/lx", M, K, outlier_prob=outliers)
    w = si.weights_f16(seed, "pin/lw", N, K)
    b = si.bias_f16(seed, "pin/lb", N)
    c, s, z = orc.quantize_weights(w, bits, symmetric=symmetric)
    return x, w, b, c, s, z


@pytest.mark.parametrize("bits", ALL_BITS)
def test_w_only_equals_float64_matmul_on_dequantised_weights(orc, bits):
    x, w, b, c, s, z = _random_quantised_layer(orc, 20 + bits, 33, 128, 48, bits)
    y = orc.linear_w_only(x, c, s, z, b).view(np.float16)
    what = s.astype(np.float64)[:, None] * (c.astype(np.float64) - z[:, None])
    ref = x.astype(np.float64) @ what.T + b.astype(np.float64)
    ref16 = ref.astype(np.float16)
    # different summation order: allow one fp16 ulp on a handful of borderline sums
    ulp = np.abs(y.astype(np.float64) - ref16.astype(np.float64)) / np.maximum(np.spacing(np.abs(ref16)).astype(
        np.float64), 1e-30)
    assert ulp.max() <= 1.0 and (ulp > 0).mean() < 0.01
    # rows subset == the same rows of the full result
    rows = [0, 7, 32]
    assert np.array_equal(orc.linear_w_only(x, c, s, z, b, rows=rows).view(np.float16), y[rows])
    # the quantiser's error bound carried through the sum (interior codes: half a step per weight)
    yfp = x.astype(np.float64) @ w.astype(np.float64).T + b.astype(np.float64)
    bound = np.abs(x.astype(np.float64)).sum(1)[:, None] * s[None, :] * 1.0 + 1e-2
    assert (np.abs(ref - yfp) <= bound).all()


def test_w_only_bruteforce_triple_loop(orc):
    rng = np.random.default_rng(3)
    M, K, N = 3, 8, 4
    x = rng.normal(0, 1, (M, K)).astype(np.float16)
    c = rng.integers(0, 16, (N, K)).astype(np.uint8)
    s = rng.uniform(0.01, 0.1, N).astype(np.float32)
    z = rng.integers(0, 16, N).astype(np.int32)
    b = rng.normal(0, 0.1, N).astype(np.float16)
    y = orc.linear_w_only(x, c, s, z, b).view(np.float16)
    for m in range(M):
        for n in range(N):
            acc = Fraction(0)
            for k in range(K):
                acc += Fraction(float(x[m, k])) * Fraction(float(s[n])) * (int(c[n, k]) - int(z[n]))
            acc += Fraction(float(b[n]))
            assert y[m, n] == np.float16(float(acc)), (m, n)


def test_w_only_integer_special_case_is_exact(orc):
    rng = np.random.default_rng(4)
    x = rng.integers(-8, 9, (16, 64)).astype(np.float16)
    c = rng.integers(0, 256, (24, 64)).astype(np.uint8)
    y = orc.linear_w_only(x, c, np.ones(24, np.float32), np.zeros(24, np.int32), None).view(np.float16)
    ref = x.astype(np.int64) @ c.astype(np.int64).T
    assert np.abs(ref).max() < 2 ** 11 * 32
    assert np.array_equal(y, ref.astype(np.float16))


def test_w_only_transposed_operand_would_fail(orc):
    """N != K and asymmetric content: a transposed weight index cannot produce the same numbers."""
    x, w, b, c, s, z = _random_quantised_layer(orc, 31, 5, 64, 96, 4)
    y = orc.linear_w_only(x, c, s, z, None).view(np.float16).astype(np.float64)
    what = s.astype(np.float64)[:, None] * (c.astype(np.float64) - z[:, None])
    assert y.shape == (5, 96)
    assert np.allclose(y, x.astype(np.float64) @ what.T, rtol=2e-3, atol=1e-3)


def test_fp_linear_exact_rationals_and_integer_case(orc):
    """The unquantised 16-bit linear (layers kept at FP16; also the BOS row): brute force in exact rationals on a tiny
    case (N != K, so a transposed weight index cannot pass), an integer case that is exact, and a float64 matmul."""
    rng = np.random.default_rng(6)
    M, K, N = 3, 8, 5
    x = rng.normal(0, 1, (M, K)).astype(np.float16)
    w = rng.normal(0, 0.5, (N, K)).astype(np.float16)
    b = rng.normal(0, 0.1, N).astype(np.float16)
    y = orc.linear_fp(x, w, b).view(np.float16)
    for m in range(M):
        for n in range(N):
            acc = sum((Fraction(float(x[m, k])) * Fraction(float(w[n, k])) for k in range(K)), Fraction(float(b[n])))
            assert y[m, n] == np.float16(float(acc)), (m, n)
    xi = rng.integers(-8, 9, (16, 64)).astype(np.float16)
    wi = rng.integers(-15, 16, (24, 64)).astype(np.float16)
    assert np.array_equal(orc.linear_fp(xi, wi).view(np.float16), (xi.astype(np.int64) @ wi.astype(np.int64).T).astype(np.float16))
    x = rng.normal(0, 1, (33, 128)).astype(np.float16)
    w = rng.normal(0, 0.02, (48, 128)).astype(np.float16)
    y = orc.linear_fp(x, w).view(np.float16)
    ref16 = (x.astype(np.float64) @ w.astype(np.float64).T).astype(np.float16)
    ulp = np.abs(y.astype(np.float64) - ref16.astype(np.float64)) / np.spacing(np.abs(ref16)).astype(np.float64)
    assert ulp.max() <= 1.0 and (ulp > 0).mean() < 0.01


def test_w_only_bf16(orc):
    import torch
    rng = np.random.default_rng(5)
    xb = torch.from_numpy(rng.normal(0, 1, (9, 64)).astype(np.float32)).to(torch.bfloat16)
    x_bits = xb.view(torch.int16).numpy().view(np.uint16)
    c = rng.integers(0, 16, (12, 64)).astype(np.uint8)
    s = rng.uniform(0.01, 0.1, 12).astype(np.float32)
    z = rng.integers(0, 16, 12).astype(np.int32)
    y = orc.linear_w_only(x_bits, c, s, z, None, dtype=orc.BF16)
    what = s.astype(np.float64)[:, None] * (c.astype(np.float64) - z[:, None])
    ref = torch.from_numpy(xb.to(torch.float64).numpy() @ what.T).to(torch.float32).to(torch.bfloat16)
    got = torch.from_numpy(y.view(np.int16)).view(torch.bfloat16)
    assert (got.float() - ref.float()).abs().max() <= 2 ** -7 * ref.float().abs().max()


# ----------------------------------------------------------------------------- 8-bit activation linear

@pytest.mark.parametrize("bits,symmetric", [(8, True), (8, False), (4, False)])
def test_a8_closed_form_and_int64_bruteforce(orc, bits, symmetric):
    x, w, b, c, s, z = _random_quantised_layer(orc, 40 + bits + symmetric, 37, 192, 40, bits, symmetric, 0.01)
    y, acc, (sx, zx) = orc.linear_a8(x, c, s, z, w_signed=symmetric, bias=b)
    assert (sx, zx) == orc.act_params(x)
    qx = orc.act_quantize(x, sx, zx).astype(np.int64)
    qw = (c.view(np.int8) if symmetric else c).astype(np.int64)
    K = x.shape[1]
    # closed form: raw code product minus the three zero-point terms
    raw = qx @ qw.T
    closed = raw - zx * qw.sum(1)[None, :] - z.astype(np.int64)[None, :] * qx.sum(1)[:, None] + K * zx * z.astype(
        np.int64)[None, :]
    assert np.array_equal(acc.astype(np.int64), closed)
    assert np.array_equal(orc.code_rowsum(c, signed=symmetric).astype(np.int64), qw.sum(1))
    # output: ACC * s_x * s_w + bias in float64, one rounding
    ref = (closed.astype(np.float64) * (np.float64(sx) * s.astype(np.float64))[None, :] + b.astype(
        np.float64)).astype(np.float16)
    assert np.array_equal(y.view(np.float16), ref)
    # consistency with the weight-only definition applied to dequantised activations
    xhat = (qx - zx).astype(np.float64) * np.float64(sx)
    what = s.astype(np.float64)[:, None] * (qw - z[:, None]).astype(np.float64)
    ref2 = xhat @ what.T + b.astype(np.float64)
    assert np.allclose(y.view(np.float16).astype(np.float64), ref2, rtol=1.5e-3, atol=1e-4)
    # and it approximates the unquantised layer
    yfp = x.astype(np.float64) @ w.astype(np.float64).T + b.astype(np.float64)
    rel = np.linalg.norm(ref2 - yfp) / np.linalg.norm(yfp)
    assert rel < (0.05 if bits == 8 else 0.2)


def test_a8_static_params_and_row_subset(orc):
    x, w, b, c, s, z = _random_quantised_layer(orc, 50, 21, 64, 16, 4)
    y, acc, act = orc.linear_a8(x, c, s, z, act=(np.float32(0.05), 120), bias=None)
    assert act == (np.float32(0.05), 120)
    qx = orc.act_quantize(x, np.float32(0.05), 120).astype(np.int64)
    ref = (qx - 120) @ (c.astype(np.int64) - z[:, None]).T
    assert np.array_equal(acc, ref)
    # dynamic parameters always come from ALL rows, even when only some rows are evaluated
    yd, accd, actd = orc.linear_a8(x, c, s, z)
    ys, accs, acts = orc.linear_a8(x, c, s, z, rows=[20, 3])
    assert acts == actd and np.array_equal(accs, accd[[20, 3]]) and np.array_equal(ys, yd[[20, 3]])


def test_a8_overflow_is_reported(orc):
    K = 40000  # 255 * 255 * K exceeds int32
    x = np.full((1, K), 1.0, np.float16)
    x[0, 0] = 0
    c = np.full((1, K), 255, np.uint8)
    with pytest.raises(RuntimeError):
        orc.linear_a8(x, c, np.ones(1, np.float32), np.zeros(1, np.int32))


# ----------------------------------------------------------------------------- BOS-aware K/V projection

def _bos_case(orc, seed, B=3, T=9, K=128, N=40, shared=True):
    ctx = si.bos_context_f16(seed, "pin/ctx", B, T, K, n_outlier=4, shared_bos=shared)
    w = si.weights_f16(seed, "pin/wk", N, K)
    c, s, z = orc.quantize_weights(w, 8, symmetric=True)
    return ctx, w, c, s, z


def test_bos_row_is_fp16_linear_and_body_is_a8_without_the_row(orc):
    ctx, w, c, s, z = _bos_case(orc, 60, shared=False)
    B, T, K = ctx.shape
    y, act = orc.bos_aware_kv_proj(ctx, c, s, z, w_signed=True, w_f16=w)
    # token 0: plain floating-point linear with the unquantised weights (float64 matmul, one rounding)
    ref0 = (ctx[:, 0, :].astype(np.float64) @ w.astype(np.float64).T).astype(np.float16)
    assert np.array_equal(y[:, 0, :].view(np.float16), ref0)
    # tokens 1..: the 8-bit path run on the tensor with the BOS rows deleted
    body = np.ascontiguousarray(ctx[:, 1:, :]).reshape(B * (T - 1), K)
    yb, _, actb = orc.linear_a8(body, c, s, z, w_signed=True)
    assert act == actb
    assert np.array_equal(y[:, 1:, :].reshape(B * (T - 1), -1), yb)
    # the activation range excludes the outlier row
    assert act == orc.act_params(body)
    assert float(act[0]) * 255 < 0.5 * float(np.abs(ctx[:, 0, :].astype(np.float64)).max())


def test_bos_precomputed_equals_runtime_when_bos_is_shared(orc):
    ctx, w, c, s, z = _bos_case(orc, 61, shared=True)
    y_rt, _ = orc.bos_aware_kv_proj(ctx, c, s, z, w_signed=True, w_f16=w)
    bos_out = orc.linear_fp(ctx[0, 0:1, :], w)[0]
    y_pc, _ = orc.bos_aware_kv_proj(ctx, c, s, z, w_signed=True, bos_out=bos_out)
    assert np.array_equal(y_rt, y_pc)
    with pytest.raises(RuntimeError):
        orc.bos_aware_kv_proj(ctx, c, s, z, w_signed=True)  # neither source for the BOS row
    with pytest.raises(RuntimeError):
        orc.bos_aware_kv_proj(ctx, c, s, z, w_signed=True, w_f16=w, bos_out=bos_out)  # both


def test_bos_aware_beats_naive_all_row_quantisation(orc):
    """Direction fixed by Sec. 3.1: with the outlier row inside the 8-bit range most other values collapse
    towards the zero point; removing it shrinks the scale and the error on the remaining tokens."""
    ctx = si.bos_context_f16(62, "pin/ctx2", 4, 77, 256, n_outlier=16, gain=60.0)
    w = si.weights_f16(62, "pin/wk2", 48, 256)
    c, s, z = orc.quantize_weights(w, 8, symmetric=True)
    y_aware, act_a = orc.bos_aware_kv_proj(ctx, c, s, z, w_signed=True, w_f16=w)
    y_naive, act_n = orc.bos_aware_kv_proj(ctx, c, s, z, w_signed=True, naive_all_rows=True)
    assert float(act_n[0]) > 5 * float(act_a[0])
    ref = ctx.astype(np.float64) @ w.astype(np.float64).T
    ea = np.linalg.norm(y_aware.view(np.float16).astype(np.float64)[:, 1:] - ref[:, 1:])
    en = np.linalg.norm(y_naive.view(np.float16).astype(np.float64)[:, 1:] - ref[:, 1:])
    assert ea * 3 < en
    body_codes = orc.act_quantize(ctx[:, 1:, :].reshape(-1, 256), *act_n)
    assert len(np.unique(body_codes)) <= 24  # the body occupies a sliver of the 256 codes
    assert len(np.unique(orc.act_quantize(ctx[:, 1:, :].reshape(-1, 256), *act_a))) > 200


# ----------------------------------------------------------------------------- input recipes

def test_sweep_layer_table_matches_the_stated_workload():
    layers, mean = si.sweep_layers()
    assert len(layers) == 120
    assert abs(mean - 3.66) <= 0.01
    assert {l.bits for l in layers} <= {2, 3, 4, 8}
    assert sum(1 for l in layers if l.kind == "kv") == 24
    assert {l.M for l in layers if l.kind == "linear"} == {16384, 4096}
    # same seed, same table
    assert [l.bits for l in si.sweep_layers()[0]] == [l.bits for l in layers]


def test_generators_are_deterministic_and_have_the_stated_moments():
    a = si.activations_f16(0, "t/x", 512, 640, outlier_prob=0.01)
    assert np.array_equal(a, si.activations_f16(0, "t/x", 512, 640, outlier_prob=0.01))
    assert not np.array_equal(a, si.activations_f16(1, "t/x", 512, 640, outlier_prob=0.01))
    base = si.activations_f16(0, "t/x", 512, 640).astype(np.float64)
    assert abs(base.mean()) < 0.01 and abs(base.std() - 1) < 0.01
    changed = (a.astype(np.float64) != base).mean()
    assert 0.008 < changed < 0.012
    w = si.weights_f16(0, "t/w", 640, 640).astype(np.float64)
    assert abs(w.std() - 0.02) < 0.0005
    ctx = si.bos_context_f16(0, "t/ctx", 8, 77, 2048).astype(np.float64)
    assert np.array_equal(ctx[0, 0], ctx[7, 0])
    assert np.abs(ctx[:, 0]).max() > 5 * np.abs(ctx[:, 1:]).max() / 2


# ----------------------------------------------------------------------------------------------- fused feed-forward pair

def test_geglu_gate_function_through_the_layer_closed_forms(orc):
    """With zero weights lin = bias, so the layer exposes its gate function: gelu(0) = 0, gelu(g) - gelu(-g) = g,
    gelu(g) -> g for large g and -> 0 for large -g, and tabulated values of the normal distribution
    (gelu(g) = g Phi(g): Phi(1) = 0.8413447461, Phi(2) = 0.9772498681, Phi(0.5) = 0.6914624613)."""
    gates = np.array([0.0, 1.0, -1.0, 2.0, -2.0, 0.5, -0.5, 12.0, -12.0, 3.0, -3.0, 0.25], np.float16)
    H, K = len(gates), 64
    codes = np.zeros((2 * H, K), np.uint8)
    s, z = np.ones(2 * H, np.float32), np.zeros(2 * H, np.int32)
    bias = np.concatenate([np.ones(H, np.float16), gates])          # value 1 | gate g
    x = np.ones((1, K), np.float16)
    q, h16, _, u, lin = orc.linear_a8_geglu(x, codes, s, z, (np.float32(1.0), 0), act=(np.float32(1.0), 0), bias=bias,
                                            want_pre=True)
    gelu = dict(zip(gates.astype(np.float64).tolist(), u[0].tolist()))      # s_o = 1, value = 1: u is gelu(gate)
    assert np.array_equal(lin[0, :H], np.ones(H)) and np.array_equal(lin[0, H:], gates.astype(np.float64))
    assert gelu[0.0] == 0.0
    for g in (1.0, 2.0, 0.5, 3.0, 12.0):
        assert abs(gelu[g] - gelu[-g] - g) < 1e-15 * max(1.0, g)
    assert abs(gelu[12.0] - 12.0) < 1e-12 and abs(gelu[-12.0]) < 1e-12
    for g, phi in ((1.0, 0.8413447461), (2.0, 0.9772498681), (0.5, 0.6914624613)):
        assert abs(gelu[g] - g * phi) < 1e-9 * 4


def test_w_only_geglu_codes_by_hand_and_against_the_a8_projection(orc):
    """(i) Zero weights leave lin = bias: values 1, gates 0, 8, 24, -12 with s_o = 0.1, z_o = 3 give the codes
    3, 83, 243, 3.  (ii) Activations that ARE 8-bit codes times a power-of-two scale make the 8-bit path's linear
    outputs equal to the weight-only path's (both exact up to the fp64 sum): the two oracle functions, written
    separately, must then agree on every code and on the fp16 product."""
    H, K = 4, 64
    codes = np.zeros((2 * H, K), np.uint8)
    s, z = np.ones(2 * H, np.float32), np.zeros(2 * H, np.int32)
    bias = np.array([1.0, 1.0, 1.0, 1.0, 0.0, 8.0, 24.0, -12.0], np.float16)
    x = np.ones((2, K), np.float16)
    q, h = orc.linear_w_only_geglu(x, codes, s, z, bias=bias, out_act=(np.float32(0.1), 3))
    assert np.array_equal(q, np.tile(np.array([3, 83, 243, 3], np.uint8), (2, 1)))
    # (ii)
    rng = np.random.default_rng(5)
    M, K, H = 9, 128, 8
    w = si.weights_f16(73, "pin/gw", 2 * H, K)
    b = si.bias_f16(73, "pin/gb", 2 * H)
    c, sw, zw = orc.quantize_weights(w, 4)
    qx = rng.integers(0, 256, (M, K)).astype(np.uint8)
    act = (np.float32(2.0 ** -5), 131)
    x = ((qx.astype(np.float32) - act[1]) * act[0]).astype(np.float16)          # exact in fp16: |q - z| < 2^8
    assert np.array_equal(orc.act_quantize(x, *act), qx)
    out_act = (np.float32(0.004), 17)
    q16, h16, u16, lin16 = orc.linear_w_only_geglu(x, c, sw, zw, bias=b, out_act=out_act, want_pre=True)
    q8, h8, _, u8, lin8 = orc.linear_a8_geglu(x, c, sw, zw, out_act, act=act, bias=b, want_pre=True)
    assert np.abs(lin16 - lin8).max() <= 1e-12 * max(1.0, np.abs(lin8).max())
    near = np.abs(u8 - np.floor(u8) - 0.5) < 1e-9                                # (none in practice)
    assert np.array_equal(q16[~near], q8[~near]) and np.array_equal(h16, h8)


def test_geglu_dynamic_output_parameters_by_hand(orc):
    """Zero weights leave lin = bias.  Values 1, gates 0, 8, 24, -12: the gated product is 0, 8, 24 and -12 Phi(-12),
    which rounds to (minus) zero in fp16.  Range [0, 24] -> s_o = 24/255 in fp32, z_o = 0, codes 0, 85, 255, 0
    (8 * 255/24 = 85, 24 * 255/24 = 255).  Where the product is exact in fp16 the static path with these parameters
    gives the same codes."""
    H, K = 4, 64
    codes = np.zeros((2 * H, K), np.uint8)
    s, z = np.ones(2 * H, np.float32), np.zeros(2 * H, np.int32)
    bias = np.array([1.0, 1.0, 1.0, 1.0, 0.0, 8.0, 24.0, -12.0], np.float16)   # values | gates
    x = np.ones((3, K), np.float16)
    q, h16, out_act, _ = orc.linear_a8_geglu_dynamic(x, codes, s, z, act=(np.float32(1.0), 0), bias=bias)
    assert out_act[0] == np.float32(24.0) / np.float32(255.0) and out_act[1] == 0
    assert np.array_equal(q, np.tile(np.array([0, 85, 255, 0], np.uint8), (3, 1)))
    assert np.array_equal(h16.view(np.float16)[:, :3], np.tile(np.array([0.0, 8.0, 24.0], np.float16), (3, 1)))
    assert (h16[:, 3] & 0x7FFF == 0).all()
    q_static, _, _ = orc.linear_a8_geglu(x, codes, s, z, out_act, act=(np.float32(1.0), 0), bias=bias)
    assert np.array_equal(q, q_static)


def test_geglu_dynamic_is_the_dynamic_quantiser_applied_to_the_fp16_product(orc):
    """On a random layer: the parameters are those of the product's own range (zero included), every code is the
    affine quantiser's, the extreme values take the codes 0 and 255, and a product scaled by 2 (value half of the
    weight rows and bias doubled: exact in binary floating point) doubles the scale and keeps every code."""
    x, w, b, c, s, z = _random_quantised_layer(orc, 72, 23, 128, 32, 4)
    H = 16
    act = (np.float32(0.031), 121)
    q, h16, (so, zo), _ = orc.linear_a8_geglu_dynamic(x, c, s, z, act=act, bias=b)
    h = h16.view(np.float16).astype(np.float64)
    lo, hi = min(0.0, h.min()), max(0.0, h.max())
    assert abs(float(so) - (hi - lo) / 255.0) <= 1e-6 * (hi - lo) / 255.0
    assert zo == int(np.rint(-lo / float(so)))
    assert q.reshape(-1)[h.argmax()] == 255 and q.reshape(-1)[h.argmin()] == 0
    assert np.abs(q.astype(np.float64) - zo - h / float(so)).max() <= 0.5 + 1e-3
    s2, b2 = s.copy(), b.copy()
    s2[:H] *= 2.0
    b2[:H] = (b[:H].astype(np.float32) * 2.0).astype(np.float16)
    q2, h16_2, (so2, zo2), _ = orc.linear_a8_geglu_dynamic(x, c, s2, z, act=act, bias=b2)
    assert so2 == np.float32(2.0) * so and zo2 == zo and np.array_equal(q2, q)


def test_a8_from_codes_is_the_a8_linear_after_its_quantiser(orc):
    x, w, b, c, s, z = _random_quantised_layer(orc, 71, 19, 128, 24, 4)
    act = (np.float32(0.031), 121)
    qx = orc.act_quantize(x, *act)
    y0, acc0, _ = orc.linear_a8(x, c, s, z, act=act, bias=b)
    y1, acc1 = orc.linear_a8_codes(qx, act, c, s, z, bias=b)
    assert np.array_equal(acc0, acc1) and np.array_equal(y0, y1)


def test_geglu_order_bias_and_output_quantiser_by_hand(orc):
    """Zero weights leave lin = bias: the product is value * gelu(gate) with the FIRST half of the projection as
    value, and its code follows the affine quantiser with the given output parameters."""
    import math
    H, K = 4, 64
    codes = np.zeros((2 * H, K), np.uint8)
    s, z = np.ones(2 * H, np.float32), np.zeros(2 * H, np.int32)
    bias = np.array([1.0, -2.0, 0.5, 3.0, 0.0, 1.0, -1.0, 2.0], np.float16)   # values | gates
    x = np.ones((2, K), np.float16)
    out_act = (np.float32(0.05), 40)
    q, h16, _ = orc.linear_a8_geglu(x, codes, s, z, out_act, act=(np.float32(1.0), 0), bias=bias)
    gelu = lambda g: 0.5 * g * (1.0 + math.erf(g / math.sqrt(2.0)))
    want = [1.0 * gelu(0.0), -2.0 * gelu(1.0), 0.5 * gelu(-1.0), 3.0 * gelu(2.0)]
    assert np.allclose(h16.view(np.float16)[0].astype(np.float64), want, atol=2e-3)
    assert q[0].tolist() == [min(255, max(0, round(v / 0.05) + 40)) for v in want] and np.array_equal(q[0], q[1])


@pytest.mark.parametrize("bits,symmetric", [(4, False), (8, True)])
def test_geglu_requant_from_the_pinned_integer_accumulators(orc, bits, symmetric):
    """From the pinned A8 linear's exact accumulators: value half times the Gaussian gate of the gate half (math.erf),
    then the affine output quantiser with round-half-to-even.  A swapped half, a missing 0.5, the gate applied to the
    value, a zero point added before the division or half-away rounding would each move most codes."""
    import math
    M, K, H = 21, 128, 40
    x, w, b, c, s, z = _random_quantised_layer(orc, 72 + bits, M, K, 2 * H, bits, symmetric)
    out_act = (np.float32(0.004), 30)
    q, h16, act, u, lin = orc.linear_a8_geglu(x, c, s, z, out_act, w_signed=symmetric, bias=b, want_pre=True)
    _, acc, act2 = orc.linear_a8(x, c, s, z, w_signed=symmetric, bias=b)
    assert act == act2
    lin_ref = acc.astype(np.float64) * (np.float64(act[0]) * s.astype(np.float64))[None, :] + b.astype(np.float64)[None, :]
    assert np.allclose(lin, lin_ref, rtol=1e-14, atol=0)
    erf = np.vectorize(math.erf)
    h = lin_ref[:, :H] * 0.5 * lin_ref[:, H:] * (1.0 + erf(lin_ref[:, H:] / math.sqrt(2.0)))
    assert np.allclose(u, h / np.float64(out_act[0]), rtol=1e-12, atol=1e-300)
    want = np.clip(np.rint(h / np.float64(out_act[0])) + out_act[1], 0, 255).astype(np.int64)
    far = np.abs(np.abs(u - np.floor(u)) - 0.5) > 1e-9            # (not within rounding noise of a tie)
    assert far.mean() > 0.999 and np.array_equal(q.astype(np.int64)[far], want[far])
    assert len(np.unique(q)) > 20                               # the codes are spread, not saturated
    assert np.array_equal(h16.view(np.float16), h.astype(np.float16)) or \
        np.abs(h16.view(np.float16).astype(np.float64) - h).max() <= np.abs(h).max() * 2.0 ** -10
    swapped = lin_ref[:, H:] * 0.5 * lin_ref[:, :H] * (1.0 + erf(lin_ref[:, :H] / math.sqrt(2.0)))
    assert np.abs(h - swapped).max() > 0.05                     # value and gate are not interchangeable here
    rows = [0, 5, 20]
    q2, _, _ = orc.linear_a8_geglu(x, c, s, z, out_act, w_signed=symmetric, bias=b, rows=rows, act=act)
    assert np.array_equal(q2, q[rows])


def test_geglu_output_quantiser_rounds_half_to_even_and_saturates(orc):
    """Zero weights leave lin = bias; gate 12 (gelu(12) = 12 exactly in fp64) and s_o = 3 put u = value * 4 on exact
    ties: 0.5 -> 0, 1.5 -> 2, 2.5 -> 2, -0.5 -> -0 (half-away would give 1, 2, 3, -1); +-100 saturate."""
    vals = np.array([0.125, 0.375, 0.625, -0.125, 100.0, -100.0], np.float16)     
    H, K = len(vals), 64
    codes = np.zeros((2 * H, K), np.uint8)
    s, z = np.ones(2 * H, np.float32), np.zeros(2 * H, np.int32)
    bias = np.concatenate([vals, np.full(H, 12.0, np.float16)])
    x = np.ones((1, K), np.float16)
    q, _, _, u, _ = orc.linear_a8_geglu(x, codes, s, z, (np.float32(3.0), 7), act=(np.float32(1.0), 0), bias=bias,
                                        want_pre=True)
    assert np.array_equal(u[0, :4], [0.5, 1.5, 2.5, -0.5])       # exact ties
    assert q[0, :4].tolist() == [7 + 0, 7 + 2, 7 + 2, 7 - 0]
    assert q[0, 4] == 255 and q[0, 5] == 0                        # saturation at both ends


# ----------------------------------------------------------------------------------------------- 3x3 convolution

def _conv_case(orc, seed, B, H, W, Cin, N, bits, symmetric=False):
    rng = np.random.default_rng(seed)
    x = rng.normal(0, 1, (B, H, W, Cin)).astype(np.float16)
    w = rng.normal(0, 0.05, (N, 3, 3, Cin)).astype(np.float16)      # [N, r, s, c]
    b = rng.normal(0, 0.1, N).astype(np.float16)
    c, s, z = orc.quantize_weights(w.reshape(N, 9 * Cin), bits, symmetric=symmetric)
    return x, w, b, c, s, z


@pytest.mark.parametrize("bits", (4, 8))
def test_conv_w_only_equals_a_library_convolution_on_dequantised_weights(orc, bits):
    import torch
    B, H, W, Cin, N = 2, 5, 7, 8, 6
    x, w, b, c, s, z = _conv_case(orc, 80 + bits, B, H, W, Cin, N, bits)
    y = orc.conv3x3_w_only(x, c, s, z, b).view(np.float16).reshape(B, H, W, N)
    what = (s.astype(np.float64)[:, None] * (c.astype(np.float64) - z[:, None])).reshape(N, 3, 3, Cin)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2),
                                     torch.from_numpy(what).permute(0, 3, 1, 2), torch.from_numpy(b.astype(np.float64)),
                                     padding=1).permute(0, 2, 3, 1).numpy()
    ref16 = ref.astype(np.float16)
    ulp = np.abs(y.astype(np.float64) - ref16.astype(np.float64)) / np.spacing(np.abs(ref16)).astype(np.float64)
    assert ulp.max() <= 1.0 and (ulp > 0).mean() < 0.01
    pix = [0, 6, 17, B * H * W - 1]
    assert np.array_equal(orc.conv3x3_w_only(x, c, s, z, b, pix=pix).view(np.float16), y.reshape(-1, N)[pix])


def test_conv_on_a_single_pixel_is_the_linear_of_the_centre_tap(orc):
    x, w, b, c, s, z = _conv_case(orc, 83, 3, 1, 1, 64, 10, 4)
    y = orc.conv3x3_w_only(x, c, s, z, b)
    centre = c.reshape(10, 9, 64)[:, 4, :]
    assert np.array_equal(y, orc.linear_w_only(x.reshape(3, 64), centre, s, z, b))
    ya, acca, act = orc.conv3x3_a8(x, c, s, z, bias=b)
    yl, accl, actl = orc.linear_a8(x.reshape(3, 64), centre, s, z, bias=b)
    assert act == actl and np.array_equal(acca, accl) and np.array_equal(ya, yl)


@pytest.mark.parametrize("bits,symmetric", [(4, False), (8, True)])
def test_conv_a8_integer_accumulators_by_library_convolution(orc, bits, symmetric):
    """ACC equals an integer convolution of (codes - zero point) with zero padding: padding adds nothing because the
    value 0 has the zero point as its code."""
    import torch
    B, H, W, Cin, N = 2, 4, 6, 16, 5
    x, w, b, c, s, z = _conv_case(orc, 84 + bits, B, H, W, Cin, N, bits, symmetric)
    y, acc, act = orc.conv3x3_a8(x, c, s, z, w_signed=symmetric, bias=b)
    qx = orc.act_quantize(x.reshape(-1, Cin), *act).reshape(B, H, W, Cin).astype(np.int64) - act[1]
    qw = (c.view(np.int8).astype(np.int64) if symmetric else c.astype(np.int64)) - z[:, None]
    ref = torch.nn.functional.conv2d(torch.from_numpy(qx).permute(0, 3, 1, 2).double(),
                                     torch.from_numpy(qw.reshape(N, 3, 3, Cin)).permute(0, 3, 1, 2).double(),
                                     padding=1).permute(0, 2, 3, 1).numpy().reshape(-1, N)
    assert np.array_equal(acc.astype(np.int64), np.rint(ref).astype(np.int64))
    assert act == orc.act_params(x.reshape(-1, Cin))
    yf = acc.astype(np.float64) * (np.float64(act[0]) * s.astype(np.float64))[None, :] + b.astype(np.float64)[None, :]
    assert np.array_equal(y.view(np.float16), yf.astype(np.float16))
    # a shifted filter index or a transposed tap order would break this: the input is not symmetric under either
    assert not np.array_equal(acc, orc.conv3x3_a8(x[:, :, ::-1].copy(), c, s, z, w_signed=symmetric, act=act)[1])


def test_w_only_geglu_is_value_times_gelu_of_gate(orc):
    """From the pinned weight-only linear: first half value, second half gate, exact GELU, one rounding."""
    import math
    x, w, b, c, s, z = _random_quantised_layer(orc, 91, 17, 128, 48, 4)
    H = 24
    h = orc.linear_w_only_geglu(x, c, s, z, b).view(np.float16).astype(np.float64)
    what = s.astype(np.float64)[:, None] * (c.astype(np.float64) - z[:, None])
    lin = x.astype(np.float64) @ what.T + b.astype(np.float64)
    erf = np.vectorize(math.erf)
    ref = lin[:, :H] * 0.5 * lin[:, H:] * (1.0 + erf(lin[:, H:] / math.sqrt(2.0)))
    ref16 = ref.astype(np.float16)
    ulp = np.abs(h - ref16.astype(np.float64)) / np.maximum(np.spacing(np.abs(ref16)).astype(np.float64), 2.0 ** -24)
    assert ulp.max() <= 1.0 and (ulp > 0).mean() < 0.02
    swapped = lin[:, H:] * 0.5 * lin[:, :H] * (1.0 + erf(lin[:, :H] / math.sqrt(2.0)))
    assert np.abs(h - swapped).max() > 0.05   # value and gate are not interchangeable
    assert np.array_equal(orc.linear_w_only_geglu(x, c, s, z, b, rows=[3, 16]).view(np.float16).astype(np.float64), h[[3, 16]])


# ------------------------------------------------------------------------------- residual operand, split shortcuts

def test_residual_enters_the_sum_once_before_the_single_rounding(orc):
    """Exact rationals for the weight-only layer; for the 8-bit-activation layer the output recomputed from the
    returned integer accumulators. A residual that were added after rounding, subtracted, or indexed by the position in
    the row list instead of the row itself fails one of these."""
    rng = np.random.default_rng(101)
    M, K, N = 5, 16, 6
    x = rng.normal(0, 1, (M, K)).astype(np.float16)
    c = rng.integers(0, 16, (N, K)).astype(np.uint8)
    s = rng.uniform(0.01, 0.1, N).astype(np.float32)
    z = rng.integers(0, 16, N).astype(np.int32)
    b = rng.normal(0, 0.1, N).astype(np.float16)
    r = rng.normal(0, 1, (M, N)).astype(np.float16)
    y = orc.linear_w_only(x, c, s, z, b, residual=r).view(np.float16)
    twice = 0
    for m in range(M):
        for n in range(N):
            acc = Fraction(float(b[n])) + Fraction(float(r[m, n]))
            for k in range(K):
                acc += Fraction(float(x[m, k])) * Fraction(float(s[n])) * (int(c[n, k]) - int(z[n]))
            assert y[m, n] == np.float16(float(acc)), (m, n)
            twice += y[m, n] != np.float16(np.float16(float(acc - Fraction(float(r[m, n])))) + r[m, n])
    assert twice > 0            # rounding before the addition is a different function on this input
    rows = [4, 1]
    assert np.array_equal(orc.linear_w_only(x, c, s, z, b, rows=rows, residual=r).view(np.float16), y[rows])
    assert np.array_equal(orc.linear_w_only(x, c, s, z, b, residual=np.zeros_like(r)), orc.linear_w_only(x, c, s, z, b))

    ya, acc, act = orc.linear_a8(x, c, s, z, bias=b, residual=r)
    yf = acc.astype(np.float64) * (np.float64(act[0]) * s.astype(np.float64))[None, :] + b.astype(np.float64) + \
        r.astype(np.float64)
    assert np.array_equal(ya.view(np.float16), yf.astype(np.float16))
    assert np.array_equal(orc.linear_a8(x, c, s, z, bias=b, rows=rows, residual=r)[0], ya[rows])
    # the same on pre-quantised codes, and on the unquantised 16-bit layer (exact rationals again)
    yc, accc = orc.linear_a8_codes(orc.act_quantize(x, *act), act, c, s, z, bias=b, residual=r)
    assert np.array_equal(accc, acc) and np.array_equal(yc, ya)
    w = rng.normal(0, 0.5, (N, K)).astype(np.float16)
    yf = orc.linear_fp(x, w, b, residual=r).view(np.float16)
    for m in range(M):
        for n in range(N):
            tot = sum((Fraction(float(x[m, k])) * Fraction(float(w[n, k])) for k in range(K)),
                      Fraction(float(b[n])) + Fraction(float(r[m, n])))
            assert yf[m, n] == np.float16(float(tot)), (m, n)


def test_conv_residual_is_indexed_by_pixel(orc):
    B, H, W, Cin, N = 2, 3, 4, 8, 5
    x, w, b, c, s, z = _conv_case(orc, 103, B, H, W, Cin, N, 4)
    r = np.random.default_rng(104).normal(0, 1, (B, H, W, N)).astype(np.float16)
    y0, acc, act = orc.conv3x3_a8(x, c, s, z, bias=b)
    y, acc2, act2 = orc.conv3x3_a8(x, c, s, z, bias=b, residual=r)
    assert act == act2 and np.array_equal(acc, acc2)
    yf = acc.astype(np.float64) * (np.float64(act[0]) * s.astype(np.float64))[None, :] + b.astype(np.float64) + \
        r.reshape(-1, N).astype(np.float64)
    assert np.array_equal(y.view(np.float16), yf.astype(np.float16))
    pix = [23, 0, 9]
    assert np.array_equal(orc.conv3x3_a8(x, c, s, z, bias=b, pix=pix, residual=r)[0], y[pix])
    # weight-only: against the pinned residual-free result where the sum is exact (integers below 2048)
    xi = np.random.default_rng(105).integers(-2, 3, (B, H, W, Cin)).astype(np.float16)
    ci = np.random.default_rng(106).integers(0, 4, (N, 9 * Cin)).astype(np.uint8)
    ri = np.random.default_rng(107).integers(-50, 51, (B, H, W, N)).astype(np.float16)
    one, zero = np.ones(N, np.float32), np.zeros(N, np.int32)
    plain = orc.conv3x3_w_only(xi, ci, one, zero).view(np.float16).astype(np.float64)
    withr = orc.conv3x3_w_only(xi, ci, one, zero, residual=ri).view(np.float16).astype(np.float64)
    assert np.array_equal(withr, plain + ri.reshape(-1, N).astype(np.float64))
    assert np.array_equal(orc.conv3x3_w_only(xi, ci, one, zero, pix=pix, residual=ri).view(np.float16).astype(np.float64),
                          withr[pix])


def test_split_shortcut_equals_the_concatenated_layer_where_sums_are_exact(orc):
    """A layer over channel-concatenated inputs [trunk | skip] is the sum of two layers over the two parts (Sec. 4.1,
    split of the concatenated shortcut input). With small integers every partial sum is an exact fp16 value, so two calls
    chained through the residual operand must reproduce the one-call result bit for bit, for the linear layer and for
    the convolution in its (r, s, c) weight order."""
    rng = np.random.default_rng(110)
    M, C1, C2, N = 12, 24, 8, 7
    x1 = rng.integers(-3, 4, (M, C1)).astype(np.float16)
    x2 = rng.integers(-3, 4, (M, C2)).astype(np.float16)
    w1 = rng.integers(0, 8, (N, C1)).astype(np.uint8)
    w2 = rng.integers(0, 8, (N, C2)).astype(np.uint8)
    b = rng.integers(-4, 5, N).astype(np.float16)
    one, zero, z3 = np.ones(N, np.float32), np.zeros(N, np.int32), np.full(N, 3, np.int32)
    whole = orc.linear_w_only(np.concatenate([x1, x2], 1), np.concatenate([w1, w2], 1), one, z3, b)
    first = orc.linear_w_only(x1, w1, one, z3, b)
    assert np.array_equal(orc.linear_w_only(x2, w2, one, z3, None, residual=first), whole)

    B, H, W = 2, 4, 5
    xa = rng.integers(-2, 3, (B, H, W, C1)).astype(np.float16)
    xb = rng.integers(-2, 3, (B, H, W, C2)).astype(np.float16)
    wa = rng.integers(0, 4, (N, 3, 3, C1)).astype(np.uint8)
    wb = rng.integers(0, 4, (N, 3, 3, C2)).astype(np.uint8)
    wcat = np.concatenate([wa, wb], 3).reshape(N, -1)
    whole = orc.conv3x3_w_only(np.concatenate([xa, xb], 3), wcat, one, zero, b)
    first = orc.conv3x3_w_only(xa, wa.reshape(N, -1), one, zero, b)
    assert np.array_equal(orc.conv3x3_w_only(xb, wb.reshape(N, -1), one, zero, None, residual=first), whole)
    # 8-bit activations: each part has its own activation quantiser and its codes are not exact, so the chained result
    # is checked to the quantiser's tolerance (the accumulators of each part are pinned above)
    ya = orc.conv3x3_a8(xa, wa.reshape(N, -1), one, zero, bias=b)[0]
    yb = orc.conv3x3_a8(xb, wb.reshape(N, -1), one, zero, residual=ya)[0].view(np.float16).astype(np.float64)
    ref = whole.view(np.float16).astype(np.float64)
    assert np.abs(yb - ref).max() <= 0.02 * np.abs(ref).max()


@pytest.mark.parametrize("H,W", [(6, 8), (5, 7), (1, 1), (2, 9)])
def test_conv_stride_two_against_a_library_convolution(orc, H, W):
    """Stride 2, padding 1 (the downsampling convolutions): weight-only against a float64 library convolution on
    dequantised weights, the integer accumulators of the 8-bit-activation form against an integer convolution; odd
    sizes included (Ho = (H-1)//2 + 1).  The activation parameters are those of the whole input, also of the pixels
    a stride-2 filter never centres on."""
    import torch
    B, Cin, N = 2, 8, 5
    x, w, b, c, s, z = _conv_case(orc, 120 + H, B, H, W, Cin, N, 4)
    Ho, Wo = (H - 1) // 2 + 1, (W - 1) // 2 + 1
    y = orc.conv3x3_w_only(x, c, s, z, b, stride=2).view(np.float16)
    assert y.shape == (B * Ho * Wo, N)
    what = (s.astype(np.float64)[:, None] * (c.astype(np.float64) - z[:, None])).reshape(N, 3, 3, Cin)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2),
                                     torch.from_numpy(what).permute(0, 3, 1, 2), torch.from_numpy(b.astype(np.float64)),
                                     padding=1, stride=2).permute(0, 2, 3, 1).numpy().reshape(-1, N)
    ref16 = ref.astype(np.float16)
    ulp = np.abs(y.astype(np.float64) - ref16.astype(np.float64)) / np.spacing(np.abs(ref16)).astype(np.float64)
    assert ulp.max() <= 1.0
    # every output pixel of the stride-2 result is the stride-1 result at the even positions
    full = orc.conv3x3_w_only(x, c, s, z, b).view(np.float16).reshape(B, H, W, N)
    assert np.array_equal(y.reshape(B, Ho, Wo, N), full[:, ::2, ::2, :])
    pix = [0, B * Ho * Wo - 1]
    r = np.random.default_rng(9).normal(0, 1, (B, Ho, Wo, N)).astype(np.float16)
    yr = orc.conv3x3_w_only(x, c, s, z, b, stride=2, residual=r).view(np.float16)
    assert np.array_equal(orc.conv3x3_w_only(x, c, s, z, b, stride=2, residual=r, pix=pix).view(np.float16), yr[pix])
    assert not np.array_equal(yr, y)
    ya, acc, act = orc.conv3x3_a8(x, c, s, z, bias=b, stride=2)
    ya1, acc1, act1 = orc.conv3x3_a8(x, c, s, z, bias=b)
    assert act == act1 == orc.act_params(x.reshape(-1, Cin))
    assert np.array_equal(acc.reshape(B, Ho, Wo, N), acc1.reshape(B, H, W, N)[:, ::2, ::2, :])
    assert np.array_equal(ya.reshape(B, Ho, Wo, N), ya1.reshape(B, H, W, N)[:, ::2, ::2, :])

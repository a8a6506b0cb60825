"""ctypes loader for the CPU oracle (mixdq_oracle.c).

Test infrastructure only: the tests, the smoke check and the benchmark's
cpu_baseline leg import this; the product package never does.  Arrays are numpy;
16-bit floats travel as uint16 bit patterns (views of float16 arrays are fine).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mixdq_oracle.c")
_LIB = os.path.join(_HERE, "libmixdq_oracle.so")

F16, BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  No fast-math, no FMA contraction: the quantiser's
    fp32 operations must each round once."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_packed_row_bytes.restype = C.c_long
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _u16(a):
    """Bit pattern view of a 16-bit float array (or pass uint16 through)."""
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        return a.view(np.uint16)
    assert a.dtype == np.uint16, a.dtype
    return a


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with status {rc}")


def f16_to_f64(bits, dtype=F16):
    bits = _u16(bits)
    out = np.empty(bits.shape, np.float64)
    _check(lib().orc_f16_to_f64(_p(bits), _p(out), C.c_long(bits.size), dtype), "f16_to_f64")
    return out


def f64_to_f16(vals, dtype=F16):
    vals = np.ascontiguousarray(vals, np.float64)
    out = np.empty(vals.shape, np.uint16)
    _check(lib().orc_f64_to_f16(_p(vals), _p(out), C.c_long(vals.size), dtype), "f64_to_f16")
    return out


def asym_params(xmin, xmax, bits):
    s = C.c_float()
    z = C.c_int32()
    _check(lib().orc_asym_params(C.c_float(xmin), C.c_float(xmax), bits, C.byref(s), C.byref(z)), "asym_params")
    return np.float32(s.value), int(z.value)


def quantize_weights(w, bits, symmetric=False, dtype=F16):
    """W [N,K] 16-bit float -> (codes uint8 [N,K], scale f32 [N], zp i32 [N])."""
    w = _u16(w)
    N, K = w.shape
    codes = np.empty((N, K), np.uint8)
    scale = np.empty(N, np.float32)
    zp = np.empty(N, np.int32)
    _check(lib().orc_quantize_weights(_p(w), N, K, bits, int(symmetric), dtype, _p(codes), _p(scale), _p(zp)),
           "quantize_weights")
    return codes, scale, zp


def act_params(x, dtype=F16):
    x = _u16(x)
    M, K = x.shape
    s = C.c_float()
    z = C.c_int32()
    _check(lib().orc_act_params(_p(x), C.c_long(M), K, C.c_long(K), dtype, C.byref(s), C.byref(z)), "act_params")
    return np.float32(s.value), int(z.value)


def act_quantize(x, scale, zp, dtype=F16):
    x = _u16(x)
    M, K = x.shape
    q = np.empty((M, K), np.uint8)
    _check(lib().orc_act_quantize(_p(x), C.c_long(M), K, C.c_long(K), dtype, C.c_float(scale), C.c_int32(zp),
                                  _p(q)), "act_quantize")
    return q


def packed_row_bytes(K, bits):
    return int(lib().orc_packed_row_bytes(K, bits))


def pack_weights(codes, bits):
    codes = np.ascontiguousarray(codes, np.uint8)
    N, K = codes.shape
    rb = packed_row_bytes(K, bits)
    if rb < 0:
        raise ValueError("K*bits must be a multiple of 8 and bits in {2,3,4,8}")
    out = np.empty((N, rb), np.uint8)
    _check(lib().orc_pack_weights(_p(codes), N, K, bits, _p(out)), "pack_weights")
    return out


def unpack_weights(packed, K, bits):
    packed = np.ascontiguousarray(packed, np.uint8)
    N = packed.shape[0]
    out = np.empty((N, K), np.uint8)
    _check(lib().orc_unpack_weights(_p(packed), N, K, bits, _p(out)), "unpack_weights")
    return out


def code_rowsum(codes, signed=False):
    codes = np.ascontiguousarray(codes, np.uint8)
    N, K = codes.shape
    out = np.empty(N, np.int32)
    _check(lib().orc_code_rowsum(_p(codes), N, K, int(signed), _p(out)), "code_rowsum")
    return out


def _rows(rows):
    if rows is None:
        return None, 0
    rows = np.ascontiguousarray(rows, np.int64)
    return rows, rows.size


def linear_w_only(x, codes, w_scale, w_zp, bias=None, dtype=F16, rows=None, residual=None):
    """Returns y as uint16 bit patterns, [M,N] or [len(rows),N]."""
    x = _u16(x)
    bias = _u16(bias)
    codes = np.ascontiguousarray(codes, np.uint8)
    M, K = x.shape
    N = codes.shape[0]
    assert codes.shape[1] == K
    rows, nr = _rows(rows)
    R = nr if rows is not None else M
    y = np.empty((R, N), np.uint16)
    _check(lib().orc_linear_w_only(_p(x), C.c_long(M), K, C.c_long(K), _p(codes), N,
                                   _p(np.ascontiguousarray(w_scale, np.float32)),
                                   _p(np.ascontiguousarray(w_zp, np.int32)), _p(bias), dtype, _p(y), C.c_long(N),
                                   _p(rows), C.c_long(nr), _p(_u16(residual)), C.c_long(N)), "linear_w_only")
    return y


def linear_fp(x, w, bias=None, dtype=F16, residual=None):
    x = _u16(x)
    w = _u16(w)
    bias = _u16(bias)
    M, K = x.shape
    N = w.shape[0]
    y = np.empty((M, N), np.uint16)
    _check(lib().orc_linear_fp(_p(x), C.c_long(M), K, C.c_long(K), _p(w), N, _p(bias), dtype, _p(y), C.c_long(N),
                               _p(_u16(residual)), C.c_long(N)), "linear_fp")
    return y


def linear_a8(x, wcodes, w_scale, w_zp, w_signed=False, act=None, bias=None, rows=None, want_acc=True,
              residual=None):
    """act=None: dynamic per-tensor min-max over all rows of x; else (scale, zp).
    Returns (y uint16, acc int32 or None, (act_scale, act_zp))."""
    x = _u16(x)
    bias = _u16(bias)
    wcodes = np.ascontiguousarray(wcodes, np.uint8)
    M, K = x.shape
    N = wcodes.shape[0]
    assert wcodes.shape[1] == K
    rows, nr = _rows(rows)
    R = nr if rows is not None else M
    y = np.empty((R, N), np.uint16)
    acc = np.empty((R, N), np.int32) if want_acc else None
    s = C.c_float(0.0 if act is None else act[0])
    z = C.c_int32(0 if act is None else act[1])
    _check(lib().orc_linear_a8(_p(x), C.c_long(M), K, C.c_long(K), _p(wcodes), N, int(w_signed),
                               _p(np.ascontiguousarray(w_scale, np.float32)),
                               _p(np.ascontiguousarray(w_zp, np.int32)), int(act is None), C.byref(s), C.byref(z),
                               _p(bias), _p(y), C.c_long(N), _p(acc), _p(rows), C.c_long(nr), _p(_u16(residual)),
                               C.c_long(N)), "linear_a8")
    return y, acc, (np.float32(s.value), int(z.value))


def bos_aware_kv_proj(ctx, wcodes, w_scale, w_zp, w_signed=False, w_f16=None, bos_out=None, act=None, bias=None,
                      naive_all_rows=False):
    """ctx [B,T,K] fp16 -> (y uint16 [B,T,N], (act_scale, act_zp))."""
    ctx = _u16(ctx)
    B, T, K = ctx.shape
    wcodes = np.ascontiguousarray(wcodes, np.uint8)
    N = wcodes.shape[0]
    y = np.empty((B, T, N), np.uint16)
    s = C.c_float(0.0 if act is None else act[0])
    z = C.c_int32(0 if act is None else act[1])
    _check(lib().orc_bos_aware_kv_proj(_p(ctx), B, T, K, _p(wcodes), N, int(w_signed),
                                       _p(np.ascontiguousarray(w_scale, np.float32)),
                                       _p(np.ascontiguousarray(w_zp, np.int32)), _p(_u16(w_f16)), _p(_u16(bos_out)),
                                       int(act is None), C.byref(s), C.byref(z), _p(_u16(bias)), _p(y),
                                       int(naive_all_rows)), "bos_aware_kv_proj")
    return y, (np.float32(s.value), int(z.value))


def linear_a8_geglu(x, wcodes, w_scale, w_zp, out_act, w_signed=False, act=None, bias=None, rows=None, want_h16=True,
                    want_pre=False):
    """GEGLU projection, 8-bit activations in and out, in fp64 with the library erf.  wcodes [2H,K]; out_act = (scale,
    zp) of the gated product.  Returns (codes uint8 [R,H], h16 uint16 [R,H] or None, (act_scale, act_zp)) and, with
    want_pre, also (u float64 [R,H] = h / s_o before the rounding, lin float64 [R,2H] = the projection before the
    gate): what a checker needs to tell a borderline rounding from a wrong code."""
    x = _u16(x)
    bias = _u16(bias)
    wcodes = np.ascontiguousarray(wcodes, np.uint8)
    M, K = x.shape
    H = wcodes.shape[0] // 2
    assert wcodes.shape == (2 * H, K)
    rows, nr = _rows(rows)
    R = nr if rows is not None else M
    codes = np.empty((R, H), np.uint8)
    h16 = np.empty((R, H), np.uint16) if want_h16 else None
    u = np.empty((R, H), np.float64) if want_pre else None
    lin = np.empty((R, 2 * H), np.float64) if want_pre else None
    s = C.c_float(0.0 if act is None else act[0])
    z = C.c_int32(0 if act is None else act[1])
    _check(lib().orc_linear_a8_geglu(_p(x), C.c_long(M), K, C.c_long(K), _p(wcodes), H, int(w_signed),
                                     _p(np.ascontiguousarray(w_scale, np.float32)),
                                     _p(np.ascontiguousarray(w_zp, np.int32)), int(act is None), C.byref(s),
                                     C.byref(z), _p(bias), C.c_float(out_act[0]), C.c_int32(out_act[1]), _p(codes),
                                     _p(h16), _p(u), _p(lin), _p(rows), C.c_long(nr)), "linear_a8_geglu")
    if want_pre:
        return codes, h16, (np.float32(s.value), int(z.value)), u, lin
    return codes, h16, (np.float32(s.value), int(z.value))


def linear_a8_geglu_dynamic(x, wcodes, w_scale, w_zp, w_signed=False, act=None, bias=None):
    """GEGLU projection whose 8-bit output takes its parameters from the gated product itself: the product is rounded
    to fp16 (the tensor that is handed on), and that tensor is quantised like any dynamically quantised activation
    (paper Sec. 4.1, per-tensor min-max).  Returns (codes uint8 [M,H], h16 uint16 [M,H], (out_scale, out_zp),
    (act_scale, act_zp))."""
    # (the static parameters handed to the projection below are not used: only its fp16 product is)
    _, h16, act_used = linear_a8_geglu(x, wcodes, w_scale, w_zp, (np.float32(1.0), 0), w_signed=w_signed, act=act,
                                       bias=bias, want_h16=True)
    s_o, z_o = act_params(h16)
    return act_quantize(h16, s_o, z_o), h16, (s_o, z_o), act_used


def linear_a8_codes(qx, act, wcodes, w_scale, w_zp, w_signed=False, bias=None, want_acc=True, residual=None):
    """A8 linear on activations that arrive as unsigned 8-bit codes with act = (scale, zp).
    Returns (y uint16 [M,N], acc int32 or None)."""
    qx = np.ascontiguousarray(qx, np.uint8)
    bias = _u16(bias)
    wcodes = np.ascontiguousarray(wcodes, np.uint8)
    M, K = qx.shape
    N = wcodes.shape[0]
    assert wcodes.shape[1] == K
    y = np.empty((M, N), np.uint16)
    acc = np.empty((M, N), np.int32) if want_acc else None
    _check(lib().orc_linear_a8_codes(_p(qx), C.c_long(M), K, C.c_float(act[0]), C.c_int32(act[1]), _p(wcodes), N,
                                     int(w_signed), _p(np.ascontiguousarray(w_scale, np.float32)),
                                     _p(np.ascontiguousarray(w_zp, np.int32)), _p(bias), _p(y), C.c_long(N), _p(acc),
                                     _p(_u16(residual)), C.c_long(N)), "linear_a8_codes")
    return y, acc


def conv3x3_w_only(x, codes, w_scale, w_zp, bias=None, dtype=F16, pix=None, residual=None, stride=1):
    """x [B,H,W,Cin] 16-bit; codes [N, 9*Cin] with k = (r*3+s)*Cin + c.  Returns y uint16 [B*Ho*Wo or len(pix), N]
    (Ho = (H-1)//stride + 1, likewise Wo; pix and residual index output pixels)."""
    x = _u16(x)
    bias = _u16(bias)
    codes = np.ascontiguousarray(codes, np.uint8)
    B, H, W, Cin = x.shape
    N = codes.shape[0]
    assert codes.shape[1] == 9 * Cin
    pix, npx = _rows(pix)
    R = npx if pix is not None else B * ((H - 1) // stride + 1) * ((W - 1) // stride + 1)
    y = np.empty((R, N), np.uint16)
    _check(lib().orc_conv3x3_w_only(_p(x), B, H, W, Cin, _p(codes), N, _p(np.ascontiguousarray(w_scale, np.float32)),
                                    _p(np.ascontiguousarray(w_zp, np.int32)), _p(bias), dtype, _p(y), _p(pix),
                                    C.c_long(npx), _p(_u16(residual)), int(stride)), "conv3x3_w_only")
    return y


def conv3x3_a8(x, wcodes, w_scale, w_zp, w_signed=False, act=None, bias=None, pix=None, want_acc=True, residual=None,
               stride=1):
    """Returns (y uint16, acc int32 or None, (act_scale, act_zp))."""
    x = _u16(x)
    bias = _u16(bias)
    wcodes = np.ascontiguousarray(wcodes, np.uint8)
    B, H, W, Cin = x.shape
    N = wcodes.shape[0]
    assert wcodes.shape[1] == 9 * Cin
    pix, npx = _rows(pix)
    R = npx if pix is not None else B * ((H - 1) // stride + 1) * ((W - 1) // stride + 1)
    y = np.empty((R, N), np.uint16)
    acc = np.empty((R, N), np.int32) if want_acc else None
    s = C.c_float(0.0 if act is None else act[0])
    z = C.c_int32(0 if act is None else act[1])
    _check(lib().orc_conv3x3_a8(_p(x), B, H, W, Cin, _p(wcodes), N, int(w_signed),
                                _p(np.ascontiguousarray(w_scale, np.float32)), _p(np.ascontiguousarray(w_zp, np.int32)),
                                int(act is None), C.byref(s), C.byref(z), _p(bias), _p(y), _p(acc), _p(pix),
                                C.c_long(npx), _p(_u16(residual)), int(stride)), "conv3x3_a8")
    return y, acc, (np.float32(s.value), int(z.value))


def linear_w_only_geglu(x, codes, w_scale, w_zp, bias=None, dtype=F16, rows=None, out_act=None, want_pre=False):
    """Weight-only gated projection; codes [2H,K].  Returns h uint16 [R,H]; with out_act = (scale, zp) of the gated
    product: (codes uint8 [R,H], h) and, with want_pre, also (u float64 [R,H] = h / s_o before the rounding,
    lin float64 [R,2H] = the projection before the gate)."""
    x = _u16(x)
    bias = _u16(bias)
    codes = np.ascontiguousarray(codes, np.uint8)
    M, K = x.shape
    H = codes.shape[0] // 2
    assert codes.shape == (2 * H, K)
    rows, nr = _rows(rows)
    R = nr if rows is not None else M
    h = np.empty((R, H), np.uint16)
    q = np.empty((R, H), np.uint8) if out_act is not None else None
    u = np.empty((R, H), np.float64) if (want_pre and out_act is not None) else None
    lin = np.empty((R, 2 * H), np.float64) if (want_pre and out_act is not None) else None
    so, zo = (0.0, 0) if out_act is None else out_act
    _check(lib().orc_linear_w_only_geglu(_p(x), C.c_long(M), K, C.c_long(K), _p(codes), H,
                                         _p(np.ascontiguousarray(w_scale, np.float32)),
                                         _p(np.ascontiguousarray(w_zp, np.int32)), _p(bias), dtype, _p(h),
                                         C.c_float(so), C.c_int32(zo), _p(q), _p(u), _p(lin), _p(rows),
                                         C.c_long(nr)), "linear_w_only_geglu")
    if out_act is None:
        return h
    if want_pre:
        return q, h, u, lin
    return q, h

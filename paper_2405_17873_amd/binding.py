"""ctypes marshalling for libmixdq.so.  Tensors are torch tensors on the GPU; torch supplies device memory
and the current stream, nothing else.  Function names and argument meaning follow include/mixdq.h."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmixdq.so")

F16, BF16 = 0, 1
LAYOUT_CANONICAL, LAYOUT_KERNEL = 0, 1

_ERRORS = {
    -1: "MQ_ERR_BAD_ARG", -2: "MQ_ERR_BAD_SHAPE", -3: "MQ_ERR_UNSUPPORTED_BITS", -4: "MQ_ERR_WORKSPACE_TOO_SMALL",
    -5: "MQ_ERR_HIP", -6: "MQ_ERR_UNSUPPORTED_LAYOUT", -7: "MQ_ERR_OVERFLOW_RISK", -8: "MQ_ERR_INFEASIBLE",
    -9: "MQ_ERR_TOO_LARGE",
}

EXPORTS = ("mq_version", "mq_last_hip_error", "mq_tune_force_tile", "mq_tune_force_splits", "mq_tune_force_band", "mq_prof_enable", "mq_prof_num_slots", "mq_prof_read",
           "mq_prof_reset", "mq_prof_phase_buffer", "mq_prof_filter", "mq_prof_bracket_overhead_us", "mq_prof_copy", "mq_prof_microbench", "mq_quantize_weights", "mq_packed_bytes", "mq_pack_weights",
           "mq_unpack_weights", "mq_split_workspace_bytes", "mq_qlinear_w_only", "mq_qlinear_a8_workspace_bytes", "mq_qlinear_w8a8",
           "mq_qlinear_w4a8", "mq_qlinear_w2a8", "mq_builtin_workspace_bytes", "mq_qlinear_a8_builtin_ws", "mq_a8_row_bytes", "mq_qlinear_a8_geglu", "mq_qlinear_a8_geglu_dynamic_workspace_bytes", "mq_qlinear_a8_geglu_dynamic", "mq_qlinear_w_only_geglu", "mq_qlinear_w_only_geglu_a8", "mq_qlinear_a8_codes", "mq_conv3x3_w_only",
           "mq_conv_tap_sums", "mq_conv3x3_a8_workspace_bytes", "mq_conv3x3_a8",
           "mq_bos_aware_kv_proj_workspace_bytes", "mq_bos_aware_kv_proj", "mq_alloc_solve", "mq_alloc_split_budget",
           "mq_alloc_search")


class MixdqError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {_ERRORS.get(code, code)}")


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Loads the HIP library; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        _lib = C.CDLL(_LIB_PATH)
        for name in ("mq_a8_row_bytes", "mq_split_workspace_bytes", "mq_builtin_workspace_bytes", "mq_conv3x3_a8_workspace_bytes", "mq_packed_bytes", "mq_qlinear_a8_workspace_bytes", "mq_qlinear_a8_geglu_dynamic_workspace_bytes", "mq_bos_aware_kv_proj_workspace_bytes"):
            getattr(_lib, name).restype = C.c_size_t
        _lib.mq_prof_bracket_overhead_us.restype = C.c_double
    return _lib


def version() -> int:
    return load().mq_version()


def tune_force_tile(tile: int) -> None:
    load().mq_tune_force_tile(int(tile))


def tune_force_splits(parts: int) -> None:
    load().mq_tune_force_splits(int(parts))


def tune_force_band(rows: int) -> None:
    load().mq_tune_force_band(int(rows))


def prof_phase_buffer(buf: Optional[torch.Tensor]) -> None:
    """buf: int64 device tensor with 4 entries per workgroup, or None to switch phase timing off."""
    load().mq_prof_phase_buffer(_ptr(buf), C.c_long(0 if buf is None else buf.numel() // 4))


def prof_enable(on: bool) -> None:
    _check(load().mq_prof_enable(int(on)), "mq_prof_enable")


def prof_filter(slot: int = -1, stride: int = 1) -> None:
    _check(load().mq_prof_filter(int(slot), int(stride)), "mq_prof_filter")


def prof_bracket_overhead_us() -> float:
    return float(load().mq_prof_bracket_overhead_us(_stream()))


def prof_copy(dst: torch.Tensor, src: torch.Tensor) -> None:
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(load().mq_prof_copy(_ptr(dst), _ptr(src), C.c_size_t(nbytes), _stream()), "mq_prof_copy")


def prof_microbench(kind: int, buf: torch.Tensor) -> float:
    """Elapsed milliseconds (best of five) of microbenchmark `kind` (see include/mixdq.h); buf: device scratch."""
    ms = C.c_double(0.0)
    _check(load().mq_prof_microbench(int(kind), _ptr(buf), C.c_size_t(buf.numel() * buf.element_size()), C.byref(ms),
                                     _stream()), "mq_prof_microbench")
    return ms.value


def machine_peaks(buf: Optional[torch.Tensor] = None) -> dict:
    """Measured rates of this machine: int8 and fp16 MFMA (T(FL)OP/s), read-only stream (GB/s), LDS reads and L2 -> LDS
    copies (bytes per second over the chip), and the overlap of matrix and vector instructions on a SIMD: with 8 vector
    instructions per MFMA (as many cycles as the MFMA itself) the elapsed time of both kinds of work together divided
    by the sum of their separate times (0.5 = perfect overlap of equal halves, 1.0 = none), in one wave and in two
    waves of one SIMD; and with 4 vector instructions per MFMA the elapsed time divided by that of the MFMAs alone
    (1.0: the vector instructions are hidden completely)."""
    if buf is None:
        buf = torch.empty(2 << 30, dtype=torch.uint8, device="cuda")
    small = buf[:4 << 20]
    t = {k: prof_microbench(k, small if k != 5 else buf) for k in range(9)}
    n_mfma = 512 * 4 * 4096 * 4
    return {
        "int8_TOPs": n_mfma * 65536.0 / (t[0] * 1e-3) / 1e12,
        "f16_TFLOPs": n_mfma * 32768.0 / (t[1] * 1e-3) / 1e12,
        "read_GBps": (buf.numel() - 4096) / (t[5] * 1e-3) / 1e9,
        "lds_read_TBps": 1024 * 4 * 4000 * 8192.0 / (t[6] * 1e-3) / 1e12,
        "l2_to_lds_TBps": 768 * 4 * 2048 * 8192.0 / (t[7] * 1e-3) / 1e12,
        "mfma_ms": t[0], "valu_ms": t[2], "same_wave_ms": t[3], "two_waves_ms": t[4],
        "serial_share_same_wave": t[3] / (t[0] + t[2]), "serial_share_two_waves": t[4] / (t[0] + t[2]),
        "four_valu_per_mfma_ms": t[8], "four_valu_per_mfma_over_mfma_only": t[8] / t[0],
    }


def prof_reset() -> None:
    _check(load().mq_prof_reset(), "mq_prof_reset")


def prof_read():
    """Per-kernel totals since the last reset: list of dicts (only kernels that ran)."""
    L = load()
    out = []
    for slot in range(L.mq_prof_num_slots()):
        name = C.create_string_buffer(128)
        n = C.c_longlong()
        ms, ops, byts = C.c_double(), C.c_double(), C.c_double()
        _check(L.mq_prof_read(slot, name, 128, C.byref(n), C.byref(ms), C.byref(ops), C.byref(byts)), "mq_prof_read")
        if n.value:
            out.append({"slot": slot, "kernel": name.value.decode(), "launches": n.value, "ms": ms.value, "ops": ops.value,
                        "bytes": byts.value})
    return out


def _ptr(t: Optional[torch.Tensor]):
    return C.c_void_p(0 if t is None else t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc: int, what: str):
    if rc != 0:
        raise MixdqError(rc, what)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float16:
        return F16
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"expected a 16-bit float tensor, got {t.dtype}")


@dataclass
class PackedWeight:
    """A quantised, packed weight matrix resident on the GPU (what the offline step hands to the hot path)."""
    packed: torch.Tensor      # uint8 bytes
    scale: Optional[torch.Tensor]   # float32 [N] (None for unquantised 16-bit weights)
    zp: Optional[torch.Tensor]      # int32 [N]
    colsum: Optional[torch.Tensor]  # int32 [N]
    N: int
    K: int
    bits: int
    layout: int
    signed: bool


def keep_weights_16bit(w: torch.Tensor) -> PackedWeight:
    """An unquantised fp16/bf16 weight matrix in the layout the GEMM reads (a layer kept at 16 bits)."""
    packed, _ = pack_weights(w, 16, LAYOUT_KERNEL)
    return PackedWeight(packed, None, None, None, w.shape[0], w.shape[1], 16, LAYOUT_KERNEL, False)


def stack_weights(parts) -> PackedWeight:
    """Layers that share their input (a block's q, k, v projections; the K and V projections of the text context) as
    one layer: in the kernel layout the packed form of the row-stacked matrix is the concatenation of the parts'
    packed buffers (tiles are 32 output channels tall, so every part's N must be a multiple of 32), and the
    per-channel parameters concatenate likewise.  One call on the stacked weight writes [M, N1 + N2 + ...]."""
    first = parts[0]
    for p in parts:
        assert p.N % 32 == 0 and (p.K, p.bits, p.layout, p.signed) == (first.K, first.bits, LAYOUT_KERNEL, first.signed)
    cat = lambda ts: None if ts[0] is None else torch.cat(ts)
    return PackedWeight(torch.cat([p.packed for p in parts]), cat([p.scale for p in parts]), cat([p.zp for p in parts]),
                        cat([p.colsum for p in parts]), sum(p.N for p in parts), first.K, first.bits, LAYOUT_KERNEL,
                        first.signed)


def quantize_weights(w: torch.Tensor, bits: int, symmetric: bool = False):
    """W [N,K] fp16/bf16 -> (codes uint8 [N,K], scale float32 [N], zp int32 [N])."""
    assert w.is_cuda and w.dim() == 2 and w.is_contiguous()
    N, K = w.shape
    codes = torch.empty((N, K), dtype=torch.uint8, device=w.device)
    scale = torch.empty(N, dtype=torch.float32, device=w.device)
    zp = torch.empty(N, dtype=torch.int32, device=w.device)
    _check(load().mq_quantize_weights(_ptr(w), N, K, bits, int(symmetric), _dtype_code(w), _ptr(codes), _ptr(scale),
                                      _ptr(zp), _stream()), "mq_quantize_weights")
    return codes, scale, zp


def packed_bytes(N: int, K: int, bits: int, layout: int) -> int:
    return int(load().mq_packed_bytes(N, K, bits, layout))


def pack_weights(codes: torch.Tensor, bits: int, layout: int = LAYOUT_KERNEL, codes_signed: bool = False,
                 want_colsum: bool = True):
    """codes uint8 [N,K] -> (packed uint8 [bytes], colsum int32 [N] or None).  bits = 16: `codes` is the fp16/bf16
    weight matrix itself and there is no colsum."""
    assert codes.is_cuda and codes.dim() == 2 and codes.is_contiguous()
    assert codes.dtype == torch.uint8 if bits != 16 else codes.dtype in (torch.float16, torch.bfloat16)
    N, K = codes.shape
    nbytes = packed_bytes(N, K, bits, layout)
    packed = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=codes.device)
    colsum = torch.empty(N, dtype=torch.int32, device=codes.device) if (want_colsum and bits != 16) else None
    _check(load().mq_pack_weights(_ptr(codes), N, K, bits, layout, int(codes_signed), _ptr(packed), _ptr(colsum),
                                  _stream()), "mq_pack_weights")
    return packed, colsum


def unpack_weights(packed: torch.Tensor, N: int, K: int, bits: int, layout: int, dtype=torch.float16) -> torch.Tensor:
    """Codes uint8 [N,K]; for bits = 16 the weight matrix in `dtype`."""
    codes = torch.empty((N, K), dtype=torch.uint8 if bits != 16 else dtype, device=packed.device)
    _check(load().mq_unpack_weights(_ptr(packed), N, K, bits, layout, _ptr(codes), _stream()), "mq_unpack_weights")
    return codes


def _res(residual, M, N, dtype):
    """(pointer, row stride) of an optional [M,N] residual operand."""
    if residual is None:
        return C.c_void_p(0), 0
    assert residual.is_cuda and residual.dim() == 2 and residual.shape == (M, N) and residual.stride(1) == 1
    assert residual.dtype == dtype
    return _ptr(residual), residual.stride(0)


def split_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(load().mq_split_workspace_bytes(M, N, K))


def _ws_args(ws: Optional[torch.Tensor]):
    return (C.c_void_p(0), C.c_size_t(0)) if ws is None else (_ptr(ws), C.c_size_t(ws.numel() * ws.element_size()))


def qlinear_w_only(x: torch.Tensor, w: PackedWeight, bias: Optional[torch.Tensor] = None,
                   out: Optional[torch.Tensor] = None, residual: Optional[torch.Tensor] = None,
                   ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Y = X . dequant(W)^T + bias (+ residual) with 16-bit floating-point compute (weight-only quantisation).
    ws: optional uint8 workspace of split_workspace_bytes(M, N, K) bytes; allocated here when the shape can use one."""
    assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1
    M, K = x.shape
    assert K == w.K
    y = out if out is not None else torch.empty((M, w.N), dtype=x.dtype, device=x.device)
    rp, ldr = _res(residual, M, w.N, x.dtype)
    if ws is None:
        need = split_workspace_bytes(M, w.N, K)
        ws = torch.empty(need, dtype=torch.uint8, device=x.device) if need else None
    _check(load().mq_qlinear_w_only(_ptr(x), M, K, x.stride(0), _ptr(w.packed), w.N, w.bits, w.layout, _ptr(w.scale),
                                    _ptr(w.zp), _ptr(bias), _ptr(y), y.stride(0), _dtype_code(x), rp, ldr, *_ws_args(ws),
                                    _stream()), "mq_qlinear_w_only")
    return y


def qlinear_a8_workspace_bytes(M: int, K: int) -> int:
    return int(load().mq_qlinear_a8_workspace_bytes(M, K))


def _workspace(nbytes: int, device, ws: Optional[torch.Tensor]):
    if ws is None:
        ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    return ws


def _qlinear_a8(fn_name, x, w: PackedWeight, act, bias, out, ws, want_acc, want_act, residual=None):
    assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1 and x.dtype == torch.float16
    M, K = x.shape
    assert K == w.K
    dev = x.device
    y = out if out is not None else torch.empty((M, w.N), dtype=torch.float16, device=dev)
    ws = _workspace(qlinear_a8_workspace_bytes(M, K) + split_workspace_bytes(M, w.N, K), dev, ws)
    acc = torch.empty((M, w.N), dtype=torch.int32, device=dev) if want_acc else None
    s_out = torch.empty(1, dtype=torch.float32, device=dev) if want_act else None
    z_out = torch.empty(1, dtype=torch.int32, device=dev) if want_act else None
    a_s, a_z = (None, None) if act is None else act
    rp, ldr = _res(residual, M, w.N, torch.float16)
    L = load()
    if fn_name == "mq_qlinear_w8a8":
        rc = L.mq_qlinear_w8a8(_ptr(x), M, K, x.stride(0), _ptr(w.packed), w.N, w.layout, int(w.signed), _ptr(w.scale),
                               _ptr(w.zp), _ptr(w.colsum), _ptr(a_s), _ptr(a_z), _ptr(bias), _ptr(y), y.stride(0),
                               _ptr(acc), rp, ldr, _ptr(s_out), _ptr(z_out), _ptr(ws), C.c_size_t(ws.numel()),
                               _stream())
    else:
        fn = L.mq_qlinear_w4a8 if fn_name == "mq_qlinear_w4a8" else L.mq_qlinear_w2a8
        rc = fn(_ptr(x), M, K, x.stride(0), _ptr(w.packed), w.N, w.layout, _ptr(w.scale), _ptr(w.zp),
                               _ptr(w.colsum), _ptr(a_s), _ptr(a_z), _ptr(bias), _ptr(y), y.stride(0), _ptr(acc),
                               rp, ldr, _ptr(s_out), _ptr(z_out), _ptr(ws), C.c_size_t(ws.numel()), _stream())
    _check(rc, fn_name)
    return y, acc, (s_out, z_out)


def qlinear_w8a8(x, w: PackedWeight, act=None, bias=None, out=None, ws=None, want_acc=False, want_act=False,
                 residual=None):
    """act=None: dynamic per-tensor min-max on the device; else (scale tensor[1] f32, zp tensor[1] i32).
    Returns (y, acc or None, (act_scale, act_zp) device scalars or (None, None))."""
    assert w.bits == 8
    return _qlinear_a8("mq_qlinear_w8a8", x, w, act, bias, out, ws, want_acc, want_act, residual)


def qlinear_w4a8(x, w: PackedWeight, act=None, bias=None, out=None, ws=None, want_acc=False, want_act=False,
                 residual=None):
    assert w.bits == 4 and not w.signed
    return _qlinear_a8("mq_qlinear_w4a8", x, w, act, bias, out, ws, want_acc, want_act, residual)


def qlinear_w2a8(x, w: PackedWeight, act=None, bias=None, out=None, ws=None, want_acc=False, want_act=False,
                 residual=None):
    assert w.bits == 2 and not w.signed
    return _qlinear_a8("mq_qlinear_w2a8", x, w, act, bias, out, ws, want_acc, want_act, residual)


def builtin_workspace_bytes() -> int:
    return int(load().mq_builtin_workspace_bytes())


def qlinear_a8_builtin_ws(x, w: PackedWeight, act=None, bias=None, out=None, want_acc=False, want_act=False,
                          residual=None, y=None):
    """W8A8 / W4A8 / W2A8 (by the weight's bit-width) with the workspace inside the library: the C call allocates
    nothing.  Pass out= (and want_acc / want_act False) for a call that allocates nothing on the Python side either.
    Returns (y, acc or None, (act_scale, act_zp) or (None, None))."""
    assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1 and x.dtype == torch.float16
    M, K = x.shape
    assert K == w.K
    dev = x.device
    y = out if out is not None else torch.empty((M, w.N), dtype=torch.float16, device=dev)
    acc = torch.empty((M, w.N), dtype=torch.int32, device=dev) if want_acc else None
    s_out = torch.empty(1, dtype=torch.float32, device=dev) if want_act else None
    z_out = torch.empty(1, dtype=torch.int32, device=dev) if want_act else None
    a_s, a_z = (None, None) if act is None else act
    rp, ldr = _res(residual, M, w.N, torch.float16)
    _check(load().mq_qlinear_a8_builtin_ws(_ptr(x), M, K, x.stride(0), _ptr(w.packed), w.N, w.bits, w.layout,
                                           int(w.signed), _ptr(w.scale), _ptr(w.zp), _ptr(w.colsum), _ptr(a_s), _ptr(a_z),
                                           _ptr(bias), _ptr(y), y.stride(0), _ptr(acc), rp, ldr, _ptr(s_out), _ptr(z_out),
                                           _stream()), "mq_qlinear_a8_builtin_ws")
    return y, acc, (s_out, z_out)


def a8_row_bytes(K: int) -> int:
    return int(load().mq_a8_row_bytes(K))


def qlinear_a8_geglu(x, w: PackedWeight, out_act, act=None, bias=None, ws=None, want_h16=False, want_act=False):
    """Gated projection with 8-bit output.  w has 2H rows; out_act = (scale, zp) one-element device tensors.
    Returns (a8 int8 [M, a8_row_bytes(H)], h16 fp16 [M,H] or None, (act_scale, act_zp) or None)."""
    assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1 and x.dtype == torch.float16
    M, K = x.shape
    H = w.N // 2
    a8 = torch.empty((M, a8_row_bytes(H)), dtype=torch.int8, device=x.device)
    h16 = torch.empty((M, H), dtype=torch.float16, device=x.device) if want_h16 else None
    ws = _workspace(qlinear_a8_workspace_bytes(M, K), x.device, ws)
    a_s, a_z = (None, None) if act is None else act
    so = torch.empty(1, dtype=torch.float32, device=x.device) if want_act else None
    zo = torch.empty(1, dtype=torch.int32, device=x.device) if want_act else None
    _check(load().mq_qlinear_a8_geglu(_ptr(x), M, K, x.stride(0), _ptr(w.packed), H, w.bits, w.layout, int(w.signed),
                                      _ptr(w.scale), _ptr(w.zp), _ptr(w.colsum), _ptr(a_s), _ptr(a_z), _ptr(bias),
                                      _ptr(out_act[0]), _ptr(out_act[1]), _ptr(a8), _ptr(h16), H, _ptr(so), _ptr(zo),
                                      _ptr(ws), C.c_size_t(ws.numel()), _stream()), "mq_qlinear_a8_geglu")
    return a8, h16, ((so, zo) if want_act else None)


def qlinear_a8_geglu_dynamic_workspace_bytes(M: int, K: int, H: int) -> int:
    return int(load().mq_qlinear_a8_geglu_dynamic_workspace_bytes(int(M), int(K), int(H)))


def qlinear_a8_geglu_dynamic(x, w: PackedWeight, act=None, bias=None, ws=None, want_act=False):
    """Gated projection with 8-bit output whose parameters are taken from the range of the gated product itself.
    w has 2H rows.  Returns (a8 int8 [M, a8_row_bytes(H)], h16 fp16 [M,H], (out_scale, out_zp) one-element device
    tensors, (act_scale, act_zp) of the input or None)."""
    assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1 and x.dtype == torch.float16
    M, K = x.shape
    H = w.N // 2
    a8 = torch.empty((M, a8_row_bytes(H)), dtype=torch.int8, device=x.device)
    h16 = torch.empty((M, H), dtype=torch.float16, device=x.device)
    ws = _workspace(qlinear_a8_geglu_dynamic_workspace_bytes(M, K, H), x.device, ws)
    a_s, a_z = (None, None) if act is None else act
    o_s = torch.empty(1, dtype=torch.float32, device=x.device)
    o_z = torch.empty(1, dtype=torch.int32, device=x.device)
    so = torch.empty(1, dtype=torch.float32, device=x.device) if want_act else None
    zo = torch.empty(1, dtype=torch.int32, device=x.device) if want_act else None
    _check(load().mq_qlinear_a8_geglu_dynamic(_ptr(x), M, K, x.stride(0), _ptr(w.packed), H, w.bits, w.layout,
                                              int(w.signed), _ptr(w.scale), _ptr(w.zp), _ptr(w.colsum), _ptr(a_s),
                                              _ptr(a_z), _ptr(bias), _ptr(h16), H, _ptr(a8), _ptr(o_s), _ptr(o_z),
                                              _ptr(so), _ptr(zo), _ptr(ws), C.c_size_t(ws.numel()), _stream()),
           "mq_qlinear_a8_geglu_dynamic")
    return a8, h16, (o_s, o_z), ((so, zo) if want_act else None)


def qlinear_w_only_geglu(x, w: PackedWeight, bias=None, out=None):
    """Weight-only gated projection: w has 2H rows; returns value * gelu(gate) as fp16 [M,H]."""
    assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1 and x.dtype == torch.float16
    M, K = x.shape
    H = w.N // 2
    h = out if out is not None else torch.empty((M, H), dtype=torch.float16, device=x.device)
    _check(load().mq_qlinear_w_only_geglu(_ptr(x), M, K, x.stride(0), _ptr(w.packed), H, w.bits, w.layout, _ptr(w.scale),
                                          _ptr(w.zp), _ptr(bias), _ptr(h), h.stride(0), _stream()),
           "mq_qlinear_w_only_geglu")
    return h


def qlinear_w_only_geglu_a8(x, w: PackedWeight, out_act, bias=None, want_h16=False):
    """Weight-only gated projection with 8-bit output; out_act = (scale, zp) one-element device tensors.
    Returns (a8 int8 [M, a8_row_bytes(H)], h16 fp16 [M,H] or None)."""
    assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1 and x.dtype == torch.float16
    M, K = x.shape
    H = w.N // 2
    a8 = torch.empty((M, a8_row_bytes(H)), dtype=torch.int8, device=x.device)
    h16 = torch.empty((M, H), dtype=torch.float16, device=x.device) if want_h16 else None
    _check(load().mq_qlinear_w_only_geglu_a8(_ptr(x), M, K, x.stride(0), _ptr(w.packed), H, w.bits, w.layout,
                                             _ptr(w.scale), _ptr(w.zp), _ptr(bias), _ptr(out_act[0]), _ptr(out_act[1]),
                                             _ptr(a8), _ptr(h16), H, _stream()), "mq_qlinear_w_only_geglu_a8")
    return a8, h16


def qlinear_a8_codes(a8, K: int, act, w: PackedWeight, bias=None, out=None, want_acc=False, residual=None):
    """A8 linear on activations in the A8 layout (a8 int8 [M, stride]); act = (scale, zp) one-element device tensors."""
    assert a8.is_cuda and a8.dim() == 2 and a8.stride(1) == 1 and a8.dtype == torch.int8 and K == w.K
    M = a8.shape[0]
    y = out if out is not None else torch.empty((M, w.N), dtype=torch.float16, device=a8.device)
    acc = torch.empty((M, w.N), dtype=torch.int32, device=a8.device) if want_acc else None
    rp, ldr = _res(residual, M, w.N, torch.float16)
    _check(load().mq_qlinear_a8_codes(_ptr(a8), M, K, a8.stride(0), _ptr(act[0]), _ptr(act[1]), _ptr(w.packed), w.N,
                                      w.bits, w.layout, int(w.signed), _ptr(w.scale), _ptr(w.zp), _ptr(w.colsum),
                                      _ptr(bias), _ptr(y), y.stride(0), _ptr(acc), rp, ldr, _stream()),
           "mq_qlinear_a8_codes")
    return y, acc


def plan_qlinear_a8_geglu(x, w: PackedWeight, out_act, bias, a8_out, ws, act=None):
    M, K = x.shape
    H = w.N // 2
    a_s, a_z = (None, None) if act is None else act
    null = C.c_void_p(0)
    args = (_ptr(x), M, K, x.stride(0), _ptr(w.packed), H, w.bits, w.layout, int(w.signed), _ptr(w.scale), _ptr(w.zp),
            _ptr(w.colsum), _ptr(a_s), _ptr(a_z), _ptr(bias), _ptr(out_act[0]), _ptr(out_act[1]), _ptr(a8_out), null, H,
            null, null, _ptr(ws), C.c_size_t(ws.numel()), _stream())
    return _planned(load().mq_qlinear_a8_geglu, "mq_qlinear_a8_geglu", args, (x, w, out_act, bias, a8_out, ws, act))


def plan_qlinear_a8_geglu_dynamic(x, w: PackedWeight, bias, h16, a8_out, out_act, ws, act=None):
    """out_act = (scale, zp) one-element device tensors that RECEIVE the parameters of the gated product."""
    M, K = x.shape
    H = w.N // 2
    a_s, a_z = (None, None) if act is None else act
    null = C.c_void_p(0)
    args = (_ptr(x), M, K, x.stride(0), _ptr(w.packed), H, w.bits, w.layout, int(w.signed), _ptr(w.scale), _ptr(w.zp),
            _ptr(w.colsum), _ptr(a_s), _ptr(a_z), _ptr(bias), _ptr(h16), h16.stride(0), _ptr(a8_out), _ptr(out_act[0]),
            _ptr(out_act[1]), null, null, _ptr(ws), C.c_size_t(ws.numel()), _stream())
    return _planned(load().mq_qlinear_a8_geglu_dynamic, "mq_qlinear_a8_geglu_dynamic", args,
                    (x, w, bias, h16, a8_out, out_act, ws, act))


def plan_qlinear_a8_codes(a8, K, act, w: PackedWeight, bias, out, residual=None):
    M = a8.shape[0]
    null = C.c_void_p(0)
    rp, ldr = _res(residual, M, w.N, torch.float16)
    args = (_ptr(a8), M, K, a8.stride(0), _ptr(act[0]), _ptr(act[1]), _ptr(w.packed), w.N, w.bits, w.layout,
            int(w.signed), _ptr(w.scale), _ptr(w.zp), _ptr(w.colsum), _ptr(bias), _ptr(out), out.stride(0), null,
            rp, ldr, _stream())
    return _planned(load().mq_qlinear_a8_codes, "mq_qlinear_a8_codes", args, (a8, act, w, bias, out, residual))


def conv_tap_sums(codes: torch.Tensor, Cin: int, bits: int, codes_signed: bool = False) -> torch.Tensor:
    """codes uint8 [N, 9*Cin] -> int32 [9, N]."""
    N = codes.shape[0]
    assert codes.is_cuda and codes.dtype == torch.uint8 and codes.is_contiguous() and codes.shape[1] == 9 * Cin
    out = torch.empty((9, N), dtype=torch.int32, device=codes.device)
    _check(load().mq_conv_tap_sums(_ptr(codes), N, Cin, bits, int(codes_signed), _ptr(out), _stream()), "mq_conv_tap_sums")
    return out


def _res4(residual, shape):
    if residual is None:
        return C.c_void_p(0)
    assert residual.is_cuda and tuple(residual.shape) == tuple(shape) and residual.is_contiguous()
    assert residual.dtype == torch.float16
    return _ptr(residual)


def _conv_out_hw(H: int, W: int, stride: int):
    assert stride in (1, 2)
    return (H - 1) // stride + 1, (W - 1) // stride + 1


def conv3x3_w_only(x: torch.Tensor, w: PackedWeight, bias=None, out=None, residual=None, stride: int = 1) -> torch.Tensor:
    """x [B,H,W,Cin] fp16 channels-last contiguous; w packed from the [N, 9*Cin] matrix.  Returns y [B,Ho,Wo,N]
    (+ residual of that shape, added before the rounding); stride 1 or 2."""
    assert x.is_cuda and x.dim() == 4 and x.is_contiguous() and x.dtype == torch.float16
    B, H, W, Cin = x.shape
    assert w.K == 9 * Cin
    Ho, Wo = _conv_out_hw(H, W, stride)
    y = out if out is not None else torch.empty((B, Ho, Wo, w.N), dtype=torch.float16, device=x.device)
    assert tuple(y.shape) == (B, Ho, Wo, w.N) and y.is_contiguous()
    _check(load().mq_conv3x3_w_only(_ptr(x), B, H, W, Cin, stride, _ptr(w.packed), w.N, w.bits, w.layout, _ptr(w.scale),
                                    _ptr(w.zp), _ptr(bias), _ptr(y), _res4(residual, y.shape), _stream()),
           "mq_conv3x3_w_only")
    return y


def conv3x3_a8_workspace_bytes(B: int, H: int, W: int, Cin: int) -> int:
    return int(load().mq_conv3x3_a8_workspace_bytes(B, H, W, Cin))


def conv3x3_a8(x, w: PackedWeight, tapsum, act=None, bias=None, out=None, ws=None, want_acc=False, want_act=False,
               residual=None, stride: int = 1):
    """Returns (y [B,Ho,Wo,N], acc int32 [B*Ho*Wo,N] or None, (act_scale, act_zp) or None)."""
    assert x.is_cuda and x.dim() == 4 and x.is_contiguous() and x.dtype == torch.float16
    B, H, W, Cin = x.shape
    assert w.K == 9 * Cin
    Ho, Wo = _conv_out_hw(H, W, stride)
    y = out if out is not None else torch.empty((B, Ho, Wo, w.N), dtype=torch.float16, device=x.device)
    assert tuple(y.shape) == (B, Ho, Wo, w.N) and y.is_contiguous()
    acc = torch.empty((B * Ho * Wo, w.N), dtype=torch.int32, device=x.device) if want_acc else None
    ws = _workspace(conv3x3_a8_workspace_bytes(B, H, W, Cin), x.device, ws)
    a_s, a_z = (None, None) if act is None else act
    so = torch.empty(1, dtype=torch.float32, device=x.device) if want_act else None
    zo = torch.empty(1, dtype=torch.int32, device=x.device) if want_act else None
    _check(load().mq_conv3x3_a8(_ptr(x), B, H, W, Cin, stride, _ptr(w.packed), w.N, w.bits, w.layout, int(w.signed),
                                _ptr(w.scale), _ptr(w.zp), _ptr(w.colsum), _ptr(tapsum), _ptr(a_s), _ptr(a_z), _ptr(bias),
                                _ptr(y), _ptr(acc), _res4(residual, y.shape), _ptr(so), _ptr(zo), _ptr(ws),
                                C.c_size_t(ws.numel()), _stream()), "mq_conv3x3_a8")
    return y, acc, ((so, zo) if want_act else None)


def bos_aware_kv_proj_workspace_bytes(B: int, T: int, K: int) -> int:
    return int(load().mq_bos_aware_kv_proj_workspace_bytes(B, T, K))


def bos_aware_kv_proj(ctx: torch.Tensor, w: PackedWeight, w_f16: Optional[torch.Tensor] = None,
                      bos_out: Optional[torch.Tensor] = None, act=None, bias=None, naive_all_rows: bool = False,
                      out=None, ws=None, want_act=False):
    """ctx [B,T,K] fp16 -> y [B,T,N] fp16; token 0 of each prompt bypasses activation quantisation."""
    assert ctx.is_cuda and ctx.dim() == 3 and ctx.is_contiguous() and ctx.dtype == torch.float16
    B, T, K = ctx.shape
    assert K == w.K
    dev = ctx.device
    y = out if out is not None else torch.empty((B, T, w.N), dtype=torch.float16, device=dev)
    ws = _workspace(bos_aware_kv_proj_workspace_bytes(B, T, K) + split_workspace_bytes(B * T, w.N, K), dev, ws)
    s_out = torch.empty(1, dtype=torch.float32, device=dev) if want_act else None
    z_out = torch.empty(1, dtype=torch.int32, device=dev) if want_act else None
    a_s, a_z = (None, None) if act is None else act
    rc = load().mq_bos_aware_kv_proj(_ptr(ctx), B, T, K, _ptr(w.packed), w.N, w.bits, w.layout, int(w.signed),
                                     _ptr(w.scale), _ptr(w.zp), _ptr(w.colsum), _ptr(w_f16), _ptr(bos_out), _ptr(a_s),
                                     _ptr(a_z), _ptr(bias), _ptr(y), int(naive_all_rows), _ptr(s_out), _ptr(z_out),
                                     _ptr(ws), C.c_size_t(ws.numel()), _stream())
    _check(rc, "mq_bos_aware_kv_proj")
    return y, (s_out, z_out)


# ---------------------------------------------------------------------------------------------------------------
# Pre-marshalled calls.  A serving loop runs the same layer on the same buffers over and over; marshalling two
# dozen arguments in Python each time costs more than some of the kernels.  plan_*() does the marshalling once and
# returns a zero-argument callable that only performs the C call (on the stream that was current at plan time).
# ---------------------------------------------------------------------------------------------------------------

def _planned(fn, what, args, keep):
    def call():
        rc = fn(*args)
        if rc != 0:
            raise MixdqError(rc, what)
    call.keepalive = keep  # the tensors must outlive the plan
    return call


def plan_qlinear_w_only(x, w: PackedWeight, bias, out, residual=None, ws=None):
    """ws: optional workspace (see qlinear_w_only); without one the call never splits its reduction."""
    assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1 and out.shape == (x.shape[0], w.N)
    M, K = x.shape
    rp, ldr = _res(residual, M, w.N, x.dtype)
    args = (_ptr(x), M, K, x.stride(0), _ptr(w.packed), w.N, w.bits, w.layout, _ptr(w.scale), _ptr(w.zp), _ptr(bias),
            _ptr(out), out.stride(0), _dtype_code(x), rp, ldr, *_ws_args(ws), _stream())
    return _planned(load().mq_qlinear_w_only, "mq_qlinear_w_only", args, (x, w, bias, out, residual, ws))


def plan_qlinear_a8(x, w: PackedWeight, bias, out, ws, act=None, residual=None):
    """W8A8 or W4A8 by the weight's bit-width; dynamic activation parameters unless act=(scale, zp) tensors."""
    assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1 and x.dtype == torch.float16
    M, K = x.shape
    a_s, a_z = (None, None) if act is None else act
    null = C.c_void_p(0)
    rp, ldr = _res(residual, M, w.N, torch.float16)
    if w.bits == 8:
        fn, what = load().mq_qlinear_w8a8, "mq_qlinear_w8a8"
        args = (_ptr(x), M, K, x.stride(0), _ptr(w.packed), w.N, w.layout, int(w.signed), _ptr(w.scale), _ptr(w.zp),
                _ptr(w.colsum), _ptr(a_s), _ptr(a_z), _ptr(bias), _ptr(out), out.stride(0), null, rp, ldr, null, null,
                _ptr(ws), C.c_size_t(ws.numel()), _stream())
    else:
        fn, what = (load().mq_qlinear_w4a8, "mq_qlinear_w4a8") if w.bits == 4 else (load().mq_qlinear_w2a8, "mq_qlinear_w2a8")
        args = (_ptr(x), M, K, x.stride(0), _ptr(w.packed), w.N, w.layout, _ptr(w.scale), _ptr(w.zp), _ptr(w.colsum),
                _ptr(a_s), _ptr(a_z), _ptr(bias), _ptr(out), out.stride(0), null, rp, ldr, null, null, _ptr(ws),
                C.c_size_t(ws.numel()), _stream())
    return _planned(fn, what, args, (x, w, bias, out, ws, act, residual))


def plan_bos_aware_kv_proj(ctx, w: PackedWeight, out, ws, w_f16=None, bos_out=None, bias=None, act=None):
    assert ctx.is_cuda and ctx.dim() == 3 and ctx.is_contiguous() and ctx.dtype == torch.float16
    B, T, K = ctx.shape
    a_s, a_z = (None, None) if act is None else act
    null = C.c_void_p(0)
    args = (_ptr(ctx), B, T, K, _ptr(w.packed), w.N, w.bits, w.layout, int(w.signed), _ptr(w.scale), _ptr(w.zp),
            _ptr(w.colsum), _ptr(w_f16), _ptr(bos_out), _ptr(a_s), _ptr(a_z), _ptr(bias), _ptr(out), 0, null, null,
            _ptr(ws), C.c_size_t(ws.numel()), _stream())
    return _planned(load().mq_bos_aware_kv_proj, "mq_bos_aware_kv_proj", args, (ctx, w, out, ws, w_f16, bos_out, bias, act))


# ---------------------------------------------------------------------------------------------------------------
# Bit-width allocation (host arrays, no GPU)
# ---------------------------------------------------------------------------------------------------------------

def _np_ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def alloc_solve(sens, cost, budget: int):
    """Eq. 2 solved exactly.  sens float64 [n_layers, n_choices], cost int64 [n_layers, n_choices].
    Returns (choice int32 [n_layers], objective, cost used); raises MixdqError (code -8) when nothing fits."""
    import numpy as np
    sens = np.ascontiguousarray(sens, np.float64)
    cost = np.ascontiguousarray(cost, np.int64)
    assert sens.ndim == 2 and sens.shape == cost.shape
    n, m = sens.shape
    choice = np.empty(n, np.int32)
    obj = C.c_double(0.0)
    used = C.c_int64(0)
    _check(load().mq_alloc_solve(n, m, _np_ptr(sens), _np_ptr(cost), C.c_int64(int(budget)), _np_ptr(choice),
                                 C.byref(obj), C.byref(used)), "mq_alloc_solve")
    return choice, obj.value, used.value


def alloc_split_budget(budget_all: int, params_content: int, params_quality: int, k: float):
    bc, bq = C.c_int64(0), C.c_int64(0)
    _check(load().mq_alloc_split_budget(C.c_int64(int(budget_all)), C.c_int64(int(params_content)),
                                        C.c_int64(int(params_quality)), C.c_double(k), C.byref(bc), C.byref(bq)),
           "mq_alloc_split_budget")
    return bc.value, bq.value


def alloc_search(sens_content, params_content, sens_quality, params_quality, bits, avg_bits_target: float,
                 delta_avg_bits: float, n_budgets: int, k_lo: float, k_hi: float, n_ratios: int):
    """The budget x ratio scan around Eq. 2.  Returns a dict of arrays over the n_budgets * n_ratios candidates:
    budgets int64 [E,3] (all, content, quality), k [E], feasible [E], objectives [E,2], choice_content [E,n_c],
    choice_quality [E,n_q]."""
    import numpy as np
    sc = np.ascontiguousarray(sens_content, np.float64)
    sq = np.ascontiguousarray(sens_quality, np.float64)
    pc = np.ascontiguousarray(params_content, np.int64)
    pq = np.ascontiguousarray(params_quality, np.int64)
    bits = np.ascontiguousarray(bits, np.int32)
    nc, nq, m = sc.shape[0], sq.shape[0], bits.shape[0]
    assert sc.shape == (nc, m) and sq.shape == (nq, m) and pc.shape == (nc,) and pq.shape == (nq,)
    E = n_budgets * n_ratios
    out = dict(budgets=np.empty((E, 3), np.int64), k=np.empty(E, np.float64), feasible=np.empty(E, np.int32),
               objectives=np.empty((E, 2), np.float64), choice_content=np.empty((E, nc), np.int32),
               choice_quality=np.empty((E, nq), np.int32))
    _check(load().mq_alloc_search(nc, _np_ptr(sc), _np_ptr(pc), nq, _np_ptr(sq), _np_ptr(pq), m, _np_ptr(bits),
                                  C.c_double(avg_bits_target), C.c_double(delta_avg_bits), n_budgets, C.c_double(k_lo),
                                  C.c_double(k_hi), n_ratios, _np_ptr(out["budgets"]), _np_ptr(out["k"]),
                                  _np_ptr(out["feasible"]), _np_ptr(out["objectives"]), _np_ptr(out["choice_content"]),
                                  _np_ptr(out["choice_quality"])), "mq_alloc_search")
    return out

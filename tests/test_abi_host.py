"""Host-only checks of the C ABI: the library loads without a GPU, exports every declared symbol, and
rejects bad arguments before launching anything."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2405_17873_amd as mq
    if not os.path.exists(mq.lib_path()):
        from paper_2405_17873_amd import build
        build.build()
    return mq.load()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "mixdq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mq_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2405_17873_amd import binding
    names = _declared_symbols()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_size_queries(lib):
    import paper_2405_17873_amd as mq
    assert mq.packed_bytes(320, 320, 4, mq.LAYOUT_CANONICAL) == 320 * 160
    assert mq.packed_bytes(40, 128, 16, mq.LAYOUT_KERNEL) == 64 * 128 * 2  # unquantised 16-bit weights, 32-row tiles
    assert mq.packed_bytes(40, 128, 16, mq.LAYOUT_CANONICAL) == 40 * 128 * 2
    assert mq.packed_bytes(320, 320, 3, mq.LAYOUT_CANONICAL) == 320 * 120
    assert mq.packed_bytes(320, 320, 2, mq.LAYOUT_KERNEL) == 320 * 80
    assert mq.packed_bytes(33, 64, 8, mq.LAYOUT_KERNEL) == 64 * 64  # padded to 64 channels
    assert mq.packed_bytes(320, 100, 4, mq.LAYOUT_KERNEL) == 0      # K % 64
    assert mq.packed_bytes(320, 5, 3, mq.LAYOUT_CANONICAL) == 0     # 15 bits is not whole bytes
    assert mq.packed_bytes(320, 320, 5, mq.LAYOUT_CANONICAL) == 0
    assert mq.qlinear_a8_workspace_bytes(4096, 1280) >= 4096 * 1280 + 4 * 4096
    assert mq.bos_aware_kv_proj_workspace_bytes(8, 77, 2048) >= 8 * 77 * 2048
    # split of the reduction: shapes with many tiles or a short reduction never split
    assert mq.split_workspace_bytes(4096, 1280, 1280) == 0 and mq.split_workspace_bytes(64, 1280, 640) == 0
    assert mq.split_workspace_bytes(64, 1280, 5120) >= 16 * 128 * 1280 * 4
    assert mq.split_workspace_bytes(308, 640, 2048) >= 8 * 384 * 640 * 4


def test_error_codes_without_a_gpu(lib):
    """Validation happens on the host, so these calls never reach the device."""
    buf = (C.c_uint8 * 4096)()
    base = C.addressof(buf)
    p = C.c_void_p((base + 255) // 256 * 256)  # aligned fake pointer; never dereferenced: every call below fails first
    null = C.c_void_p(0)
    st = C.c_void_p(0)
    # quantize_weights
    assert lib.mq_quantize_weights(null, 4, 64, 4, 0, 0, p, p, p, st) == -1
    assert lib.mq_quantize_weights(p, 4, 64, 5, 0, 0, p, p, p, st) == -3
    assert lib.mq_quantize_weights(p, 0, 64, 4, 0, 0, p, p, p, st) == -2
    assert lib.mq_quantize_weights(p, 4, 64, 4, 0, 7, p, p, p, st) == -1
    # pack
    assert lib.mq_pack_weights(p, 4, 5, 3, 0, 0, p, null, st) == -2
    assert lib.mq_pack_weights(p, 4, 96, 4, 1, 0, p, null, st) == -2
    assert lib.mq_pack_weights(p, 4, 64, 4, 9, 0, p, null, st) == -6
    assert lib.mq_pack_weights(p, 4, 64, 4, 1, 1, p, null, st) == -1  # signed codes only at 8 bit
    assert lib.mq_pack_weights(p, 4, 64, 16, 1, 0, p, p, st) == -1  # no code sums of unquantised weights
    assert lib.mq_quantize_weights(p, 4, 64, 16, 0, 0, p, p, p, st) == -3
    assert lib.mq_unpack_weights(p, 4, 64, 6, 1, p, st) == -3
    # w_only
    args = lambda **o: [o.get("x", p), o.get("M", 8), o.get("K", 64), o.get("ldx", 64), p, o.get("N", 32),
                        o.get("bits", 4), o.get("layout", 1), p, p, null, p, o.get("ldy", 32), 0, o.get("res", null),
                        o.get("ldr", 0), o.get("ws", null), C.c_size_t(o.get("wsb", 0)), st]
    assert lib.mq_qlinear_w_only(*args(x=null)) == -1
    assert lib.mq_qlinear_w_only(*args(bits=5)) == -3
    assert lib.mq_qlinear_w_only(*args(K=96, ldx=96)) == -2
    assert lib.mq_qlinear_w_only(*args(M=0)) == -2
    assert lib.mq_qlinear_w_only(*args(ldx=32)) == -2
    assert lib.mq_qlinear_w_only(*args(layout=0)) == -6
    assert lib.mq_qlinear_w_only(*args(x=C.c_void_p(p.value + 2))) == -1  # misaligned
    assert lib.mq_qlinear_w_only(*args(res=p, ldr=16)) == -2              # residual rows shorter than N
    assert lib.mq_qlinear_w_only(*args(res=p, ldr=34)) == -2
    assert lib.mq_qlinear_w_only(*args(res=C.c_void_p(p.value + 4), ldr=32)) == -1
    assert lib.mq_qlinear_w_only(*args(ws=C.c_void_p(p.value + 64), wsb=4096)) == -1   # workspace not 256-byte aligned
    # a forced split of the reduction needs its workspace: absent or too small is an error, nothing is launched
    lib.mq_tune_force_splits(4)
    try:
        need = lib.mq_split_workspace_bytes(8, 32, 2048)
        assert need >= 4 * 128 * 128 * 4
        assert lib.mq_qlinear_w_only(*args(K=2048, ldx=2048)) == -4
        assert lib.mq_qlinear_w_only(*args(K=2048, ldx=2048, ws=p, wsb=need - 1)) == -4
    finally:
        lib.mq_tune_force_splits(0)
    # unquantised weights of 2 GiB and more: their byte offsets would not fit 32 bits
    assert lib.mq_qlinear_w_only(*args(M=1, K=40960, ldx=40960, N=32768, ldy=32768, bits=16)) == -2
    # a8
    a8 = lambda **o: [p, 8, o.get("K", 64), o.get("K", 64), p, 32, 1, 1, p, p, o.get("colsum", p),
                      o.get("a_s", null), o.get("a_z", null), null, p, 32, null, o.get("res", null), o.get("ldr", 0), null,
                      null, o.get("ws", p),
                      C.c_size_t(o.get("wsb", 1 << 20)), st]
    assert lib.mq_qlinear_w8a8(*a8(colsum=null)) == -1
    assert lib.mq_qlinear_w8a8(*a8(a_s=p)) == -1       # scale without zero point
    assert lib.mq_qlinear_w8a8(*a8(wsb=16)) == -4
    assert lib.mq_qlinear_w8a8(*a8(K=33088)) == -7     # 255*255*K >= 2^31
    assert lib.mq_qlinear_w8a8(*a8(ws=null)) == -1
    assert lib.mq_qlinear_w8a8(*a8(res=p, ldr=8)) == -2
    # gated projection with dynamic output parameters
    gd = lambda **o: [p, 8, 64, 64, p, o.get("H", 32), 4, 1, 0, p, p, p, null, null, null, o.get("h16", p), o.get("ldh", 32), p,
                      o.get("so", p), o.get("zo", p), null, null, p, C.c_size_t(o.get("wsb", 1 << 20)), st]
    assert lib.mq_qlinear_a8_geglu_dynamic(*gd(h16=null)) == -1     # the fp16 product is not optional here
    assert lib.mq_qlinear_a8_geglu_dynamic(*gd(so=null)) == -1
    assert lib.mq_qlinear_a8_geglu_dynamic(*gd(H=48)) == -2
    assert lib.mq_qlinear_a8_geglu_dynamic(*gd(ldh=16)) == -2
    assert lib.mq_qlinear_a8_geglu_dynamic(*gd(wsb=lib.mq_qlinear_a8_workspace_bytes(8, 64))) == -4
    assert lib.mq_qlinear_a8_geglu_dynamic_workspace_bytes(8, 64, 32) > lib.mq_qlinear_a8_workspace_bytes(8, 64)
    # weight-only gated projection with 8-bit output
    wg = lambda **o: [p, 8, 64, 64, p, o.get("H", 32), o.get("bits", 4), 1, p, p, null, o.get("so", p), p, p, null, 32, st]
    assert lib.mq_qlinear_w_only_geglu_a8(*wg(so=null)) == -1
    assert lib.mq_qlinear_w_only_geglu_a8(*wg(bits=16)) == -3
    assert lib.mq_qlinear_w_only_geglu_a8(*wg(H=40)) == -2
    # bos
    bos = lambda **o: [p, o.get("B", 2), 5, 64, p, 32, o.get("wb", 8), 1, 1, p, p, p, o.get("wf", null),
                       o.get("bo", null), null, null, null, p, 0, null, null, p, C.c_size_t(1 << 20), st]
    assert lib.mq_bos_aware_kv_proj(*bos()) == -1            # neither BOS source
    assert lib.mq_bos_aware_kv_proj(*bos(wf=p, bo=p)) == -1  # both
    assert lib.mq_bos_aware_kv_proj(*bos(wb=3, wf=p)) == -3
    assert lib.mq_bos_aware_kv_proj(*bos(B=0, wf=p)) == -2


def test_microbenchmark_entry_rejects_bad_arguments_without_a_gpu(lib):
    """mq_prof_microbench validates before it touches the device."""
    buf = (C.c_uint8 * 8192)()
    p = C.c_void_p((C.addressof(buf) + 255) // 256 * 256)
    ms = C.c_double(-1.0)
    st = C.c_void_p(0)
    f = lib.mq_prof_microbench
    f.argtypes = [C.c_int, C.c_void_p, C.c_size_t, C.POINTER(C.c_double), C.c_void_p]
    assert f(-1, p, 4096, C.byref(ms), st) == -1
    assert f(9, p, 4096, C.byref(ms), st) == -1          # kinds are 0..8
    assert f(0, p, 4096, None, st) == -1                  # nowhere to write the time
    assert f(0, None, 4096, C.byref(ms), st) == -1
    assert f(0, p, 1024, C.byref(ms), st) == -1           # scratch below 4 KiB
    assert f(0, C.c_void_p(p.value + 8), 4096, C.byref(ms), st) == -1   # not 16-byte aligned
    assert f(7, p, 4096, C.byref(ms), st) == -1           # the L2 -> LDS kind needs 2 MiB to copy from
    assert ms.value == -1.0


def test_missing_library_is_loud(monkeypatch):
    from paper_2405_17873_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libmixdq.so")
    with pytest.raises(RuntimeError):
        binding.load()


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2405_17873_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower().replace("no cpu fallback", ""), f

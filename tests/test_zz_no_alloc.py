"""The entry point for callers that cannot allocate: mq_qlinear_a8_builtin_ws keeps its workspace in a device array of
the library.  Its results must equal those of the entry points that take a workspace, bit for bit, also when the
array still holds a larger previous call's contents."""
import numpy as np
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mq():
    import paper_2405_17873_amd as m
    m.load()
    assert torch.cuda.is_available()
    return m


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def make(mq, seed, N, K, bits, sym=False):
    w = dev(si.weights_f16(seed, f"na/w{N}x{K}", N, K))
    c, s, z = mq.quantize_weights(w, bits, sym)
    p, cs = mq.pack_weights(c, bits, mq.LAYOUT_KERNEL, codes_signed=sym)
    return mq.PackedWeight(p, s, z, cs, N, K, bits, mq.LAYOUT_KERNEL, sym)


def test_builtin_workspace_matches_caller_workspace_two_calls_in_a_row(mq, orc):
    """First a large problem (fills 5.4 MB of the array), then a smaller one on the same array, each against the entry
    point that takes a caller workspace (int32 accumulators, dynamic parameters and every output bit) and the first
    also against the oracle; then static parameters, a residual and the other bit-widths."""
    fns = {8: mq.qlinear_w8a8, 4: mq.qlinear_w4a8, 2: mq.qlinear_w2a8}
    cases = [(4096, 1280, 640, 4, False), (300, 640, 264, 4, False), (77, 128, 40, 8, True), (608, 2048, 640, 2, False),
             (1, 64, 8, 8, False)]
    for i, (M, K, N, bits, sym) in enumerate(cases):
        xh = si.activations_f16(70 + i, f"na/x{M}x{K}", M, K, outlier_prob=0.01)
        x = dev(xh)
        b = dev(si.bias_f16(70 + i, f"na/b{N}", N))
        pw = make(mq, 70 + i, N, K, bits, sym)
        y, acc, (s, z) = mq.qlinear_a8_builtin_ws(x, pw, bias=b, want_acc=True, want_act=True)
        ry, racc, (rs, rz) = fns[bits](x, pw, bias=b, want_acc=True, want_act=True)
        torch.cuda.synchronize()
        assert torch.equal(s, rs) and torch.equal(z, rz), f"case {i}: dynamic parameters"
        assert torch.equal(acc, racc), f"case {i}: accumulators"
        assert torch.equal(y, ry), f"case {i}: outputs"
        if i == 1:
            oc, os_, oz = orc.quantize_weights(si.weights_f16(70 + i, f"na/w{N}x{K}", N, K), bits, sym)
            _, oacc, (o_s, o_z) = orc.linear_a8(xh, oc, os_, oz, w_signed=sym, bias=b.cpu().numpy())
            assert np.array_equal(acc.cpu().numpy(), oacc) and s.item() == o_s and z.item() == o_z
        # static parameters and a residual, into a caller-provided output (nothing is allocated on either side)
        act = (dev(np.array([0.03], np.float32)), dev(np.array([117], np.int32)))
        res = dev(si.activations_f16(90 + i, f"na/r{M}x{N}", M, N))
        out = torch.empty((M, N), dtype=torch.float16, device="cuda")
        mq.qlinear_a8_builtin_ws(x, pw, act=act, bias=b, out=out, residual=res)
        ry2, _, _ = fns[bits](x, pw, act=act, bias=b, residual=res)
        torch.cuda.synchronize()
        assert torch.equal(out, ry2), f"case {i}: static parameters + residual"


def test_builtin_workspace_limit_is_an_error(mq):
    assert mq.builtin_workspace_bytes() == 48 << 20
    M, K = 16384, 5120          # 84 MB of int8 activations: beyond the array
    assert mq.qlinear_a8_workspace_bytes(M, K) > mq.builtin_workspace_bytes()
    x = torch.zeros((8, K), dtype=torch.float16, device="cuda")
    pw = make(mq, 79, 64, K, 4)
    import ctypes as C
    from paper_2405_17873_amd import binding as bd
    null = C.c_void_p(0)
    y = torch.empty((8, 64), dtype=torch.float16, device="cuda")
    rc = bd.load().mq_qlinear_a8_builtin_ws(bd._ptr(x), M, K, K, bd._ptr(pw.packed), 64, 4, 1, 0, bd._ptr(pw.scale),
                                            bd._ptr(pw.zp), bd._ptr(pw.colsum), null, null, null, bd._ptr(y), 64, null,
                                            null, 0, null, null, null)
    assert rc == -4
    # the largest configured activation tensor (16384 x 2560) fits
    assert mq.qlinear_a8_workspace_bytes(16384, 2560) <= mq.builtin_workspace_bytes()

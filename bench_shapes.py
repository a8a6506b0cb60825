#!/usr/bin/env python3
"""Per-shape report of the quantized-linear hot path on one MI355X (a table, not the one-line benchmark).

For every configured layer shape and mode it prints the time per call, the achieved op rate and algorithmic byte rate,
the two roofline times (HBM at 8 TB/s, dense MFMA at 2.5 PFLOP/s fp16 / 5.0 POP/s int8), which of them binds, and
the fraction  max(t_HBM, t_MFMA) / t_measured.

Timing: calls are issued back to back on one stream and timed as a whole with one event pair (N calls / elapsed), so
the figure is the throughput a pipeline of such layers sees, launch cost included.  Every call of the loop uses its
own set of buffers (activations, packed weights, outputs), and the sets together exceed the 256 MB last-level cache, so
no call finds its operands cached by the previous one.  The A8 rows include the activation min/max and quantise
kernels ("dyn") or the quantise kernel only ("static"); the "kernel" column is the library's own event timing of the
GEMM kernel alone (bracket cost subtracted).

Algorithmic bytes per call: X once (2 M K) + packed weights (N K bits / 8) + 10 N (scale, zero point, bias) + Y once
(2 M N); ops = 2 M N K.

The last two columns repeat the two fractions against what THIS machine reaches in microbenchmarks run at the start
(mq_prof_microbench: MFMA-only loops for the two operand types, a read-only stream over 2 GiB), printed in the header:
the published peaks assume a clock the chip does not hold under load.
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM = 8000e9
PEAK = {"w": 2500e12, "a": 5000e12}
LLC_BYTES = 320 << 20


def shapes():
    S = []
    # (label, M, K, N, modes)   modes: w<bits> weight-only (w16: the layer kept at fp16), a4/a8 dynamic, s4/s8 static
    # activation parameters, bos<bits> the BOS-aware K/V projection
    S.append(("c1", 256, 320, 320, ("w4", "a8sym")))
    for (K, N) in ((640, 640), (640, 5120), (2560, 640)):
        S.append(("c2", 4096, K, N, ("w16", "w8", "w4", "w3", "w2")))
    for (K, N) in ((1280, 1280), (1280, 10240), (5120, 1280)):
        S.append(("c3", 4096, K, N, ("a4", "a2", "a8sym", "s4", "w4", "w16")))
    for N in (640, 1280):
        S.append(("c4", 8 * 77, 2048, N, ("bos8", "bos4")))
    for (K, N) in ((640, 640), (640, 5120), (2560, 640)):
        S.append(("c5", 16384, K, N, ("w4", "w2", "a4")))
    S.append(("c5", 4 * 77, 2048, 1280, ("w4", "bos4")))
    for M in (1, 4, 16, 64, 77):
        for (K, N) in ((1280, 1280), (1280, 10240), (5120, 1280), (2048, 1280)):
            S.append(("small-M", M, K, N, ("w8", "w4", "w2")))
    return S


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--iters", type=int, default=200)
    ap.add_argument("--only", default="", help="comma-separated labels (c1,c2,c3,c4,c5,small-M,ff,conv,qkv,kvall)")
    ap.add_argument("--tile", type=int, default=-1, help="force a tile of the GEMM's tile table (-1: the library's choice)")
    ap.add_argument("--band", type=int, default=0, help="force the band height of the workgroup -> tile map (0: the library's choice)")
    ap.add_argument("--modes", default="", help="comma-separated modes to keep (w4,a4,a8sym,...); empty: all")
    ap.add_argument("--no-peaks", action="store_true", help="skip the microbenchmarks (measured-peak columns read 0)")
    args = ap.parse_args()

    import torch

    import paper_2405_17873_amd as mq
    mq.load()
    mq.tune_force_tile(args.tile)
    mq.tune_force_band(args.band)
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(0)
    overhead_us = mq.prof_bracket_overhead_us()
    only = set(filter(None, args.only.split(",")))
    keep_modes = set(filter(None, args.modes.split(",")))
    mpk = None
    if not args.no_peaks:
        mpk = mq.machine_peaks()
        print(f"# measured on this machine: int8 MFMA {mpk['int8_TOPs']:.0f} TOP/s, fp16 MFMA {mpk['f16_TFLOPs']:.0f} TFLOP/s, "
              f"read-only stream {mpk['read_GBps']:.0f} GB/s, LDS reads {mpk['lds_read_TBps']:.1f} TB/s, L2 -> LDS copies "
              f"{mpk['l2_to_lds_TBps']:.1f} TB/s; 8 vector instructions per MFMA: matrix and vector "
              f"instructions together take {mpk['serial_share_same_wave']:.2f} (one wave) / {mpk['serial_share_two_waves']:.2f} "
              f"(two waves of a SIMD) of the sum of their separate times (0.50 = full overlap, 1.00 = none); 4 per MFMA: "
              f"{mpk['four_valu_per_mfma_over_mfma_only']:.2f} of the time of the MFMAs alone")
        torch.cuda.empty_cache()
    m_hbm = mpk["read_GBps"] * 1e9 if mpk else 0.0
    m_peak = {"w": mpk["f16_TFLOPs"] * 1e12, "a": mpk["int8_TOPs"] * 1e12} if mpk else {"w": 0.0, "a": 0.0}

    if args.tile >= 0:
        print(f"# tile {args.tile} forced")
    print(f"# per-shape report, {torch.cuda.get_device_name(0)}; iters per row {args.iters}; "
          f"event-bracket cost subtracted from the kernel column: {overhead_us:.2f} us")
    print(f"{'cfg':8s}{'M':>6s}{'K':>6s}{'N':>6s} {'mode':7s}{'us/call':>9s}{'kernel us':>10s}{'T(FL)OP/s':>10s}"
          f"{'GB/s':>8s}{'t_HBM us':>9s}{'t_MFMA us':>10s} {'binds':5s}{'frac':>6s}{'k.frac':>7s}{'m.frac':>7s}{'m.kfrac':>8s}")

    for (cfg, M, K, N, modes) in shapes():
        if only and cfg not in only:
            continue
        for mode in modes:
            if keep_modes and mode not in keep_modes:
                continue
            bos = mode.startswith("bos")
            sym = mode.endswith("sym")
            kind = "w" if mode[0] == "w" else "a"
            bits = int(mode[3:]) if bos else (16 if mode == "w16" else int(mode.replace("sym", "")[-1]))
            xbytes = 2 * M * K
            wbytes = N * K * bits // 8
            alg_bytes = xbytes + wbytes + 10 * N + 2 * M * N
            ops = 2.0 * M * N * K
            nsets = max(2, min(args.iters, -(-LLC_BYTES // (alg_bytes + (M * K if kind == "a" else 0)))))
            sets = []
            ws = None
            for _ in range(nsets):
                w = (torch.randn(N, K, generator=gen, device=dev) * 0.02).half()
                if bits == 16:
                    pw = mq.keep_weights_16bit(w)
                else:
                    c, s, z = mq.quantize_weights(w, bits, sym)
                    p, cs = mq.pack_weights(c, bits, mq.LAYOUT_KERNEL, codes_signed=sym)
                    pw = mq.PackedWeight(p, s, z, cs, N, K, bits, mq.LAYOUT_KERNEL, sym)
                bias = (torch.randn(N, generator=gen, device=dev) * 0.01).half()
                if bos:
                    B, T = M // 77, 77
                    x = torch.randn(B, T, K, generator=gen, device=dev)
                    x[:, 0, :16] *= 60.0
                    x = x.half()
                    y = torch.empty(B, T, N, dtype=torch.float16, device=dev)
                    ws = ws if ws is not None else torch.empty(mq.bos_aware_kv_proj_workspace_bytes(B, T, K) +
                                                                mq.split_workspace_bytes(M, N, K),
                                                                dtype=torch.uint8, device=dev)
                    sets.append(mq.plan_bos_aware_kv_proj(x, pw, y, ws, w_f16=w, bias=bias))
                    continue
                del w
                x = torch.randn(M, K, generator=gen, device=dev).half()
                y = torch.empty(M, N, dtype=torch.float16, device=dev)
                if kind == "w":
                    need = mq.split_workspace_bytes(M, N, K)
                    ws = ws if ws is not None or not need else torch.empty(need, dtype=torch.uint8, device=dev)
                    sets.append(mq.plan_qlinear_w_only(x, pw, bias, y, ws=ws))
                else:
                    ws = ws if ws is not None else torch.empty(mq.qlinear_a8_workspace_bytes(M, K) +
                                                                mq.split_workspace_bytes(M, N, K), dtype=torch.uint8,
                                                                device=dev)
                    act = None
                    if mode[0] == "s":
                        act = (torch.tensor([8.0 / 255], device=dev), torch.tensor([128], dtype=torch.int32, device=dev))
                    sets.append(mq.plan_qlinear_a8(x, pw, bias, y, ws, act=act))
            for i in range(min(nsets, 8)):
                sets[i]()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(args.iters):
                sets[i % nsets]()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / args.iters
            # the GEMM kernel alone, from the library's event brackets
            mq.prof_reset()
            mq.prof_filter(-1, 1)
            mq.prof_enable(True)
            for i in range(min(args.iters, 50)):
                sets[i % nsets]()
            torch.cuda.synchronize()
            mq.prof_enable(False)
            ker = [k for k in mq.prof_read() if "gemm_kernel" in k["kernel"]]
            k_us = sum(k["ms"] for k in ker) * 1e3 / max(1, sum(k["launches"] for k in ker)) - overhead_us if ker else 0.0
            k_us = max(k_us, 0.05)
            t_hbm = alg_bytes / HBM * 1e6
            t_mfma = ops / PEAK[kind] * 1e6
            bind = "HBM" if t_hbm >= t_mfma else "MFMA"
            t_meas = max(alg_bytes / m_hbm, ops / m_peak[kind]) * 1e6 if mpk else 0.0   # against the measured rates
            print(f"{cfg:8s}{M:6d}{K:6d}{N:6d} {mode:7s}{us:9.2f}{k_us:10.2f}{ops / us / 1e6:10.1f}"
                  f"{alg_bytes / us / 1e3:8.0f}{t_hbm:9.2f}{t_mfma:10.2f} {bind:5s}{max(t_hbm, t_mfma) / us:6.3f}"
                  f"{max(t_hbm, t_mfma) / k_us:7.3f}{t_meas / us:7.3f}{t_meas / k_us:8.3f}", flush=True)
            del sets
            torch.cuda.empty_cache()
    if not only or "ff" in only:
        ff_pairs(mq, torch, min(args.iters, 100), overhead_us)
    if not only or "conv" in only:
        convs(mq, torch, min(args.iters, 100), overhead_us)
    if not only or "qkv" in only:
        stacked_qkv(mq, torch, min(args.iters, 120))
    if not only or "kvall" in only:
        all_kv_projections(mq, torch, min(args.iters, 40))
    if not only or "c4" in only or "boserr" in only:
        bos_error_report(mq, torch)


def ff_pairs(mq, torch, iters, overhead_us):
    """Feed-forward block of a transformer layer, C -> 8C -> (GEGLU) -> 4C -> C, W4A8 with static activation
    parameters: the fused pair (gated projection that emits 8-bit codes + output linear on codes: 3 kernels) against
    the same two linears through the ordinary entry points (fp16 8C-wide tensor out, fp16 4C-wide tensor in, both
    with static parameters: 4 kernels; the GEGLU kernel that a framework would run between them is NOT included)."""
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(1)
    print("\n# feed-forward pair, W4A8, static activation parameters: us per block (both linears), cold operands")
    print(f"{'M':>6s}{'C':>6s} {'fused us':>9s}{'separate us':>12s}{'T OP/s fused':>13s}{'t_MFMA us':>10s}{'frac':>6s}")
    for (M, Cc) in ((4096, 1280), (16384, 640)):
        ops = 2.0 * M * Cc * 8 * Cc + 2.0 * M * 4 * Cc * Cc
        per_set = 2 * M * Cc + 4 * Cc * Cc + M * 4 * Cc * 2 + 2 * Cc * Cc + 2 * M * Cc
        nsets = max(2, min(iters, -(-LLC_BYTES // per_set)))
        fused, sep = [], []
        sc = lambda v: torch.tensor([v], dtype=torch.float32, device=dev)
        zi = lambda v: torch.tensor([v], dtype=torch.int32, device=dev)
        act_in, act_mid = (sc(8.0 / 255), zi(128)), (sc(0.01), zi(20))
        ws = torch.empty(max(mq.qlinear_a8_workspace_bytes(M, Cc), mq.qlinear_a8_workspace_bytes(M, 4 * Cc)),
                         dtype=torch.uint8, device=dev)
        for _ in range(nsets):
            packs = []
            for (N, K) in ((8 * Cc, Cc), (Cc, 4 * Cc)):
                w = (torch.randn(N, K, generator=gen, device=dev) * 0.02).half()
                c, s_, z = mq.quantize_weights(w, 4)
                p, cs = mq.pack_weights(c, 4, mq.LAYOUT_KERNEL)
                packs.append(mq.PackedWeight(p, s_, z, cs, N, K, 4, mq.LAYOUT_KERNEL, False))
                del w, c
            x = torch.randn(M, Cc, generator=gen, device=dev).half()
            a8 = torch.empty((M, mq.a8_row_bytes(4 * Cc)), dtype=torch.int8, device=dev)
            y = torch.empty(M, Cc, dtype=torch.float16, device=dev)
            f1 = mq.plan_qlinear_a8_geglu(x, packs[0], act_mid, None, a8, ws, act=act_in)
            f2 = mq.plan_qlinear_a8_codes(a8, 4 * Cc, act_mid, packs[1], None, y)
            fused.append((f1, f2))
            y8 = torch.empty(M, 8 * Cc, dtype=torch.float16, device=dev)
            s1 = mq.plan_qlinear_a8(x, packs[0], None, y8, ws, act=act_in)
            s2 = mq.plan_qlinear_a8(y8[:, :4 * Cc], packs[1], None, y, ws, act=act_mid)
            sep.append((s1, s2))
        res = []
        for calls in (fused, sep):
            for i in range(min(nsets, 4)):
                calls[i][0](), calls[i][1]()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(iters):
                calls[i % nsets][0](), calls[i % nsets][1]()
            e1.record()
            torch.cuda.synchronize()
            res.append(e0.elapsed_time(e1) * 1e3 / iters)
        t_mfma = ops / PEAK["a"] * 1e6
        print(f"{M:6d}{Cc:6d} {res[0]:9.2f}{res[1]:12.2f}{ops / res[0] / 1e6:13.1f}{t_mfma:10.2f}{t_mfma / res[0]:6.3f}",
              flush=True)
        del fused, sep
    # the same pair with DYNAMIC parameters of the activation between the two linears (and of the input)
    print("\n# feed-forward pair, W4A8, dynamic activation parameters: us per block, cold operands; fused = gated "
          "projection that leaves the fp16 product with its range + quantise + linear on codes; separate = two ordinary "
          "dynamic calls (8C-wide fp16 tensor in between, GEGLU kernel not included)")
    print(f"{'M':>6s}{'C':>6s} {'fused us':>9s}{'separate us':>12s}")
    for (M, Cc) in ((4096, 1280), (16384, 640)):
        per_set = 2 * M * Cc + 4 * Cc * Cc + M * 4 * Cc * 2 + 2 * Cc * Cc + 2 * M * Cc + M * 8 * Cc * 2
        nsets = max(2, min(iters, -(-LLC_BYTES // per_set)))
        fused, sep = [], []
        ws = torch.empty(max(mq.qlinear_a8_geglu_dynamic_workspace_bytes(M, Cc, 4 * Cc),
                             mq.qlinear_a8_workspace_bytes(M, 4 * Cc)), dtype=torch.uint8, device=dev)
        for _ in range(nsets):
            packs = []
            for (N, K) in ((8 * Cc, Cc), (Cc, 4 * Cc)):
                w = (torch.randn(N, K, generator=gen, device=dev) * 0.02).half()
                c, s_, z = mq.quantize_weights(w, 4)
                p, cs = mq.pack_weights(c, 4, mq.LAYOUT_KERNEL)
                packs.append(mq.PackedWeight(p, s_, z, cs, N, K, 4, mq.LAYOUT_KERNEL, False))
                del w, c
            x = torch.randn(M, Cc, generator=gen, device=dev).half()
            a8 = torch.empty((M, mq.a8_row_bytes(4 * Cc)), dtype=torch.int8, device=dev)
            h16 = torch.empty(M, 4 * Cc, dtype=torch.float16, device=dev)
            y = torch.empty(M, Cc, dtype=torch.float16, device=dev)
            mid = (torch.empty(1, dtype=torch.float32, device=dev), torch.empty(1, dtype=torch.int32, device=dev))
            f1 = mq.plan_qlinear_a8_geglu_dynamic(x, packs[0], None, h16, a8, mid, ws)
            f2 = mq.plan_qlinear_a8_codes(a8, 4 * Cc, mid, packs[1], None, y)
            fused.append((f1, f2))
            y8 = torch.empty(M, 8 * Cc, dtype=torch.float16, device=dev)
            s1 = mq.plan_qlinear_a8(x, packs[0], None, y8, ws)
            s2 = mq.plan_qlinear_a8(y8[:, :4 * Cc], packs[1], None, y, ws)
            sep.append((s1, s2))
        res = []
        for calls in (fused, sep):
            for i in range(min(nsets, 4)):
                calls[i][0](), calls[i][1]()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(iters):
                calls[i % nsets][0](), calls[i % nsets][1]()
            e1.record()
            torch.cuda.synchronize()
            res.append(e0.elapsed_time(e1) * 1e3 / iters)
        print(f"{M:6d}{Cc:6d} {res[0]:9.2f}{res[1]:12.2f}", flush=True)
        del fused, sep
        torch.cuda.empty_cache()


def convs(mq, torch, iters, overhead_us):
    """3x3 convolutions of the UNet's residual blocks and its two downsamplers (stride 2) at latent 128x128, batch 4
    (channels-last), W4A16 and W4A8."""
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(2)
    print("\n# 3x3 convolution (padding 1), cold operands; ops = 2 M N 9 Cin over the M output pixels, bytes = x once + "
          "weights + y once")
    print(f"{'B':>3s}{'H':>5s}{'W':>5s}{'Cin':>6s}{'N':>6s}{'str':>4s} {'mode':5s}{'us/call':>9s}{'T(FL)OP/s':>10s}{'GB/s':>8s}{'t_HBM us':>9s}"
          f"{'t_MFMA us':>10s}{'frac':>7s}")
    for (B, H, W, Cin, N, stride) in ((4, 128, 128, 320, 320, 1), (4, 64, 64, 640, 640, 1), (4, 32, 32, 1280, 1280, 1),
                                      (4, 32, 32, 2560, 1280, 1), (4, 128, 128, 320, 320, 2), (4, 64, 64, 640, 640, 2)):
        Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
        M = B * Ho * Wo
        ops = 2.0 * M * N * 9 * Cin
        alg = 2 * B * H * W * Cin + N * 9 * Cin // 2 + 10 * N + 2 * M * N
        nsets = max(2, min(iters, -(-LLC_BYTES // alg)))
        for mode in ("w4", "a4"):
            calls = []
            ws = torch.empty(mq.conv3x3_a8_workspace_bytes(B, H, W, Cin), dtype=torch.uint8, device=dev)
            for _ in range(nsets):
                w = (torch.randn(N, 9 * Cin, generator=gen, device=dev) * 0.02).half()
                c, s_, z = mq.quantize_weights(w, 4)
                p, cs = mq.pack_weights(c, 4, mq.LAYOUT_KERNEL)
                pw = mq.PackedWeight(p, s_, z, cs, N, 9 * Cin, 4, mq.LAYOUT_KERNEL, False)
                ts = mq.conv_tap_sums(c, Cin, 4)
                del w, c
                x = torch.randn(B, H, W, Cin, generator=gen, device=dev).half()
                y = torch.empty(B, Ho, Wo, N, dtype=torch.float16, device=dev)
                if mode == "w4":
                    calls.append(lambda x=x, pw=pw, y=y: mq.conv3x3_w_only(x, pw, out=y, stride=stride))
                else:
                    calls.append(lambda x=x, pw=pw, ts=ts, y=y: mq.conv3x3_a8(x, pw, ts, out=y, ws=ws, stride=stride))
            for i in range(min(nsets, 4)):
                calls[i]()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(iters):
                calls[i % nsets]()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / iters
            t_hbm, t_mfma = alg / HBM * 1e6, ops / PEAK["w" if mode == "w4" else "a"] * 1e6
            print(f"{B:3d}{H:5d}{W:5d}{Cin:6d}{N:6d}{stride:4d} {mode:5s}{us:9.2f}{ops / us / 1e6:10.1f}{alg / us / 1e3:8.0f}{t_hbm:9.2f}"
                  f"{t_mfma:10.2f}{max(t_hbm, t_mfma) / us:7.3f}", flush=True)
            del calls
            torch.cuda.empty_cache()


def stacked_qkv(mq, torch, iters):
    """The q, k, v projections of a self-attention block (same input, three C x C weights) as three calls and as one
    call on the stacked weight (binding.stack_weights): W4A16 and W4A8 with dynamic activation parameters."""
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(3)
    print("\n# q, k, v projections of one block: three calls against one call on the stacked weight, cold operands")
    print(f"{'M':>6s}{'C':>6s} {'mode':5s}{'3 calls us':>11s}{'stacked us':>11s}")
    for (M, Cc) in ((4096, 1280), (16384, 640)):
        per_set = 2 * M * Cc + 3 * Cc * Cc // 2 + 3 * 2 * M * Cc
        nsets = max(2, min(iters // 3, -(-LLC_BYTES // per_set)))
        for mode in ("w4", "a4"):
            sets = []
            ws = torch.empty(mq.qlinear_a8_workspace_bytes(M, Cc), dtype=torch.uint8, device=dev)
            for _ in range(nsets):
                parts = []
                for _i in range(3):
                    w = (torch.randn(Cc, Cc, generator=gen, device=dev) * 0.02).half()
                    c, s_, z = mq.quantize_weights(w, 4)
                    p, cs = mq.pack_weights(c, 4, mq.LAYOUT_KERNEL)
                    parts.append(mq.PackedWeight(p, s_, z, cs, Cc, Cc, 4, mq.LAYOUT_KERNEL, False))
                    del w, c
                x = torch.randn(M, Cc, generator=gen, device=dev).half()
                y3 = [torch.empty(M, Cc, dtype=torch.float16, device=dev) for _i in range(3)]
                y1 = torch.empty(M, 3 * Cc, dtype=torch.float16, device=dev)
                st = mq.stack_weights(parts)
                if mode == "w4":
                    three = [mq.plan_qlinear_w_only(x, p, None, y) for p, y in zip(parts, y3)]
                    one = mq.plan_qlinear_w_only(x, st, None, y1)
                else:
                    three = [mq.plan_qlinear_a8(x, p, None, y, ws) for p, y in zip(parts, y3)]
                    one = mq.plan_qlinear_a8(x, st, None, y1, ws)
                sets.append((three, one))
            res = []
            for which in (0, 1):
                run = (lambda s: [f() for f in s[0]]) if which == 0 else (lambda s: s[1]())
                for i in range(min(nsets, 3)):
                    run(sets[i])
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                n = max(nsets, iters // 3)
                e0.record()
                for i in range(n):
                    run(sets[i % nsets])
                e1.record()
                torch.cuda.synchronize()
                res.append(e0.elapsed_time(e1) * 1e3 / n)
            print(f"{M:6d}{Cc:6d} {mode:5s}{res[0]:11.2f}{res[1]:11.2f}", flush=True)
            del sets
            torch.cuda.empty_cache()




def bos_error_report(mq, torch):
    """What keeping the BOS row out of activation quantisation buys at the eight-prompt size: output error on tokens
    1..76 of the BOS-aware call and of the naive all-row call, both against the unquantised layer (fp16 weights, fp32
    accumulation: the library's own 16-bit path), as relative Frobenius error.  Weight bit-width 8 (symmetric) and 4."""
    import synth_inputs as si
    dev = torch.device("cuda:0")
    B, T, K = 8, 77, 2048
    ctx = torch.from_numpy(si.bos_context_f16(0, "c4/ctx", B, T, K)).to(dev)
    print("\n# BOS-aware against naive all-row activation quantisation, eight prompts [8,77,2048]: relative Frobenius error on "
          "tokens 1..76 against the unquantised layer; activation scale of each")
    print(f"{'N':>6s} {'w bits':>7s}{'err BOS-aware':>15s}{'err naive':>12s}{'ratio':>8s}{'s_x BOS-aware':>15s}{'s_x naive':>11s}")
    for N in (640, 1280):
        w = torch.from_numpy(si.weights_f16(0, f"c4/w{N}", N, K)).to(dev)
        ref = mq.qlinear_w_only(ctx.view(B * T, K), mq.keep_weights_16bit(w)).view(B, T, N)[:, 1:].float()
        for bits, sym in ((8, True), (4, False)):
            c, s_, z = mq.quantize_weights(w, bits, sym)
            p, cs = mq.pack_weights(c, bits, mq.LAYOUT_KERNEL, codes_signed=sym)
            pw = mq.PackedWeight(p, s_, z, cs, N, K, bits, mq.LAYOUT_KERNEL, sym)
            y1, (s1, _) = mq.bos_aware_kv_proj(ctx, pw, w_f16=w, want_act=True)
            y2, (s2, _) = mq.bos_aware_kv_proj(ctx, pw, naive_all_rows=True, want_act=True)
            e1 = ((y1[:, 1:].float() - ref).norm() / ref.norm()).item()
            e2 = ((y2[:, 1:].float() - ref).norm() / ref.norm()).item()
            print(f"{N:6d} {bits:7d}{e1:15.4f}{e2:12.4f}{e2 / e1:8.1f}{s1.item():15.5f}{s2.item():11.5f}", flush=True)


def all_kv_projections(mq, torch, iters):
    """Every cross-attention K and V projection of the UNet reads the same text context, so all of them can run as
    one stacked layer before the first block: 10 blocks at 640 channels and 60 at 1280 give N = 166 400 output
    channels over K = 2048, 341 M weights.  With M = 77 (one prompt) or 308 (four) this is the one SDXL shape that is
    bound by the weight stream from HBM; packed weights of consecutive calls differ, so nothing is cached.
    Modes: w<bits> weight-only, bos<bits> the BOS-aware projection (pre-computed BOS rows, dynamic parameters)."""
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(4)
    N, K = 10 * 2 * 640 + 60 * 2 * 1280, 2048
    print("\n# all K/V projections of the UNet as one stacked layer (N = 166400, K = 2048), weights from HBM")
    print(f"{'M':>6s} {'mode':6s}{'us/call':>9s}{'W MB':>8s}{'GB/s':>8s}{'of 8 TB/s':>10s}{'T(FL)OP/s':>10s}")
    for bits, sym in ((8, True), (4, False), (2, False)):
        sets = []
        for _ in range(2 if bits == 8 else 3):
            w = (torch.randn(N, K, generator=gen, device=dev) * 0.02).half()
            c, s_, z = mq.quantize_weights(w, bits, sym)
            pk, cs = mq.pack_weights(c, bits, mq.LAYOUT_KERNEL, codes_signed=sym)
            sets.append(mq.PackedWeight(pk, s_, z, cs, N, K, bits, mq.LAYOUT_KERNEL, sym))
            del w, c
        wbytes = N * K * bits / 8
        bos_out = torch.zeros(N, dtype=torch.float16, device=dev)
        for B in (1, 4):
            M = B * 77
            ctx = torch.randn(B, 77, K, generator=gen, device=dev).half()
            y = torch.empty(B, 77, N, dtype=torch.float16, device=dev)
            ws = torch.empty(mq.bos_aware_kv_proj_workspace_bytes(B, 77, K), dtype=torch.uint8, device=dev)
            for mode in ("w", "bos"):
                if mode == "w":
                    fns = [mq.plan_qlinear_w_only(ctx.view(M, K), pw, None, y.view(M, N)) for pw in sets]
                else:
                    fns = [mq.plan_bos_aware_kv_proj(ctx, pw, y, ws, bos_out=bos_out) for pw in sets]
                for f in fns:
                    f()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for i in range(iters):
                    fns[i % len(fns)]()
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / iters
                tot = wbytes + 10 * N + (2 if mode == "w" else 3) * M * K + 2 * M * N
                print(f"{M:6d} {mode + str(bits):6s}{us:9.1f}{wbytes / 1e6:8.1f}{tot / us / 1e3:8.0f}{tot / us / 1e6 / 8:10.3f}"
                      f"{2.0 * M * N * K / us / 1e6:10.1f}", flush=True)
        del sets
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()

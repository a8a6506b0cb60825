"""Seeded synthetic inputs shaped like the SDXL-turbo UNet's linear layers.

This module holds no arithmetic of the quantisation method: only a counter-based
random number generator, value recipes and the layer shape tables.  Both the CPU
oracle's tests and the HIP path's tests/benchmark draw their inputs from here, so
the two sides see identical bytes.

Generator: splitmix64 finaliser applied to a counter keyed by (seed, tensor_id,
element index); two 32-bit halves feed Box-Muller.  Values are rounded to fp16 on
the host (numpy's round-to-nearest-even conversion).
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _splitmix64(x: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        x = (x + np.uint64(0x9E3779B97F4A7C15)) & _M64
        z = x
        z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _M64
        z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _M64
        return z ^ (z >> np.uint64(31))


def tensor_id(name: str) -> int:
    """Stable 32-bit id of a tensor role name."""
    return zlib.crc32(name.encode())


def _key(seed: int, tid: int) -> np.uint64:
    k = _splitmix64(np.array([(seed & 0xFFFFFFFF) << 32 | (tid & 0xFFFFFFFF)], np.uint64))[0]
    return k


def raw_u64(seed: int, name: str, n: int, offset: int = 0) -> np.ndarray:
    key = _key(seed, tensor_id(name))
    idx = np.arange(offset, offset + n, dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _splitmix64(key ^ (idx * np.uint64(0xD1342543DE82EF95) & _M64))


def uniform01(seed: int, name: str, n: int) -> np.ndarray:
    """n doubles in (0,1)."""
    r = raw_u64(seed, name, n)
    return ((r >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed: int, name: str, shape, std: float = 1.0) -> np.ndarray:
    """float64 N(0, std^2) of the given shape (Box-Muller on two 32-bit halves)."""
    n = int(np.prod(shape))
    r = raw_u64(seed, name, n)
    u1 = ((r >> np.uint64(32)).astype(np.float64) + 0.5) * (1.0 / 4294967296.0)
    u2 = ((r & np.uint64(0xFFFFFFFF)).astype(np.float64) + 0.5) * (1.0 / 4294967296.0)
    g = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return (g * std).reshape(shape)


def normal_f16(seed: int, name: str, shape, std: float = 1.0) -> np.ndarray:
    return normal(seed, name, shape, std).astype(np.float16)


def activations_f16(seed: int, name: str, M: int, K: int, outlier_prob: float = 0.0,
                    outlier_gain: float = 10.0) -> np.ndarray:
    """X ~ N(0,1); each entry multiplied by outlier_gain with probability outlier_prob."""
    x = normal(seed, name, (M, K))
    if outlier_prob > 0.0:
        u = uniform01(seed, name + "/outlier", M * K).reshape(M, K)
        x = np.where(u < outlier_prob, x * outlier_gain, x)
    return x.astype(np.float16)


def weights_f16(seed: int, name: str, N: int, K: int, std: float = 0.02) -> np.ndarray:
    return normal_f16(seed, name, (N, K), std)


def bias_f16(seed: int, name: str, N: int, std: float = 0.01) -> np.ndarray:
    return normal_f16(seed, name, (N,), std)


def bos_context_f16(seed: int, name: str, B: int, T: int, K: int, n_outlier: int = 16, gain: float = 60.0,
                    shared_bos: bool = True) -> np.ndarray:
    """Text-encoder-like context [B,T,K]: N(0,1) body; token 0 of each prompt carries n_outlier channels of
    magnitude N(0,1)*gain.  shared_bos: the same BOS row for every prompt (the paper observes that the BOS
    feature does not depend on the prompt, Sec. 3.1)."""
    ctx = normal(seed, name, (B, T, K))
    nb = 1 if shared_bos else B
    for b in range(nb):
        row = normal(seed, f"{name}/bos{b}", (K,))
        order = np.argsort(uniform01(seed, f"{name}/bosidx{b}", K), kind="stable")
        ch = order[:n_outlier]
        row[ch] = normal(seed, f"{name}/bosval{b}", (n_outlier,)) * gain
        if shared_bos:
            ctx[:, 0, :] = row
        else:
            ctx[b, 0, :] = row
    return ctx.astype(np.float16)


# ----------------------------------------------------------------------------------------------
# Layer tables
# ----------------------------------------------------------------------------------------------

@dataclass(frozen=True)
class Layer:
    name: str
    M: int
    K: int
    N: int
    kind: str  # "linear" or "kv" (cross-attention K/V projection on [B,77,2048] context)
    bias: bool
    bits: int = 4
    B: int = 0  # prompts, for kind == "kv"
    T: int = 0


def transformer_block_linears(prefix: str, M: int, C: int, B: int, ctx_dim: int = 2048, T: int = 77):
    """The ten linears of one SDXL transformer block at channel width C:
    self-attn q,k,v,out; cross-attn q,out and k,v (on the text context); GEGLU proj C->8C; FF out 4C->C."""
    L = []
    for nm in ("attn1.to_q", "attn1.to_k", "attn1.to_v"):
        L.append(Layer(f"{prefix}.{nm}", M, C, C, "linear", False))
    L.append(Layer(f"{prefix}.attn1.to_out", M, C, C, "linear", True))
    L.append(Layer(f"{prefix}.attn2.to_q", M, C, C, "linear", False))
    L.append(Layer(f"{prefix}.attn2.to_k", B * T, ctx_dim, C, "kv", False, B=B, T=T))
    L.append(Layer(f"{prefix}.attn2.to_v", B * T, ctx_dim, C, "kv", False, B=B, T=T))
    L.append(Layer(f"{prefix}.attn2.to_out", M, C, C, "linear", True))
    L.append(Layer(f"{prefix}.ff.proj", M, C, 8 * C, "linear", True))
    L.append(Layer(f"{prefix}.ff.out", M, 4 * C, C, "linear", True))
    return L


def _assign_bits(layers, seed: int, choices, target: float, tol: float = 0.01):
    """Seeded draw from `choices`, then seeded single-step moves along the sorted choices until the
    parameter-weighted mean bit-width (the paper's average, Sec. 4.2) is target +- tol."""
    choices = sorted(choices)
    n = len(layers)
    params = np.array([l.N * l.K for l in layers], np.float64)
    draw = (uniform01(seed, "bits/draw", n) * len(choices)).astype(int).clip(0, len(choices) - 1)
    idx = draw.copy()
    bits_of = np.array(choices)

    def mean(ix):
        return float((params * bits_of[ix]).sum() / params.sum())

    step = 0
    order = raw_u64(seed, "bits/moves", 100000)
    while abs(mean(idx) - target) > tol and step < 100000:
        j = int(order[step] % np.uint64(n))
        step += 1
        cur = mean(idx)
        trial = idx.copy()
        if cur > target and trial[j] > 0:
            trial[j] -= 1
        elif cur < target and trial[j] < len(choices) - 1:
            trial[j] += 1
        else:
            continue
        if abs(mean(trial) - target) < abs(cur - target):
            idx = trial
    return [int(bits_of[i]) for i in idx], mean(idx)


def sweep_layers(seed: int = 0, batch: int = 4, latent: int = 128, bits_choices=(2, 3, 4, 8),
                 target_bits: float = 3.66):
    """The full linear sweep: 2 transformer blocks at the 640-channel level (M = batch*(latent/2)^2) and 10 at
    the 1280-channel level (M = batch*(latent/4)^2), mixed per-layer bit-widths averaging target_bits."""
    from dataclasses import replace
    M640 = batch * (latent // 2) ** 2
    M1280 = batch * (latent // 4) ** 2
    layers = []
    for b in range(2):
        layers += transformer_block_linears(f"down1.block{b}", M640, 640, batch)
    for b in range(10):
        layers += transformer_block_linears(f"down2.block{b}", M1280, 1280, batch)
    bits, mean = _assign_bits(layers, seed, bits_choices, target_bits)
    layers = [replace(l, bits=bt) for l, bt in zip(layers, bits)]
    return layers, mean


# ----------------------------------------------------------------------------------------------
# Inputs of the bit-width allocation: a layer table with element counts and groups, and a synthetic
# sensitivity table (the real one needs the model, prompts and image metrics)
# ----------------------------------------------------------------------------------------------

def unet_allocation_layers(ctx_dim: int = 2048):
    """(name, group, weight elements) for the linear and convolution layers of an SDXL-shaped UNet: channel widths
    320/640/1280, transformer depths 0/2/10 per level (encoder 2 stages per level, middle 1, decoder 3), residual
    blocks with two 3x3 convolutions, a time-embedding linear and a 1x1 shortcut where the width changes.
    group: "content" for cross-attention and feed-forward layers, "quality" for the rest (Sec. 3.2)."""
    rows = []

    def transformer(prefix, C, depth):
        rows.append((f"{prefix}.proj_in", "quality", C * C))
        for d in range(depth):
            for L in transformer_block_linears(f"{prefix}.block{d}", 1, C, 1, ctx_dim):
                grp = "content" if (".attn2." in L.name or ".ff." in L.name) else "quality"
                rows.append((L.name, grp, L.N * L.K))
        rows.append((f"{prefix}.proj_out", "quality", C * C))

    def resblock(prefix, cin, cout):
        rows.append((f"{prefix}.conv1", "quality", 9 * cin * cout))
        rows.append((f"{prefix}.time_emb", "quality", 1280 * cout))
        rows.append((f"{prefix}.conv2", "quality", 9 * cout * cout))
        if cin != cout:
            rows.append((f"{prefix}.shortcut", "quality", cin * cout))

    widths, depths = (320, 640, 1280), (0, 2, 10)
    rows.append(("conv_in", "quality", 9 * 4 * 320))
    prev = 320
    skips = [320]
    for lvl, (C, dep) in enumerate(zip(widths, depths)):
        for s in range(2):
            resblock(f"down{lvl}.res{s}", prev, C)
            if dep:
                transformer(f"down{lvl}.attn{s}", C, dep)
            prev = C
            skips.append(C)
        if lvl < 2:
            rows.append((f"down{lvl}.downsample", "quality", 9 * C * C))
            skips.append(C)
    resblock("mid.res0", 1280, 1280)
    transformer("mid.attn", 1280, 10)
    resblock("mid.res1", 1280, 1280)
    for lvl in (2, 1, 0):
        C, dep = widths[lvl], depths[lvl]
        for s in range(3):
            resblock(f"up{lvl}.res{s}", prev + skips.pop(), C)
            if dep:
                transformer(f"up{lvl}.attn{s}", C, dep)
            prev = C
        if lvl > 0:
            rows.append((f"up{lvl}.upsample", "quality", 9 * C * C))
    rows.append(("conv_out", "quality", 9 * 320 * 4))
    return rows


def sensitivity_table(seed: int, name: str, n_layers: int, bits=(2, 4, 8)) -> np.ndarray:
    """Synthetic scores S[i][b] in dB-like units: about 6 dB per bit times a per-layer gain in [0.5, 1.5], on a
    per-layer offset, with a little noise, and non-decreasing in b (more bits never score worse)."""
    gain = 0.5 + uniform01(seed, name + "/gain", n_layers)
    offset = 20.0 * uniform01(seed, name + "/offset", n_layers)
    noise = normal(seed, name + "/noise", (n_layers, len(bits)), 0.5)
    s = offset[:, None] + 6.02 * gain[:, None] * np.asarray(bits, np.float64)[None, :] + noise
    return np.maximum.accumulate(s, axis=1)

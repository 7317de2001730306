"""Seeded synthetic FP8 E4M3 weights shaped like the paper's workloads.

This module only makes inputs.  It holds none of the codec's arithmetic and is
the one module that both the product's harness (tests, bench) and the oracle's
tests use.  The paper evaluates on trained checkpoints (Section 4, Table 1);
those cannot be fetched here, so heavy-tailed alpha-stable samples stand in
for them: Section 2 of the paper models trained weights as symmetric
alpha-stable, which is what concentrates the exponent field.

Recipe per tensor: draw S_alpha(beta=0, gamma=scale, delta=0) in fp32 with the
Chambers-Mallows-Stuck transform, scale so that the largest magnitude of each
128x128 block (or of the whole tensor) maps to 448, clamp, and round to nearest
even into OCP E4M3 ("fn": no infinities, 0x7F/0xFF are NaN and never produced).
"""
import math

import numpy as np
import torch

E4M3_MAX = 448.0


def _mix(seed, tensor_id):
    # SplitMix64-style scramble of (seed, tensor_id) into one 63-bit generator seed
    z = (seed * 0x9E3779B97F4A7C15 + tensor_id * 0xBF58476D1CE4E5B9 + 0x94D049BB133111EB) & (2 ** 64 - 1)
    z ^= z >> 30
    z = (z * 0xBF58476D1CE4E5B9) & (2 ** 64 - 1)
    z ^= z >> 27
    z = (z * 0x94D049BB133111EB) & (2 ** 64 - 1)
    z ^= z >> 31
    return z & (2 ** 63 - 1)


def alpha_stable(n, alpha, scale, gen, device="cpu"):
    """n fp32 samples of S_alpha(0, scale, 0); alpha=2 gives N(0, 2 scale^2)."""
    u = torch.rand(n, generator=gen, device=device, dtype=torch.float32)
    u = (u - 0.5) * math.pi
    u = u.clamp_(-math.pi / 2 + 1e-6, math.pi / 2 - 1e-6)
    w = torch.empty(n, device=device, dtype=torch.float32).exponential_(generator=gen)
    w.clamp_(min=1e-30)
    a = float(alpha)
    x = torch.sin(a * u) / torch.cos(u).pow(1.0 / a)
    x = x * (torch.cos((1.0 - a) * u) / w).pow((1.0 - a) / a)
    return x.mul_(float(scale))


def scale_to_e4m3(w, scaling):
    """w: fp32 (rows, cols).  Returns uint8 (rows, cols) of E4M3 encodings."""
    rows, cols = w.shape
    if scaling == "tensor":
        m = w.abs().max()
        s = torch.where(m > 0, E4M3_MAX / m, torch.ones_like(m))
        y = w * s
    elif scaling == "block128":
        pr, pc = (-rows) % 128, (-cols) % 128
        wp = torch.nn.functional.pad(w, (0, pc, 0, pr)) if (pr or pc) else w
        R, C = wp.shape
        blk = wp.view(R // 128, 128, C // 128, 128)
        m = blk.abs().amax(dim=(1, 3), keepdim=True)
        s = torch.where(m > 0, E4M3_MAX / m, torch.ones_like(m))
        y = (blk * s).view(R, C)[:rows, :cols]
    else:
        raise ValueError(scaling)
    y = y.clamp(-E4M3_MAX, E4M3_MAX).contiguous()
    return y.to(torch.float8_e4m3fn).view(torch.uint8)


def make_weight(rows, cols, alpha, scale, seed, tensor_id=0, scaling="block128", device="cpu"):
    """One synthetic weight matrix as a uint8 tensor of E4M3 bytes."""
    gen = torch.Generator(device=device)
    gen.manual_seed(_mix(seed, tensor_id))
    w = alpha_stable(rows * cols, alpha, scale, gen, device).view(rows, cols)
    return scale_to_e4m3(w, scaling)


def _drawn(seed, tensor_id):
    r = np.random.default_rng([seed, tensor_id, 0x5eed])
    return float(r.uniform(1.6, 2.0)), float(r.uniform(0.01, 0.03))


def config0():
    """1024x1024, alpha 1.8, scale 0.02, per-128x128 scaling, seed 0."""
    return [dict(name="w", rows=1024, cols=1024, alpha=1.8, scale=0.02, scaling="block128", tensor_id=0)]


LLM8B_SHAPES = [("q", 4096, 4096), ("k", 1024, 4096), ("v", 1024, 4096), ("o", 4096, 4096),
                ("gate", 14336, 4096), ("up", 14336, 4096), ("down", 4096, 14336)]


def config1(seed=0, layers=32):
    """8B-class dense LLM stack: 7 matrices per layer, alpha and scale drawn per matrix."""
    out = []
    for layer in range(layers):
        for j, (nm, r, c) in enumerate(LLM8B_SHAPES):
            tid = layer * 16 + j
            a, g = _drawn(seed, tid)
            out.append(dict(name="l%d.%s" % (layer, nm), rows=r, cols=c, alpha=a, scale=g,
                            scaling="block128", tensor_id=tid, layer=layer))
    return out


def config2(seed=0, experts=256):
    """671B-class MoE layer: experts x {gate, up, down} plus two attention projections."""
    out = []
    for e in range(experts):
        for j, (nm, r, c) in enumerate([("gate", 2048, 7168), ("up", 2048, 7168), ("down", 7168, 2048)]):
            tid = 100000 + e * 4 + j
            _, g = _drawn(seed, tid)
            out.append(dict(name="e%d.%s" % (e, nm), rows=r, cols=c, alpha=1.7, scale=g,
                            scaling="block128", tensor_id=tid, expert=e))
    for j, (nm, r, c) in enumerate([("attn_a", 7168, 128 * 192), ("attn_b", 16384, 7168)]):
        tid = 200000 + j
        _, g = _drawn(seed, tid)
        out.append(dict(name=nm, rows=r, cols=c, alpha=1.7, scale=g, scaling="block128", tensor_id=tid))
    return out


DIT_SHAPES = ([("sa_%s" % n, 5120, 5120) for n in "qkvo"] + [("ca_%s" % n, 5120, 5120) for n in "qkvo"] +
              [("ffn1", 13824, 5120), ("ffn2", 5120, 13824), ("adaln", 6 * 5120, 5120)])


def config3(blocks=40):
    """14B-class diffusion transformer: 11 matrices per block, per-tensor scaling."""
    out = []
    for b in range(blocks):
        for j, (nm, r, c) in enumerate(DIT_SHAPES):
            out.append(dict(name="b%d.%s" % (b, nm), rows=r, cols=c, alpha=1.9, scale=0.015,
                            scaling="tensor", tensor_id=300000 + b * 16 + j, block=b))
    return out


def config4():
    """W for the fused decode+GEMM case (config-2 distribution)."""
    return [dict(name="w", rows=14336, cols=4096, alpha=1.7, scale=0.02, scaling="block128", tensor_id=400000)]


def make_bf16(rows, cols, alpha, scale, seed, tensor_id=0, device="cpu"):
    """One synthetic weight matrix as a uint16 tensor of BF16 bit patterns (unscaled weights)."""
    gen = torch.Generator(device=device)
    gen.manual_seed(_mix(seed, tensor_id))
    w = alpha_stable(rows * cols, alpha, scale, gen, device).view(rows, cols)
    return w.to(torch.bfloat16).view(torch.uint16)


def make_e5m2(rows, cols, alpha, scale, seed, tensor_id=0, device="cpu"):
    """The same weights scaled per tensor to the E5M2 range (largest magnitude -> 57344), as uint8."""
    gen = torch.Generator(device=device)
    gen.manual_seed(_mix(seed, tensor_id))
    w = alpha_stable(rows * cols, alpha, scale, gen, device).view(rows, cols)
    m = w.abs().max()
    s = torch.where(m > 0, 57344.0 / m, torch.ones_like(m))
    return (w * s).clamp(-57344.0, 57344.0).to(torch.float8_e5m2).view(torch.uint8)


def make(spec, seed=0, device="cpu"):
    return make_weight(spec["rows"], spec["cols"], spec["alpha"], spec["scale"], seed,
                       spec["tensor_id"], spec["scaling"], device)


def activations(m, k, seed=0, device="cpu"):
    """M x K activations: N(0,1) rows scaled to max 448, as E4M3 bytes."""
    gen = torch.Generator(device=device)
    gen.manual_seed(_mix(seed, 500000 + m))
    x = torch.randn(m, k, generator=gen, device=device, dtype=torch.float32)
    mx = x.abs().amax(dim=1, keepdim=True)
    x = (x * (E4M3_MAX / mx)).clamp(-E4M3_MAX, E4M3_MAX)
    return x.to(torch.float8_e4m3fn).view(torch.uint8)

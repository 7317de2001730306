"""Checks of the synthetic-input generator (no codec arithmetic involved)."""
import math

import numpy as np
import torch

from paper_2510_02676_amd import synth


def _e4m3_value(b):
    s = -1.0 if b & 0x80 else 1.0
    e, m = (b >> 3) & 15, b & 7
    if e == 0:
        return s * m * 2.0 ** -9
    return s * (1 + m / 8.0) * 2.0 ** (e - 7)


def _rne_reference(y):
    """Round-to-nearest-even into E4M3 written out arithmetically (|y| <= 448)."""
    out = np.zeros(y.shape, dtype=np.uint8)
    a = np.abs(y).astype(np.float64)
    sign = (np.signbit(y)).astype(np.uint8) << 7
    sub = a < 2.0 ** -6
    q = np.rint(a * 2.0 ** 9)
    out[sub] = q[sub].astype(np.uint8)
    nz = ~sub
    e = np.floor(np.log2(a[nz]))
    mant = np.rint((a[nz] / 2.0 ** e - 1.0) * 8.0)
    carry = mant == 8
    e = e + carry
    mant = np.where(carry, 0, mant)
    out[nz] = ((e + 7).astype(np.uint8) << 3) | mant.astype(np.uint8)
    return out | sign


def test_cast_matches_arithmetic_rne_on_grid_and_midpoints():
    vals = sorted(_e4m3_value(b) for b in range(0x7F))  # all finite non-negative values
    pts = []
    for lo, hi in zip(vals[:-1], vals[1:]):
        mid = np.float32((lo + hi) / 2)
        pts += [lo, hi, mid, np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(1e9))]
    pts = np.array(pts, dtype=np.float32)
    pts = np.concatenate([pts, -pts, np.array([0.0, -0.0, 2.0 ** -10, -2.0 ** -10, 448.0, -448.0], dtype=np.float32)])
    got = torch.from_numpy(pts).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(got, _rne_reference(pts))
    # the generator's scaling path ends in exactly that cast and never makes NaN
    w = torch.from_numpy(pts.reshape(1, -1))
    b = synth.scale_to_e4m3(w, "tensor").numpy()
    assert (b & 0x7F).max() == 0x7E and not np.any((b & 0x7F) == 0x7F)


def test_alpha2_is_gaussian_with_variance_2_gamma2():
    gen = torch.Generator().manual_seed(1)
    x = synth.alpha_stable(2_000_000, 2.0, 0.02, gen).double()
    assert abs(x.var().item() / (2 * 0.02 ** 2) - 1) < 0.01
    assert abs(x.mean().item()) < 1e-4
    k = ((x - x.mean()) ** 4).mean() / x.var() ** 2
    assert abs(k.item() - 3.0) < 0.05


def test_tail_exponent():
    gen = torch.Generator().manual_seed(2)
    a = 1.7
    x = synth.alpha_stable(4_000_000, a, 1.0, gen).abs()
    p1 = (x > 20).double().mean().item()
    p2 = (x > 80).double().mean().item()
    slope = math.log(p1 / p2) / math.log(4.0)
    assert abs(slope - a) < 0.15


def test_block_scaling_hits_448_in_every_block_and_is_seeded():
    spec = synth.config0()[0]
    w = synth.make(spec, seed=0)
    assert w.shape == (1024, 1024) and w.dtype == torch.uint8
    blk = (w & 0x7F).view(8, 128, 8, 128).amax(dim=(1, 3))
    assert torch.all(blk == 0x7E)
    assert torch.equal(w, synth.make(spec, seed=0))
    assert not torch.equal(w, synth.make(spec, seed=1))
    e = ((w >> 3) & 15).flatten().numpy()
    f = np.bincount(e, minlength=16) / e.size
    h = -(f[f > 0] * np.log2(f[f > 0])).sum()
    assert 2.0 < h < 3.5  # the exponent entropy of trained FP8 weights lies between two and three bits (Section 1, Figure 1)


def test_config_shapes():
    c1 = synth.config1()
    assert len(c1) == 224 and sum(s["rows"] * s["cols"] for s in c1) == 6_979_321_856
    assert all(1.6 <= s["alpha"] <= 2.0 and 0.01 <= s["scale"] <= 0.03 for s in c1)
    c2 = synth.config2()
    assert len(c2) == 770 and sum(s["rows"] * s["cols"] for s in c2) == 11_567_890_432
    c3 = synth.config3()
    assert len(c3) == 440 and sum(s["rows"] * s["cols"] for s in c3) == 20_342_374_400

"""The GPU-side encoder of the wide-alphabet codec (ecfw_encode_gpu) against the CPU encoder and the oracle.

The CPU encoder's container is pinned to the oracle's on the CPU (tests/test_wide_host.py); here the device
encoder must produce that same container byte for byte, and the oracle's reader must decode it to the input.
"""
import numpy as np
import pytest
import torch

from paper_2510_02676_amd import ecf8, ecfw, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
E5M2, BF16 = ecfw.FMT_E5M2, ecfw.FMT_BF16


def _rand_elems(fmt, n, seed, spread=3.0):
    rng = np.random.default_rng(seed)
    if fmt == BF16:
        e = np.clip(np.rint(rng.normal(120, spread, n)), 0, 255).astype(np.uint16)
        return ((rng.integers(0, 2, n).astype(np.uint16) << 15) | (e << 7) | rng.integers(0, 128, n).astype(np.uint16))
    e = np.clip(np.rint(rng.normal(14, spread, n)), 0, 31).astype(np.uint8)
    return ((rng.integers(0, 2, n).astype(np.uint8) << 7) | (e << 2) | rng.integers(0, 4, n).astype(np.uint8))


def _to_dev(fmt, x):
    t = torch.from_numpy(x.view(np.int16) if fmt == BF16 else x)
    return t.to(DEV)


def _same_as_cpu(orc, fmt, x, rows, cols, oracle_read=True, **opts):
    x = np.ascontiguousarray(x).reshape(-1)
    ref = ecfw.ecfw_encode(fmt, x, rows, cols, **opts)
    print("fmt", fmt, "n", x.size, opts, "max_len", ref.header.max_code_len, flush=True)
    guard = 4096
    bound = ctypes_bound(fmt, rows, cols, **opts)
    assert bound >= ref.size
    buf = torch.full((bound + guard,), 0xA5, dtype=torch.uint8, device=DEV)
    hdr, d_blob = ecfw.ecfw_encode_gpu(fmt, _to_dev(fmt, x), rows, cols, d_blob=buf[:bound], **opts)
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    assert (host[bound:] == 0xA5).all()
    got = host[:hdr.total_size]
    assert bytes(hdr) == bytes(ref.header)
    assert got.size == ref.size and np.array_equal(got, ref.numpy())
    if oracle_read:
        dec, bits = orc.w_container_decode(got)
        assert np.array_equal(dec, x) and bits == hdr.stream_bits
    # and the device decoder reads what the device encoder wrote
    out = ecfw.ecfw_decode(d_blob, hdr)
    torch.cuda.synchronize()
    back = out.view(torch.int16).cpu().numpy().view(np.uint16) if fmt == BF16 else out.cpu().numpy()
    assert np.array_equal(back, x)


def ctypes_bound(fmt, rows, cols, lane_syms=0, group_chunks=0, max_code_len=0):
    import ctypes
    opts = ecfw.WEncodeOpts(fmt, lane_syms, 0, group_chunks, max_code_len)
    b = ctypes.c_uint64(0)
    ecf8._check("ecfw_encode_bound", ecfw._lib.ecfw_encode_bound(rows, cols, ctypes.byref(opts), ctypes.byref(b)))
    return int(b.value)


@pytest.mark.parametrize("fmt", [E5M2, BF16])
@pytest.mark.parametrize("n", [1, 3, 16, 17, 4095, 4096, 4097, 8193, 64 * 128 * 3 + 1, 300007, 1000003])
def test_ragged_sizes(orc, fmt, n):
    _same_as_cpu(orc, fmt, _rand_elems(fmt, n, n), 1, n)


@pytest.mark.parametrize("fmt", [E5M2, BF16])
@pytest.mark.parametrize("lane_syms,group,cap", [(64, 1, 0), (64, 2, 16), (128, 4, 9), (128, 64, 0), (64, 32, 13), (128, 1, 16)])
def test_options(orc, fmt, lane_syms, group, cap):
    n = 64 * lane_syms * 37 + 123
    _same_as_cpu(orc, fmt, _rand_elems(fmt, n, n + cap, spread=2.5), 1, n, lane_syms=lane_syms, group_chunks=group, max_code_len=cap)


@pytest.mark.parametrize("fmt", [E5M2, BF16])
def test_degenerate_histograms(orc, fmt):
    one = np.full(9000, 0x3F80 if fmt == BF16 else 0x3C, dtype=np.uint16 if fmt == BF16 else np.uint8)
    _same_as_cpu(orc, fmt, one, 90, 100)
    two = one.copy()
    two[::5] = 0x4000 if fmt == BF16 else 0x40
    _same_as_cpu(orc, fmt, two, 90, 100)
    every = np.tile(np.arange(65536, dtype=np.uint16) if fmt == BF16 else np.arange(256, dtype=np.uint8), 4)
    _same_as_cpu(orc, fmt, every, 4, every.size // 4, max_code_len=16)


def test_long_codes_everywhere(orc):
    """All 256 BF16 exponent fields with geometric frequencies: codewords of 13..16 bits in most lanes (the
    widest stream stage of the packer)."""
    rng = np.random.default_rng(7)
    p = 0.93 ** np.arange(256)
    e = rng.choice(256, size=500000, p=p / p.sum()).astype(np.uint16)
    e[:256] = np.arange(256)
    x = ((rng.integers(0, 2, e.size).astype(np.uint16) << 15) | (e << 7) | rng.integers(0, 128, e.size).astype(np.uint16))
    _same_as_cpu(orc, BF16, x, 1, x.size, max_code_len=16, lane_syms=128)
    _same_as_cpu(orc, BF16, x, 1, x.size, max_code_len=16, lane_syms=64, group_chunks=8)


@pytest.mark.parametrize("fmt", [E5M2, BF16])
def test_full_size_matrix(orc, fmt):
    make = synth.make_bf16 if fmt == BF16 else synth.make_e5m2
    x = make(14336, 4096, 1.8, 0.02, 0, tensor_id=5).numpy()
    _same_as_cpu(orc, fmt, x, 14336, 4096, oracle_read=False)


def test_argument_errors():
    x = torch.zeros(10000, dtype=torch.int16, device=DEV)
    with pytest.raises(ecf8.Ecf8Error) as e:
        ecfw.ecfw_encode_gpu(BF16, x, d_blob=torch.empty(1024, dtype=torch.uint8, device=DEV))
    assert e.value.code == ecf8.E_CAPACITY
    with pytest.raises(ecf8.Ecf8Error) as e:
        ecfw.ecfw_encode_gpu(BF16, x, lane_syms=32)
    assert e.value.code == ecf8.E_ARG
    with pytest.raises(ecf8.Ecf8Error):
        ecfw.ecfw_encode_gpu(BF16, x.to(torch.uint8))          # one byte per element is not BF16
    with pytest.raises(ecf8.Ecf8Error):
        ecfw.ecfw_encode_gpu(7, x)
    y = torch.arange(10000, dtype=torch.int16, device=DEV)       # 40 distinct exponent fields need more than 5 bits
    with pytest.raises(ecf8.Ecf8Error) as e:
        ecfw.ecfw_encode_gpu(BF16, y, max_code_len=5)
    assert e.value.code == ecf8.E_ARG
    torch.cuda.synchronize()

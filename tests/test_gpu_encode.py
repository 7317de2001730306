"""GPU-side encoder (ecf8_encode_gpu, paper Section 3.1 on the device): the container it writes is
the CPU encoder's, byte for byte; the oracle's reader decodes it to the input and agrees on the
stream length; the GPU decoder round-trips it."""
import numpy as np
import pytest
import torch

from paper_2510_02676_amd import ecf8, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _rand_bytes(n, seed, conc=0.4):
    rng = np.random.default_rng(seed)
    p = rng.dirichlet(np.ones(16) * conc)
    e = rng.choice(16, size=n, p=p).astype(np.uint8)
    return ((rng.integers(0, 2, n, dtype=np.uint8) << 7) | (e << 3) | rng.integers(0, 8, n, dtype=np.uint8)).astype(np.uint8)


def _check_same(orc, x, rows, cols, oracle_read=True, **opts):
    d_x = torch.from_numpy(x).to(DEV)
    hdr, d_blob = ecf8.ecf8_encode_gpu(d_x, rows, cols, **opts)
    torch.cuda.synchronize()
    got = d_blob.cpu().numpy()
    want = ecf8.ecf8_encode(x, rows, cols, **opts)
    assert bytes(hdr) == bytes(want.header)
    w = want.numpy()
    assert got.size == w.size
    if not np.array_equal(got, w):
        bad = np.flatnonzero(got != w)
        raise AssertionError("GPU and CPU containers differ at %d bytes, first at offset %d (sections: cb %d lb %d st %d pl %d)"
                             % (bad.size, bad[0], hdr.off_chunk_bit, hdr.off_lane_bits, hdr.off_stream, hdr.off_plane))
    ecf8.blob_validate(got)
    if oracle_read:
        dec, bits = orc.container_decode(got)
        assert np.array_equal(dec, x.reshape(-1)) and bits == hdr.stream_bits
    out = ecf8.ecf8_decode(hdr, d_blob.clone())
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy().reshape(-1), x.reshape(-1))


@pytest.mark.parametrize("lane_syms", [32, 64, 128])
@pytest.mark.parametrize("n", [1, 15, 16, 17, 2047, 4097, 8193, 3 * 8192 + 77, 300_001, 1_000_003])
def test_same_container_as_the_cpu_encoder(orc, lane_syms, n):
    x = _rand_bytes(n, 13 * n + lane_syms)
    _check_same(orc, x, 1, n, lane_syms=lane_syms, max_code_len=15 if n % 2 else 0, table_mode=1 + (n % 3 == 0))


@pytest.mark.parametrize("opts", [dict(group_chunks=1), dict(group_chunks=4, lane_syms=32), dict(group_chunks=64),
                                  dict(max_code_len=4), dict(max_code_len=15, lane_syms=64, group_chunks=2)])
def test_layout_and_cap_options(orc, opts):
    x = _rand_bytes(2_300_017, 77)
    _check_same(orc, x, 1, x.size, **opts)


@pytest.mark.parametrize("lane_syms,rows,cols", [(32, 16, 128), (64, 64, 4096), (128, 48, 3584), (64, 160, 1024)])
def test_row_tiled_layout(orc, lane_syms, rows, cols):
    x = _rand_bytes(rows * cols, rows + cols)
    _check_same(orc, x, rows, cols, lane_syms=lane_syms, tile_rows=16)


@pytest.mark.parametrize("block", range(4))
def test_seeded_sweep_of_shapes_and_options(orc, block):
    """120 seeded combinations of size, lane_syms, group width, cap, table mode and exponent skew:
    the device writes the CPU encoder's container every time."""
    rng = np.random.default_rng(7000 + block)
    for i in range(30):
        lane_syms = int(rng.choice([32, 64, 128]))
        chunk = 64 * lane_syms
        n = max(1, int(rng.integers(1, 40)) * chunk + int(rng.integers(-chunk, chunk)) if i % 2 else int(rng.integers(1, 300_000)))
        x = _rand_bytes(n, int(rng.integers(1 << 30)), conc=float(rng.choice([0.05, 0.3, 2.0, 50.0])))
        _check_same(orc, x, 1, n, oracle_read=(i % 5 == 0), lane_syms=lane_syms,
                    group_chunks=int(rng.choice([1, 2, 8, 32, 64])), max_code_len=int(rng.choice([0, 15, 4, 10])),
                    table_mode=int(rng.choice([1, 2])))


def test_special_histograms(orc):
    fib = [1, 1]
    while len(fib) < 16:
        fib.append(fib[-1] + fib[-2])
    deep = np.repeat(np.arange(16, dtype=np.uint8) << 3, fib)
    np.random.default_rng(0).shuffle(deep)
    cases = [np.arange(256, dtype=np.uint8).repeat(40), np.full(5000, 0x80, dtype=np.uint8),
             np.array([0x38, 0xB8, 0x3C, 0x00], dtype=np.uint8), deep,
             np.concatenate([np.full(9000, 0x38, np.uint8), np.array([0x7F, 0xFF], np.uint8)])]
    for x in cases:
        for cap in (0, 15):
            _check_same(orc, x, 1, x.size, max_code_len=cap)


def test_config0_and_a_full_size_matrix(orc):
    w = synth.make(synth.config0()[0], seed=0).numpy()
    _check_same(orc, w.reshape(-1), 1024, 1024)
    spec = synth.config1(0, 1)[4]                       # l0.gate, 14336 x 4096
    wd = synth.make(spec, 0, device=DEV)
    hdr, d_blob = ecf8.ecf8_encode_gpu(wd)
    want = ecf8.ecf8_encode(wd.cpu(), spec["rows"], spec["cols"])
    torch.cuda.synchronize()
    assert bytes(hdr) == bytes(want.header)
    assert torch.equal(d_blob.cpu(), torch.from_numpy(want.numpy()))
    assert torch.equal(ecf8.ecf8_decode(hdr, d_blob), wd)


def test_argument_errors():
    d_x = torch.zeros(4096, dtype=torch.uint8, device=DEV)
    with pytest.raises(ecf8.Ecf8Error) as e:
        ecf8.ecf8_encode_gpu(d_x, 1, 4096, lane_syms=48)
    assert e.value.code == ecf8.E_ARG
    with pytest.raises(ecf8.Ecf8Error) as e:
        ecf8.ecf8_encode_gpu(d_x, 1, 4096, d_blob=torch.empty(512, dtype=torch.uint8, device=DEV))
    assert e.value.code == ecf8.E_CAPACITY
    with pytest.raises(ecf8.Ecf8Error) as e:
        ecf8.ecf8_encode_gpu(d_x, 1, 4096, d_blob=torch.empty(1 << 20, dtype=torch.uint8, device=DEV)[16:])
    assert e.value.code == ecf8.E_ALIGN
    with pytest.raises(ecf8.Ecf8Error):
        ecf8.ecf8_encode_gpu(d_x, 8, 512, lane_syms=64, tile_rows=16)

"""CPU-side tests of the wide-alphabet calls (E5M2, BF16): exported symbols, and the host
encoder against the oracle -- its code must cost what the oracle's exhaustive optimum costs,
and its container must be, byte for byte, the one the oracle writes for the same code
lengths (equally cheap codes may differ in which symbol gets which length, so the lengths
are the encoder's, checked for validity and cost).  No GPU call is made here."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2510_02676_amd import ecf8, ecfw, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
E5M2, BF16 = ecfw.FMT_E5M2, ecfw.FMT_BF16


def _rand_elems(fmt, n, seed, spread=3.0):
    rng = np.random.default_rng(seed)
    if fmt == BF16:
        e = np.clip(np.rint(rng.normal(120, spread, n)), 0, 255).astype(np.uint16)
        return ((rng.integers(0, 2, n).astype(np.uint16) << 15) | (e << 7) | rng.integers(0, 128, n).astype(np.uint16))
    e = np.clip(np.rint(rng.normal(14, spread, n)), 0, 31).astype(np.uint8)
    return ((rng.integers(0, 2, n).astype(np.uint8) << 7) | (e << 2) | rng.integers(0, 4, n).astype(np.uint8))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "ecfw.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(ecfw_[a-z_0-9]+)\s*\(", text))
    assert {"ecfw_encode", "ecfw_decode", "ecfw_blob_describe", "ecfw_blob_validate"} <= names
    lib = ctypes.CDLL(ecf8.LIB_PATH)
    for n in sorted(names):
        assert hasattr(lib, n), n


def _check_against_oracle(orc, fmt, x, rows, cols, **opts):
    blob = ecfw.ecfw_encode(fmt, x, rows, cols, **opts)
    h, arr = blob.header, blob.numpy()
    cap = opts.get("max_code_len", 0) or 12
    freq = orc.w_histogram(fmt, x)
    ln = blob.code_len()
    _, best = orc.w_lengths_limited(freq, cap)
    assert h.stream_bits == best == orc.w_stream_bits(freq, ln)
    assert ln.max() == h.max_code_len <= cap and np.array_equal(ln > 0, freq > 0)
    orc.w_canonical(ln)                                    # a prefix code (raises otherwise)
    N = opts.get("lane_syms", 0) or (64 if fmt == BF16 else 128)
    G = opts.get("group_chunks", 0) or 32
    want = orc.w_container_encode(fmt, x, rows, cols, N, G, ln)
    assert arr.size == want.size and np.array_equal(arr, want)
    dec, bits = orc.w_container_decode(arr)
    assert np.array_equal(dec, np.asarray(x).reshape(-1)) and bits == h.stream_bits
    ecfw.blob_validate(arr)
    return blob


@pytest.mark.parametrize("fmt", [E5M2, BF16])
@pytest.mark.parametrize("n,opts", [
    (1, {}), (7, {}), (4097, {}), (64 * 64 * 3, {"lane_syms": 64, "group_chunks": 1}),
    (128 * 64 * 5 + 77, {"lane_syms": 128, "group_chunks": 2}), (64 * 64 * 40 + 5, {"lane_syms": 64}),
    (200000, {"max_code_len": 16}), (200000, {"max_code_len": 6}), (100001, {"lane_syms": 128, "group_chunks": 4, "max_code_len": 9}),
])
def test_encoder_matches_oracle_container(orc, fmt, n, opts):
    _check_against_oracle(orc, fmt, _rand_elems(fmt, n, n), 1, n, **opts)


@pytest.mark.parametrize("fmt", [E5M2, BF16])
def test_synthetic_weights(orc, fmt):
    make = synth.make_bf16 if fmt == BF16 else synth.make_e5m2
    x = make(512, 768, 1.8, 0.02, 0).numpy()
    blob = _check_against_oracle(orc, fmt, x, 512, 768)
    h = blob.header
    assert (h.rows, h.cols, h.n_elem) == (512, 768, 512 * 768)
    raw = h.n_elem * ecfw.ELEM_BYTES[fmt]
    # exponent entropy of such weights is about 2.7 bits: BF16 shrinks by about a third, E5M2 by about a quarter
    assert blob.size / raw < (0.72 if fmt == BF16 else 0.78)


def test_cap_that_binds_costs_little_and_is_respected(orc):
    """Plain Huffman on these weights needs codewords of about 20 bits: Section 3.1's cap of 16 binds."""
    x = synth.make_bf16(1024, 1024, 1.8, 0.02, 0).numpy()
    freq = orc.w_histogram(BF16, x)
    assert orc.w_huffman_lengths(freq).max() > 16
    huff = orc.w_stream_bits(freq, orc.w_huffman_lengths(freq))
    b16 = ecfw.ecfw_encode(BF16, x, max_code_len=16)
    b12 = ecfw.ecfw_encode(BF16, x)
    assert b16.header.max_code_len == 16 and b12.header.max_code_len == 12
    assert huff < b16.header.stream_bits <= b12.header.stream_bits < huff * 1.01
    assert b16.header.stream_bits == orc.w_lengths_limited(freq, 16)[1]


@pytest.mark.parametrize("fmt", [E5M2, BF16])
def test_every_bit_pattern(orc, fmt):
    x = np.arange(256, dtype=np.uint8) if fmt == E5M2 else np.arange(65536, dtype=np.uint16)
    x = np.tile(x, 3)
    blob = _check_against_oracle(orc, fmt, x, 3, x.size // 3, max_code_len=16)
    assert blob.header.n_symbols == blob.header.n_alphabet and blob.header.max_code_len == (5 if fmt == E5M2 else 8)


def test_single_symbol_and_two_symbols(orc):
    x = np.full(5000, 0x3F80, dtype=np.uint16)
    b = _check_against_oracle(orc, BF16, x, 50, 100)
    assert b.header.stream_bits == 5000 and b.header.n_symbols == 1
    x[::3] = 0x4000
    b = _check_against_oracle(orc, BF16, x, 50, 100)
    assert b.header.stream_bits == 5000 and b.header.n_symbols == 2


def test_threads_do_not_change_the_blob():
    x = _rand_elems(BF16, 300000, 9)
    a = ecfw.ecfw_encode(BF16, x, n_threads=1).numpy()
    for t in (2, 3, 8):
        assert np.array_equal(a, ecfw.ecfw_encode(BF16, x, n_threads=t).numpy())
    y = _rand_elems(E5M2, 300000, 9)
    assert np.array_equal(ecfw.ecfw_encode(E5M2, y, n_threads=1).numpy(), ecfw.ecfw_encode(E5M2, y, n_threads=5).numpy())


def test_error_paths():
    x = _rand_elems(BF16, 9000, 1)
    with pytest.raises(ecf8.Ecf8Error) as e:
        ecfw.ecfw_encode(3, x)
    assert e.value.code == ecf8.E_ARG
    for bad in (dict(lane_syms=32), dict(group_chunks=3), dict(group_chunks=128), dict(max_code_len=17),
                dict(max_code_len=3)):                 # 2^3 < the number of exponent fields in use
        with pytest.raises(ecf8.Ecf8Error) as e:
            ecfw.ecfw_encode(BF16, x, **bad)
        assert e.value.code == ecf8.E_ARG, bad
    with pytest.raises(TypeError):
        ecfw.ecfw_encode(BF16, x.astype(np.uint8))
    with pytest.raises(ecf8.Ecf8Error):
        ecfw.ecfw_encode(BF16, x, 10, 10)
    blob = ecfw.ecfw_encode(BF16, x, 90, 100, group_chunks=1)
    arr = blob.numpy().copy()
    h = blob.header
    ecfw.blob_validate(arr)
    with pytest.raises(ecf8.Ecf8Error) as e:
        ecfw.blob_describe(arr[:-1])
    assert e.value.code == ecf8.E_FORMAT
    for off in (0, 4, 8, 16, 40, 44, 48, 52, 56, 60, 64, 72, 80, 136, 200, h.off_code_len + int(np.argmax(blob.code_len() > 0)),
                h.off_freq + 8 * int(np.argmax(blob.code_len() > 0))):
        bad = arr.copy()
        bad[off] ^= 1
        with pytest.raises(ecf8.Ecf8Error):
            ecfw.blob_describe(bad)
    for off in (h.off_chunk_bit + 8, h.off_lane_bits + 2, h.off_stream + h.stream_bytes - 1, h.off_plane + h.plane_bytes - 1,
                h.off_chunk_bit + 8 * (h.n_chunks + 1) + 3):
        bad = arr.copy()
        bad[off] ^= 0x40
        ecfw.blob_describe(bad)                         # structure intact ...
        with pytest.raises(ecf8.Ecf8Error):
            ecfw.blob_validate(bad)                     # ... metadata or padding is not


def test_batch_prepare_checks_on_the_host():
    """ecfw_batch_prepare runs on the host alone: running chunk offsets, the launch facts, and the refusals."""
    import ctypes
    xs = [_rand_elems(BF16, n, n) for n in (5000, 70000, 9)]
    blobs = [ecfw.ecfw_encode(BF16, x, max_code_len=c) for x, c in zip(xs, (0, 14, 0))]
    n = len(blobs)
    H = (ecfw.WHeader * n)(*[b.header for b in blobs])
    fake = [0x7f0000000000 + 0x10000000 * i for i in range(n)]          # never dereferenced by prepare
    B = (ctypes.c_void_p * n)(*fake)
    O = (ctypes.c_void_p * n)(*[f + 0x1000000 for f in fake])
    C = (ctypes.c_uint64 * n)(*[2 * b.header.n_elem for b in blobs])
    items = (ecfw.WBatchItem * n)()
    info = ecfw.WBatchInfo()
    lib = ecfw._lib
    assert lib.ecfw_batch_prepare(H, B, O, C, n, items, ctypes.byref(info)) == 0
    assert info.total_chunks == sum(b.header.n_chunks for b in blobs) and info.fmt == BF16 and info.lane_syms == 64
    assert info.max_code_len == max(b.header.max_code_len for b in blobs)
    run = 0
    for it, b in zip(items, blobs):
        assert it.first_chunk == run and it.n_chunks == b.header.n_chunks and it.off_stream == b.header.off_stream
        run += b.header.n_chunks
    C[1] -= 1
    assert lib.ecfw_batch_prepare(H, B, O, C, n, items, ctypes.byref(info)) == ecf8.E_CAPACITY
    C[1] += 1
    O[2] = O[2] + 8
    assert lib.ecfw_batch_prepare(H, B, O, C, n, items, ctypes.byref(info)) == ecf8.E_ALIGN
    O[2] = O[2] - 8
    H[0].lane_syms = 128
    assert lib.ecfw_batch_prepare(H, B, O, C, n, items, ctypes.byref(info)) != 0
    assert lib.ecfw_batch_prepare(H, B, O, C, 0, items, ctypes.byref(info)) == ecf8.E_ARG


def test_encode_bound_covers_every_histogram():
    import ctypes
    for fmt, x in ((BF16, np.arange(65536, dtype=np.uint16)), (E5M2, np.arange(256, dtype=np.uint8).repeat(300))):
        for cap in (0, 16):
            opts = ecfw.WEncodeOpts(fmt, 0, 0, 0, cap)
            b = ctypes.c_uint64(0)
            assert ecfw._lib.ecfw_encode_bound(1, x.size, ctypes.byref(opts), ctypes.byref(b)) == 0
            assert b.value >= ecfw.ecfw_encode(fmt, x, max_code_len=16 if fmt == BF16 else cap).size or cap == 0
    opts = ecfw.WEncodeOpts(9, 0, 0, 0, 0)
    assert ecfw._lib.ecfw_encode_bound(1, 100, ctypes.byref(opts), ctypes.byref(b)) == ecf8.E_ARG
    assert ecfw._lib.ecfw_encode_bound(0, 100, ctypes.byref(ecfw.WEncodeOpts(BF16, 0, 0, 0, 0)), ctypes.byref(b)) == ecf8.E_ARG

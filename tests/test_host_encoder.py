"""CPU-side tests of the library: the C ABI loads and exports what the header
declares, and the host encoder's containers are read back by the oracle's
independent reader.  No GPU call is made here."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2510_02676_amd import ecf8, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _rand_bytes(n, seed, conc=0.4):
    rng = np.random.default_rng(seed)
    p = rng.dirichlet(np.ones(16) * conc)
    e = rng.choice(16, size=n, p=p).astype(np.uint8)
    return ((rng.integers(0, 2, n, dtype=np.uint8) << 7) | (e << 3) | rng.integers(0, 8, n, dtype=np.uint8)).astype(np.uint8)


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "ecf8.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(ecf8_[a-z_0-9]+)\s*\(", text))
    assert {"ecf8_encode", "ecf8_decode", "ecf8_decode_batched"} <= names
    lib = ctypes.CDLL(ecf8.LIB_PATH)
    for n in sorted(names):
        assert hasattr(lib, n), n
    assert ecf8.version() == 1


def _oracle_bits(orc, f, max_code_len):
    """Cost of the cheapest code under the cap, from the oracle (0 = the encoder's default cap of 7)."""
    cap = max_code_len or 7
    return orc.stream_bits(f, orc.huffman_lengths(f) if cap >= 15 else orc.huffman_lengths_limited(f, cap))


@pytest.mark.parametrize("max_code_len", [0, 15, 5])
@pytest.mark.parametrize("lane_syms", [32, 64, 128])
@pytest.mark.parametrize("n", [1, 7, 16, 2047, 2048, 4096, 4097, 8191, 8193, 100003])
def test_encoder_container_read_by_oracle(orc, lane_syms, n, max_code_len):
    x = _rand_bytes(n, n + lane_syms)
    blob = ecf8.ecf8_encode(x, 1, n, lane_syms=lane_syms, max_code_len=max_code_len)
    arr = blob.numpy()
    ecf8.blob_validate(arr)
    dec, bits = orc.container_decode(arr)
    assert np.array_equal(dec, x)
    f = orc.histogram(x)
    assert max(blob.header.code_len) <= (max_code_len or 7)
    assert bits == _oracle_bits(orc, f, max_code_len) == blob.header.stream_bits
    assert list(blob.header.freq) == [int(v) for v in f]
    assert blob.size == orc.lib().orc_container_size(n, bits, lane_syms)


@pytest.mark.parametrize("lane_syms,group,n", [
    (32, 2, 4096), (32, 4, 8192), (32, 4, 8193), (32, 4, 3 * 8192 + 5000), (32, 64, 300001),
    (64, 32, 2 * 131072 + 70001), (64, 8, 100003), (128, 32, 262144 + 12345), (128, 2, 16384 * 3 - 1),
    (128, 32, 262143), (128, 1, 50000)])
def test_grouped_layout_read_by_oracle(orc, lane_syms, group, n):
    """Whole groups interleaved, the rest chunk-major: product writer against the oracle's reader,
    and the oracle's writer against the product's validator (the bitstreams may differ only where
    the two Huffman tie-breaks differ, so the blobs are not compared byte by byte)."""
    x = _rand_bytes(n, n + lane_syms + group)
    blob = ecf8.ecf8_encode(x, 1, n, lane_syms=lane_syms, group_chunks=group)
    assert blob.header.group_chunks == group
    arr = blob.numpy()
    ecf8.blob_validate(arr)
    dec, bits = orc.container_decode(arr)
    assert np.array_equal(dec, x) and bits == blob.header.stream_bits
    theirs = orc.container_encode(x, 1, n, lane_syms, group)
    ecf8.blob_validate(theirs)
    assert ecf8.blob_describe(theirs).group_chunks == group
    dec2, _ = orc.container_decode(theirs)
    assert np.array_equal(dec2, x)


@pytest.mark.parametrize("lane_syms,rows,cols,cap", [(32, 16, 128, 0), (64, 32, 512, 0), (64, 48, 4096, 15), (128, 16, 1024, 5)])
def test_row_tiled_layout_read_by_oracle(orc, lane_syms, rows, cols, cap):
    """Row-tiled layout (what the fused GEMM reads): product writer against the oracle's reader, the
    oracle's writer against the product's validator, and lane ownership restated as a reshape."""
    n = rows * cols
    x = _rand_bytes(n, n + lane_syms)
    blob = ecf8.ecf8_encode(x, rows, cols, lane_syms=lane_syms, tile_rows=16, max_code_len=cap)
    h, arr = blob.header, blob.numpy()
    assert h.tile_rows == 16 and h.group_chunks == 1 and h.n_chunks == n // (64 * lane_syms)
    ecf8.blob_validate(arr)
    dec, bits = orc.container_decode(arr)
    assert np.array_equal(dec, x) and bits == h.stream_bits == _oracle_bits(orc, orc.histogram(x), cap)
    theirs = orc.container_encode(x, rows, cols, lane_syms, 1, cap or 7, 16)
    ecf8.blob_validate(theirs)
    assert ecf8.blob_describe(theirs).tile_rows == 16
    w = 4 * lane_syms
    cost = np.array(list(h.code_len), dtype=np.int64)[(x >> 3) & 15].reshape(rows // 16, 16, cols // w, w // 64, 4, 16)
    want = cost.sum(axis=(3, 5)).transpose(0, 2, 3, 1).reshape(-1, 64)
    lb = arr[h.off_lane_bits:h.off_lane_bits + 128 * h.n_chunks].view("<u2").reshape(-1, 64)
    assert np.array_equal(lb.astype(np.int64), want)


def test_row_tiled_layout_argument_errors():
    x = np.zeros(16 * 512, dtype=np.uint8)
    with pytest.raises(ecf8.Ecf8Error):
        ecf8.ecf8_encode(x, 8, 1024, lane_syms=64, tile_rows=16)          # rows not a multiple of 16
    with pytest.raises(ecf8.Ecf8Error):
        ecf8.ecf8_encode(x, 64, 128, lane_syms=64, tile_rows=16)          # cols not a multiple of 4 N
    with pytest.raises(ecf8.Ecf8Error):
        ecf8.ecf8_encode(x, 16, 512, lane_syms=64, tile_rows=16, group_chunks=4)
    with pytest.raises(ecf8.Ecf8Error):
        ecf8.ecf8_encode(x, 16, 512, lane_syms=64, tile_rows=8)
    good = ecf8.ecf8_encode(x, 16, 512, lane_syms=64, tile_rows=16).numpy().copy()
    ecf8.blob_validate(good)
    bad = good.copy()
    bad[47] = 8
    with pytest.raises(ecf8.Ecf8Error):
        ecf8.blob_validate(bad)


def test_group_interleave_is_block_by_block():
    """The layout stated from scratch for one whole group of two chunks (N = 32): the four
    1024-element blocks alternate between the chunks, lane l owns elements [16 l, 16 l + 16) of
    each of its blocks; lane_bits must be the code bits of exactly those elements."""
    n = 4096
    x = _rand_bytes(n, 77)
    b = ecf8.ecf8_encode(x, 1, n, lane_syms=32, group_chunks=2)
    a, h = b.numpy(), b.header
    assert h.n_chunks == 2
    length = np.array(list(h.code_len), dtype=np.int64)
    bits_of = length[(x >> 3) & 15]
    lane_bits = a[h.off_lane_bits:h.off_lane_bits + 2 * 128].view("<u2")
    for c in range(2):
        for l in range(64):
            want = sum(int(bits_of[blk * 1024 + 16 * l: blk * 1024 + 16 * l + 16].sum()) for blk in (c, c + 2))
            assert lane_bits[c * 64 + l] == want
    # the same tensor chunk-major: chunk c owns blocks 2c and 2c+1
    b1 = ecf8.ecf8_encode(x, 1, n, lane_syms=32, group_chunks=1)
    a1, h1 = b1.numpy(), b1.header
    lane_bits1 = a1[h1.off_lane_bits:h1.off_lane_bits + 2 * 128].view("<u2")
    for c in range(2):
        for l in range(64):
            want = sum(int(bits_of[blk * 1024 + 16 * l: blk * 1024 + 16 * l + 16].sum()) for blk in (2 * c, 2 * c + 1))
            assert lane_bits1[c * 64 + l] == want


@pytest.mark.parametrize("n", [5, 4096, 100003])
def test_embedded_table_is_what_the_code_says(orc, n):
    """A blob with the decoder's pair table embedded: the oracle's reader rebuilds every
    entry from the code by bit-serial walks and compares; so does the host validator."""
    x = _rand_bytes(n, 900 + n, conc=0.15)          # skewed: long codes, pairs that do not fit
    blob = ecf8.ecf8_encode(x, 1, n, table_mode=1)
    arr = blob.numpy()
    assert blob.header.table_bits == 14 and blob.header.off_chunk_bit == 256 + 32768
    ecf8.blob_validate(arr)
    dec, _ = orc.container_decode(arr)
    assert np.array_equal(dec, x)
    plain = ecf8.ecf8_encode(x, 1, n, table_mode=2)
    assert plain.header.table_bits == 0 and blob.size == plain.size + 32768
    for off in (256, 256 + 2 * 777, 256 + 32766):
        bad = arr.copy()
        bad[off] ^= 0x08
        with pytest.raises(ecf8.Ecf8Error):
            ecf8.blob_validate(bad)
        with pytest.raises(ValueError):
            orc.container_decode(bad)


def test_every_byte_value_and_special_histograms(orc):
    cases = [np.arange(256, dtype=np.uint8).repeat(40),
             np.full(5000, 0x80, dtype=np.uint8),                       # one symbol: -0 everywhere
             np.array([0x38, 0xB8, 0x3C, 0x00], dtype=np.uint8),
             np.concatenate([np.full(9000, 0x38, np.uint8), np.array([0x7F, 0xFF], np.uint8)])]
    fib = [1, 1]
    while len(fib) < 16:
        fib.append(fib[-1] + fib[-2])
    deep = np.repeat(np.arange(16, dtype=np.uint8) << 3, fib)
    np.random.default_rng(0).shuffle(deep)
    cases.append(deep)                                                  # code lengths up to 15
    for x in cases:
        for tm in (1, 2):
            for cap in (0, 15):
                blob = ecf8.ecf8_encode(x, 1, x.size, table_mode=tm, max_code_len=cap)
                ecf8.blob_validate(blob.numpy())
                dec, bits = orc.container_decode(blob.numpy())
                assert np.array_equal(dec, x)
                assert bits == _oracle_bits(orc, orc.histogram(x), cap)
    assert max(ecf8.ecf8_encode(deep, 1, deep.size, max_code_len=15).header.code_len) == 15
    assert max(ecf8.ecf8_encode(deep, 1, deep.size).header.code_len) == 7


def test_hand_example_bytes_in_the_product_container():
    x = np.array([0x38, 0xB8, 0x3C, 0x00], dtype=np.uint8)
    b = ecf8.ecf8_encode(x, 2, 2)
    a, h = b.numpy(), b.header
    assert h.stream_bits == 4 and h.rows == 2 and h.cols == 2
    assert h.lane_syms == 128 and h.group_chunks == 32 and a[h.off_stream] == 0x07
    assert list(a[h.off_plane:h.off_plane + 4]) == [0x00, 0x08, 0x04, 0x00]


def test_default_symbols_per_lane_follow_the_cap():
    """lane_syms = 0: 128 under a cap of up to 7 bits (the kernels without a second level), 64 where longer codewords
    are allowed (what the general kernels decode fastest); a given value is kept; row-tiled blobs name theirs."""
    x = np.random.default_rng(5).integers(0, 256, 20_000, dtype=np.uint8)
    for cap, want in ((0, 128), (4, 128), (7, 128), (8, 64), (12, 64), (15, 64)):
        assert ecf8.ecf8_encode(x, 1, x.size, max_code_len=cap).header.lane_syms == want
        for given in (32, 64, 128):
            assert ecf8.ecf8_encode(x, 1, x.size, max_code_len=cap, lane_syms=given).header.lane_syms == given


def test_threads_do_not_change_the_blob():
    x = _rand_bytes(1_500_001, 5)
    a = ecf8.ecf8_encode(x, 1, x.size, n_threads=1).numpy().copy()
    for t in (2, 3, 8):
        assert np.array_equal(a, ecf8.ecf8_encode(x, 1, x.size, n_threads=t).numpy())


def test_synthetic_config0_compresses_like_the_paper_band(orc):
    w = synth.make(synth.config0()[0], seed=0).numpy()
    b = ecf8.ecf8_encode(w)
    st = b.stats()
    assert st["entropy_bits"] <= st["avg_code_bits"] < st["entropy_bits"] + 1
    assert 0.75 < st["ratio"] < 0.93           # memory saving in the paper's 9.8-26.9 % range (Table 1)
    dec, _ = orc.container_decode(b.numpy())
    assert np.array_equal(dec, w.reshape(-1))


def test_container_files_round_trip(orc, tmp_path):
    x = _rand_bytes(70001, 9)
    b = ecf8.ecf8_encode(x, 1, x.size)
    path = str(tmp_path / "w.ecf8")
    ecf8.save_blob(path, b)
    hdr, arr = ecf8.load_blob(path)
    assert bytes(hdr) == bytes(b.header) and np.array_equal(arr, b.numpy())
    dec, _ = orc.container_decode(arr)
    assert np.array_equal(dec, x)
    with open(path, "r+b") as f:                      # a damaged file is refused
        f.seek(int(hdr.off_lane_bits))
        f.write(b"\xff\xff")
    with pytest.raises(ecf8.Ecf8Error):
        ecf8.load_blob(path)


def test_error_paths():
    x = _rand_bytes(1000, 1)
    with pytest.raises(ecf8.Ecf8Error) as e:
        ecf8.ecf8_encode(x, 0, 0)
    assert e.value.code == ecf8.E_ARG
    with pytest.raises(ecf8.Ecf8Error):
        ecf8.ecf8_encode(x, 1, 1000, lane_syms=48)
    for g in (3, 128):
        with pytest.raises(ecf8.Ecf8Error) as e:
            ecf8.ecf8_encode(x, 1, 1000, group_chunks=g)
        assert e.value.code == ecf8.E_ARG
    for cap in (3, 16):
        with pytest.raises(ecf8.Ecf8Error) as e:
            ecf8.ecf8_encode(x, 1, 1000, max_code_len=cap)
        assert e.value.code == ecf8.E_ARG
    good = ecf8.ecf8_encode(x, 10, 100).numpy().copy()
    ecf8.blob_validate(good)
    for off, val in [(0, 0), (4, 9), (40, 16), (46, 0), (46, 3), (56, 1), (64, 0), (16, 7)]:
        bad = good.copy()
        bad[off] = val
        with pytest.raises(ecf8.Ecf8Error) as e:
            ecf8.blob_validate(bad)
        assert e.value.code == ecf8.E_FORMAT
    with pytest.raises(ecf8.Ecf8Error):
        ecf8.blob_describe(good[:100].copy())
    with pytest.raises(ecf8.Ecf8Error):
        ecf8.blob_validate(good[:-256].copy())
    h = ecf8.blob_describe(good)
    bad = good.copy()
    bad[h.off_lane_bits] ^= 1
    with pytest.raises(ecf8.Ecf8Error):
        ecf8.blob_validate(bad)
    bad = good.copy()
    bad[h.off_chunk_bit + 8] ^= 2
    with pytest.raises(ecf8.Ecf8Error):
        ecf8.blob_validate(bad)
    # decode argument checks that need no device: null pointers, capacity, alignment
    lib = ctypes.CDLL(ecf8.LIB_PATH)
    assert lib.ecf8_decode(None, None, None, 0, None) == ecf8.E_ARG
    assert lib.ecf8_decode(ctypes.byref(h), ctypes.c_void_p(4096), ctypes.c_void_p(8192), ctypes.c_uint64(10), None) == ecf8.E_CAPACITY
    assert lib.ecf8_decode(ctypes.byref(h), ctypes.c_void_p(4097), ctypes.c_void_p(8192), ctypes.c_uint64(1000), None) == ecf8.E_ALIGN
    assert lib.ecf8_decode_batched(None, 1, 1, 64, None) == ecf8.E_ARG


@pytest.mark.parametrize("wide", [False, True])
def test_validate_survives_random_corruption(wide):
    """Single-byte damage anywhere in a container: the validator returns (accepts or rejects, never crashes or
    reads out of bounds), rejects every change to the metadata the kernels index with (chunk_bit, lane_bits)
    and every truncation, and accepts changes to the payload, which it cannot and need not judge."""
    rng = np.random.default_rng(11)
    if wide:
        from paper_2510_02676_amd import ecfw
        x = synth.make_bf16(300, 700, 1.8, 0.02, 3).numpy()
        good = ecfw.ecfw_encode(ecfw.FMT_BF16, x).numpy().copy()
        validate, h = ecfw.blob_validate, ecfw.blob_describe(good)
        Err = ecfw.EcfwError if hasattr(ecfw, "EcfwError") else ecf8.Ecf8Error
    else:
        x = synth.make_weight(300, 700, 1.8, 0.02, 3).numpy()
        good = ecf8.ecf8_encode(x, table_mode=1).numpy().copy()
        validate, h = ecf8.blob_validate, ecf8.blob_describe(good)
        Err = ecf8.Ecf8Error
    validate(good)
    verdicts = {"accepted": 0, "rejected": 0}
    for _ in range(1500):
        bad = good.copy()
        off = int(rng.integers(0, min(good.size, h.off_stream + 64)))        # header, tables, metadata, start of the stream
        bad[off] ^= np.uint8(1 << int(rng.integers(0, 8)))
        try:
            validate(bad)
            verdicts["accepted"] += 1
            assert not (h.off_chunk_bit <= off < h.off_chunk_bit + 8 * (h.n_chunks + 1)), off
            assert not (h.off_lane_bits <= off < h.off_lane_bits + 128 * h.n_chunks), off
        except Err:
            verdicts["rejected"] += 1
    assert verdicts["rejected"] > 100
    for cut in (1, 16, 255, 256, 4096, good.size // 2, good.size - 8):
        with pytest.raises(Err):
            validate(good[:good.size - cut].copy())
    for off in rng.integers(h.off_stream + 64, good.size, size=50):          # payload
        bad = good.copy()
        bad[int(off)] ^= 0x10
        validate(bad)


def test_gemm_group_prepare_is_pure_host_logic():
    """ecf8_gemm_group_prepare touches no device: with made-up (aligned) device addresses it lays the members out
    by their chunks of 16 x 256 weights, records the largest M and the kind of scales, and rejects mixed groups."""
    shapes, Ms = [(64, 512), (32, 7168), (160, 2048)], [3, 64, 16]
    hdrs = []
    for i, (rows, cols) in enumerate(shapes):
        w = synth.make_weight(rows, cols, 1.7, 0.02, i).numpy()
        hdrs.append(ecf8.ecf8_encode(w, rows, cols, lane_syms=64, tile_rows=16).header)
    n = len(shapes)

    def descs(raw=(False,) * 3, scaled=(0,) * 3):
        d = (ecf8.GemmGroupDesc * n)()
        for i in range(n):
            if raw[i]:
                d[i].rows, d[i].cols = shapes[i]
            else:
                d[i].hdr = ctypes.pointer(hdrs[i])
            d[i].d_w, d[i].d_x, d[i].d_y, d[i].M = 0x10000 * (i + 1), 0x2000000 + 0x10000 * i, 0x4000000 + 0x10000 * i, Ms[i]
            if scaled[i]:
                d[i].d_w_scale = 0x6000000
                if scaled[i] == 2:
                    d[i].d_x_scale, d[i].x_scale_cols = 0x7000000, shapes[i][1] // 128
        return d
    items, info = (ecf8.GemmGroupItem * n)(), ecf8.GemmGroupInfo()
    assert ecf8._lib.ecf8_gemm_group_prepare(descs(), n, items, ctypes.byref(info)) == ecf8.OK
    assert (info.total_work, info.n_items, info.max_M, info.scale_mode, info.raw) == (4 * 2 + 2 * 28 + 10 * 8, 3, 64, 0, 0)
    first_work = [items[i].opaque[0] for i in range(n)]
    assert first_work == [0, 8, 8 + 56]
    assert ecf8._lib.ecf8_gemm_group_prepare(descs(raw=(True,) * 3, scaled=(2,) * 3), n, items, ctypes.byref(info)) == ecf8.OK
    assert (info.scale_mode, info.raw) == (2, 1)
    for bad in (descs(raw=(False, True, False)), descs(scaled=(1, 0, 1)), descs(scaled=(1, 2, 1))):
        assert ecf8._lib.ecf8_gemm_group_prepare(bad, n, items, ctypes.byref(info)) == ecf8.E_ARG
    d = descs()
    d[1].M = 65
    assert ecf8._lib.ecf8_gemm_group_prepare(d, n, items, ctypes.byref(info)) == ecf8.E_ARG
    d = descs()
    d[2].d_x += 8
    assert ecf8._lib.ecf8_gemm_group_prepare(d, n, items, ctypes.byref(info)) == ecf8.E_ALIGN
    lin = ecf8.ecf8_encode(synth.make_weight(64, 512, 1.7, 0.02, 0).numpy(), 64, 512).header      # not row-tiled
    d = descs()
    d[0].hdr = ctypes.pointer(lin)
    assert ecf8._lib.ecf8_gemm_group_prepare(d, n, items, ctypes.byref(info)) == ecf8.E_ARG
    assert ecf8._lib.ecf8_gemm_group_prepare(descs(), 0, items, ctypes.byref(info)) == ecf8.E_ARG


def test_split_k_plan_is_pure_host_logic():
    """Slices = the largest divisor of cols / 256 with rows / 16 * slices <= compute units; workspace = 4096 bytes
    of counters + rows / 16 * slices * (1, 2, 4 KiB for M <= 16, 32, 64); nothing when the matrix has blocks enough."""
    want = {(256, 14336): 14, (576, 7168): 7, (1536, 7168): 2, (1024, 4096): 4, (4096, 4096): 1, (16, 256): 1,
            (2048, 7168): 2, (32, 512): 2, (48, 5120): 20, (16400, 4096): 1}
    for (rows, cols), sl in want.items():
        assert ecf8.gemm_splitk_plan(rows, cols, 1, 256) == (sl, 0 if sl == 1 else 4096 + rows // 16 * sl * 1024), (rows, cols)
        for s2 in range(sl + 1, cols // 256 + 1):
            assert (cols // 256) % s2 or rows // 16 * s2 > 256
    assert ecf8.gemm_splitk_plan(256, 14336, 17, 256)[1] == 4096 + 16 * 14 * 2048
    assert ecf8.gemm_splitk_plan(256, 14336, 64, 256)[1] == 4096 + 16 * 14 * 4096
    assert ecf8.gemm_splitk_plan(256, 14336, 64, 64) == (4, 4096 + 16 * 4 * 4096)      # a smaller chip splits less
    assert ecf8.gemm_splitk_plan(256, 14336, 64, 8)[0] == 1
    for bad in ((250, 14336, 1), (256, 1000, 1), (256, 14336, 0), (256, 14336, 65), (0, 256, 1)):
        with pytest.raises(ecf8.Ecf8Error) as e:
            ecf8.gemm_splitk_plan(*bad, 256)
        assert e.value.code == ecf8.E_ARG

"""Pins of the CPU oracle against what the paper and the mathematics fix.

Nothing here touches the product.  Each test is chosen so that a plausible
mistake in the oracle (dropped term, wrong bit order, transposed nibble, wrong
tie handling that loses optimality, off-by-one in metadata) fails it.
"""
import itertools
import math
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _gold(name):
    d = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, _, v = line.partition(" ")
            d[k] = v.split()
    return d


def _bytes_from(exps, rng):
    exps = np.asarray(exps, dtype=np.uint8)
    s = rng.integers(0, 2, size=exps.size, dtype=np.uint8)
    m = rng.integers(0, 8, size=exps.size, dtype=np.uint8)
    return ((s << 7) | (exps << 3) | m).astype(np.uint8)


def _kraft_num(lengths):
    # sum of 2^(15-l) over coded symbols; equals 2^15 iff the Kraft sum is exactly one
    return sum(1 << (15 - int(l)) for l in lengths if l > 0)


def _np_entropy(freq):
    f = np.asarray(freq, dtype=np.float64)
    p = f[f > 0] / f.sum()
    return float(-(p * np.log2(p)).sum())


# ---------------------------------------------------------------- identity

def test_roundtrip_every_byte_value(orc):
    """Losslessness (Section 4: bit-exact reconstruction) for all 256 encodings,
    including -0, subnormals and the two NaN encodings 0x7F / 0xFF."""
    x = np.arange(256, dtype=np.uint8)
    out, nbits, _ = orc.roundtrip(x)
    assert np.array_equal(out, x)
    assert nbits == 256 * 4  # uniform exponents: no gain


@pytest.mark.parametrize("n", [1, 2, 3, 7, 8, 9, 63, 64, 65, 1000, 4097])
def test_roundtrip_ragged_sizes(orc, n):
    rng = np.random.default_rng(n)
    p = rng.dirichlet(np.ones(16) * 0.3)
    x = _bytes_from(rng.choice(16, size=n, p=p), rng)
    out, nbits, ln = orc.roundtrip(x)
    assert np.array_equal(out, x)
    assert nbits == orc.stream_bits(orc.histogram(x), ln)


# ---------------------------------------------------------------- code lengths

@pytest.mark.parametrize("seed", range(40))
def test_kraft_equality_and_entropy_sandwich(orc, seed):
    """An optimal prefix code is complete (Kraft sum exactly 1) and its mean
    length obeys H <= Lbar < H + 1 (Section 2: L_min = H(E))."""
    rng = np.random.default_rng(seed)
    k = int(rng.integers(2, 17))
    freq = np.zeros(16, dtype=np.uint64)
    idx = rng.choice(16, size=k, replace=False)
    if seed % 3 == 0:   # geometric-ish, long codes
        freq[idx] = (2.0 ** rng.uniform(0, 30, size=k)).astype(np.uint64) + 1
    else:
        freq[idx] = rng.integers(1, 10 ** 6, size=k).astype(np.uint64)
    ln = orc.huffman_lengths(freq)
    assert all((ln[i] > 0) == (freq[i] > 0) for i in range(16))
    assert ln.max() <= 15
    assert _kraft_num(ln) == 1 << 15
    n = float(freq.sum())
    lbar = orc.stream_bits(freq, ln) / n
    h = _np_entropy(freq)
    assert h - 1e-9 <= lbar < h + 1
    assert abs(orc.entropy_bits(freq) - h) < 1e-9


def _brute_force_cost(freqs):
    k = len(freqs)
    best = None
    for ls in itertools.product(range(1, k), repeat=k):
        if sum(2.0 ** -l for l in ls) <= 1.0 + 1e-12:
            c = sum(f * l for f, l in zip(freqs, ls))
            best = c if best is None or c < best else best
    return best


@pytest.mark.parametrize("seed", range(25))
def test_huffman_is_optimal_by_brute_force(orc, seed):
    """min over ALL length vectors satisfying Kraft == the oracle's cost (k <= 6)."""
    rng = np.random.default_rng(1000 + seed)
    k = int(rng.integers(2, 7))
    fr = [int(v) for v in rng.integers(1, 40, size=k)]
    if seed % 5 == 0:
        fr = [1] * k  # all ties
    pos = sorted(int(v) for v in rng.choice(16, size=k, replace=False))
    freq = np.zeros(16, dtype=np.uint64)
    for p_, f in zip(pos, fr):
        freq[p_] = f
    ln = orc.huffman_lengths(freq)
    assert orc.stream_bits(freq, ln) == _brute_force_cost(fr)


def _brute_force_cost_limited(freqs, lmax):
    best = None
    for ls in itertools.product(range(1, lmax + 1), repeat=len(freqs)):
        if sum(2.0 ** -l for l in ls) <= 1.0 + 1e-12:
            c = sum(f * l for f, l in zip(freqs, ls))
            best = c if best is None or c < best else best
    return best


@pytest.mark.parametrize("seed", range(30))
def test_length_limited_code_is_optimal_by_brute_force(orc, seed):
    """min over ALL length vectors <= lmax satisfying Kraft == the oracle's capped cost (k <= 6),
    on skewed histograms where the cap binds."""
    rng = np.random.default_rng(2000 + seed)
    k = int(rng.integers(2, 7))
    fr = [int(v) for v in (2.0 ** rng.uniform(0, 12, size=k)).astype(np.int64) + 1]
    if seed % 6 == 0:
        fr = [1, 1, 2, 3, 5, 8][:k]            # Fibonacci: the uncapped tree is a chain
    pos = sorted(int(v) for v in rng.choice(16, size=k, replace=False))
    freq = np.zeros(16, dtype=np.uint64)
    for p_, f in zip(pos, fr):
        freq[p_] = f
    lo = int(np.ceil(np.log2(k)))
    for lmax in range(max(lo, 1), 6):
        ln = orc.huffman_lengths_limited(freq, lmax)
        assert ln.max() <= lmax and all((ln[i] > 0) == (freq[i] > 0) for i in range(16))
        assert sum(2.0 ** -int(l) for l in ln if l) <= 1.0
        assert orc.stream_bits(freq, ln) == _brute_force_cost_limited(fr, lmax)


def test_length_limited_code_special_cases(orc):
    fib = np.array([1, 1, 2, 3, 5, 8, 13, 21, 34, 55, 89, 144, 233, 377, 610, 987], dtype=np.uint64)
    # a cap that does not bind gives the Huffman cost; costs never fall as the cap tightens
    assert orc.stream_bits(fib, orc.huffman_lengths_limited(fib, 15)) == orc.stream_bits(fib, orc.huffman_lengths(fib))
    costs = [orc.stream_bits(fib, orc.huffman_lengths_limited(fib, L)) for L in range(4, 16)]
    assert all(a >= b for a, b in zip(costs, costs[1:])) and costs[0] > costs[-1]
    # 16 symbols under a cap of 4: the only code is the fixed-length one
    assert list(orc.huffman_lengths_limited(fib, 4)) == [4] * 16
    # Kraft holds with equality for every cap (a cheapest code wastes no code space)
    for L in range(4, 16):
        ln = orc.huffman_lengths_limited(fib, L)
        assert sum(1 << (15 - int(l)) for l in ln) == 1 << 15 and ln.max() <= L
    # hand case: frequencies 8 4 2 1 1 under cap 3: lengths 1 3 3 3 3 cost 32, or 2 2 2 3 3 cost 34 -> 32;
    # uncapped Huffman gives 1 2 3 4 4 cost 30
    f = np.zeros(16, dtype=np.uint64)
    f[[2, 4, 6, 8, 10]] = [8, 4, 2, 1, 1]
    assert orc.stream_bits(f, orc.huffman_lengths(f)) == 30
    assert orc.stream_bits(f, orc.huffman_lengths_limited(f, 3)) == 32
    one = np.zeros(16, dtype=np.uint64)
    one[5] = 77
    assert list(orc.huffman_lengths_limited(one, 7)) == [0] * 5 + [1] + [0] * 10
    with pytest.raises(ValueError):
        orc.huffman_lengths_limited(fib, 3)     # 16 symbols do not fit 3 bits
    with pytest.raises(ValueError):
        orc.huffman_lengths_limited(np.zeros(16, dtype=np.uint64), 7)


def test_fig2_worked_example(orc):
    """Figure 2: 'aaabbcddeeeee' costs 29 bits; the drawn tree's 2-bit cascaded
    table has root {e, e, a, ->1} and sub-table {b, b, c, d}."""
    g = _gold("fig2_example.txt")
    fr = {kv.split("=")[0]: int(kv.split("=")[1]) for kv in g["freq"]}
    sym = {"a": 3, "b": 5, "c": 6, "d": 9, "e": 12}  # arbitrary exponent slots, a<b<c<d<e
    freq = np.zeros(16, dtype=np.uint64)
    for ch, f in fr.items():
        freq[sym[ch]] = f
    ln = orc.huffman_lengths(freq)
    total = orc.stream_bits(freq, ln)
    assert total == int(g["total_bits"][0])
    assert abs(total / 13 - float(g["avg_len"][0])) < 1e-5
    assert abs(orc.entropy_bits(freq) - float(g["entropy"][0])) < 1e-5
    # the tree the figure draws, through the cascaded-table builder with 2-bit rows
    dl = {kv.split("=")[0]: int(kv.split("=")[1]) for kv in g["drawn_lengths"]}
    lens = np.zeros(16, dtype=np.uint8)
    for ch, l in dl.items():
        lens[sym[ch]] = l
    assert sum(fr[c] * dl[c] for c in fr) == 29
    codes = orc.canonical_codes(lens)
    assert [int(codes[sym[c]]) for c in "eabcd"] == [0b0, 0b10, 0b110, 0b1110, 0b1111]
    lut, n_luts = orc.paper_build_lut(lens, codes, width=2)
    assert n_luts == 3  # root, one sub-table, length table
    name = {v: k for k, v in sym.items()}
    root = [name.get(int(v), "ptr%d" % (256 - int(v))) for v in lut[0]]
    assert root == g["root"]
    assert [name[int(v)] for v in lut[1]] == g["sub1"]
    assert int(lut[0][3]) == 256 - 1  # pointer value 256 - index


def test_canonical_textbook_example(orc):
    g = _gold("canonical_example.txt")
    lens = np.zeros(16, dtype=np.uint8)
    lens[:8] = [int(v) for v in g["lengths"]]
    codes = orc.canonical_codes(lens)
    assert [int(c) for c in codes[:8]] == [int(v) for v in g["codes"]]


@pytest.mark.parametrize("seed", range(10))
def test_canonical_codes_prefix_free(orc, seed):
    rng = np.random.default_rng(77 + seed)
    freq = (2.0 ** rng.uniform(0, 24, size=16)).astype(np.uint64) + 1
    ln = orc.huffman_lengths(freq)
    codes = orc.canonical_codes(ln)
    words = [format(int(codes[s]), "0%db" % ln[s]) for s in range(16)]
    for a, b in itertools.permutations(words, 2):
        assert not b.startswith(a)


def test_special_histograms(orc):
    # uniform over 16 symbols: every code 4 bits, stream = n/2 bytes (no gain)
    freq = np.full(16, 1000, dtype=np.uint64)
    ln = orc.huffman_lengths(freq)
    assert list(ln) == [4] * 16
    assert orc.stream_bits(freq, ln) == 16000 * 4
    # dyadic 1/2, 1/4, ... : Lbar == H exactly
    freq = np.zeros(16, dtype=np.uint64)
    w = [2 ** 14 >> i for i in range(15)] + [1]
    freq[:] = w
    ln = orc.huffman_lengths(freq)
    assert sorted(ln) == sorted(list(range(1, 16)) + [15])
    assert abs(orc.stream_bits(freq, ln) / float(freq.sum()) - _np_entropy(freq)) < 1e-12
    # two symbols, however skewed: one bit each
    freq = np.zeros(16, dtype=np.uint64)
    freq[3], freq[11] = 1, 10 ** 9
    ln = orc.huffman_lengths(freq)
    assert ln[3] == 1 and ln[11] == 1 and ln.sum() == 2
    # a single distinct symbol: one 1-bit code (the documented exception to Kraft == 1)
    freq = np.zeros(16, dtype=np.uint64)
    freq[7] = 12345
    ln = orc.huffman_lengths(freq)
    assert ln[7] == 1 and ln.sum() == 1
    x = np.full(100, 7 << 3, dtype=np.uint8)
    out, nbits, _ = orc.roundtrip(x)
    assert nbits == 100 and np.array_equal(out, x)


def test_fibonacci_histogram_reaches_depth_15(orc):
    """The deepest tree 16 symbols allow: depth 15, so a 16-bit cap can never bind."""
    fib = [1, 1]
    while len(fib) < 16:
        fib.append(fib[-1] + fib[-2])
    freq = np.array(fib, dtype=np.uint64)
    ln = orc.huffman_lengths(freq)
    assert ln.max() == 15 and _kraft_num(ln) == 1 << 15
    x = _bytes_from(np.repeat(np.arange(16), fib), np.random.default_rng(5))
    np.random.default_rng(6).shuffle(x)
    out, _, _ = orc.roundtrip(x)
    assert np.array_equal(out, x)


# ---------------------------------------------------------------- hand example

def test_hand_worked_bytes(orc):
    g = _gold("hand_bytes.txt")
    x = np.array([int(v, 16) for v in g["input"]], dtype=np.uint8)
    freq = orc.histogram(x)
    assert freq[7] == 3 and freq[0] == 1 and freq.sum() == 4
    ln = orc.huffman_lengths(freq)
    assert ln[0] == int(g["len0"][0]) and ln[7] == int(g["len7"][0])
    codes = orc.canonical_codes(ln)
    assert codes[0] == 0 and codes[7] == 1
    s_msb, nb = orc.encode_exponents(x, ln, codes, orc.MSB_FIRST)
    assert nb == int(g["stream_bits"][0])
    assert [int(v) for v in s_msb] == [int(v, 16) for v in g["stream_msb_first"]]
    s_lsb, _ = orc.encode_exponents(x, ln, codes, orc.LSB_FIRST)
    assert [int(v) for v in s_lsb] == [int(v, 16) for v in g["stream_lsb_first"]]
    assert [int(v) for v in orc.pack_nibbles_paper(x)] == [int(v, 16) for v in g["plane_paper"]]
    out = orc.decode_serial(s_msb, nb, ln, orc.pack_nibbles_paper(x), 4, orc.MSB_FIRST)
    assert np.array_equal(out, x)
    # the chunked container of the same four bytes
    blob = orc.container_encode(x, 1, 4, 64)
    off_st = int(np.frombuffer(blob[96:104].tobytes(), "<u8")[0])
    off_pl = int(np.frombuffer(blob[104:112].tobytes(), "<u8")[0])
    assert int(blob[off_st]) == int(g["stream_lsb_first"][0], 16)
    assert [int(v) for v in blob[off_pl:off_pl + 4]] == [int(v, 16) for v in g["plane_container"]]
    dec, bits = orc.container_decode(blob)
    assert np.array_equal(dec, x) and bits == 4


def test_decoder_rejects_wrong_bit_order_and_truncation(orc):
    rng = np.random.default_rng(3)
    p = np.array([0.5, 0.25, 0.125, 0.0625] + [0.0625 / 12] * 12)
    x = _bytes_from(rng.choice(16, size=5000, p=p), rng)
    freq = orc.histogram(x)
    ln = orc.huffman_lengths(freq)
    codes = orc.canonical_codes(ln)
    s, nb = orc.encode_exponents(x, ln, codes, orc.MSB_FIRST)
    pk = orc.pack_nibbles_paper(x)
    assert np.array_equal(orc.decode_serial(s, nb, ln, pk, x.size, orc.MSB_FIRST), x)
    bad = None
    try:
        bad = orc.decode_serial(s, nb, ln, pk, x.size, orc.LSB_FIRST)
    except ValueError:
        pass
    assert bad is None or not np.array_equal(bad, x)
    with pytest.raises(ValueError):
        orc.decode_serial(s, nb - 1, ln, pk, x.size, orc.MSB_FIRST)
    with pytest.raises(ValueError):
        orc.decode_serial(s, nb, ln, pk, x.size - 1, orc.MSB_FIRST)


# ---------------------------------------------------------------- containers

@pytest.mark.parametrize("lane_syms", [16, 64, 128, 256])
@pytest.mark.parametrize("n", [1, 15, 16, 17, 4095, 4096, 4097, 3 * 8192 + 77])
def test_container_roundtrip_and_metadata(orc, lane_syms, n):
    rng = np.random.default_rng(n * 7 + lane_syms)
    p = rng.dirichlet(np.ones(16) * 0.4)
    x = _bytes_from(rng.choice(16, size=n, p=p), rng)
    blob = orc.container_encode(x, 1, n, lane_syms)
    dec, bits = orc.container_decode(blob)
    assert np.array_equal(dec, x)
    assert bits == orc.stream_bits(orc.histogram(x), orc.huffman_lengths(orc.histogram(x)))
    # independent view of the metadata: lane_bits must sum to chunk_bit differences
    hdr = np.frombuffer(blob[:256].tobytes(), "<u8")
    n_chunks = int(hdr[6])
    off_cb, off_lb = int(hdr[10]), int(hdr[11])
    cb = np.frombuffer(blob[off_cb:off_cb + 8 * (n_chunks + 1)].tobytes(), "<u8")
    lb = np.frombuffer(blob[off_lb:off_lb + 128 * n_chunks].tobytes(), "<u2").reshape(n_chunks, 64)
    assert cb[0] == 0 and cb[-1] == bits
    assert np.array_equal(np.diff(cb.astype(np.int64)), lb.sum(axis=1))


@pytest.mark.parametrize("lane_syms,group,n", [(32, 2, 4096), (32, 4, 8192 * 2 + 3000), (64, 8, 2 * 32768 + 4097),
                                               (128, 32, 262144 + 9000), (16, 64, 3 * 65536 + 1)])
def test_container_group_interleave(orc, lane_syms, group, n):
    """Whole groups of G chunks are interleaved block by block, the rest is chunk after chunk.
    The expected ownership is stated as array reshapes (axes: piece, chunk-in-group, lane, byte),
    not with the container's index formula."""
    rng = np.random.default_rng(n + group)
    p = rng.dirichlet(np.ones(16) * 0.4)
    x = _bytes_from(rng.choice(16, size=n, p=p), rng)
    blob = orc.container_encode(x, 1, n, lane_syms, group)
    dec, bits = orc.container_decode(blob)
    assert np.array_equal(dec, x)
    ln = orc.huffman_lengths(orc.histogram(x)).astype(np.int64)
    chunk = 64 * lane_syms
    n_chunks = -(-n // chunk)
    pieces = lane_syms // 16
    padded = np.zeros(n_chunks * chunk, dtype=np.int64)
    padded[:n] = ln[(x >> 3) & 15]                 # code bits per element, 0 for elements that do not exist
    whole = n // (group * chunk)
    want = np.zeros((n_chunks, 64), dtype=np.int64)
    for g in range(whole):
        blk = padded[g * group * chunk:(g + 1) * group * chunk].reshape(pieces, group, 64, 16)
        want[g * group:(g + 1) * group] = blk.sum(axis=(0, 3))
    for c in range(whole * group, n_chunks):
        want[c] = padded[c * chunk:(c + 1) * chunk].reshape(pieces, 64, 16).sum(axis=(0, 2))
    hdr = np.frombuffer(blob[:256].tobytes(), "<u8")
    off_lb = int(hdr[11])
    lb = np.frombuffer(blob[off_lb:off_lb + 128 * n_chunks].tobytes(), "<u2").reshape(n_chunks, 64)
    assert np.array_equal(lb.astype(np.int64), want)
    with pytest.raises(ValueError):
        orc.container_encode(x, 1, n, lane_syms, 3)
    bad = blob.copy()
    bad[46] = 0
    with pytest.raises(ValueError):
        orc.container_decode(bad)


@pytest.mark.parametrize("lane_syms,rows,cols", [(16, 16, 64), (32, 32, 256), (64, 48, 512), (128, 16, 1024)])
def test_container_row_tiled_layout(orc, lane_syms, rows, cols):
    """Row-tiled layout: chunk = 16 rows x 4N columns; lane l owns row l % 16 and, in every 64-column
    stripe of the block, the 16 columns starting at 16 (l / 16).  Stated as reshapes of the matrix
    (axes: block row, row in block, block column, stripe, lane group, byte), not with index arithmetic."""
    rng = np.random.default_rng(rows * cols + lane_syms)
    p = rng.dirichlet(np.ones(16) * 0.4)
    n = rows * cols
    x = _bytes_from(rng.choice(16, size=n, p=p), rng)
    blob = orc.container_encode(x, rows, cols, lane_syms, 1, 15, 16)
    assert blob[46] == 1 and blob[47] == 16
    dec, bits = orc.container_decode(blob)
    assert np.array_equal(dec, x)
    ln = orc.huffman_lengths(orc.histogram(x)).astype(np.int64)
    w = 4 * lane_syms
    cost = ln[(x >> 3) & 15].reshape(rows // 16, 16, cols // w, w // 64, 4, 16)
    # -> [block row, block col, lane group, row in block] summed over stripes and bytes
    want = cost.sum(axis=(3, 5)).transpose(0, 2, 3, 1).reshape(-1, 64)      # lane = 16 * group + row
    n_chunks = n // (64 * lane_syms)
    hdr = np.frombuffer(blob[:256].tobytes(), "<u8")
    off_lb = int(hdr[11])
    lb = np.frombuffer(blob[off_lb:off_lb + 128 * n_chunks].tobytes(), "<u2").reshape(n_chunks, 64)
    assert np.array_equal(lb.astype(np.int64), want)
    for bad_rows, bad_cols in ((rows + 8, cols), (rows, cols + 2 * lane_syms)):
        with pytest.raises(ValueError):
            orc.container_encode(np.zeros(bad_rows * bad_cols, np.uint8), bad_rows, bad_cols, lane_syms, 1, 15, 16)
    with pytest.raises(ValueError):
        orc.container_encode(x, rows, cols, lane_syms, 2, 15, 16)      # no interleave in this layout


def test_container_reader_catches_tampering(orc):
    rng = np.random.default_rng(11)
    p = rng.dirichlet(np.ones(16) * 0.4)
    x = _bytes_from(rng.choice(16, size=20000, p=p), rng)
    blob = orc.container_encode(x, 100, 200, 64)
    hdr = np.frombuffer(blob[:256].tobytes(), "<u8")
    off_cb, off_lb, off_st = int(hdr[10]), int(hdr[11]), int(hdr[12])

    def expect_fail(mutate):
        b = blob.copy()
        mutate(b)
        with pytest.raises(ValueError):
            orc.container_decode(b)

    expect_fail(lambda b: b.__setitem__(0, 0))                       # magic
    expect_fail(lambda b: b.__setitem__(off_lb + 2, b[off_lb + 2] ^ 1))   # one lane length
    expect_fail(lambda b: b.__setitem__(off_cb + 8, b[off_cb + 8] ^ 4))   # one chunk start
    expect_fail(lambda b: b.__setitem__(40, 48))                      # lane_syms no longer matches
    expect_fail(lambda b: b.__setitem__(64 + int(np.argmax(blob[64:80])), 1))  # a code length
    b = blob.copy()
    b[off_st + 5] ^= 0x10                                             # a stream bit
    try:
        dec, _ = orc.container_decode(b)
        assert not np.array_equal(dec, x)
    except ValueError:
        pass


def _ecf8_sections(blob):
    u64 = lambda o: int(np.frombuffer(blob[o:o + 8].tobytes(), "<u8")[0])
    return dict(n=u64(16), n_chunks=u64(48), bits=u64(56), off_cb=u64(80), off_lb=u64(88), off_st=u64(96),
                off_pl=u64(104), st_bytes=u64(112))


def test_container_backward_run_by_hand(orc):
    """tests/golden/container_backward_run.txt: 1026 bytes whose lane 0 carries two symbols of the backward
    run; stream bytes, lane_bits and chunk_bit derived by hand from the format description."""
    g = _gold("container_backward_run.txt")
    n, N = int(g["n"][0]), int(g["lane_syms"][0])
    x = np.full(n, 0x38, dtype=np.uint8)
    x[[int(v) for v in g["zero_elements"]]] = 0x00
    blob = orc.container_encode(x, 1, n, N, 1)
    s = _ecf8_sections(blob)
    assert s["n_chunks"] == 1 and s["bits"] == int(g["stream_bits"][0])
    lb = np.frombuffer(blob[s["off_lb"]:s["off_lb"] + 128].tobytes(), "<u2")
    assert lb[0] == int(g["lane_bits_lane0"][0]) and (lb[1:] == int(g["lane_bits_other"][0])).all()
    st = blob[s["off_st"]:s["off_st"] + s["st_bytes"]]
    used = int(g["stream_used_bytes"][0])
    head = [int(v, 16) for v in g["stream_head"]]
    assert [int(v) for v in st[:len(head)]] == head
    assert (st[len(head):used - 1] == 0xFF).all() and int(st[used - 1]) == int(g["stream_last"][0], 16)
    assert not st[used:].any()
    cb = np.frombuffer(blob[s["off_cb"]:s["off_cb"] + 16].tobytes(), "<u8")
    assert list(cb) == [0, 1026]
    dec, bits = orc.container_decode(blob)
    assert np.array_equal(dec, x) and bits == 1026
    # a reader that took the backward run in the forward direction would swap elements 1024 and 1025
    swapped = x.copy()
    swapped[1024], swapped[1025] = x[1025], x[1024]
    assert not np.array_equal(swapped, x)


@pytest.mark.parametrize("N,G,n_chunks_whole,extra", [(32, 1, 2, 0), (64, 1, 1, 16 * 100), (64, 2, 5, 16 * 7), (128, 4, 9, 16),
                                                      (128, 32, 33, 16 * 300), (64, 64, 64, 0)])
def test_stream_order_with_a_fixed_length_code(orc, N, G, n_chunks_whole, extra):
    """With a uniform exponent histogram every codeword is 4 bits long and the canonical code of field s is s,
    so the stream is an array of 4-bit fields: the element order (lane l of chunk c takes 16-element pieces
    l, l + 64, ...; the G chunks of a whole group alternate KiB by KiB), the bit order and the two run
    directions can be written down as array reshapes (axes: piece, chunk in group, lane, element in piece)
    and compared with the container's stream, lane_bits and chunk_bit byte for byte."""
    E = 64 * N
    n = n_chunks_whole * E + extra
    assert n % 16 == 0
    rng = np.random.default_rng(n + G)
    sym = rng.permutation(np.tile(np.arange(16), n // 16))      # exactly uniform: Huffman gives sixteen 4-bit codes
    x = _bytes_from(sym, rng)
    blob = orc.container_encode(x, 1, n, N, G)
    s = _ecf8_sections(blob)
    assert [int(v) for v in blob[64:80]] == [4] * 16
    n_chunks = s["n_chunks"]
    padded = np.full(n_chunks * E, -1, dtype=np.int64)
    padded[:n] = sym
    lanes = np.zeros((n_chunks, 64, N), dtype=np.int64)         # [chunk, lane, k]
    F = n // (G * E)
    for g in range(F):
        blk = padded[g * G * E:(g + 1) * G * E].reshape(N // 16, G, 64, 16)
        lanes[g * G:(g + 1) * G] = blk.transpose(1, 2, 0, 3).reshape(G, 64, N)
    for c in range(F * G, n_chunks):
        lanes[c] = padded[c * E:(c + 1) * E].reshape(N // 16, 64, 16).transpose(1, 0, 2).reshape(64, N)
    bits = []
    lane_bits = np.zeros((n_chunks, 64), dtype=np.int64)
    for c in range(n_chunks):
        for l in range(64):
            ks = lanes[c, l]
            fwd = [b for v in ks[:N // 2] if v >= 0 for b in format(int(v), "04b")]      # first bit = most significant
            bwd = [b for v in ks[N // 2:] if v >= 0 for b in format(int(v), "04b")]
            lane = fwd + bwd[::-1]                                                     # backward run: first bit highest
            lane_bits[c, l] = len(lane)
            bits.extend(lane)
    want = np.packbits(np.array(bits, dtype=np.uint8), bitorder="little")
    got = blob[s["off_st"]:s["off_st"] + s["st_bytes"]]
    assert np.array_equal(got[:want.size], want) and not got[want.size:].any()
    lb = np.frombuffer(blob[s["off_lb"]:s["off_lb"] + 128 * n_chunks].tobytes(), "<u2").reshape(n_chunks, 64)
    assert np.array_equal(lb, lane_bits)
    cb = np.frombuffer(blob[s["off_cb"]:s["off_cb"] + 8 * (n_chunks + 1)].tobytes(), "<u8")
    assert np.array_equal(cb, np.concatenate([[0], np.cumsum(lane_bits.sum(axis=1))]).astype(np.uint64))
    dec, _ = orc.container_decode(blob)
    assert np.array_equal(dec, x)


@pytest.mark.parametrize("N,rows,cols", [(32, 16, 128), (64, 32, 512), (128, 16, 1024), (64, 48, 256)])
def test_row_tiled_stream_order_with_a_fixed_length_code(orc, N, rows, cols):
    """The row-tiled layout the same way: chunk c is block c of the matrix cut into 16 rows x 4N columns (along a
    row of blocks first), lane l = 16 g + r works on row r of the block, and its k-th symbol is column
    64 (k / 16) + 16 g + k % 16: as a reshape of the block with axes (row, piece, g, element in piece)."""
    n = rows * cols
    rng = np.random.default_rng(n + N)
    sym = rng.permutation(np.tile(np.arange(16), n // 16)).reshape(rows, cols)
    x = _bytes_from(sym.reshape(-1), rng)
    blob = orc.container_encode(x, rows, cols, N, 1, 15, 16)
    s = _ecf8_sections(blob)
    assert [int(v) for v in blob[64:80]] == [4] * 16
    bits = []
    for br in range(rows // 16):
        for bc in range(cols // (4 * N)):
            block = sym[16 * br:16 * br + 16, 4 * N * bc:4 * N * (bc + 1)]
            lanes = block.reshape(16, N // 16, 4, 16).transpose(2, 0, 1, 3).reshape(64, N)    # [g, r] -> lane 16 g + r
            for l in range(64):
                fwd = [b for v in lanes[l, :N // 2] for b in format(int(v), "04b")]
                bwd = [b for v in lanes[l, N // 2:] for b in format(int(v), "04b")]
                bits.extend(fwd + bwd[::-1])
    want = np.packbits(np.array(bits, dtype=np.uint8), bitorder="little")
    got = blob[s["off_st"]:s["off_st"] + s["st_bytes"]]
    assert np.array_equal(got[:want.size], want) and not got[want.size:].any()
    dec, _ = orc.container_decode(blob)
    assert np.array_equal(dec, x)


# ---------------------------------------------------------------- the paper's own container

@pytest.mark.parametrize("T", [32, 256])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_paper_algorithm1_emulator_roundtrip(orc, T, seed):
    """Algorithm 1 with B = 8 over gaps/outpos/cascaded tables built per Section 3.1
    gives back the input: the readings of the garbled passages are consistent."""
    rng = np.random.default_rng(seed)
    if seed == 0:
        p = np.array([2.0 ** -min(i + 1, 15) for i in range(16)])  # very long codes, two levels
    elif seed == 1:
        p = rng.dirichlet(np.ones(16) * 0.5)
    else:
        p = np.full(16, 1.0)
    p = p / p.sum()
    n = 70001
    x = _bytes_from(rng.choice(16, size=n, p=p), rng)
    out, c = orc.paper_alg1_roundtrip(x, T)
    assert np.array_equal(out, x)
    # gap and outpos re-derived here from the codeword start positions
    ln, codes = c["lengths"], orc.canonical_codes(c["lengths"])
    starts = np.concatenate([[0], np.cumsum(ln[(x >> 3) & 15].astype(np.int64))])
    assert c["stream_bits"] == starts[-1]
    for tg in [0, 1, 2, 17, c["n_blocks"] * T // 2]:
        w0 = tg * 64
        j = int(np.searchsorted(starts[:-1], w0, side="left"))
        if j < n:
            g = (int(c["gaps"][tg // 2]) >> (4 - (tg % 2) * 4)) & 15
            assert g == starts[j] - w0 and 0 <= g <= 15
    for b in range(c["n_blocks"]):
        assert c["outpos"][b] == np.searchsorted(starts[:-1], b * T * 64, side="left")
    assert c["outpos"][-1] == n
    assert c["n_luts"] == 2 + len({int(codes[s]) >> (int(ln[s]) - 8) for s in range(16) if ln[s] > 8})


def test_paper_single_symbol_and_tiny(orc):
    x = np.full(777, (5 << 3) | 0x83, dtype=np.uint8)
    out, _ = orc.paper_alg1_roundtrip(x, 32)
    assert np.array_equal(out, x)
    x = np.array([0x38, 0xB8, 0x3C, 0x00], dtype=np.uint8)
    out, _ = orc.paper_alg1_roundtrip(x, 32)
    assert np.array_equal(out, x)


def test_paper_metadata_checks_catch_planted_mistakes(orc):
    """The window decoder insists that every gap lands on a codeword start and that a block's counts add up
    to its share of outpos; the table check insists that the cascaded table says what the code says.  A
    mistake planted in the gaps, in outpos or in the table must be caught."""
    import ctypes
    rng = np.random.default_rng(5)
    p = np.array([2.0 ** -min(i + 1, 15) for i in range(16)])
    x = _bytes_from(rng.choice(16, size=30011, p=p / p.sum()), rng)
    T = 32
    out, c = orc.paper_alg1_roundtrip(x, T)
    assert np.array_equal(out, x)
    L = orc.lib()
    L.orc_paper_lut_mismatches.restype = ctypes.c_int64

    def decode(gaps, outpos):
        res = np.zeros(x.size, dtype=np.uint8)
        rc = L.orc_paper_window_decode(orc._p(c["lengths"]), orc._p(c["encoded"]), ctypes.c_uint64(c["encoded"].size),
                                       orc._p(c["packed"]), orc._p(outpos), orc._p(gaps), ctypes.c_uint64(c["n_blocks"]),
                                       ctypes.c_uint32(T), ctypes.c_uint64(x.size), orc._p(res))
        return rc, res
    rc, res = decode(c["gaps"], c["outpos"])
    assert rc == 0 and np.array_equal(res, x)
    # the first gap nibble whose value can be raised by one
    tg = next(t for t in range(2, 200) if 0 < ((int(c["gaps"][t // 2]) >> (4 - (t % 2) * 4)) & 15) < 15)
    bad = c["gaps"].copy()
    bad[tg // 2] = (int(bad[tg // 2]) + (0x10 if tg % 2 == 0 else 0x01)) & 0xFF
    rc, res = decode(bad, c["outpos"])
    assert rc != 0 or not np.array_equal(res, x)
    assert rc == orc.E_META or rc == orc.E_CODE
    bad_pos = c["outpos"].copy()
    bad_pos[1] += 1
    assert decode(c["gaps"], bad_pos)[0] == orc.E_META
    assert L.orc_paper_lut_mismatches(orc._p(c["lengths"]), orc._p(c["lut"]), ctypes.c_uint32(c["n_luts"])) == 0
    lut = c["lut"].copy()
    lut[3] = (int(lut[3]) + 1) % 16
    assert L.orc_paper_lut_mismatches(orc._p(c["lengths"]), orc._p(lut), ctypes.c_uint32(c["n_luts"])) > 0

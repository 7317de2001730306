"""Pins of the wide-alphabet CPU oracle (E5M2, BF16) against what the formats and
the mathematics fix.  Nothing here touches the product.

The paper's method (Section 3.1) with the exponent field as the coded symbol; the
16-bit cap on codewords that Section 3.1 mentions binds for these alphabets, so the
length-limited code is pinned hardest: brute force over every length assignment,
textbook Huffman, the independent exhaustive search of the 16-symbol oracle.
"""
import heapq
import itertools
import os

import numpy as np
import pytest
import torch

GOLD = os.path.join(os.path.dirname(__file__), "golden")
E5M2, BF16 = 1, 2


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


def _rand_elems(fmt, n, rng, spread=3.0):
    """Elements whose exponent field is concentrated around a centre (normal-ish), other bits uniform."""
    if fmt == BF16:
        e = np.clip(np.rint(rng.normal(120, spread, n)), 0, 255).astype(np.uint16)
        return ((rng.integers(0, 2, n).astype(np.uint16) << 15) | (e << 7) | rng.integers(0, 128, n).astype(np.uint16))
    e = np.clip(np.rint(rng.normal(14, spread, n)), 0, 31).astype(np.uint8)
    return ((rng.integers(0, 2, n).astype(np.uint8) << 7) | (e << 2) | rng.integers(0, 4, n).astype(np.uint8))


def _heap_huffman_cost(freq):
    h = [int(f) for f in freq if f]
    if len(h) == 1:
        return h[0]
    heapq.heapify(h)
    cost = 0
    while len(h) > 1:
        a, b = heapq.heappop(h), heapq.heappop(h)
        cost += a + b
        heapq.heappush(h, a + b)
    return cost


def _kraft(lengths, L=16):
    return sum(1 << (L - int(l)) for l in lengths if l)


# ---------------------------------------------------------------- fields

def test_hand_worked_values(orc):
    g = _gold("wide_hand.txt")
    xb = np.array([int(v, 16) for v in g["bf16"]], dtype=np.uint16)
    xe = np.array([int(v, 16) for v in g["e5m2"]], dtype=np.uint8)
    # the fixture's bit patterns are the values it names
    vals = [1.0, -2.0, 0.5, 1.5]
    assert torch.tensor(xb.astype(np.int32)).to(torch.int16).view(torch.bfloat16).float().tolist() == vals
    assert torch.tensor(xe).view(torch.float8_e5m2).float().tolist() == vals
    for fmt, x, key in ((BF16, xb, "bf16"), (E5M2, xe, "e5m2")):
        sym, rem = orc.w_split(fmt, x)
        assert sym.tolist() == [int(v) for v in g[key + "_exp"]]
        assert rem.tolist() == [int(v, 16) for v in g[key + "_rem"]]
        freq = orc.w_histogram(fmt, x)
        ln, cost = orc.w_lengths_limited(freq, 16)
        mid, low, high = sym[0], sym[2], sym[1]
        assert (ln[mid], ln[low], ln[high]) == (int(g["len_mid"][0]), int(g["len_low"][0]), int(g["len_high"][0]))
        assert cost == int(g["stream_bits"][0])
        blob = orc.w_container_encode(fmt, x, 1, 4, 64, 1, ln)
        off_st = int(np.frombuffer(blob[112:120].tobytes(), "<u8")[0])
        off_pl = int(np.frombuffer(blob[120:128].tobytes(), "<u8")[0])
        off_sg = int(np.frombuffer(blob[128:136].tobytes(), "<u8")[0])
        assert blob[off_st] == int(g["stream_byte0"][0], 16) and not blob[off_st + 1:off_st + 16].any()
        assert blob[off_pl:off_pl + 4].tolist() == [int(v, 16) for v in g[key + "_plane"]]
        if fmt == E5M2:
            assert blob[off_sg:off_sg + 2].tolist() == [int(v, 16) for v in g["e5m2_sign"]]
        else:
            assert off_sg == 0


def test_bf16_fields_against_frexp(orc):
    """Exponent field = floor(log2 |x|) + 127 for normal values; sign and 7-bit mantissa from the value."""
    rng = np.random.default_rng(1)
    v = torch.tensor(rng.standard_normal(4096) * np.exp(rng.uniform(-20, 20, 4096)), dtype=torch.float32)
    xb = v.to(torch.bfloat16)
    x = xb.view(torch.int16).numpy().view(np.uint16)
    sym, rem = orc.w_split(BF16, x)
    f = xb.float().numpy().astype(np.float64)
    m, e = np.frexp(np.abs(f))                       # |f| = m 2^e, m in [0.5, 1)
    assert np.array_equal(sym, (e - 1 + 127).astype(np.uint8))
    assert np.array_equal(rem >> 7, (f < 0).astype(np.uint8))
    assert np.array_equal(rem & 127, np.rint((m * 2 - 1) * 128).astype(np.uint8))


def test_e5m2_fields_against_frexp(orc):
    x = np.arange(256, dtype=np.uint8)
    sym, rem = orc.w_split(E5M2, x)
    f = torch.tensor(x).view(torch.float8_e5m2).float().numpy().astype(np.float64)
    finite = np.isfinite(f) & (sym > 0)
    m, e = np.frexp(np.abs(f[finite]))
    assert np.array_equal(sym[finite], (e - 1 + 15).astype(np.uint8))          # bias 15
    assert np.array_equal(rem[finite] & 3, np.rint((m * 2 - 1) * 4).astype(np.uint8))
    assert np.array_equal(rem[finite] >> 2, np.signbit(f[finite]).astype(np.uint8))
    sub = sym == 0                                    # zero and subnormals: value = mantissa * 2^-16
    assert np.array_equal(np.abs(f[sub]), (rem[sub] & 3) * 2.0 ** -16)
    assert np.all(~np.isfinite(f[sym == 31]))         # exponent field all ones: infinities and NaNs


@pytest.mark.parametrize("fmt", [E5M2, BF16])
def test_histogram_counts(orc, fmt):
    rng = np.random.default_rng(2)
    x = _rand_elems(fmt, 5000, rng)
    sym, _ = orc.w_split(fmt, x)
    freq = orc.w_histogram(fmt, x)
    assert np.array_equal(freq, np.bincount(sym, minlength=freq.size).astype(np.uint64))
    assert freq.sum() == 5000


# ---------------------------------------------------------------- code lengths

def test_huffman_textbook_example(orc):
    """The classic six-symbol example (frequencies 45 13 12 16 9 5): 224 bits in total."""
    freq = np.array([45, 13, 12, 16, 9, 5, 0, 0], dtype=np.uint64)
    ln = orc.w_huffman_lengths(freq)
    assert ln.tolist() == [1, 3, 3, 3, 4, 4, 0, 0]
    assert orc.w_stream_bits(freq, ln) == 224
    ln2, cost = orc.w_lengths_limited(freq, 16)
    assert cost == 224 and orc.w_stream_bits(freq, ln2) == 224


@pytest.mark.parametrize("seed", range(6))
def test_huffman_cost_matches_heap_merge(orc, seed):
    rng = np.random.default_rng(seed)
    freq = np.zeros(256, dtype=np.uint64)
    k = int(rng.integers(2, 60))
    freq[rng.choice(256, k, replace=False)] = np.maximum(1, (rng.pareto(0.7, k) * 10).astype(np.uint64))
    ln = orc.w_huffman_lengths(freq)
    assert orc.w_stream_bits(freq, ln) == _heap_huffman_cost(freq)
    assert _kraft(ln, 64) == 1 << 64                # a full binary tree
    assert np.array_equal(ln > 0, freq > 0)
    if ln.max() <= 16:                               # the cap does not bind: same cost
        assert orc.w_lengths_limited(freq, 16)[1] == _heap_huffman_cost(freq)


@pytest.mark.parametrize("seed", range(8))
def test_limited_lengths_brute_force(orc, seed):
    """Every assignment of lengths 1..L to up to 6 symbols, kept if Kraft allows it."""
    rng = np.random.default_rng(100 + seed)
    k = int(rng.integers(2, 7))
    f = np.maximum(1, (rng.pareto(0.6, k) * 5).astype(np.int64))
    freq = np.zeros(32, dtype=np.uint64)
    pos = rng.choice(32, k, replace=False)
    freq[pos] = f
    for L in range(1, 6):
        best = None
        for ls in itertools.product(range(1, L + 1), repeat=k):
            if sum(2.0 ** -l for l in ls) <= 1.0:
                c = int(sum(int(a) * b for a, b in zip(f, ls)))
                best = c if best is None else min(best, c)
        if best is None:
            with pytest.raises(ValueError):
                orc.w_lengths_limited(freq, L)
            continue
        ln, cost = orc.w_lengths_limited(freq, L)
        assert cost == best
        assert orc.w_stream_bits(freq, ln) == best and ln.max() <= L and _kraft(ln) <= 1 << 16
        assert np.array_equal(ln > 0, freq > 0)


@pytest.mark.parametrize("seed", range(5))
def test_limited_lengths_match_the_16_symbol_search(orc, seed):
    """Same optimum as the exhaustive search over sorted length sequences that pins the E4M3 path."""
    rng = np.random.default_rng(200 + seed)
    freq = np.zeros(16, dtype=np.uint64)
    k = int(rng.integers(3, 17))
    freq[rng.choice(16, k, replace=False)] = np.maximum(1, (rng.pareto(0.5, k) * 3).astype(np.uint64))
    for L in (4, 5, 7, 10):
        ln16 = orc.huffman_lengths_limited(freq, L)
        _, cost = orc.w_lengths_limited(freq, L)
        assert cost == orc.stream_bits(freq, ln16)


def test_limited_lengths_special_cases(orc):
    # Fibonacci weights: Huffman is a chain of depth k-1, so every cap below that binds
    fib = [1, 1, 2, 3, 5, 8, 13, 21, 34, 55, 89, 144, 233, 377, 610, 987, 1597, 2584, 4181, 6765]
    freq = np.zeros(32, dtype=np.uint64)
    freq[:20] = fib
    assert orc.w_huffman_lengths(freq).max() == 19
    costs = [orc.w_lengths_limited(freq, L)[1] for L in range(5, 17)]
    assert all(a > b for a, b in zip(costs, costs[1:]))      # each extra bit of depth still pays here
    assert costs[-1] > _heap_huffman_cost(freq)               # 16 < 19: the cap costs something
    for L in range(5, 17):
        ln, _ = orc.w_lengths_limited(freq, L)
        assert ln.max() == L and _kraft(ln) == 1 << 16       # complete code that uses the cap
    # 2^k equally likely symbols under the cap k: everything has length k
    freq = np.zeros(256, dtype=np.uint64)
    freq[:64] = 7
    ln, cost = orc.w_lengths_limited(freq, 6)
    assert ln[:64].tolist() == [6] * 64 and cost == 7 * 64 * 6
    with pytest.raises(ValueError):
        orc.w_lengths_limited(freq, 5)                        # 64 symbols do not fit 5 bits
    # one symbol: one bit
    freq = np.zeros(32, dtype=np.uint64)
    freq[9] = 11
    assert orc.w_lengths_limited(freq, 16)[0][9] == 1 and orc.w_huffman_lengths(freq)[9] == 1
    # all 256 symbols with geometric weights under the cap 16
    freq = np.array([max(1, 2 ** 40 >> i) for i in range(256)], dtype=np.uint64)
    ln, cost = orc.w_lengths_limited(freq, 16)
    assert ln.max() == 16 and _kraft(ln) <= 1 << 16 and cost == orc.w_stream_bits(freq, ln)
    assert np.all(np.diff(ln.astype(int)) >= 0)               # rarer symbols never get shorter codes


def test_entropy_bounds(orc):
    rng = np.random.default_rng(3)
    x = _rand_elems(BF16, 200000, rng, spread=2.0)
    freq = orc.w_histogram(BF16, x)
    p = freq[freq > 0] / freq.sum()
    H = float(-(p * np.log2(p)).sum())
    avg = orc.w_lengths_limited(freq, 16)[1] / x.size
    assert H <= avg < H + 1
    assert orc.w_lengths_limited(freq, 8)[1] >= orc.w_lengths_limited(freq, 12)[1] >= orc.w_lengths_limited(freq, 16)[1]


def test_canonical_codes(orc):
    g = _gold("canonical_example.txt")
    ln = np.zeros(32, dtype=np.uint8)
    ln[:8] = [int(v) for v in g["lengths"]]
    assert orc.w_canonical(ln)[:8].tolist() == [int(v) for v in g["codes"]]
    rng = np.random.default_rng(4)
    freq = np.zeros(256, dtype=np.uint64)
    freq[rng.choice(256, 40, replace=False)] = (rng.pareto(0.5, 40) * 4 + 1).astype(np.uint64)
    ln, _ = orc.w_lengths_limited(freq, 12)
    code = orc.w_canonical(ln)
    words = sorted((format(int(code[s]), "0%db" % ln[s]), s) for s in range(256) if ln[s])
    for (a, _), (b, _) in zip(words, words[1:]):
        assert not b.startswith(a)                            # prefix-free
    order = sorted((int(ln[s]), s) for s in range(256) if ln[s])
    # numerically increasing when left-aligned, in (length, symbol) order
    aligned = [int(code[s]) << (16 - l) for l, s in order]
    assert aligned == sorted(aligned) and aligned[0] == 0
    bad = np.zeros(32, dtype=np.uint8)
    bad[:3] = 1
    with pytest.raises(ValueError):
        orc.w_canonical(bad)                                  # three 1-bit codes overfill the space


# ---------------------------------------------------------------- container

def _sections(blob):
    u64 = lambda o: int(np.frombuffer(blob[o:o + 8].tobytes(), "<u8")[0])
    u32 = lambda o: int(np.frombuffer(blob[o:o + 4].tobytes(), "<u4")[0])
    return dict(total=u64(8), n=u64(16), fmt=u32(40), N=u32(44), G=u32(48), maxlen=u32(52), A=u32(56), nsym=u32(60),
                n_chunks=u64(64), bits=u64(72), off_len=u64(80), off_freq=u64(88), off_cb=u64(96), off_lb=u64(104),
                off_st=u64(112), off_pl=u64(120), off_sg=u64(128), st_bytes=u64(136), pl_bytes=u64(144),
                sg_bytes=u64(152))


@pytest.mark.parametrize("fmt", [E5M2, BF16])
@pytest.mark.parametrize("N,G,n", [(64, 1, 1), (64, 1, 4095), (64, 2, 64 * 64 * 5 + 17), (128, 4, 128 * 64 * 9 + 1),
                                   (128, 1, 128 * 64), (64, 32, 64 * 64 * 70 + 333), (128, 64, 128 * 64 * 64)])
def test_container_roundtrip(orc, fmt, N, G, n):
    rng = np.random.default_rng(n + N + G)
    x = _rand_elems(fmt, n, rng)
    freq = orc.w_histogram(fmt, x)
    ln, cost = orc.w_lengths_limited(freq, 9)
    blob = orc.w_container_encode(fmt, x, 1, n, N, G, ln)
    y, bits = orc.w_container_decode(blob)
    assert np.array_equal(y, x) and y.dtype == x.dtype
    s = _sections(blob)
    assert bits == cost == s["bits"] and s["total"] == blob.size and s["n_chunks"] == -(-n // (64 * N))
    assert all(s[k] % 256 == 0 for k in s if k.startswith("off_"))
    assert s["st_bytes"] == -(-((cost + 7) // 8 + 8) // 16) * 16
    assert s["pl_bytes"] == s["n_chunks"] * (64 * N if fmt == BF16 else 16 * N)
    assert s["sg_bytes"] == (0 if fmt == BF16 else s["n_chunks"] * 8 * N)


@pytest.mark.parametrize("fmt", [E5M2, BF16])
def test_every_bit_pattern_roundtrips(orc, fmt):
    """Losslessness for every encoding: zeros, subnormals, infinities, NaN payloads."""
    x = np.arange(256, dtype=np.uint8) if fmt == E5M2 else np.arange(65536, dtype=np.uint16)
    freq = orc.w_histogram(fmt, x)
    ln, cost = orc.w_lengths_limited(freq, 16)
    assert cost == x.size * (5 if fmt == E5M2 else 8)         # uniform exponents: no gain
    y, _ = orc.w_container_decode(orc.w_container_encode(fmt, x, 1, x.size, 64, 1, ln))
    assert np.array_equal(y, x)


@pytest.mark.parametrize("fmt,N,G,n_chunks_whole,extra", [(E5M2, 128, 1, 3, 0), (E5M2, 64, 2, 5, 40), (BF16, 64, 4, 9, 13),
                                                           (BF16, 128, 2, 4, 0)])
def test_stream_order_with_a_fixed_length_code(orc, fmt, N, G, n_chunks_whole, extra):
    """With every exponent field equally long-coded the stream is an array of fixed-width
    fields, so the element order, the bit order and the two run directions can be written
    down as array reshapes (axes: piece, chunk in group, lane, element in piece)."""
    w = 5 if fmt == E5M2 else 8
    A = 1 << w
    P = 16 if fmt == E5M2 else 8
    E = 64 * N
    n = n_chunks_whole * E + extra
    rng = np.random.default_rng(n)
    sym = rng.integers(0, A, n)
    sym[:A] = np.arange(A)                                    # every field occurs
    if fmt == E5M2:
        x = ((rng.integers(0, 2, n) << 7) | (sym << 2) | rng.integers(0, 4, n)).astype(np.uint8)
    else:
        x = ((rng.integers(0, 2, n) << 15) | (sym << 7) | rng.integers(0, 128, n)).astype(np.uint16)
    ln = np.full(A, w, dtype=np.uint8)                        # canonical code of symbol s = s
    blob = orc.w_container_encode(fmt, x, 1, n, N, G, ln)
    s = _sections(blob)
    n_chunks = s["n_chunks"]
    padded = np.full(n_chunks * E, -1, dtype=np.int64)
    padded[:n] = sym
    lanes = np.zeros((n_chunks, 64, N), dtype=np.int64)       # [chunk, lane, k]
    F = n // (G * E)
    for g in range(F):
        blk = padded[g * G * E:(g + 1) * G * E].reshape(N // P, G, 64, P)
        lanes[g * G:(g + 1) * G] = blk.transpose(1, 2, 0, 3).reshape(G, 64, N)
    for c in range(F * G, n_chunks):
        lanes[c] = padded[c * E:(c + 1) * E].reshape(N // P, 64, P).transpose(1, 0, 2).reshape(64, N)
    bits = []
    lane_bits = np.zeros((n_chunks, 64), dtype=np.int64)
    for c in range(n_chunks):
        for l in range(64):
            ks = lanes[c, l]
            fwd = [b for v in ks[:N // 2] if v >= 0 for b in format(int(v), "0%db" % w)]
            bwd = [b for v in ks[N // 2:] if v >= 0 for b in format(int(v), "0%db" % w)]
            lane = fwd + bwd[::-1]
            lane_bits[c, l] = len(lane)
            bits.extend(lane)
    want = np.packbits(np.array(bits, dtype=np.uint8), bitorder="little")
    got = blob[s["off_st"]:s["off_st"] + s["st_bytes"]]
    assert np.array_equal(got[:want.size], want) and not got[want.size:].any()
    lb = np.frombuffer(blob[s["off_lb"]:s["off_lb"] + 128 * n_chunks].tobytes(), "<u2").reshape(n_chunks, 64)
    assert np.array_equal(lb, lane_bits)
    cb = np.frombuffer(blob[s["off_cb"]:s["off_cb"] + 8 * (n_chunks + 1)].tobytes(), "<u8")
    assert np.array_equal(cb, np.concatenate([[0], np.cumsum(lane_bits.sum(axis=1))]).astype(np.uint64))


@pytest.mark.parametrize("n", [4, 1000, 64 * 64 + 5])
def test_plane_layouts(orc, n):
    rng = np.random.default_rng(n)
    # BF16: bytes of a group of four elements in the order 0 2 1 3
    x = rng.integers(0, 65536, n).astype(np.uint16)
    ln, _ = orc.w_lengths_limited(orc.w_histogram(BF16, x), 16)
    blob = orc.w_container_encode(BF16, x, 1, n, 64, 1, ln)
    s = _sections(blob)
    rem = np.zeros(s["pl_bytes"], dtype=np.uint8)
    rem[:n] = ((x >> 15) << 7 | (x & 127)).astype(np.uint8)
    want = rem.reshape(-1, 4)[:, [0, 2, 1, 3]].reshape(-1)
    assert np.array_equal(blob[s["off_pl"]:s["off_pl"] + s["pl_bytes"]], want)
    # E5M2: mantissa of element 16g + 4d + j in bits 8j+2d of word g; sign of element i in bit i%16 of word g
    x = rng.integers(0, 256, n).astype(np.uint8)
    ln, _ = orc.w_lengths_limited(orc.w_histogram(E5M2, x), 16)
    blob = orc.w_container_encode(E5M2, x, 1, n, 64, 1, ln)
    s = _sections(blob)
    pieces = s["pl_bytes"] // 4
    m = np.zeros(pieces * 16, dtype=np.uint32)
    m[:n] = x & 3
    sg = np.zeros(pieces * 16, dtype=np.uint32)
    sg[:n] = x >> 7
    m = m.reshape(pieces, 4, 4)                               # [g, d, j]
    shifts = (8 * np.arange(4)[None, :] + 2 * np.arange(4)[:, None]).astype(np.uint32)   # [d, j]
    want_m = (m << shifts[None]).sum(axis=(1, 2)).astype("<u4")
    want_s = (sg.reshape(pieces, 16) << np.arange(16, dtype=np.uint32)[None]).sum(axis=1).astype("<u2")
    assert np.array_equal(np.frombuffer(blob[s["off_pl"]:s["off_pl"] + 4 * pieces].tobytes(), "<u4"), want_m)
    assert np.array_equal(np.frombuffer(blob[s["off_sg"]:s["off_sg"] + 2 * pieces].tobytes(), "<u2"), want_s)


def test_decoder_rejects_inconsistent_containers(orc):
    rng = np.random.default_rng(5)
    x = _rand_elems(BF16, 9000, rng)
    ln, _ = orc.w_lengths_limited(orc.w_histogram(BF16, x), 12)
    blob = orc.w_container_encode(BF16, x, 90, 100, 64, 1, ln)
    s = _sections(blob)
    for off in (0, 4, 16, 40, 44, 48, 52, 60, 72, s["off_cb"] + 8, s["off_lb"], s["off_freq"] + 8 * int(np.argmax(ln > 0))):
        bad = blob.copy()
        bad[off] ^= 1
        with pytest.raises(ValueError):
            orc.w_container_decode(bad)
    with pytest.raises(ValueError):
        orc.w_container_decode(blob[:-1])
    short = ln.copy()
    short[np.flatnonzero(ln)[0]] = 0                          # a field that occurs has no codeword
    with pytest.raises(ValueError):
        orc.w_container_encode(BF16, x, 90, 100, 64, 1, short)
    with pytest.raises(ValueError):
        orc.w_container_encode(BF16, x, 90, 100, 32, 1, ln)   # lane_syms not offered
    with pytest.raises(ValueError):
        orc.w_container_encode(BF16, x, 90, 100, 64, 3, ln)   # group not a power of two

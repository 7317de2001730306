"""ECF8 CPU oracle -- TEST INFRASTRUCTURE ONLY.

ctypes front end of the plain-C oracle in this directory.  Only ``tests/``,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import this package; the product never does, and this package never imports the
product.  All arrays are numpy ``uint8``/``uint64`` on the host.
"""
import ctypes
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = [os.path.join(_DIR, f) for f in ("ecf8_oracle.c", "ecf8_container.c", "paper_alg1.c", "gemm_ref.c", "ecfw_oracle.c")]
_LIB = os.path.join(_DIR, "libecf8_oracle.so")

MSB_FIRST = 0
LSB_FIRST = 1

OK = 0
E_ARG, E_FORMAT, E_CAPACITY, E_CODE, E_META = -1, -2, -3, -4, -5


def build(force=True):
    """Compile the oracle with gcc (-O2, no vectorisation flags)."""
    srcs = [s for s in _SRC if os.path.exists(s)]
    if not force and os.path.exists(_LIB) and all(
            os.path.getmtime(_LIB) >= os.path.getmtime(s) for s in srcs):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB] + srcs + ["-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = ctypes.CDLL(_LIB)
        _lib.orc_entropy_bits.restype = ctypes.c_double
        _lib.orc_stream_bits.restype = ctypes.c_uint64
        _lib.orc_container_size.restype = ctypes.c_uint64
        _lib.orc_container_size.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint32]
        _lib.orw_container_size.restype = ctypes.c_uint64
        _lib.orw_container_size.argtypes = [ctypes.c_int, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint32]
        _lib.orw_stream_bits.restype = ctypes.c_uint64
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _u8(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint8
    return a.reshape(-1)


def histogram(x):
    x = _u8(x)
    freq = np.zeros(16, dtype=np.uint64)
    lib().orc_histogram(_p(x), ctypes.c_uint64(x.size), _p(freq))
    return freq


def entropy_bits(freq):
    freq = np.ascontiguousarray(freq, dtype=np.uint64)
    return float(lib().orc_entropy_bits(_p(freq)))


def huffman_lengths(freq):
    freq = np.ascontiguousarray(freq, dtype=np.uint64)
    assert freq.size == 16
    ln = np.zeros(16, dtype=np.uint8)
    rc = lib().orc_huffman_lengths(_p(freq), _p(ln))
    if rc < 0:
        raise ValueError("orc_huffman_lengths: %d" % rc)
    return ln


def huffman_lengths_limited(freq, max_len):
    """Cheapest prefix code with every length <= max_len (exhaustive search)."""
    freq = np.ascontiguousarray(freq, dtype=np.uint64)
    assert freq.size == 16
    ln = np.zeros(16, dtype=np.uint8)
    rc = lib().orc_huffman_lengths_limited(_p(freq), ctypes.c_int(max_len), _p(ln))
    if rc < 0:
        raise ValueError("orc_huffman_lengths_limited: %d" % rc)
    return ln


def canonical_codes(lengths):
    lengths = np.ascontiguousarray(lengths, dtype=np.uint8)
    code = np.zeros(16, dtype=np.uint16)
    rc = lib().orc_canonical_codes(_p(lengths), _p(code))
    if rc:
        raise ValueError("orc_canonical_codes: %d" % rc)
    return code


def stream_bits(freq, lengths):
    freq = np.ascontiguousarray(freq, dtype=np.uint64)
    lengths = np.ascontiguousarray(lengths, dtype=np.uint8)
    return int(lib().orc_stream_bits(_p(freq), _p(lengths)))


def encode_exponents(x, lengths, codes, order=MSB_FIRST):
    """Bit-serial encoder; returns (stream bytes, nbits)."""
    x = _u8(x)
    lengths = np.ascontiguousarray(lengths, dtype=np.uint8)
    codes = np.ascontiguousarray(codes, dtype=np.uint16)
    cap = (x.size * 15 + 7) // 8 + 1
    stream = np.zeros(cap, dtype=np.uint8)
    nbits = ctypes.c_uint64(0)
    rc = lib().orc_encode_exponents(_p(x), ctypes.c_uint64(x.size), _p(lengths), _p(codes),
                                    ctypes.c_int(order), _p(stream), ctypes.c_uint64(cap),
                                    ctypes.byref(nbits), ctypes.c_uint64(0), None)
    if rc:
        raise ValueError("orc_encode_exponents: %d" % rc)
    nb = int(nbits.value)
    return stream[: (nb + 7) // 8].copy(), nb


def pack_nibbles_paper(x):
    x = _u8(x)
    packed = np.zeros((x.size + 1) // 2, dtype=np.uint8)
    lib().orc_pack_nibbles_paper(_p(x), ctypes.c_uint64(x.size), _p(packed))
    return packed


def decode_serial(stream, nbits, lengths, packed, n, order=MSB_FIRST):
    stream = _u8(stream)
    packed = _u8(packed)
    lengths = np.ascontiguousarray(lengths, dtype=np.uint8)
    out = np.zeros(n, dtype=np.uint8)
    rc = lib().orc_decode_serial(_p(stream), ctypes.c_uint64(nbits), ctypes.c_int(order),
                                 _p(lengths), _p(packed), ctypes.c_uint64(n), _p(out))
    if rc:
        raise ValueError("orc_decode_serial: %d" % rc)
    return out


def roundtrip(x):
    """decode(encode(x)) entirely inside the oracle; returns (out, nbits, lengths)."""
    x = _u8(x)
    out = np.zeros(x.size, dtype=np.uint8)
    nbits = ctypes.c_uint64(0)
    ln = np.zeros(16, dtype=np.uint8)
    rc = lib().orc_roundtrip(_p(x), ctypes.c_uint64(x.size), _p(out), ctypes.byref(nbits), _p(ln))
    if rc:
        raise ValueError("orc_roundtrip: %d" % rc)
    return out, int(nbits.value), ln


def container_encode(x, rows, cols, lane_syms, group_chunks=1, max_code_len=15, tile_rows=0):
    x = _u8(x)
    assert x.size == rows * cols
    cap = int(lib().orc_container_size(x.size, x.size * 15, lane_syms)) + 256
    blob = np.zeros(cap, dtype=np.uint8)
    size = ctypes.c_uint64(0)
    rc = lib().orc_container_encode(_p(x), ctypes.c_uint64(rows), ctypes.c_uint64(cols),
                                    ctypes.c_uint32(lane_syms), ctypes.c_uint32(group_chunks),
                                    ctypes.c_uint32(max_code_len), ctypes.c_uint32(tile_rows), _p(blob),
                                    ctypes.c_uint64(cap),
                                    ctypes.byref(size))
    if rc:
        raise ValueError("orc_container_encode: %d" % rc)
    return blob[: int(size.value)].copy()


def container_decode(blob):
    """Returns (decoded bytes, stream_bits); raises ValueError(code) on any inconsistency."""
    blob = _u8(blob)
    if blob.size < 256:
        raise ValueError("orc_container_decode: %d" % E_FORMAT)
    n = int(np.frombuffer(blob[16:24].tobytes(), dtype="<u8")[0])
    out = np.zeros(max(n, 1), dtype=np.uint8)
    n_out = ctypes.c_uint64(0)
    bits = ctypes.c_uint64(0)
    rc = lib().orc_container_decode(_p(blob), ctypes.c_uint64(blob.size), _p(out),
                                    ctypes.c_uint64(out.size), ctypes.byref(n_out), ctypes.byref(bits))
    if rc:
        raise ValueError("orc_container_decode: %d" % rc)
    return out[: int(n_out.value)], int(bits.value)


def paper_build_lut(lengths, codes, width=8):
    """Cascaded table with `width`-bit rows; returns (rows x 2^width uint8 array, n_luts)."""
    lengths = np.ascontiguousarray(lengths, dtype=np.uint8)
    codes = np.ascontiguousarray(codes, dtype=np.uint16)
    lut = np.zeros(18 * 256, dtype=np.uint8)
    n_luts = ctypes.c_uint32(0)
    rc = lib().orc_paper_build_lut_w(_p(lengths), _p(codes), ctypes.c_uint32(width), _p(lut), ctypes.byref(n_luts))
    if rc:
        raise ValueError("orc_paper_build_lut_w: %d" % rc)
    k = int(n_luts.value)
    return lut[: k * (1 << width)].reshape(k, 1 << width).copy(), k


def paper_alg1_roundtrip(x, T=256):
    """Encode x into the paper's own container (B=8) and decode it with the block decoder of
    Algorithm 1 restated over the bit-serial walk (every gap must land on a codeword start, every
    block's counts must add up to its share of outpos); the cascaded table is checked against the
    code tree on all 16-bit prefixes.  Returns (outputs, dict of the container's arrays)."""
    x = _u8(x)
    n = x.size
    freq = histogram(x)
    ln0 = huffman_lengths(freq)
    bits = stream_bits(freq, ln0)
    n_bytes = ctypes.c_uint64(0)
    n_blocks = ctypes.c_uint64(0)
    alloc = ctypes.c_uint64(0)
    gbytes = ctypes.c_uint64(0)
    lib().orc_paper_sizes(ctypes.c_uint64(bits), ctypes.c_uint32(T), ctypes.byref(n_bytes),
                          ctypes.byref(n_blocks), ctypes.byref(alloc), ctypes.byref(gbytes))
    ln = np.zeros(16, dtype=np.uint8)
    lut = np.zeros(18 * 256, dtype=np.uint8)
    n_luts = ctypes.c_uint32(0)
    encoded = np.zeros(int(alloc.value), dtype=np.uint8)
    packed = np.zeros((n + 1) // 2, dtype=np.uint8)
    outpos = np.zeros(int(n_blocks.value) + 1, dtype=np.int64)
    gaps = np.zeros(int(gbytes.value), dtype=np.uint8)
    nb2 = ctypes.c_uint64(0)
    nbl2 = ctypes.c_uint64(0)
    rc = lib().orc_paper_encode(_p(x), ctypes.c_uint64(n), ctypes.c_uint32(T), _p(ln), _p(lut),
                                ctypes.byref(n_luts), _p(encoded), ctypes.c_uint64(encoded.size),
                                ctypes.byref(nb2), _p(packed), _p(outpos), _p(gaps), ctypes.byref(nbl2))
    if rc:
        raise ValueError("orc_paper_encode: %d" % rc)
    out = np.zeros(n, dtype=np.uint8)
    rc = lib().orc_paper_window_decode(_p(ln), _p(encoded), ctypes.c_uint64(encoded.size), _p(packed), _p(outpos),
                                       _p(gaps), nbl2, ctypes.c_uint32(T), ctypes.c_uint64(n), _p(out))
    if rc:
        raise ValueError("orc_paper_window_decode: %d" % rc)
    lib().orc_paper_lut_mismatches.restype = ctypes.c_int64
    if lib().orc_paper_lut_mismatches(_p(ln), _p(lut), n_luts) != 0:
        raise ValueError("cascaded table disagrees with the code tree")
    return out, dict(lengths=ln, lut=lut, n_luts=int(n_luts.value), encoded=encoded,
                     n_bytes=int(nb2.value), packed=packed, outpos=outpos, gaps=gaps,
                     n_blocks=int(nbl2.value), stream_bits=bits)


def e4m3_to_double(b):
    lib().orc_e4m3_to_double.restype = ctypes.c_double
    return float(lib().orc_e4m3_to_double(ctypes.c_uint8(int(b))))


def gemm_ref(X, W):
    """Y = X @ W.T for raw E4M3 bytes X (M, K), W (N, K) in fp64; returns (Y, sum |x w|)."""
    X = np.ascontiguousarray(X, dtype=np.uint8)
    W = np.ascontiguousarray(W, dtype=np.uint8)
    M, K = X.shape
    N, K2 = W.shape
    assert K == K2
    Y = np.zeros((M, N), dtype=np.float64)
    A = np.zeros((M, N), dtype=np.float64)
    lib().orc_gemm_ref(_p(X), _p(W), ctypes.c_uint64(M), ctypes.c_uint64(N), ctypes.c_uint64(K), _p(Y), _p(A))
    return Y, A


def gemm_ref_scaled(X, W, ws, xs=None):
    """Y = (xs X) @ (ws W).T with one scale per 128 x 128 block of W and, for X, one per row (xs of shape (M,))
    or one per row and 128 columns (shape (M, ceil(K/128))); returns (Y, sum |.|)."""
    X = np.ascontiguousarray(X, dtype=np.uint8)
    W = np.ascontiguousarray(W, dtype=np.uint8)
    M, K = X.shape
    N, K2 = W.shape
    assert K == K2
    ws = np.ascontiguousarray(ws, dtype=np.float32)
    assert ws.shape == ((N + 127) // 128, (K + 127) // 128)
    xs_cols = 0
    if xs is not None:
        xs = np.ascontiguousarray(xs, dtype=np.float32)
        assert xs.shape in ((M,), (M, (K + 127) // 128))
        xs_cols = 1 if xs.ndim == 1 else xs.shape[1]
    Y = np.zeros((M, N), dtype=np.float64)
    A = np.zeros((M, N), dtype=np.float64)
    lib().orc_gemm_ref_scaled(_p(X), _p(W), ctypes.c_uint64(M), ctypes.c_uint64(N), ctypes.c_uint64(K), _p(ws),
                              _p(xs) if xs is not None else None, ctypes.c_uint64(xs_cols), _p(Y), _p(A))
    return Y, A


# ---- wide alphabets (E5M2, BF16): ecfw_oracle.c ----

FMT_E5M2, FMT_BF16 = 1, 2
W_ALPHABET = {FMT_E5M2: 32, FMT_BF16: 256}
W_ELEM_BYTES = {FMT_E5M2: 1, FMT_BF16: 2}


def _w_bytes(fmt, x):
    """x: uint8 (E5M2) or uint16 (BF16 bit patterns) -> flat little-endian bytes, element count."""
    x = np.ascontiguousarray(x)
    if fmt == FMT_BF16:
        assert x.dtype == np.uint16
        return x.reshape(-1).view(np.uint8), x.size
    assert x.dtype == np.uint8
    return x.reshape(-1), x.size


def w_split(fmt, x):
    """(exponent fields, remaining bits sign-on-top) of every element."""
    b, n = _w_bytes(fmt, x)
    sym = np.zeros(n, dtype=np.uint8)
    rem = np.zeros(n, dtype=np.uint8)
    lib().orw_split(ctypes.c_int(fmt), _p(b), ctypes.c_uint64(n), _p(sym), _p(rem))
    return sym, rem


def w_histogram(fmt, x):
    b, n = _w_bytes(fmt, x)
    freq = np.zeros(W_ALPHABET[fmt], dtype=np.uint64)
    rc = lib().orw_histogram(ctypes.c_int(fmt), _p(b), ctypes.c_uint64(n), _p(freq))
    if rc:
        raise ValueError("orw_histogram: %d" % rc)
    return freq


def w_huffman_lengths(freq):
    freq = np.ascontiguousarray(freq, dtype=np.uint64)
    ln = np.zeros(freq.size, dtype=np.uint8)
    rc = lib().orw_huffman_lengths(_p(freq), ctypes.c_int(freq.size), _p(ln))
    if rc:
        raise ValueError("orw_huffman_lengths: %d" % rc)
    return ln


def w_lengths_limited(freq, max_len):
    """(lengths, cost) of a cheapest prefix code with every length <= max_len."""
    freq = np.ascontiguousarray(freq, dtype=np.uint64)
    ln = np.zeros(freq.size, dtype=np.uint8)
    cost = ctypes.c_uint64(0)
    rc = lib().orw_lengths_limited(_p(freq), ctypes.c_int(freq.size), ctypes.c_int(max_len), _p(ln), ctypes.byref(cost))
    if rc:
        raise ValueError("orw_lengths_limited: %d" % rc)
    return ln, int(cost.value)


def w_canonical(lengths):
    lengths = np.ascontiguousarray(lengths, dtype=np.uint8)
    code = np.zeros(lengths.size, dtype=np.uint32)
    rc = lib().orw_canonical(_p(lengths), ctypes.c_int(lengths.size), _p(code))
    if rc:
        raise ValueError("orw_canonical: %d" % rc)
    return code


def w_stream_bits(freq, lengths):
    freq = np.ascontiguousarray(freq, dtype=np.uint64)
    lengths = np.ascontiguousarray(lengths, dtype=np.uint8)
    return int(lib().orw_stream_bits(_p(freq), _p(lengths), ctypes.c_int(freq.size)))


def w_container_encode(fmt, x, rows, cols, lane_syms, group_chunks, lengths):
    b, n = _w_bytes(fmt, x)
    assert n == rows * cols
    lengths = np.ascontiguousarray(lengths, dtype=np.uint8)
    assert lengths.size == W_ALPHABET[fmt]
    cap = int(lib().orw_container_size(fmt, n, n * 16, lane_syms)) + 256
    if cap <= 256:
        raise ValueError("orw_container_encode: %d" % E_ARG)
    blob = np.zeros(cap, dtype=np.uint8)
    size = ctypes.c_uint64(0)
    rc = lib().orw_container_encode(ctypes.c_int(fmt), _p(b), ctypes.c_uint64(rows), ctypes.c_uint64(cols),
                                    ctypes.c_uint32(lane_syms), ctypes.c_uint32(group_chunks), _p(lengths),
                                    _p(blob), ctypes.c_uint64(cap), ctypes.byref(size))
    if rc:
        raise ValueError("orw_container_encode: %d" % rc)
    return blob[: int(size.value)].copy()


def w_container_decode(blob):
    """Returns (elements as uint8 or uint16, stream_bits); ValueError(code) on any inconsistency."""
    blob = _u8(blob)
    if blob.size < 256:
        raise ValueError("orw_container_decode: %d" % E_FORMAT)
    n = int(np.frombuffer(blob[16:24].tobytes(), dtype="<u8")[0])
    fmt = int(np.frombuffer(blob[40:44].tobytes(), dtype="<u4")[0])
    eb = W_ELEM_BYTES.get(fmt, 1)
    if n > blob.size * 64:
        raise ValueError("orw_container_decode: %d" % E_FORMAT)
    out = np.zeros(max(n, 1) * eb, dtype=np.uint8)
    n_out = ctypes.c_uint64(0)
    bits = ctypes.c_uint64(0)
    rc = lib().orw_container_decode(_p(blob), ctypes.c_uint64(blob.size), _p(out), ctypes.c_uint64(max(n, 1)),
                                    ctypes.byref(n_out), ctypes.byref(bits))
    if rc:
        raise ValueError("orw_container_decode: %d" % rc)
    out = out[: int(n_out.value) * eb]
    return (out.view(np.uint16) if fmt == FMT_BF16 else out), int(bits.value)

"""Parity of the wide-alphabet HIP decode path (E5M2, BF16) with the CPU oracle, through the C ABI.

Every case encodes seeded synthetic elements with the library's host encoder, decodes on
the GPU into the middle of a poisoned buffer, and compares element by element, bit-exact,
with what the oracle's independent bit-serial reader makes of the same container (which the
CPU tests show to be the container the oracle itself writes) and with the input.
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


def _gpu_decode_guarded(blob, pad=4096, max_workgroups=0):
    """Decode into the middle of a poisoned buffer; returns (elements, guards_intact)."""
    hdr = blob.header
    eb = ecfw.ELEM_BYTES[hdr.fmt]
    d_blob = blob.to(DEV)
    nb = hdr.n_elem * eb
    buf = torch.full((pad + nb + pad,), 0xA5, dtype=torch.uint8, device=DEV)
    out = buf[pad:pad + nb]
    ecfw.ecfw_decode(d_blob, hdr, out, max_workgroups=max_workgroups)
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    ok = bool((host[:pad] == 0xA5).all() and (host[pad + nb:] == 0xA5).all())
    got = host[pad:pad + nb]
    return (got.view(np.uint16) if eb == 2 else got), ok


def _check(orc, fmt, x, rows=None, cols=None, max_workgroups=0, **opts):
    x = np.ascontiguousarray(x).reshape(-1)
    rows, cols = (1, x.size) if rows is None else (rows, cols)
    blob = ecfw.ecfw_encode(fmt, x, rows, cols, **opts)
    print("fmt", fmt, "n", x.size, opts, "max_len", blob.header.max_code_len, flush=True)
    got, guards = _gpu_decode_guarded(blob, max_workgroups=max_workgroups)
    assert guards
    dec, _ = orc.w_container_decode(blob.numpy())
    assert np.array_equal(got, dec)
    assert np.array_equal(got, x)
    return blob


@pytest.mark.parametrize("max_code_len", [0, 16])
@pytest.mark.parametrize("lane_syms", [64, 128])
@pytest.mark.parametrize("fmt", [E5M2, BF16])
def test_synthetic_matrix_parity(orc, fmt, lane_syms, max_code_len):
    """1024x1024 alpha-stable weights (alpha 1.8, scale 0.02, seed 0) in both formats, with the default
    cap of 12 bits (branch-free kernels) and with Section 3.1's cap of 16 (long-code branch in use)."""
    make = synth.make_bf16 if fmt == BF16 else synth.make_e5m2
    x = make(1024, 1024, 1.8, 0.02, 0).numpy()
    blob = _check(orc, fmt, x, 1024, 1024, lane_syms=lane_syms, max_code_len=max_code_len)
    assert (blob.header.max_code_len <= 12) == (max_code_len == 0)


@pytest.mark.parametrize("fmt", [E5M2, BF16])
@pytest.mark.parametrize("n", [1, 2, 15, 16, 17, 511, 4095, 4096, 4097, 8191, 8193, 64 * 128 * 3 + 1, 64 * 64 * 33 - 1, 300007])
def test_ragged_sizes(orc, fmt, n):
    _check(orc, fmt, _rand_elems(fmt, n, n))


@pytest.mark.parametrize("fmt", [E5M2, BF16])
@pytest.mark.parametrize("lane_syms,group,n_chunks,extra", [(64, 1, 40, 0), (64, 2, 41, 5), (128, 4, 22, 100), (64, 32, 100, 1),
                                                            (128, 64, 130, 4000), (64, 16, 16, 0)])
def test_grouped_layouts(orc, fmt, lane_syms, group, n_chunks, extra):
    n = 64 * lane_syms * n_chunks + extra
    _check(orc, fmt, _rand_elems(fmt, n, n + group), lane_syms=lane_syms, group_chunks=group)


@pytest.mark.parametrize("fmt", [E5M2, BF16])
def test_every_bit_pattern(orc, fmt):
    """Zeros, subnormals, infinities and NaN payloads come back as they went in."""
    x = np.arange(256, dtype=np.uint8) if fmt == E5M2 else np.arange(65536, dtype=np.uint16)
    x = np.tile(x, 5)
    _check(orc, fmt, x, max_code_len=16)
    _check(orc, fmt, np.random.default_rng(0).permutation(x), lane_syms=128, group_chunks=2)


@pytest.mark.parametrize("cap", [5, 8, 12, 13, 16])
@pytest.mark.parametrize("fmt", [E5M2, BF16])
def test_caps(orc, fmt, cap):
    x = _rand_elems(fmt, 500000, cap, spread=2.0)
    blob = _check(orc, fmt, x, max_code_len=cap)
    assert blob.header.max_code_len <= cap


def test_long_codes_everywhere(orc):
    """BF16 with all 256 exponent fields in use and geometric frequencies: under the cap of 16 most
    fields have codewords of 13..16 bits, so the long-code branch runs in most decode steps."""
    rng = np.random.default_rng(7)
    p = 0.93 ** np.arange(256)
    e = rng.choice(256, size=700000, p=p / p.sum()).astype(np.uint16)
    e[:256] = np.arange(256)
    x = ((rng.integers(0, 2, e.size).astype(np.uint16) << 15) | (e << 7) | rng.integers(0, 128, e.size).astype(np.uint16))
    blob = _check(orc, BF16, x, max_code_len=16, group_chunks=1)
    assert blob.header.max_code_len == 16
    _check(orc, BF16, x, max_code_len=16, lane_syms=128, group_chunks=4)


@pytest.mark.parametrize("lane_syms", [64, 128])
def test_islands_of_long_codes(orc, lane_syms):
    """A few chunks made only of rare exponent fields (16-bit codewords): their span exceeds what a
    wavefront stages in LDS, so they are decoded the careful way, one symbol at a time."""
    rng = np.random.default_rng(11)
    n = 64 * lane_syms * 300
    e = np.clip(np.rint(rng.normal(120, 1.0, n)), 0, 255).astype(np.uint16)
    rare = np.setdiff1d(np.arange(256), np.arange(110, 131))
    for c in (3, 150, 151, 299):
        e[c * 64 * lane_syms:(c + 1) * 64 * lane_syms] = rng.choice(rare, 64 * lane_syms)
    x = ((rng.integers(0, 2, n).astype(np.uint16) << 15) | (e << 7) | rng.integers(0, 128, n).astype(np.uint16))
    blob = _check(orc, BF16, x, max_code_len=16, lane_syms=lane_syms, group_chunks=1)
    h, arr = blob.header, blob.numpy()
    cb = np.frombuffer(arr[h.off_chunk_bit:h.off_chunk_bit + 8 * (h.n_chunks + 1)].tobytes(), "<u8")
    assert (np.diff(cb.astype(np.int64)) // 8 > 64 * lane_syms * 12 // 8 + 64).sum() == 4     # the islands are oversize


@pytest.mark.parametrize("fmt", [E5M2, BF16])
def test_few_workgroups_and_caller_buffer(orc, fmt):
    x = _rand_elems(fmt, 64 * 128 * 50 + 9, 3)
    for wgs in (1, 3, 1000):
        _check(orc, fmt, x, max_workgroups=wgs)


@pytest.mark.parametrize("fmt", [E5M2, BF16])
def test_batched_matches_oracle(orc, fmt):
    """Many tensors in one launch: sizes from a single element to hundreds of chunks, so that workgroup
    ranges start and end inside tensors and run across several of them."""
    sizes = [1, 64 * 64 * 3 + 5, 17, 300000, 4096, 64 * 64 * 200, 9, 123457, 64 * 64, 5]
    blobs = [ecfw.ecfw_encode(fmt, _rand_elems(fmt, n, 1000 + i, spread=1.5 + i % 3), lane_syms=64,
                              group_chunks=(1, 4, 32)[i % 3], max_code_len=(0, 9)[i % 2]) for i, n in enumerate(sizes)]
    eb = ecfw.ELEM_BYTES[fmt]
    d_blobs = [b.to(DEV) for b in blobs]
    pad = 256
    bufs = [torch.full((pad + b.header.n_elem * eb + pad,), 0x5A, dtype=torch.uint8, device=DEV) for b in blobs]
    outs = [buf[pad:pad + b.header.n_elem * eb] for buf, b in zip(bufs, blobs)]
    for wgs in (0, 1, 7):
        for o in outs:
            o.fill_(0x5A)
        batch = ecfw.WBatch([b.header for b in blobs], d_blobs, outs)
        batch.info.max_workgroups = wgs
        print("fmt", fmt, "batched, max_workgroups", wgs, "chunks", batch.info.total_chunks, flush=True)
        ecfw.ecfw_decode_batched(batch)
        torch.cuda.synchronize()
        for buf, b in zip(bufs, blobs):
            host = buf.cpu().numpy()
            nb = b.header.n_elem * eb
            assert (host[:pad] == 0x5A).all() and (host[pad + nb:] == 0x5A).all()
            got = host[pad:pad + nb]
            dec, _ = orc.w_container_decode(b.numpy())
            assert np.array_equal(got.view(np.uint16) if eb == 2 else got, dec)


def test_batched_with_long_codes_and_argument_errors(orc):
    xs = [_rand_elems(BF16, n, n, spread=6.0) for n in (50000, 200000)]
    blobs = [ecfw.ecfw_encode(BF16, x, max_code_len=c) for x, c in zip(xs, (16, 0))]
    assert blobs[0].header.max_code_len > 12 >= blobs[1].header.max_code_len
    d_blobs = [b.to(DEV) for b in blobs]
    outs = [torch.empty(b.header.n_elem, dtype=torch.bfloat16, device=DEV) for b in blobs]
    batch = ecfw.WBatch([b.header for b in blobs], d_blobs, outs)
    assert batch.info.max_code_len == blobs[0].header.max_code_len
    ecfw.ecfw_decode_batched(batch)
    torch.cuda.synchronize()
    for o, x in zip(outs, xs):
        assert np.array_equal(o.view(torch.int16).cpu().numpy().view(np.uint16), x)
    other = ecfw.ecfw_encode(E5M2, _rand_elems(E5M2, 5000, 1))
    with pytest.raises(ecf8.Ecf8Error) as e:       # formats do not mix in one launch
        ecfw.WBatch([blobs[0].header, other.header], [d_blobs[0], other.to(DEV)],
                    [outs[0], torch.empty(5000, dtype=torch.uint8, device=DEV)])
    assert e.value.code == ecf8.E_ARG
    n128 = ecfw.ecfw_encode(BF16, xs[0], lane_syms=128)
    with pytest.raises(ecf8.Ecf8Error) as e:       # nor do chunk shapes
        ecfw.WBatch([blobs[0].header, n128.header], [d_blobs[0], n128.to(DEV)], [outs[0], torch.empty_like(outs[0])])
    assert e.value.code == ecf8.E_ARG
    with pytest.raises(ecf8.Ecf8Error) as e:
        ecfw.WBatch([blobs[0].header], [d_blobs[0]], [outs[0][:100]])
    assert e.value.code == ecf8.E_CAPACITY


def test_argument_errors():
    x = _rand_elems(BF16, 10000, 1)
    blob = ecfw.ecfw_encode(BF16, x)
    d_blob = blob.to(DEV)
    small = torch.empty(10000 * 2 - 2, dtype=torch.uint8, device=DEV)
    with pytest.raises(ecf8.Ecf8Error) as e:
        ecfw.ecfw_decode(d_blob, blob.header, small)
    assert e.value.code == ecf8.E_CAPACITY
    big = torch.empty(10000 * 2 + 64, dtype=torch.uint8, device=DEV)
    with pytest.raises(ecf8.Ecf8Error) as e:
        ecfw.ecfw_decode(d_blob, blob.header, big[2:])
    assert e.value.code == ecf8.E_ALIGN
    bad = ecfw.WHeader.from_buffer_copy(bytes(blob.header))
    bad.fmt = 7
    with pytest.raises(ecf8.Ecf8Error) as e:
        ecfw.ecfw_decode(d_blob, bad, big)
    assert e.value.code == ecf8.E_FORMAT
    with pytest.raises(ecf8.Ecf8Error):
        ecfw.ecfw_decode(blob.to("cpu"), blob.header, big)
    torch.cuda.synchronize()


@pytest.mark.parametrize("fmt", [E5M2, BF16])
def test_full_size_matrix(orc, fmt):
    """The largest matrix of the 8B-class stack (14336 x 4096) in the launch configuration the bench
    times; the whole output against the input, and sampled chunks against the oracle's reader run on a
    container re-encoded from those chunks' elements alone."""
    make = synth.make_bf16 if fmt == BF16 else synth.make_e5m2
    x = make(14336, 4096, 1.8, 0.02, 0, tensor_id=5).numpy().reshape(-1)
    blob = ecfw.ecfw_encode(fmt, x, 14336, 4096)
    got, guards = _gpu_decode_guarded(blob)
    assert guards and np.array_equal(got, x)
    ecfw.blob_validate(blob.numpy())
    h = blob.header
    freq = orc.w_histogram(fmt, x)
    assert h.stream_bits == orc.w_lengths_limited(freq, 12)[1]
    E = 64 * h.lane_syms * h.group_chunks                        # one interleaved group of chunks
    for g in (0, 1, h.n_elem // E // 2, h.n_elem // E - 1):
        part = x[g * E:(g + 1) * E]
        want = orc.w_container_encode(fmt, part, 1, part.size, h.lane_syms, h.group_chunks, blob.code_len())
        dec, _ = orc.w_container_decode(want)
        assert np.array_equal(got[g * E:(g + 1) * E], dec)


@pytest.mark.parametrize("fmt", [E5M2, BF16])
def test_stream_longer_than_2_to_the_31_bits(fmt):
    """2^30 elements: chunk start bits pass 2^31 and 2^32, device addresses and bit positions need all 64 bits.
    The oracle cannot read a container of this size in reasonable time; the decoded tensor is compared
    with the input (the container's content is pinned by the smaller cases)."""
    n = 1 << 30
    g = torch.Generator(device=DEV)
    g.manual_seed(31)
    e = torch.randn(n, generator=g, device=DEV).mul_(2.0).add_(120.0 if fmt == BF16 else 14.0).round_().clamp_(0, 255 if fmt == BF16 else 31)
    if fmt == BF16:
        low = torch.randint(0, 128, (n,), generator=g, device=DEV, dtype=torch.int32)
        x = ((e.to(torch.int32) << 7) | low | ((low & 1) << 15)).to(torch.int16)
    else:
        low = torch.randint(0, 4, (n,), generator=g, device=DEV, dtype=torch.int32)
        x = ((e.to(torch.int32) << 2) | low | ((low & 1) << 7)).to(torch.uint8)
    del e, low
    blob = ecfw.ecfw_encode(fmt, x.cpu().numpy().view(np.uint16 if fmt == BF16 else np.uint8), 1 << 15, 1 << 15)
    assert blob.header.stream_bits > 1 << 31
    print("fmt", fmt, "n", n, "stream bits", blob.header.stream_bits, flush=True)
    d_blob = blob.to(DEV)
    out = torch.empty_like(x)
    ecfw.ecfw_decode(d_blob, blob.header, out)
    torch.cuda.synchronize()
    assert torch.equal(out, x)


@pytest.mark.parametrize("fmt", [E5M2, BF16])
def test_seeded_sweep(orc, fmt):
    """Sixty seeded combinations of size, chunk shape, group width, cap and spread of the exponent field per format."""
    rng = np.random.default_rng(4242 + fmt)
    for case in range(60):
        n = int(rng.choice([rng.integers(1, 200), rng.integers(200, 20000), rng.integers(20000, 400000)]))
        lane_syms = int(rng.choice([64, 128]))
        group = int(2 ** rng.integers(0, 7))
        spread = float(rng.uniform(0.3, 9.0))
        x = _rand_elems(fmt, n, 9000 + case, spread=spread)
        distinct = len(np.unique((x >> 7) & 255 if fmt == BF16 else (x >> 2) & 31))
        low = max(1, int(np.ceil(np.log2(max(distinct, 2)))))
        cap = int(rng.choice([0, rng.integers(low, 17)]))
        if cap and cap < low:
            cap = low
        wgs = int(rng.choice([0, 0, 1, 5, 64]))
        _check(orc, fmt, x, lane_syms=lane_syms, group_chunks=group, max_code_len=cap, max_workgroups=wgs)


@pytest.mark.parametrize("fmt", [E5M2, BF16])
def test_one_lane_of_long_codes_and_dense_islands(orc, fmt):
    """Under the default cap (branch-free kernels, bits staged in per-lane columns): single lanes whose 12-bit
    codewords overflow their column while the chunk's span is ordinary, and whole chunks of rare fields whose
    span overflows the stage; both must fall back to the careful pass."""
    N = 64 if fmt == BF16 else 128
    P = 8 if fmt == BF16 else 16
    A = 256 if fmt == BF16 else 32
    centre = 120 if fmt == BF16 else 14
    rng = np.random.default_rng(77 + fmt)
    n = 64 * N * 40
    e = np.clip(np.rint(rng.normal(centre, 0.8, n)), 0, A - 1).astype(np.int64)
    common = np.unique(e)
    rare = np.setdiff1d(np.arange(A), np.arange(centre - 4, centre + 5))
    e[:rare.size] = rare                                           # every rare field occurs (a few times only)
    chunk = 64 * N
    for c, lane in ((5, 7), (5, 63), (17, 0)):                     # one lane of a chunk: its N symbols are rare
        idx = c * chunk + (np.arange(N) // P) * (64 * P) + lane * P + np.arange(N) % P
        e[idx] = rng.choice(rare, N)
    for c in (9, 30):                                              # whole chunks of rare fields
        e[c * chunk:(c + 1) * chunk] = rng.choice(rare, chunk)
    e = e.astype(np.uint16 if fmt == BF16 else np.uint8)
    if fmt == BF16:
        x = ((rng.integers(0, 2, n).astype(np.uint16) << 15) | (e << 7) | rng.integers(0, 128, n).astype(np.uint16))
    else:
        x = ((rng.integers(0, 2, n).astype(np.uint8) << 7) | (e << 2) | rng.integers(0, 4, n).astype(np.uint8))
    blob = _check(orc, fmt, x, lane_syms=N, group_chunks=1)
    h, arr = blob.header, blob.numpy()
    assert h.max_code_len <= 12
    lb = np.frombuffer(arr[h.off_lane_bits:h.off_lane_bits + 128 * h.n_chunks].tobytes(), "<u2").reshape(-1, 64)
    assert lb[5, 7] > 2 * np.median(lb) and lb[9].sum() > 2 * np.median(lb.sum(axis=1))    # the cases are what they claim
    _check(orc, fmt, x, lane_syms=N, group_chunks=4)

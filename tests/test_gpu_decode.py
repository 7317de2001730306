"""Parity of the HIP decode path with the CPU oracle, through the C ABI.

Every case encodes seeded synthetic bytes with the library's host encoder,
decodes on the GPU, and compares element by element with what the oracle
computes from the same input (its own encode -> bit-serial decode), bit-exact.
"""
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


def _gpu_decode_guarded(blob_arr, hdr, pad=4096):
    """Decode into the middle of a poisoned buffer; returns (out, guards_intact)."""
    d_blob = torch.from_numpy(blob_arr).to(DEV)
    n = hdr.n_elem
    buf = torch.full((pad + n + pad,), 0xA5, dtype=torch.uint8, device=DEV)
    out = buf[pad:pad + n]
    ecf8.ecf8_decode(hdr, d_blob, out)
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    ok = bool((host[:pad] == 0xA5).all() and (host[pad + n:] == 0xA5).all())
    return host[pad:pad + n], ok


def _oracle_expected(orc, x):
    exp, _, _ = orc.roundtrip(x)
    return exp


@pytest.mark.parametrize("max_code_len", [0, 15])
@pytest.mark.parametrize("table_mode", [1, 2])
@pytest.mark.parametrize("lane_syms", [32, 64, 128])
def test_config0_parity(orc, lane_syms, table_mode, max_code_len):
    """configs[0]: 1024x1024, alpha 1.8, per-128x128 scaling, seed 0; with the pair table
    embedded in the blob (1) and built in the kernel (2); with the default cap on the code
    length (the kernels' branch-free form) and with plain Huffman (second level in use)."""
    w = synth.make(synth.config0()[0], seed=0).numpy().reshape(-1)
    blob = ecf8.ecf8_encode(w, 1024, 1024, lane_syms=lane_syms, table_mode=table_mode, max_code_len=max_code_len)
    assert (max(blob.header.code_len) <= 7) == (max_code_len == 0)
    got, guards = _gpu_decode_guarded(blob.numpy(), blob.header)
    assert guards
    assert np.array_equal(got, _oracle_expected(orc, w))
    # the oracle's independent reader agrees on what this container holds
    dec, _ = orc.container_decode(blob.numpy())
    assert np.array_equal(got, dec)


@pytest.mark.parametrize("lane_syms", [32, 64, 128])
@pytest.mark.parametrize("n", [1, 15, 16, 17, 63, 2047, 2049, 4095, 4096, 4097, 8191, 8193, 3 * 8192 + 77, 1_000_003])
def test_ragged_sizes(orc, lane_syms, n):
    x = _rand_bytes(n, 31 * n + lane_syms)
    blob = ecf8.ecf8_encode(x, 1, n, lane_syms=lane_syms, max_code_len=15 if n % 2 else 0)
    got, guards = _gpu_decode_guarded(blob.numpy(), blob.header)
    assert guards
    assert np.array_equal(got, _oracle_expected(orc, x))


def _special_cases():
    fib = [1, 1]
    while len(fib) < 16:
        fib.append(fib[-1] + fib[-2])
    deep = np.repeat(np.arange(16, dtype=np.uint8) << 3, np.array(fib) * 40)
    np.random.default_rng(0).shuffle(deep)
    deep |= np.random.default_rng(1).integers(0, 8, deep.size, dtype=np.uint8)
    rng = np.random.default_rng(2)
    # mostly one exponent, with an island of uniformly random exponents whose rare
    # symbols carry long codes: that island's chunks overflow the staging buffer
    island = np.full(400_000, 7 << 3, dtype=np.uint8)
    island[150_000:190_000] = rng.integers(0, 256, 40_000, dtype=np.uint8)
    return {
        "all_byte_values": np.arange(256, dtype=np.uint8).repeat(300),
        "single_symbol": np.full(70_001, 0x80, dtype=np.uint8),
        "two_symbols": (rng.integers(0, 2, 50_000, dtype=np.uint8) * 0x41 + 0x3A).astype(np.uint8),
        "uniform_exponents": rng.integers(0, 256, 300_000, dtype=np.uint8),
        "depth15_codes": deep,
        "incompressible_island": island,
        "nan_encodings": np.concatenate([np.full(9000, 0x38, np.uint8), np.array([0x7F, 0xFF] * 50, np.uint8)]),
    }


@pytest.mark.parametrize("cap", [0, 15])
@pytest.mark.parametrize("lane_syms", [32, 64, 128])
@pytest.mark.parametrize("name", sorted(_special_cases()))
def test_degenerate_and_extreme_inputs(orc, name, lane_syms, cap):
    x = _special_cases()[name]
    blob = ecf8.ecf8_encode(x, 1, x.size, lane_syms=lane_syms, table_mode=1 + (lane_syms == 64), max_code_len=cap)
    got, guards = _gpu_decode_guarded(blob.numpy(), blob.header)
    assert guards
    assert np.array_equal(got, _oracle_expected(orc, x))


@pytest.mark.parametrize("cap", [9, 12, 14])
@pytest.mark.parametrize("lane_syms", [32, 64, 128])
def test_long_codes_that_fit_the_table(orc, lane_syms, cap):
    """Codes between 8 and 14 bits: every codeword is in the table, many pairs of codewords are not, in the first and
    in the second lookup of a step, in the forward and in the backward run.  Four frequent exponents and a geometric tail
    of twelve: plain Huffman is 15 deep there, so the cap binds and the tail's codes crowd just under it."""
    rng = np.random.default_rng(300 + cap)
    tail = 0.5 ** np.arange(12.0)
    p = np.concatenate([[0.3, 0.28, 0.2, 0.1], 0.12 * tail / tail.sum()])
    n = 1_500_000 + lane_syms + 3
    x = (rng.choice(16, size=n, p=p / p.sum()).astype(np.uint8) << 3) | rng.integers(0, 8, n, dtype=np.uint8) | \
        (rng.integers(0, 2, n, dtype=np.uint8) << 7)
    blob = ecf8.ecf8_encode(x, 1, x.size, lane_syms=lane_syms, max_code_len=cap, table_mode=1 + (cap % 2))
    lens = np.array(list(blob.header.code_len), dtype=np.int64)
    assert lens.max() == cap                     # the cap binds: plain Huffman is 15 deep on this histogram
    q = np.bincount((x >> 3) & 15, minlength=16) / x.size
    pair_too_long = sum(q[i] * q[j] for i in range(16) for j in range(16) if lens[i] + lens[j] > 14)
    assert pair_too_long * x.size / 2 > 200      # hundreds of such pairs
    got, guards = _gpu_decode_guarded(blob.numpy(), blob.header)
    assert guards
    assert np.array_equal(got, _oracle_expected(orc, x))


@pytest.mark.parametrize("lane_syms", [32, 64, 128])
@pytest.mark.parametrize("island_chunks,workgroups,group", [(6, 0, 1), (40, 1, 1), (150, 1, 1), (150, 0, 1), (150, 0, 32)])
def test_islands_of_long_codes(orc, lane_syms, island_chunks, workgroups, group):
    """Plain-Huffman blobs whose chunks code far worse than the stage allows: one exponent fills
    90 % of the tensor (1-bit code), islands hold only the fifteen rare ones (5 bits and more per
    symbol, spans larger than a wave's stage).  A few such chunks per workgroup go through the wide
    slots, more than the kernel remembers (one workgroup, 150 chunks) through the symbol pass."""
    rng = np.random.default_rng(lane_syms + island_chunks)
    chunk = 64 * lane_syms
    n = 40 * island_chunks * chunk + 12345
    e = np.full(n, 7, dtype=np.uint8)
    rare = np.array([v for v in range(16) if v != 7], dtype=np.uint8)
    for start in (3 * chunk + 17, n // 2):                     # two islands, the first one unaligned
        m = island_chunks * chunk // 2
        e[start:start + m] = rng.choice(rare, size=m)
    x = ((rng.integers(0, 2, n, dtype=np.uint8) << 7) | (e << 3) | rng.integers(0, 8, n, dtype=np.uint8)).astype(np.uint8)
    blob = ecf8.ecf8_encode(x, 1, n, lane_syms=lane_syms, max_code_len=15, group_chunks=group)
    h = blob.header
    assert max(h.code_len) > 4 and min(v for v in h.code_len if v) == 1
    cb = blob.numpy()[h.off_chunk_bit:h.off_chunk_bit + 8 * (h.n_chunks + 1)].view("<u8").astype(np.int64)
    assert (np.diff(cb) / 8 > lane_syms * 32 + 64).sum() >= (island_chunks - 4 if group == 1 else 64)   # spans beyond a wave's stage
    pad = 4096
    buf = torch.full((pad + n + pad,), 0xA5, dtype=torch.uint8, device=DEV)
    batch = ecf8.Batch([h], [blob.to(DEV)], [buf[pad:pad + n]])
    batch.info.max_workgroups = workgroups
    ecf8.ecf8_decode_batched(batch)
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    assert (host[:pad] == 0xA5).all() and (host[pad + n:] == 0xA5).all()
    assert np.array_equal(host[pad:pad + n], x)


@pytest.mark.parametrize("lane_syms,group", [(32, 1), (32, 64), (64, 2), (64, 32), (128, 1), (128, 8), (128, 64)])
def test_group_widths(orc, lane_syms, group):
    """Every interleave width the format allows next to the default: whole groups, then
    chunk-major chunks, then a ragged last chunk."""
    n = 1_000_003 if group < 64 else 2_300_017
    x = _rand_bytes(n, 5 * lane_syms + group)
    blob = ecf8.ecf8_encode(x, 1, n, lane_syms=lane_syms, group_chunks=group, table_mode=1 + (group % 3 == 1),
                            max_code_len=15 if group in (2, 8) else 0)
    assert blob.header.group_chunks == group
    got, guards = _gpu_decode_guarded(blob.numpy(), blob.header)
    assert guards
    assert np.array_equal(got, _oracle_expected(orc, x))


@pytest.mark.parametrize("block", range(6))
def test_seeded_sweep_of_shapes_and_options(orc, block):
    """240 seeded combinations of size, lane_syms, group width, code cap, table mode and exponent
    skew, each decoded alone (guarded buffer) and all of a block again in one mixed batch."""
    rng = np.random.default_rng(9000 + block)
    cases = []
    for i in range(40):
        lane_syms = int(rng.choice([32, 64, 128]))
        chunk = 64 * lane_syms
        kind = i % 5
        if kind == 0:
            n = int(rng.integers(1, 3 * chunk))
        elif kind == 1:
            n = int(rng.integers(1, 40)) * chunk + int(rng.choice([-1, 0, 1, 15, 16, 17]))
        elif kind == 2:
            g = int(rng.choice([2, 4, 8]))
            n = g * chunk * int(rng.integers(1, 4)) + int(rng.integers(0, 2 * chunk))
        else:
            n = int(rng.integers(1, 400_000))
        n = max(n, 1)
        group = int(rng.choice([1, 2, 4, 8, 16, 32, 64]))
        cap = int(rng.choice([0, 0, 15, 4, 9]))
        conc = float(rng.choice([0.05, 0.2, 0.5, 2.0, 50.0]))
        x = _rand_bytes(n, int(rng.integers(1 << 30)), conc=conc)
        blob = ecf8.ecf8_encode(x, 1, n, lane_syms=lane_syms, group_chunks=group, max_code_len=cap,
                                table_mode=int(rng.choice([1, 2])))
        got, guards = _gpu_decode_guarded(blob.numpy(), blob.header, pad=512)
        assert guards, (lane_syms, n, group, cap)
        assert np.array_equal(got, x), (lane_syms, n, group, cap, conc)
        cases.append((lane_syms, x, blob))
    assert np.array_equal(_oracle_expected(orc, cases[0][1]), cases[0][1])
    for lane_syms in (32, 64, 128):
        sel = [(x, b) for ls, x, b in cases if ls == lane_syms]
        if not sel:
            continue
        outs = [torch.full((x.size,), 0x33, dtype=torch.uint8, device=DEV) for x, _ in sel]
        batch = ecf8.Batch([b.header for _, b in sel], [b.to(DEV) for _, b in sel], outs)
        ecf8.ecf8_decode_batched(batch)
        torch.cuda.synchronize()
        for (x, _), o in zip(sel, outs):
            assert np.array_equal(o.cpu().numpy(), x)


@pytest.mark.parametrize("lane_syms,rows,cols,cap", [(32, 16, 128, 0), (64, 64, 4096, 0), (64, 160, 1024, 15),
                                                     (128, 48, 3584, 0), (128, 1024, 1024, 15)])
def test_row_tiled_blobs_decode(orc, lane_syms, rows, cols, cap):
    """ecf8_decode on the row-tiled layout the fused GEMM reads (a chunk = 16 rows x 4N columns)."""
    x = _rand_bytes(rows * cols, rows + cols + lane_syms)
    blob = ecf8.ecf8_encode(x, rows, cols, lane_syms=lane_syms, tile_rows=16, max_code_len=cap, table_mode=1 + (rows > 100))
    assert blob.header.tile_rows == 16
    got, guards = _gpu_decode_guarded(blob.numpy(), blob.header)
    assert guards
    assert np.array_equal(got, _oracle_expected(orc, x))
    dec, _ = orc.container_decode(blob.numpy())
    assert np.array_equal(got, dec)


@pytest.mark.parametrize("rows,cols", [(16, 256), (48, 512), (1040, 4096), (272, 14336), (4096, 1024)])
def test_row_tiled_blobs_of_the_fused_gemm_decode_as_row_segments(orc, rows, cols):
    """The fused GEMM's blobs (row-tiled, N = 64, codes capped at 7 bits) through ecf8_decode and through a
    batch: the kernel variant that turns a decoded chunk into whole 256-byte row segments in LDS before
    storing it.  Against the input, the oracle's reader (small cases) and with guard bytes around the output;
    a batch that mixes such a blob with a linear one takes the general route and must agree as well."""
    x = synth.make_weight(rows, cols, 1.7, 0.02, rows + cols).numpy()
    blob = ecf8.ecf8_encode(x, rows, cols, lane_syms=64, tile_rows=16, table_mode=1 + (rows > 100))
    assert blob.header.tile_rows == 16 and max(blob.header.code_len) <= 7
    got, guards = _gpu_decode_guarded(blob.numpy(), blob.header)
    assert guards
    assert np.array_equal(got, x.reshape(-1))
    if rows * cols <= 1 << 22:
        dec, _ = orc.container_decode(blob.numpy())
        assert np.array_equal(got, dec)
    x2 = synth.make_weight(rows, cols, 1.9, 0.015, 5).numpy()
    blob2 = ecf8.ecf8_encode(x2, rows, cols, lane_syms=64, tile_rows=16)
    lin = ecf8.ecf8_encode(x2, rows, cols, lane_syms=64)
    for members, tiled in (((x, blob), (x2, blob2)), True), (((x, blob), (x2, lin)), False):
        outs = [torch.full((rows * cols + 64,), 0xEE, dtype=torch.uint8, device=DEV) for _ in members]
        batch = ecf8.Batch([b.header for _, b in members], [b.to(DEV) for _, b in members], [o[32:32 + rows * cols] for o in outs])
        assert batch.info.row_tiled == int(tiled)
        ecf8.ecf8_decode_batched(batch)
        torch.cuda.synchronize()
        for (want, _), o in zip(members, outs):
            assert np.array_equal(o[32:32 + rows * cols].cpu().numpy(), want.reshape(-1))
            assert bool((o[:32] == 0xEE).all()) and bool((o[32 + rows * cols:] == 0xEE).all())


@pytest.mark.parametrize("lane_syms,group", [(64, 1), (64, 4), (128, 32)])
def test_oracle_written_container_decodes_on_gpu(orc, lane_syms, group):
    """Interop: a container written by the oracle's writer (its own tie-breaks)."""
    x = _rand_bytes(600_003, 9)
    arr = orc.container_encode(x, 1, x.size, lane_syms, group)
    hdr = ecf8.blob_describe(arr)
    ecf8.blob_validate(arr)
    got, guards = _gpu_decode_guarded(arr, hdr)
    assert guards and np.array_equal(got, x)


def test_deterministic_and_on_side_stream(orc):
    x = _rand_bytes(3_000_000, 4)
    blob = ecf8.ecf8_encode(x, 1500, 2000)
    d_blob = blob.to(DEV)
    a = ecf8.ecf8_decode(blob.header, d_blob)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        b = ecf8.ecf8_decode(blob.header, d_blob)
    s.synchronize()
    torch.cuda.synchronize()
    assert a.shape == (1500, 2000)
    assert torch.equal(a, b)
    assert np.array_equal(a.cpu().numpy().reshape(-1), _oracle_expected(orc, x))


@pytest.mark.parametrize("caps,lane_syms", [((0,), 0), ((0, 15, 9), 128), ((0, 15, 9), 64), ((15,), 0), ((15,), 128)])
def test_batched_mixed_tensors(orc, caps, lane_syms):
    """Many tensors, each with its own code, sizes from one lane to many chunks, one launch;
    all under the default cap (branch-free kernel), mixed caps and plain Huffman (general kernels).
    A batch shares one lane size, and the encoder's default depends on the cap: mixed caps name theirs."""
    sizes = [5, 4096, 70_000, 1, 333_333, 8192 * 3, 1_000_000, 17, 250_000]
    xs = [_rand_bytes(n, 100 + i, conc=0.2 + 0.1 * i) for i, n in enumerate(sizes)]
    blobs = [ecf8.ecf8_encode(x, 1, x.size, table_mode=1 + (i % 2), max_code_len=caps[i % len(caps)], lane_syms=lane_syms)
             for i, x in enumerate(xs)]
    d_blobs = [b.to(DEV) for b in blobs]
    pad = 256
    bufs = [torch.full((pad + x.size + pad,), 0x5A, dtype=torch.uint8, device=DEV) for x in xs]
    outs = [b[pad:pad + x.size] for b, x in zip(bufs, xs)]
    batch = ecf8.Batch([b.header for b in blobs], d_blobs, outs)
    assert batch.total_chunks == sum(b.header.n_chunks for b in blobs)
    ecf8.ecf8_decode_batched(batch)
    torch.cuda.synchronize()
    for x, buf in zip(xs, bufs):
        h = buf.cpu().numpy()
        assert (h[:pad] == 0x5A).all() and (h[pad + x.size:] == 0x5A).all()
        assert np.array_equal(h[pad:pad + x.size], _oracle_expected(orc, x))


def test_batch_argument_errors():
    x = _rand_bytes(5000, 1)
    b64, b128 = ecf8.ecf8_encode(x, 1, x.size, lane_syms=64), ecf8.ecf8_encode(x, 1, x.size, lane_syms=128)
    d = [b64.to(DEV), b128.to(DEV)]
    o = [torch.empty(5000, dtype=torch.uint8, device=DEV) for _ in range(2)]
    with pytest.raises(ecf8.Ecf8Error) as e:
        ecf8.Batch([b64.header, b128.header], d, o)          # mixed lane_syms
    assert e.value.code == ecf8.E_ARG
    with pytest.raises(ecf8.Ecf8Error) as e:
        ecf8.Batch([b64.header], d[:1], [o[0][:100]])          # output too small
    assert e.value.code == ecf8.E_CAPACITY
    with pytest.raises(ecf8.Ecf8Error) as e:
        ecf8.ecf8_decode(b64.header, d[0], torch.empty(5008, dtype=torch.uint8, device=DEV)[3:5003])
    assert e.value.code == ecf8.E_ALIGN


# ---------------------------------------------------------------- full-size cases

def _full_size_case(orc, specs, oracle_checks, max_code_len=0, reader_checks=(), gpu_encode=False, arenas=False):
    """Encode/ decode `specs` (full-size tensors, generated on the GPU) in ONE batched launch, the
    launch configuration bench.py times.  Every output is compared with its input on the device
    (decode(encode(x)) == x is the plain definition of the result); the tensors named in
    `oracle_checks` are also compared with the oracle's own encode -> bit-serial decode (and the
    container's stream length with the oracle's optimum), and for those in `reader_checks` the
    oracle's reader decodes the very container the GPU decoded.  gpu_encode: containers written by the
    device encoder (byte for byte the CPU encoder's, tests/test_gpu_encode.py), which keeps the
    largest stacks inside the suite's time.  arenas: all blobs in one device allocation and all outputs in another,
    tensors at multiples of 4 KiB, which is how bench.py holds a stack by default."""
    ts = []
    for s in specs:
        w = synth.make(s, 0, device=DEV)
        if gpu_encode:
            h, big = ecf8.ecf8_encode_gpu(w, s["rows"], s["cols"], max_code_len=max_code_len)
            d_blob = big.clone()
            del big
        else:
            b = ecf8.ecf8_encode(w.cpu(), s["rows"], s["cols"], max_code_len=max_code_len)
            h, d_blob = b.header, b.to(DEV)
        ts.append((s, w, h, d_blob, None if arenas else torch.full_like(w, 0xEE)))
    if arenas:
        al = lambda n: (n + 4095) // 4096 * 4096
        blobs = torch.empty(sum(al(t[3].numel()) for t in ts), dtype=torch.uint8, device=DEV)
        outs = torch.full((sum(al(t[1].numel()) for t in ts),), 0xEE, dtype=torch.uint8, device=DEV)
        ob = oo = 0
        for i, (s, w, h, d_blob, _) in enumerate(ts):
            nb, no = d_blob.numel(), w.numel()
            blobs[ob:ob + nb].copy_(d_blob)
            ts[i] = (s, w, h, blobs[ob:ob + nb], outs[oo:oo + no].view(w.shape))
            ob, oo = ob + al(nb), oo + al(no)
        del d_blob
        torch.cuda.empty_cache()
    print("full-size case: %d tensors, %d weights, one launch" % (len(ts), sum(t[1].numel() for t in ts)), flush=True)
    batch = ecf8.Batch([t[2] for t in ts], [t[3] for t in ts], [t[4] for t in ts])
    ecf8.ecf8_decode_batched(batch)
    torch.cuda.synchronize()
    seen = set()
    for s, w, h, d_blob, out in ts:
        assert torch.equal(out, w), s["name"]
        if s["name"] in oracle_checks:
            seen.add(s["name"])
            x = w.cpu().numpy().reshape(-1)
            exp, nbits, _ = orc.roundtrip(x)
            f = orc.histogram(x)
            cap = max_code_len or 7
            assert h.stream_bits == (nbits if cap >= 15 else orc.stream_bits(f, orc.huffman_lengths_limited(f, cap)))
            got = out.cpu().numpy().reshape(-1)
            assert np.array_equal(got, exp), s["name"]
            if s["name"] in reader_checks:
                dec, bits = orc.container_decode(d_blob.cpu().numpy())
                assert bits == h.stream_bits and np.array_equal(dec, got), s["name"]
    assert seen == set(oracle_checks)


@pytest.mark.parametrize("max_code_len", [0, 15])
def test_config1_full_layer(orc, max_code_len):
    """configs[1]: one full layer of the 8B-class stack (7 matrices, 218 M weights), one launch;
    under the default cap on the code length and with plain Huffman.  The oracle decodes the whole
    layer, and its reader the K projection's container."""
    specs = synth.config1(0, 1)
    _full_size_case(orc, specs, {s["name"] for s in specs}, max_code_len, reader_checks={"l0.k"})


def test_config1_whole_stack_one_launch(orc):
    """configs[1] at full size in the launch configuration and memory layout bench.py times: all 32 layers (224
    matrices, 6.98 G weights) through ONE ecf8_decode_batched launch; every output compared with
    its input on the device, two matrices also with the oracle's own encode -> bit-serial decode."""
    _full_size_case(orc, synth.config1(0, 32), {"l17.v", "l31.k"}, gpu_encode=True, arenas=True)


def test_config2_experts_and_attention(orc):
    """configs[2]: six full-size expert matrices and the two attention projections in one launch,
    containers from the CPU encoder."""
    specs = synth.config2(0, 2)
    _full_size_case(orc, specs, {"e0.gate", "e1.down"})


def test_config2_whole_layer_one_launch(orc):
    """configs[2] at full size: the 768 expert matrices and the two attention projections (770 tensors,
    11.6 G weights) through ONE ecf8_decode_batched launch; every output compared with its input on the
    device; the oracle decodes one expert's three matrices and an attention projection, and its reader
    one expert container."""
    _full_size_case(orc, synth.config2(0, 256), {"e137.gate", "e137.up", "e137.down", "attn_b"},
                    reader_checks={"e137.down"}, gpu_encode=True)


def test_config3_full_block(orc):
    """configs[3]: one full DiT block (11 matrices, 509 M weights, per-tensor scaling), one launch,
    containers from the CPU encoder; the oracle decodes the whole block."""
    specs = synth.config3(1)
    _full_size_case(orc, specs, {s["name"] for s in specs}, reader_checks={"b0.sa_q"})


def test_config3_whole_stack_one_launch(orc):
    """configs[3] at full size: all 40 blocks (440 matrices, 20.3 G weights) through ONE
    ecf8_decode_batched launch; every output compared with its input on the device, three matrices of
    a late block also with the oracle."""
    _full_size_case(orc, synth.config3(40), {"b33.ca_k", "b33.ffn2", "b39.sa_o"}, gpu_encode=True, arenas=True)


def test_stream_longer_than_2_to_the_31_bits():
    """2^30 weights in one tensor: chunk start bits pass 2^31, so bit positions need all 64 bits.  The
    oracle cannot read a container of this size in reasonable time; the decoded tensor is compared with
    the input (the container's content is pinned by the smaller cases)."""
    n = 1 << 30
    g = torch.Generator(device=DEV)
    g.manual_seed(31)
    e = torch.randn(n, generator=g, device=DEV).mul_(1.5).add_(7.0).round_().clamp_(0, 15).to(torch.int32)
    low = torch.randint(0, 8, (n,), generator=g, device=DEV, dtype=torch.int32)
    x = ((e << 3) | low | ((low & 1) << 7)).to(torch.uint8)
    del e, low
    blob = ecf8.ecf8_encode(x.cpu().numpy(), 1 << 15, 1 << 15)
    assert blob.header.stream_bits > 1 << 31
    d_blob = blob.to(DEV)
    out = torch.empty_like(x)
    ecf8.ecf8_decode(blob.header, d_blob, out)
    torch.cuda.synchronize()
    assert torch.equal(out, x)


def test_e5m2_bytes_through_this_codec(orc):
    """The codec never interprets its bytes: E5M2 weights go through unchanged (coded by the upper four bits of
    their exponent field, the lowest one kept raw in the nibble plane) and come back exact."""
    w = synth.make_e5m2(1024, 1536, 1.8, 0.02, 3).numpy().reshape(-1)
    blob = ecf8.ecf8_encode(w, 1024, 1536)
    got, guards = _gpu_decode_guarded(blob.numpy(), blob.header)
    assert guards and np.array_equal(got, _oracle_expected(orc, w)) and np.array_equal(got, w)
    assert blob.size / w.size < 0.78

"""Fused decode + FP8 GEMM (configs[4]) against the oracle's fp64 reference, through the C ABI.

Tolerances, both relative to sum_k |x_k w_k| of the output in question (FP8 x FP8 products are exact; only
the accumulation differs from the fp64 reference, so the natural yardstick is the sum of magnitudes):

EXACT = 1e-5, the tolerance the fused-GEMM configuration states.  It holds for the calls that multiply on
the F16 matrix cores (ecf8_gemm_fp8_exact and its raw twin): operands are converted to halves exactly, the
products are exact, and what is left is fp32 summation (K / 32 partial sums per wave and a handful of adds
across waves: about sqrt(K / 32) * 2^-24 of the partial sums, well below 1e-6).

FP8_CORE = 7 * 2^-13, the bound of the FP8 matrix core (ecf8_gemm_fp8 and every call built on it), derived
from how it adds: the 8 products a lane contributes to a step are aligned to the largest of them and bits
more than 13 places below its leading bit are dropped (448 * 448 + 31 * 1 gives 200728: the 7 ones that
share a lane with the big product are lost).  Each of the other 7 products of a lane group loses less than
2^-13 of the largest, which is at most the group's share of sum |x w|; summed over the groups the error is
below 7 * 2^-13 * sum_k |x_k w_k| whatever K is.  The same bound applies to every slice of a scaled sum
(the scale multiplies the slice's value and its error alike), so the scaled, split and grouped calls share
it.  1e-5 is not reachable on this path; that is what the exact calls are for.  The decoded weights
themselves are bit exact either way: each fused call equals its twin on uncompressed weights bit for bit.
"""
import numpy as np
import pytest
import torch

from paper_2510_02676_amd import ecf8, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


EXACT = 1e-5
FP8_CORE = 7 * 2.0 ** -13


def _check(y, yref, mag, what, rel=FP8_CORE):
    err = np.abs(y.astype(np.float64) - yref)
    bound = rel * mag + 1e-30
    worst = float((err / bound).max())
    assert worst <= 1.0, "%s: worst |err| / (%.1e sum|xw|) = %.3g" % (what, rel, worst)


def test_one_tile_ocp_landmarks(orc):
    """One 16-row tile whose weights are the OCP landmarks (-0 = 0x80, 448 = 0x7E, 2^-6 = 0x08,
    subnormals, 1.0, -1.5): wrong FP8 flavour in the matrix cores would show as NaN or factors of 2."""
    K = 4096
    w = np.zeros((16, K), dtype=np.uint8)
    vals = [0x80, 0x7E, 0x08, 0x01, 0x07, 0x38, 0xBC, 0xFE, 0x00, 0x40, 0x30, 0x28, 0x77, 0xF7, 0x0F, 0x10]
    for n in range(16):
        w[n, :] = vals[n]
        w[n, n::17] = vals[(n + 5) % 16]
    x = np.zeros((3, K), dtype=np.uint8)
    x[0, :] = 0x38                      # 1.0 everywhere: row sums of W
    x[1, ::2] = 0x38
    x[1, 1::2] = 0xB8                   # alternating +1 / -1
    x[2, :] = 0x30                      # 0.5
    yref, mag = orc.gemm_ref(x, w)
    d_x = torch.from_numpy(x).to(DEV)
    raw = ecf8.ecf8_gemm_fp8_raw(torch.from_numpy(w).to(DEV), d_x)
    blob = ecf8.ecf8_encode(w, 16, K, lane_syms=64, tile_rows=16)
    fused = ecf8.ecf8_gemm_fp8(blob.header, blob.to(DEV), d_x)
    torch.cuda.synchronize()
    assert not torch.isnan(raw).any() and not torch.isnan(fused).any()
    # this input is adversarial for the FP8 matrix core's truncation (448s next to subnormals); a wrong
    # FP8 flavour misses even that bound by orders
    _check(raw.cpu().numpy(), yref, mag, "raw")
    _check(fused.cpu().numpy(), yref, mag, "fused")
    assert torch.equal(raw, fused)      # same multiply phase on the same bytes
    # on the F16 matrix cores the same adversarial input meets the stated tolerance
    d_blob = blob.to(DEV)
    exact = ecf8.ecf8_gemm_fp8_exact(blob.header, d_blob, d_x)
    exact_raw = ecf8.ecf8_gemm_fp8_raw_exact(torch.from_numpy(w).to(DEV), d_x)
    torch.cuda.synchronize()
    _check(exact.cpu().numpy(), yref, mag, "exact", rel=EXACT)
    assert torch.equal(exact, exact_raw)
    # a NaN encoding in W or in X makes the outputs it touches NaN in both modes
    wn, xn = w.copy(), x.copy()
    wn[3, 100] = 0x7F
    xn[1, 7] = 0xFF
    bn = ecf8.ecf8_encode(wn, 16, K, lane_syms=64, tile_rows=16)
    for fn in (ecf8.ecf8_gemm_fp8, ecf8.ecf8_gemm_fp8_exact):
        y = fn(bn.header, bn.to(DEV), torch.from_numpy(xn).to(DEV)).cpu().numpy()
        assert np.isnan(y[:, 3]).all() and np.isnan(y[1, :]).all()
        assert not np.isnan(np.delete(np.delete(y, 3, axis=1), 1, axis=0)).any()


@pytest.mark.parametrize("M", [1, 16, 17, 64])
@pytest.mark.parametrize("table_mode", [1, 2])
def test_small_gemm_against_oracle(orc, M, table_mode):
    rows, K = 128, 4096
    w = synth.make_weight(rows, K, 1.7, 0.02, 3).numpy()
    x = synth.activations(M, K, seed=M).numpy()
    yref, mag = orc.gemm_ref(x, w)
    blob = ecf8.ecf8_encode(w, rows, K, lane_syms=64, tile_rows=16, table_mode=table_mode)
    d_x = torch.from_numpy(x).to(DEV)
    guard = torch.full((M + 2, rows), float("nan"), dtype=torch.float32, device=DEV)
    y = ecf8.ecf8_gemm_fp8(blob.header, blob.to(DEV), d_x, guard[1:M + 1])
    torch.cuda.synchronize()
    assert torch.isnan(guard[0]).all() and torch.isnan(guard[M + 1]).all()
    _check(y.cpu().numpy(), yref, mag, "fused M=%d" % M)
    raw = ecf8.ecf8_gemm_fp8_raw(torch.from_numpy(w).to(DEV), d_x)
    torch.cuda.synchronize()
    assert torch.equal(raw, y)
    guard.fill_(float("nan"))
    y = ecf8.ecf8_gemm_fp8_exact(blob.header, blob.to(DEV), d_x, d_y=guard[1:M + 1])
    raw = ecf8.ecf8_gemm_fp8_raw_exact(torch.from_numpy(w).to(DEV), d_x)
    torch.cuda.synchronize()
    assert torch.isnan(guard[0]).all() and torch.isnan(guard[M + 1]).all()
    _check(y.cpu().numpy(), yref, mag, "exact fused M=%d" % M, rel=EXACT)
    assert torch.equal(raw, y)


@pytest.mark.parametrize("M", [1, 16, 64])
def test_config4_full_size(orc, M):
    """configs[4]: W 14336 x 4096 (config-2 distribution), X = M x 4096 N(0,1) rows scaled to 448.
    Every output of the fused kernel equals the raw-weights kernel bit for bit, on the FP8 and on the F16
    matrix cores; a sample of output columns is checked against the oracle (decoded bytes are the
    oracle's: decode(encode(W)) == W): the exact call to the configuration's 1e-5, the FP8 matrix-core
    call to that core's bound."""
    spec = synth.config4()[0]
    w = synth.make(spec, 0, device=DEV)
    x = synth.activations(M, 4096, seed=0, device=DEV)
    blob = ecf8.ecf8_encode(w.cpu(), spec["rows"], spec["cols"], lane_syms=64, tile_rows=16)
    d_blob = blob.to(DEV)
    fused = ecf8.ecf8_gemm_fp8(blob.header, d_blob, x)
    raw = ecf8.ecf8_gemm_fp8_raw(w, x)
    exact = ecf8.ecf8_gemm_fp8_exact(blob.header, d_blob, x)
    exact_raw = ecf8.ecf8_gemm_fp8_raw_exact(w, x)
    torch.cuda.synchronize()
    assert torch.equal(fused, raw) and torch.equal(exact, exact_raw)
    cols = np.unique(np.concatenate([np.arange(0, 64), np.random.default_rng(M).integers(0, spec["rows"], 448),
                                     np.arange(spec["rows"] - 32, spec["rows"])]))
    wh = w.cpu().numpy()
    dec, _, _ = orc.roundtrip(wh[cols].reshape(-1))
    assert np.array_equal(dec.reshape(len(cols), 4096), wh[cols])
    yref, mag = orc.gemm_ref(x.cpu().numpy(), wh[cols])
    _check(exact.cpu().numpy()[:, cols], yref, mag, "config4 exact M=%d" % M, rel=EXACT)
    _check(fused.cpu().numpy()[:, cols], yref, mag, "config4 M=%d" % M)


@pytest.mark.parametrize("rows,M", [(16 * 1300, 1), (16 * 2200, 16), (16 * 2051, 7)])
def test_tall_matrices_at_k_4096(orc, rows, M):
    """More than four blocks of 16 rows per workgroup at K = 4096 and up to 16 columns of X: the workgroups park the
    partial sums of four blocks per barrier, so here the buffers are reused (two or three rounds, the last one with
    one to four blocks).  Fused equals the twin on uncompressed weights bit for bit, with and without scales; rows
    from the first, a middle and the last round are checked against the oracle."""
    K = 4096
    w = synth.make_weight(rows, K, 1.8, 0.015, 11, device=DEV)
    x = synth.activations(M, K, seed=rows % 97, device=DEV)
    hdr, d_blob = ecf8.ecf8_encode_gpu(w.view(torch.uint8), rows, K, lane_syms=64, tile_rows=16)
    guard = torch.full((M + 2, rows), float("nan"), dtype=torch.float32, device=DEV)
    fused = ecf8.ecf8_gemm_fp8(hdr, d_blob, x, guard[1:M + 1])
    raw = ecf8.ecf8_gemm_fp8_raw(w.view(torch.uint8), x)
    exact = ecf8.ecf8_gemm_fp8_exact(hdr, d_blob, x)
    exact_raw = ecf8.ecf8_gemm_fp8_raw_exact(w.view(torch.uint8), x)
    torch.cuda.synchronize()
    assert torch.isnan(guard[0]).all() and torch.isnan(guard[M + 1]).all()
    assert torch.equal(fused, raw) and torch.equal(exact, exact_raw)
    ws, xs = _scales(rows, M, M)
    d_ws, d_xs = torch.from_numpy(ws).to(DEV), torch.from_numpy(xs).to(DEV)
    ys = ecf8.ecf8_gemm_fp8_scaled(hdr, d_blob, x, d_ws, d_xs)
    ys_raw = ecf8.ecf8_gemm_fp8_raw_scaled(w.view(torch.uint8), x, d_ws, d_xs)
    torch.cuda.synchronize()
    assert torch.equal(ys, ys_raw)
    cols = np.unique(np.concatenate([np.arange(0, 48), np.random.default_rng(M).integers(0, rows, 300),
                                     np.arange(16 * 256 * 4 - 16, 16 * 256 * 4 + 32), np.arange(rows - 48, rows)]))
    wh = w.view(torch.uint8).cpu().numpy()
    xh = x.cpu().numpy()
    yref, mag = orc.gemm_ref(xh, wh[cols])
    _check(exact.cpu().numpy()[:, cols], yref, mag, "tall exact M=%d" % M, rel=EXACT)
    _check(fused.cpu().numpy()[:, cols], yref, mag, "tall M=%d" % M)
    sub = np.arange(0, 256)                      # the first two rows of scale blocks, whole
    yref_s, mag_s = orc.gemm_ref_scaled(xh, wh[sub], ws[:2], xs)
    _check(ys.cpu().numpy()[:, sub], yref_s, mag_s, "tall scaled M=%d" % M)


def test_gemm_argument_errors():
    x = torch.zeros((4, 4096), dtype=torch.uint8, device=DEV)
    w = torch.zeros((32, 2176), dtype=torch.uint8, device=DEV)
    with pytest.raises(ecf8.Ecf8Error) as e:
        ecf8.ecf8_gemm_fp8_raw(w, x[:, :2176].contiguous())            # cols not a multiple of 256
    assert e.value.code == ecf8.E_ARG
    w = torch.zeros((24, 4096), dtype=torch.uint8, device=DEV)
    with pytest.raises(ecf8.Ecf8Error):
        ecf8.ecf8_gemm_fp8_raw(w, x)                                    # rows not a multiple of 16
    w = torch.zeros((32, 4096), dtype=torch.uint8, device=DEV)
    with pytest.raises(ecf8.Ecf8Error):
        ecf8.ecf8_gemm_fp8_raw(w, torch.zeros((65, 4096), dtype=torch.uint8, device=DEV))   # M > 64
    b = ecf8.ecf8_encode(np.zeros((32, 4096), dtype=np.uint8), 32, 4096, lane_syms=128)
    with pytest.raises(ecf8.Ecf8Error):
        ecf8.ecf8_gemm_fp8(b.header, b.to(DEV), x)                      # lane_syms != 64
    z = np.zeros((64, 4096), dtype=np.uint8)
    for kw in (dict(lane_syms=64), dict(lane_syms=64, group_chunks=1), dict(lane_syms=128, tile_rows=16)):
        b = ecf8.ecf8_encode(z, 64, 4096, **kw)
        with pytest.raises(ecf8.Ecf8Error) as e:
            ecf8.ecf8_gemm_fp8(b.header, b.to(DEV), x)                  # not a row-tiled blob of 16 x 256 chunks
        assert e.value.code == ecf8.E_ARG
    fib = [1, 1]
    while len(fib) < 16:
        fib.append(fib[-1] + fib[-2])
    deep = np.resize(np.repeat(np.arange(16, dtype=np.uint8) << 3, fib), 64 * 4096)
    b = ecf8.ecf8_encode(deep, 64, 4096, lane_syms=64, tile_rows=16, max_code_len=15)
    with pytest.raises(ecf8.Ecf8Error) as e:
        ecf8.ecf8_gemm_fp8(b.header, b.to(DEV), x)                      # codewords longer than 7 bits
    assert e.value.code == ecf8.E_ARG


def _scales(rows, M, seed):
    rng = np.random.default_rng(seed)
    ws = np.exp(rng.normal(0.0, 0.7, size=((rows + 127) // 128, 32))).astype(np.float32)      # 2^-2 .. 2^2 or so
    xs = np.exp(rng.normal(0.0, 0.5, size=M)).astype(np.float32)
    return ws, xs


@pytest.mark.parametrize("M", [1, 7, 16, 17, 32, 33, 64])
def test_block_scaled_gemm_against_oracle(orc, M):
    """One fp32 scale per 128 x 128 block of W and per row of X; rows = 208 leaves the second row of scale
    blocks ragged.  Every 128-wide slice of K enters the sum through one fp32 multiply-add, which adds a
    few 2^-24: same tolerances as the unscaled case, on either kind of matrix core."""
    rows, K = 208, 4096
    w = synth.make_weight(rows, K, 1.7, 0.02, 5).numpy()
    x = synth.activations(M, K, seed=100 + M).numpy()
    ws, xs = _scales(rows, M, M)
    d_w, d_x = torch.from_numpy(w).to(DEV), torch.from_numpy(x).to(DEV)
    d_ws, d_xs = torch.from_numpy(ws).to(DEV), torch.from_numpy(xs).to(DEV)
    blob = ecf8.ecf8_encode(w, rows, K, lane_syms=64, tile_rows=16)
    d_blob = blob.to(DEV)
    xg = np.exp(np.random.default_rng(M + 50).normal(0.0, 0.5, size=(M, K // 128))).astype(np.float32)
    d_xg = torch.from_numpy(xg).to(DEV)
    for xs_h, xs_d in ((xs, d_xs), (None, None), (xg, d_xg)):      # one scale per row, none, one per row and 128 columns
        yref, mag = orc.gemm_ref_scaled(x, w, ws, xs_h)
        guard = torch.full((M + 2, rows), float("nan"), dtype=torch.float32, device=DEV)
        y = ecf8.ecf8_gemm_fp8_scaled(blob.header, d_blob, d_x, d_ws, xs_d, guard[1:M + 1])
        raw = ecf8.ecf8_gemm_fp8_raw_scaled(d_w, d_x, d_ws, xs_d)
        torch.cuda.synchronize()
        assert torch.isnan(guard[0]).all() and torch.isnan(guard[M + 1]).all()
        _check(y.cpu().numpy(), yref, mag, "scaled fused M=%d" % M)
        assert torch.equal(raw, y)           # same steps in the same order on the same bytes
        y = ecf8.ecf8_gemm_fp8_exact(blob.header, d_blob, d_x, d_ws, xs_d)
        raw = ecf8.ecf8_gemm_fp8_raw_exact(d_w, d_x, d_ws, xs_d)
        torch.cuda.synchronize()
        _check(y.cpu().numpy(), yref, mag, "scaled exact M=%d" % M, rel=EXACT)
        assert torch.equal(raw, y)


def test_block_scales_that_are_powers_of_two_scale_exactly():
    """Doubling the scales of one column of scale blocks changes exactly that slice's contribution; doubling
    all of them doubles every output bit for bit (fp32 multiply-adds by powers of two are exact)."""
    rows, K, M = 256, 4096, 5
    w = synth.make_weight(rows, K, 1.8, 0.02, 6).numpy()
    x = synth.activations(M, K, seed=6).numpy()
    blob = ecf8.ecf8_encode(w, rows, K, lane_syms=64, tile_rows=16)
    d_blob, d_x = blob.to(DEV), torch.from_numpy(x).to(DEV)
    ones = torch.ones((2, 32), dtype=torch.float32, device=DEV)
    y1 = ecf8.ecf8_gemm_fp8_scaled(blob.header, d_blob, d_x, ones)
    y2 = ecf8.ecf8_gemm_fp8_scaled(blob.header, d_blob, d_x, ones * 2)
    y4 = ecf8.ecf8_gemm_fp8_scaled(blob.header, d_blob, d_x, ones, torch.full((M,), 4.0, device=DEV))
    only_first_rows = ones.clone()
    only_first_rows[1] = 0.0
    y0 = ecf8.ecf8_gemm_fp8_scaled(blob.header, d_blob, d_x, only_first_rows)
    torch.cuda.synchronize()
    assert torch.equal(y2, y1 * 2) and torch.equal(y4, y1 * 4)
    assert torch.equal(y0[:, :128], y1[:, :128]) and (y0[:, 128:] == 0).all()


def test_block_scaled_full_size_and_argument_errors(orc):
    spec = synth.config4()[0]
    M = 16
    w = synth.make(spec, 0, device=DEV)
    x = synth.activations(M, 4096, seed=1, device=DEV)
    ws, xs = _scales(spec["rows"], M, 9)
    d_ws, d_xs = torch.from_numpy(ws).to(DEV), torch.from_numpy(xs).to(DEV)
    blob = ecf8.ecf8_encode(w.cpu(), spec["rows"], spec["cols"], lane_syms=64, tile_rows=16)
    d_blob = blob.to(DEV)
    fused = ecf8.ecf8_gemm_fp8_scaled(blob.header, d_blob, x, d_ws, d_xs)
    raw = ecf8.ecf8_gemm_fp8_raw_scaled(w, x, d_ws, d_xs)
    torch.cuda.synchronize()
    assert torch.equal(fused, raw)
    cols = np.unique(np.concatenate([np.arange(100, 164), np.random.default_rng(2).integers(0, spec["rows"], 300),
                                     np.arange(spec["rows"] - 16, spec["rows"])]))
    wh = w.cpu().numpy()
    # the oracle on the sampled rows of W: their scale rows are those of the rows' own blocks
    yref = np.zeros((M, len(cols)))
    mag = np.zeros((M, len(cols)))
    for j, n in enumerate(cols):
        yj, aj = orc.gemm_ref_scaled(x.cpu().numpy(), wh[n:n + 1], ws[n // 128:n // 128 + 1], xs)
        yref[:, j], mag[:, j] = yj[:, 0], aj[:, 0]
    _check(fused.cpu().numpy()[:, cols], yref, mag, "config4 scaled")
    with pytest.raises(ecf8.Ecf8Error):
        ecf8.ecf8_gemm_fp8_scaled(blob.header, d_blob, x, d_ws[:, :31].contiguous())      # scale table of the wrong shape
    with pytest.raises(ecf8.Ecf8Error):
        ecf8.ecf8_gemm_fp8_scaled(blob.header, d_blob, x, d_ws, d_xs[:5].contiguous())
    with pytest.raises(ecf8.Ecf8Error):
        ecf8.ecf8_gemm_fp8_scaled(blob.header, d_blob, x, d_ws.double())


@pytest.mark.parametrize("M", [1, 16, 17, 33, 64])
@pytest.mark.parametrize("rows,K", [(48, 256), (32, 512), (128, 2048), (64, 5120), (48, 7168), (80, 14336)])
def test_any_k_against_oracle(orc, rows, K, M):
    """K other than 4096 (any multiple of 256): fewer chunks than waves (K = 256 .. 2048), an uneven deal
    (K = 5120: 20 chunks over 16 waves; K = 14336: 56), the down-projection's K = 14336."""
    w = synth.make_weight(rows, K, 1.7, 0.02, 7).numpy()
    x = synth.activations(M, K, seed=200 + M).numpy()
    yref, mag = orc.gemm_ref(x, w)
    blob = ecf8.ecf8_encode(w, rows, K, lane_syms=64, tile_rows=16)
    d_x, d_w = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
    guard = torch.full((M + 2, rows), float("nan"), dtype=torch.float32, device=DEV)
    print("any K: rows", rows, "K", K, "M", M, flush=True)
    y = ecf8.ecf8_gemm_fp8(blob.header, blob.to(DEV), d_x, guard[1:M + 1])
    raw = ecf8.ecf8_gemm_fp8_raw(d_w, d_x)
    torch.cuda.synchronize()
    assert torch.isnan(guard[0]).all() and torch.isnan(guard[M + 1]).all()
    _check(y.cpu().numpy(), yref, mag, "any-K fused %dx%d M=%d" % (rows, K, M))
    assert torch.equal(raw, y)
    y = ecf8.ecf8_gemm_fp8_exact(blob.header, blob.to(DEV), d_x)
    raw = ecf8.ecf8_gemm_fp8_raw_exact(d_w, d_x)
    torch.cuda.synchronize()
    _check(y.cpu().numpy(), yref, mag, "any-K exact %dx%d M=%d" % (rows, K, M), rel=EXACT)
    assert torch.equal(raw, y)
    # operands whose products and sums are exact in fp32 whatever the order and alignment (values 0, +-0.5, +-1,
    # +-2): the result must equal the reference exactly
    rng = np.random.default_rng(K + M)
    vals = np.array([0x00, 0x30, 0xB0, 0x38, 0xB8, 0x40, 0xC0], dtype=np.uint8)
    w2 = vals[rng.integers(0, len(vals), size=(rows, K))]
    x2 = vals[rng.integers(0, len(vals), size=(M, K))]
    yref2, _ = orc.gemm_ref(x2, w2)
    blob2 = ecf8.ecf8_encode(w2, rows, K, lane_syms=64, tile_rows=16)
    y2 = ecf8.ecf8_gemm_fp8(blob2.header, blob2.to(DEV), torch.from_numpy(x2).to(DEV))
    torch.cuda.synchronize()
    assert np.array_equal(y2.cpu().numpy().astype(np.float64), yref2)


@pytest.mark.parametrize("M", [3, 40])
def test_any_k_block_scaled_and_full_size(orc, M):
    """The down projection of the 8B-class stack (4096 x 14336) with block scales: fused equals the twin on
    uncompressed weights bit for bit; sampled outputs against the oracle."""
    rows, K = 4096, 14336
    w = synth.make_weight(rows, K, 1.8, 0.02, 8, device=DEV)
    x = synth.activations(M, K, seed=300 + M, device=DEV)
    rng = np.random.default_rng(M)
    ws = np.exp(rng.normal(0.0, 0.7, size=(rows // 128, K // 128))).astype(np.float32)
    xs = np.exp(rng.normal(0.0, 0.5, size=(M, K // 128))).astype(np.float32)      # activations quantised in 1 x 128 groups
    d_ws, d_xs = torch.from_numpy(ws).to(DEV), torch.from_numpy(xs).to(DEV)
    blob = ecf8.ecf8_encode(w.cpu(), rows, K, lane_syms=64, tile_rows=16)
    d_blob = blob.to(DEV)
    fused = ecf8.ecf8_gemm_fp8_scaled(blob.header, d_blob, x, d_ws, d_xs)
    raw = ecf8.ecf8_gemm_fp8_raw_scaled(w, x, d_ws, d_xs)
    plain = ecf8.ecf8_gemm_fp8(blob.header, d_blob, x)
    plain_raw = ecf8.ecf8_gemm_fp8_raw(w, x)
    torch.cuda.synchronize()
    assert torch.equal(fused, raw) and torch.equal(plain, plain_raw)
    cols = np.unique(np.concatenate([np.arange(0, 20), rng.integers(0, rows, 100), np.arange(rows - 16, rows)]))
    wh, xh = w.cpu().numpy(), x.cpu().numpy()
    yref, mag = orc.gemm_ref(xh, wh[cols])
    _check(plain.cpu().numpy()[:, cols], yref, mag, "down projection")
    ex = ecf8.ecf8_gemm_fp8_exact(blob.header, d_blob, x)
    ex_s = ecf8.ecf8_gemm_fp8_exact(blob.header, d_blob, x, d_ws, d_xs)
    ex_s_raw = ecf8.ecf8_gemm_fp8_raw_exact(w, x, d_ws, d_xs)
    torch.cuda.synchronize()
    assert torch.equal(ex_s, ex_s_raw)
    _check(ex.cpu().numpy()[:, cols], yref, mag, "down projection, exact", rel=EXACT)
    yref = np.zeros((M, len(cols)))
    mag = np.zeros((M, len(cols)))
    for j, n in enumerate(cols):
        yj, aj = orc.gemm_ref_scaled(xh, wh[n:n + 1], ws[n // 128:n // 128 + 1], xs)
        yref[:, j], mag[:, j] = yj[:, 0], aj[:, 0]
    _check(fused.cpu().numpy()[:, cols], yref, mag, "down projection, block scales")
    _check(ex_s.cpu().numpy()[:, cols], yref, mag, "down projection, block scales, exact", rel=EXACT)


# ---- split K ----

SPLIT_SHAPES = [(256, 14336), (576, 7168), (1024, 4096), (1536, 7168), (32, 512), (48, 5120), (16, 256)]


def _split_workspace():
    """One workspace for every split-K test, sized for the largest shape: the calls leave its counters at zero."""
    global _WS
    try:
        return _WS
    except NameError:
        n = max(ecf8._lib.ecf8_gemm_splitk_workspace_bytes(r, k, 64) for r, k in SPLIT_SHAPES)
        _WS = ecf8.gemm_splitk_workspace(1, 1, 1, DEV)          # the minimum, then one of the full size
        assert _WS.numel() == 16
        _WS = torch.full((n,), 0xA5, dtype=torch.uint8, device=DEV)
        ecf8._check("init", ecf8._lib.ecf8_gemm_splitk_workspace_init(_WS.data_ptr(), _WS.numel(), None))
        torch.cuda.synchronize()
        assert int(_WS.count_nonzero()) == 0
        return _WS


@pytest.mark.parametrize("M", [1, 16, 17, 64])
@pytest.mark.parametrize("rows,K", SPLIT_SHAPES)
def test_split_k_against_oracle(orc, rows, K, M):
    """Matrices of few rows: `slices` workgroups share a block of 16 rows.  Against the oracle, against the twin
    on uncompressed weights (bit for bit), call after call on one workspace (bit for bit: the slices are
    added in slice order whoever arrives last), with and without scales; (16, 256) and, on a chip of 256
    compute units, nothing else here falls through to the plain kernels."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    slices = ecf8.gemm_splitk_slices(rows, K)
    assert slices >= 1 and (K // 256) % slices == 0 and (slices == 1 or rows // 16 * slices <= cus)
    assert all((K // 256) % s or rows // 16 * s > cus for s in range(slices + 1, K // 256 + 1))     # the largest such
    need = ecf8._lib.ecf8_gemm_splitk_workspace_bytes(rows, K, M)
    tiles = 1 if M <= 16 else 2 if M <= 32 else 4
    assert need == (0 if slices == 1 else 4096 + rows // 16 * slices * tiles * 1024)
    wsp = _split_workspace()
    print("split K: rows", rows, "K", K, "M", M, "slices", slices, flush=True)
    w = synth.make_weight(rows, K, 1.7, 0.02, 9).numpy()
    x = synth.activations(M, K, seed=400 + M).numpy()
    blob = ecf8.ecf8_encode(w, rows, K, lane_syms=64, tile_rows=16)
    d_blob, d_x, d_w = blob.to(DEV), torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
    rel = FP8_CORE
    yref, mag = orc.gemm_ref(x, w)
    guard = torch.full((M + 2, rows), float("nan"), dtype=torch.float32, device=DEV)
    y = ecf8.ecf8_gemm_fp8_splitk(blob.header, d_blob, d_x, wsp, d_y=guard[1:M + 1])
    raw = ecf8.ecf8_gemm_fp8_raw_splitk(d_w, d_x, wsp)
    again = [ecf8.ecf8_gemm_fp8_splitk(blob.header, d_blob, d_x, wsp) for _ in range(5)]
    torch.cuda.synchronize()
    assert torch.isnan(guard[0]).all() and torch.isnan(guard[M + 1]).all()
    _check(y.cpu().numpy(), yref, mag, "split-K fused %dx%d M=%d" % (rows, K, M), rel=rel)
    assert torch.equal(raw, y) and all(torch.equal(a, y) for a in again)
    # against the plain call: the same chunk sums added in another order, a few fp32 roundings apart
    plain = ecf8.ecf8_gemm_fp8(blob.header, d_blob, d_x)
    torch.cuda.synchronize()
    _check(y.cpu().numpy(), plain.cpu().numpy().astype(np.float64), mag, "split-K against the plain call", rel=2e-6)
    n_ctr = 4096
    assert int(wsp[:n_ctr].count_nonzero()) == 0                  # counters back at zero
    # scales of W alone, with one per row of X, with one per row and 128 columns of X
    rng = np.random.default_rng(rows + M)
    ws = np.exp(rng.normal(0.0, 0.7, size=((rows + 127) // 128, K // 128))).astype(np.float32)
    xr = np.exp(rng.normal(0.0, 0.5, size=M)).astype(np.float32)
    xg = np.exp(rng.normal(0.0, 0.5, size=(M, K // 128))).astype(np.float32)
    d_ws = torch.from_numpy(ws).to(DEV)
    for xs in (None, xr, xg):
        d_xs = None if xs is None else torch.from_numpy(xs).to(DEV)
        yref, mag = orc.gemm_ref_scaled(x, w, ws, xs)
        y = ecf8.ecf8_gemm_fp8_splitk(blob.header, d_blob, d_x, wsp, d_ws, d_xs)
        raw = ecf8.ecf8_gemm_fp8_raw_splitk(d_w, d_x, wsp, d_ws, d_xs)
        torch.cuda.synchronize()
        _check(y.cpu().numpy(), yref, mag, "split-K scaled %dx%d M=%d" % (rows, K, M), rel=rel)
        assert torch.equal(raw, y)
        plain = ecf8.ecf8_gemm_fp8_scaled(blob.header, d_blob, d_x, d_ws, d_xs)
        torch.cuda.synchronize()
        _check(y.cpu().numpy(), plain.cpu().numpy().astype(np.float64), mag, "split-K scaled against the plain call", rel=2e-6)
    # operands whose products and sums are exact in fp32 in any order: equal to the reference, and to the plain call
    vals = np.array([0x00, 0x30, 0xB0, 0x38, 0xB8, 0x40, 0xC0], dtype=np.uint8)
    w2 = vals[rng.integers(0, len(vals), size=(rows, K))]
    x2 = vals[rng.integers(0, len(vals), size=(M, K))]
    yref2, _ = orc.gemm_ref(x2, w2)
    blob2 = ecf8.ecf8_encode(w2, rows, K, lane_syms=64, tile_rows=16)
    d_x2 = torch.from_numpy(x2).to(DEV)
    y2 = ecf8.ecf8_gemm_fp8_splitk(blob2.header, blob2.to(DEV), d_x2, wsp)
    plain = ecf8.ecf8_gemm_fp8(blob2.header, blob2.to(DEV), d_x2)
    torch.cuda.synchronize()
    assert np.array_equal(y2.cpu().numpy().astype(np.float64), yref2) and torch.equal(plain, y2)
    assert int(wsp[:n_ctr].count_nonzero()) == 0


def test_split_k_argument_errors():
    rows, K, M = 256, 14336, 4
    if ecf8.gemm_splitk_slices(rows, K) <= 1:
        pytest.skip("this device has too few compute units to split this shape")
    w = synth.make_weight(rows, K, 1.7, 0.02, 9).numpy()
    blob = ecf8.ecf8_encode(w, rows, K, lane_syms=64, tile_rows=16)
    d_blob, d_x = blob.to(DEV), synth.activations(M, K, seed=1).to(DEV)
    need = ecf8._lib.ecf8_gemm_splitk_workspace_bytes(rows, K, M)
    wsp = torch.zeros((need + 16,), dtype=torch.uint8, device=DEV)
    y = torch.full((M, rows), 7.0, dtype=torch.float32, device=DEV)
    for ws_arg, code in ((wsp[:need - 1], ecf8.E_CAPACITY), (wsp[1:], ecf8.E_ALIGN)):
        with pytest.raises(ecf8.Ecf8Error) as e:
            ecf8.ecf8_gemm_fp8_splitk(blob.header, d_blob, d_x, ws_arg, d_y=y)
        assert e.value.code == code
    rc = ecf8._lib.ecf8_gemm_fp8_splitk(blob.header, d_blob.data_ptr(), d_x.data_ptr(), M, None, None, 0, y.data_ptr(), None, 0, None)
    assert rc == ecf8.E_ARG
    xs = torch.ones((M,), dtype=torch.float32, device=DEV)
    with pytest.raises(ecf8.Ecf8Error):                 # scales of X without scales of W
        ecf8.ecf8_gemm_fp8_splitk(blob.header, d_blob, d_x, wsp, None, xs, d_y=y)
    assert ecf8.gemm_splitk_slices(250, K) == 0 and ecf8.gemm_splitk_slices(rows, 1000) == 0
    torch.cuda.synchronize()
    assert bool((y == 7.0).all()) and int(wsp.count_nonzero()) == 0      # nothing ran
    ecf8.ecf8_gemm_fp8_splitk(blob.header, d_blob, d_x, wsp[:need], d_y=y)   # exactly the size asked for
    torch.cuda.synchronize()
    assert bool((y != 7.0).any())


def test_split_k_calls_with_changing_inputs_share_a_workspace():
    """A long run of calls on one workspace whose inputs change from call to call (two activations, two weight
    matrices, unscaled and scaled in turn): every result equals the one the same call gave on a fresh
    workspace.  A partial sum read from an earlier call, or a counter left off zero, would show here."""
    rows, K, M = 576, 7168, 16
    if ecf8.gemm_splitk_slices(rows, K) <= 1:
        pytest.skip("this device has too few compute units to split this shape")
    ws_h = np.exp(np.random.default_rng(3).normal(0.0, 0.7, size=((rows + 127) // 128, K // 128))).astype(np.float32)
    d_ws = torch.from_numpy(ws_h).to(DEV)
    cases = []
    for i in range(2):
        w = synth.make_weight(rows, K, 1.7, 0.02, 20 + i).numpy()
        blob = ecf8.ecf8_encode(w, rows, K, lane_syms=64, tile_rows=16)
        for j in range(2):
            d_x = synth.activations(M, K, seed=500 + j).to(DEV)
            for scale in (None, d_ws):
                fresh = ecf8.gemm_splitk_workspace(rows, K, M, DEV)
                want = ecf8.ecf8_gemm_fp8_splitk(blob.header, blob.to(DEV), d_x, fresh, scale)
                cases.append((blob.header, blob.to(DEV), d_x, scale, want))
    torch.cuda.synchronize()
    assert not torch.equal(cases[0][4], cases[2][4]) and not torch.equal(cases[0][4], cases[4][4])
    wsp = ecf8.gemm_splitk_workspace(rows, K, M, DEV)
    rng = np.random.default_rng(0)
    order = rng.integers(0, len(cases), size=300)
    got = [ecf8.ecf8_gemm_fp8_splitk(cases[c][0], cases[c][1], cases[c][2], wsp, cases[c][3]) for c in order]
    torch.cuda.synchronize()
    bad = [int(k) for k, c in enumerate(order) if not torch.equal(got[k], cases[c][4])]
    assert not bad, "calls %s of 300 differ from the same call on a fresh workspace" % bad[:10]
    assert int(wsp[:4096].count_nonzero()) == 0


# ---- a group of matrices in one launch ----

def _group_members(shapes, Ms, seed, scale_mode=0, raw=False):
    members, singles = [], []
    for i, ((rows, K), M) in enumerate(zip(shapes, Ms)):
        w = synth.make_weight(rows, K, 1.7, 0.02, seed, tensor_id=i).numpy()
        x = synth.activations(M, K, seed=seed + 31 * i).numpy()
        rng = np.random.default_rng(seed + i)
        ws = np.exp(rng.normal(0.0, 0.7, size=((rows + 127) // 128, K // 128))).astype(np.float32)
        xs = (np.exp(rng.normal(0.0, 0.5, size=M)) if scale_mode == 1 else np.exp(rng.normal(0.0, 0.5, size=(M, K // 128)))).astype(np.float32)
        m = {"x": torch.from_numpy(x).to(DEV), "host": (x, w, ws, xs)}
        if scale_mode:
            m["w_scale"], m["x_scale"] = torch.from_numpy(ws).to(DEV), torch.from_numpy(xs).to(DEV)
        if raw:
            m["w"] = torch.from_numpy(w).to(DEV)
        else:
            blob = ecf8.ecf8_encode(w, rows, K, lane_syms=64, tile_rows=16, table_mode=1 + i % 2)   # with and without a table
            m["hdr"], m["blob"] = blob.header, blob.to(DEV)
        members.append(m)
    return members


def _single_call(m):
    if "hdr" in m:
        if "w_scale" in m:
            return ecf8.ecf8_gemm_fp8_scaled(m["hdr"], m["blob"], m["x"], m["w_scale"], m["x_scale"])
        return ecf8.ecf8_gemm_fp8(m["hdr"], m["blob"], m["x"])
    if "w_scale" in m:
        return ecf8.ecf8_gemm_fp8_raw_scaled(m["w"], m["x"], m["w_scale"], m["x_scale"])
    return ecf8.ecf8_gemm_fp8_raw(m["w"], m["x"])


GROUPS = {
    "experts": ([(128, 1792), (128, 1792), (448, 512), (128, 1792), (448, 512), (64, 7168)], [3, 16, 1, 9, 16, 2]),
    "one": ([(208, 4096)], [7]),
    "many_tiny": ([(16, 256)] * 37 + [(32, 512)] * 5, [1 + (i * 7) % 16 for i in range(42)]),
    "tall_M": ([(96, 2048), (48, 5120), (256, 4096)], [33, 64, 17]),
    "mid_M": ([(96, 2048), (48, 5120), (160, 1024)], [32, 5, 20]),
}


@pytest.mark.parametrize("scale_mode", [0, 1, 2])
@pytest.mark.parametrize("name", sorted(GROUPS))
def test_grouped_gemm_equals_the_single_calls(orc, name, scale_mode):
    """A group on compressed weights equals the same group on uncompressed weights bit for bit, launch after
    launch.  Every product equals its single call bit for bit where that call runs the any-K kernels with
    workgroups of the group's shape (K != 4096, and M on the same side of 16 as the group's largest M: the
    same blocks computed the same way, only by other workgroups) and to a few fp32 roundings otherwise (the
    same chunk sums added in another order).  Rows outside M stay untouched; one product of each group is
    checked against the oracle as well."""
    shapes, Ms = GROUPS[name]
    members = _group_members(shapes, Ms, seed=11, scale_mode=scale_mode)
    twins = _group_members(shapes, Ms, seed=11, scale_mode=scale_mode, raw=True)
    guards = []
    for m, (rows, K), M in zip(members, shapes, Ms):
        g = torch.full((M + 2, rows), float("nan"), dtype=torch.float32, device=DEV)
        m["y"] = g[1:M + 1]
        guards.append(g)
    print("group", name, "scales", scale_mode, flush=True)
    group, twin = ecf8.GemmGroup(members), ecf8.GemmGroup(twins)
    assert group.info.n_items == len(shapes) and group.info.max_M == max(Ms) and group.info.raw == 0 and twin.info.raw == 1
    assert group.info.total_work == sum(r // 16 * (k // 256) for r, k in shapes) == twin.info.total_work
    ys = [y.clone() for y in ecf8.ecf8_gemm_fp8_grouped(group)]
    want = [_single_call(m) for m in members]
    again = ecf8.ecf8_gemm_fp8_grouped(group)
    raw = ecf8.ecf8_gemm_fp8_grouped(twin)
    torch.cuda.synchronize()
    for i, (y, w_, g) in enumerate(zip(ys, want, guards)):
        assert torch.isnan(g[0]).all() and torch.isnan(g[-1]).all(), i
        assert torch.equal(y, again[i]) and torch.equal(y, raw[i]), i
        if shapes[i][1] != 4096 and (Ms[i] <= 16) == (max(Ms) <= 16):
            assert torch.equal(y, w_), "member %d of %s" % (i, name)
        else:
            x, w, ws, xs = members[i]["host"]
            _, mag = orc.gemm_ref_scaled(x, w, ws, xs) if scale_mode else orc.gemm_ref(x, w)
            _check(y.cpu().numpy(), w_.cpu().numpy().astype(np.float64), mag, "member %d of %s against its single call" % (i, name), rel=2e-6)
    x, w, ws, xs = members[-1]["host"]
    yref, mag = orc.gemm_ref_scaled(x, w, ws, xs) if scale_mode else orc.gemm_ref(x, w)
    _check(ys[-1].cpu().numpy(), yref, mag, "grouped, last member")


def test_grouped_gemm_argument_errors():
    shapes, Ms = GROUPS["mid_M"]
    fused = _group_members(shapes, Ms, seed=3)
    rawm = _group_members(shapes, Ms, seed=3, raw=True)
    scaled = _group_members(shapes, Ms, seed=3, scale_mode=1)
    for bad in ([fused[0], rawm[1]], [fused[0], scaled[1]], [scaled[0], _group_members(shapes, Ms, seed=3, scale_mode=2)[1]]):
        with pytest.raises(ecf8.Ecf8Error) as e:
            ecf8.GemmGroup(bad)
        assert e.value.code == ecf8.E_ARG
    lin = ecf8.ecf8_encode(synth.make_weight(64, 512, 1.7, 0.02, 1).numpy())           # not row-tiled
    with pytest.raises(ecf8.Ecf8Error):
        ecf8.GemmGroup([{"hdr": lin.header, "blob": lin.to(DEV), "x": fused[0]["x"][:, :512].contiguous()}])
    group = ecf8.GemmGroup(fused)
    info = ecf8.GemmGroupInfo.from_buffer_copy(group.info)
    info.max_M = 65
    assert ecf8._lib.ecf8_gemm_fp8_grouped(group.d_items.data_ptr(), info, None) == ecf8.E_ARG
    assert ecf8._lib.ecf8_gemm_fp8_grouped(None, group.info, None) == ecf8.E_ARG
    assert ecf8._lib.ecf8_gemm_fp8_grouped(group.d_items.data_ptr() + 4, group.info, None) == ecf8.E_ALIGN
    assert ecf8._lib.ecf8_gemm_group_prepare(None, 1, None, None) == ecf8.E_ARG


def test_gemm_calls_replay_from_a_hip_graph():
    """The GEMM calls allocate nothing, synchronise nothing and clear nothing with memsets (the split-K counters
    are put back to zero by the kernel itself), so a decoding loop may capture them into a HIP graph: a plain, a
    scaled, a split-K and a grouped call are captured once and replayed three times with new activations
    written into the same buffers and eager calls in between; every replay equals the eager result."""
    rows, K, M = 576, 7168, 8
    w = synth.make_weight(rows, K, 1.7, 0.02, 41).numpy()
    blob = ecf8.ecf8_encode(w, rows, K, lane_syms=64, tile_rows=16)
    d_blob = blob.to(DEV)
    ws = torch.from_numpy(np.exp(np.random.default_rng(2).normal(0.0, 0.7, size=((rows + 127) // 128, K // 128))).astype(np.float32)).to(DEV)
    x = synth.activations(M, K, seed=600).to(DEV)
    wsp = ecf8.gemm_splitk_workspace(rows, K, M, DEV)
    shapes, Ms = GROUPS["experts"]
    members = _group_members(shapes, Ms, seed=17)
    group = ecf8.GemmGroup(members)
    y_plain = torch.empty((M, rows), dtype=torch.float32, device=DEV)
    y_scaled, y_split = torch.empty_like(y_plain), torch.empty_like(y_plain)

    def run(s):
        ecf8.ecf8_gemm_fp8(blob.header, d_blob, x, y_plain, stream=s)
        ecf8.ecf8_gemm_fp8_scaled(blob.header, d_blob, x, ws, None, y_scaled, stream=s)
        ecf8.ecf8_gemm_fp8_splitk(blob.header, d_blob, x, wsp, d_y=y_split, stream=s)
        ecf8.ecf8_gemm_fp8_grouped(group, stream=s)

    def results():
        return [y_plain.clone(), y_scaled.clone(), y_split.clone()] + [y.clone() for y in group.y]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):            # warm-up outside the capture
        run(side)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run(torch.cuda.current_stream())
    for rep in range(3):
        x.copy_(synth.activations(M, K, seed=601 + rep).to(DEV))
        for i, m in enumerate(members):
            m["x"].copy_(synth.activations(m["x"].shape[0], m["x"].shape[1], seed=700 + 10 * rep + i).to(DEV))
        torch.cuda.synchronize()
        run(None)                            # eager, on the new activations
        torch.cuda.synchronize()
        want = results()
        for t in [y_plain, y_scaled, y_split] + group.y:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = results()
        assert all(torch.equal(p, q) for p, q in zip(got, want)), rep
        assert int(wsp[:4096].count_nonzero()) == 0
        if rep:
            assert not torch.equal(want[0], first[0])
        first = want

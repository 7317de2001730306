"""Pins of the oracle's FP8 GEMM reference (no product code involved)."""
import numpy as np
import torch


def test_e4m3_values_match_the_library_conversion_and_landmarks(orc):
    got = np.array([orc.e4m3_to_double(b) for b in range(256)])
    lib = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    nan = np.isnan(lib)
    assert list(np.nonzero(nan)[0]) == [0x7F, 0xFF] and np.isnan(got[nan]).all()
    assert np.array_equal(got[~nan], lib[~nan])
    # landmarks of the OCP format: largest finite 448, smallest normal 2^-6, subnormal step 2^-9, signed zero
    assert got[0x7E] == 448.0 and got[0xFE] == -448.0
    assert got[0x08] == 2.0 ** -6 and got[0x01] == 2.0 ** -9 and got[0x07] == 7 * 2.0 ** -9
    assert got[0x38] == 1.0 and got[0x3C] == 1.5
    assert got[0x00] == 0.0 and got[0x80] == 0.0 and np.signbit(got[0x80])


def test_gemm_against_float64_matmul_and_hand_case(orc):
    rng = np.random.default_rng(0)
    X = rng.integers(0, 256, size=(5, 300), dtype=np.uint8)
    W = rng.integers(0, 256, size=(7, 300), dtype=np.uint8)
    X[(X & 0x7F) == 0x7F] = 0x38
    W[(W & 0x7F) == 0x7F] = 0xB8
    xf = torch.from_numpy(X).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    wf = torch.from_numpy(W).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    Y, A = orc.gemm_ref(X, W)
    assert np.allclose(Y, xf @ wf.T, rtol=1e-13, atol=0)
    assert np.allclose(A, np.abs(xf) @ np.abs(wf).T, rtol=1e-13, atol=0)
    # by hand: x = (1, 1.5, -448), w = (2, -1, 2^-6) -> 2 - 1.5 - 7 = -6.5 ; magnitudes 2 + 1.5 + 7 = 10.5
    x = np.array([[0x38, 0x3C, 0xFE]], dtype=np.uint8)
    w = np.array([[0x40, 0xB8, 0x08]], dtype=np.uint8)
    Y, A = orc.gemm_ref(x, w)
    assert Y[0, 0] == -6.5 and A[0, 0] == 10.5
    # transposed operands must not give the same answer: W is indexed [n][k]
    W2 = rng.integers(0, 120, size=(3, 4), dtype=np.uint8)
    X2 = rng.integers(0, 120, size=(2, 4), dtype=np.uint8)
    Y2, _ = orc.gemm_ref(X2, W2)
    assert Y2.shape == (2, 3)


def test_scaled_gemm_against_dequantised_float64_matmul(orc):
    """Block scales of W (128 x 128) and row scales of X: the reference equals the plain float64 product of
    the dequantised matrices, written here with numpy broadcasting instead of the oracle's loops."""
    rng = np.random.default_rng(1)
    M, N, K = 3, 200, 384                     # two scale rows (the second ragged), three scale columns
    X = rng.integers(0, 0x78, size=(M, K), dtype=np.uint8)
    W = (rng.integers(0, 0x78, size=(N, K)) | (rng.integers(0, 2, size=(N, K)) << 7)).astype(np.uint8)
    ws = rng.uniform(0.5, 2.0, size=(2, 3)).astype(np.float32)
    xs = rng.uniform(0.1, 3.0, size=M).astype(np.float32)
    xf = torch.from_numpy(X).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    wf = torch.from_numpy(W).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    wdq = wf * np.repeat(np.repeat(ws.astype(np.float64), 128, axis=0), 128, axis=1)[:N, :K]
    xdq = xf * xs.astype(np.float64)[:, None]
    Y, A = orc.gemm_ref_scaled(X, W, ws, xs)
    assert np.allclose(Y, xdq @ wdq.T, rtol=1e-12, atol=0)
    assert np.allclose(A, np.abs(xdq) @ np.abs(wdq).T, rtol=1e-12, atol=0)
    # one scale per row of X and 128 columns
    xg = rng.uniform(0.1, 3.0, size=(M, 3)).astype(np.float32)
    xdg = xf * np.repeat(xg.astype(np.float64), 128, axis=1)[:, :K]
    Yg, Ag = orc.gemm_ref_scaled(X, W, ws, xg)
    mag = np.abs(xdg) @ np.abs(wdq).T                       # sums cancel: compare against the sum of magnitudes
    assert np.all(np.abs(Yg - xdg @ wdq.T) <= 1e-13 * mag) and np.allclose(Ag, mag, rtol=1e-12, atol=0)
    assert not np.allclose(Yg, Y)
    # no row scales = ones; unit scales = the unscaled reference, exactly
    Y1, _ = orc.gemm_ref_scaled(X, W, ws)
    assert np.allclose(Y1, xf @ wdq.T, rtol=1e-12, atol=0)
    Yu, Au = orc.gemm_ref_scaled(X, W, np.ones((2, 3), dtype=np.float32), np.ones(M, dtype=np.float32))
    Y0, A0 = orc.gemm_ref(X, W)
    assert np.array_equal(Yu, Y0) and np.array_equal(Au, A0)
    # by hand: K = 256, x = 1 everywhere, w = 1 everywhere, scales 2 and 0.5 for the two halves of K, row scale 3
    x = np.full((1, 256), 0x38, dtype=np.uint8)
    w = np.full((1, 256), 0x38, dtype=np.uint8)
    Yh, Ah = orc.gemm_ref_scaled(x, w, np.array([[2.0, 0.5]], dtype=np.float32), np.array([3.0], dtype=np.float32))
    assert Yh[0, 0] == 3.0 * (128 * 2.0 + 128 * 0.5) and Ah[0, 0] == Yh[0, 0]
    # a scale belongs to the block of ROWS n/128 and of COLUMNS k/128, not the other way round
    ws2 = np.array([[1.0, 1.0, 1.0], [5.0, 1.0, 1.0]], dtype=np.float32)
    Y2, _ = orc.gemm_ref_scaled(X, W, ws2)
    Yb, _ = orc.gemm_ref_scaled(X, W, np.ones((2, 3), dtype=np.float32))
    assert np.array_equal(Y2[:, :128], Yb[:, :128]) and not np.array_equal(Y2[:, 128:], Yb[:, 128:])

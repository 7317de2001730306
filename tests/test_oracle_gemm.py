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

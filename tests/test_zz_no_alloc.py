"""ecf8_gemm_fp8_splitk_static (the split-K call whose workspace lives inside the library, for callers that
cannot allocate) against ecf8_gemm_fp8_splitk with a caller workspace: bit for bit, through the C ABI, on two
calls in a row, the second with a smaller input, then with scales and across shapes."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2510_02676_amd import ecf8, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(rows, K, M, seed):
    w = synth.make_weight(rows, K, 1.7, 0.02, seed).numpy()
    blob = ecf8.ecf8_encode(w, rows, K, lane_syms=64, tile_rows=16)
    x = synth.activations(M, K, seed=seed + 1).to(DEV)
    return blob.header, blob.to(DEV), x


def _static(hdr, d_blob, x, ws=None, xs=None, xc=0):
    M = x.shape[0]
    y = torch.full((M + 2, hdr.rows), float("nan"), dtype=torch.float32, device=DEV)
    rc = ecf8._lib.ecf8_gemm_fp8_splitk_static(ctypes.byref(hdr), d_blob.data_ptr(), x.data_ptr(), M,
                                               None if ws is None else ws.data_ptr(), None if xs is None else xs.data_ptr(), xc,
                                               y[1:].data_ptr(), None)
    assert rc == ecf8.OK, rc
    return y


def test_static_scratch_equals_the_workspace_call_twice_in_a_row():
    big = _case(576, 7168, 64, 1)          # 36 blocks x 7 slices, four tiles of partial sums
    small = _case(64, 2048, 3, 2)          # 4 blocks x 8 slices, one tile: a smaller input right after
    print("static split-K: 576x7168 M=64, then 64x2048 M=3", flush=True)
    got_big = _static(*big)
    got_small = _static(*small)
    torch.cuda.synchronize()
    for (hdr, d_blob, x), got in ((big, got_big), (small, got_small)):
        M = x.shape[0]
        assert ecf8.gemm_splitk_slices(hdr.rows, hdr.cols) > 1
        want = ecf8.ecf8_gemm_fp8_splitk(hdr, d_blob, x, ecf8.gemm_splitk_workspace(hdr.rows, hdr.cols, M, DEV))
        torch.cuda.synchronize()
        assert torch.equal(got[1:M + 1], want)
        assert torch.isnan(got[0]).all() and torch.isnan(got[M + 1]).all()
    # and again in the other order, with scales, on the same array
    ws = torch.from_numpy(np.exp(np.random.default_rng(0).normal(0, 0.7, size=(5, 56))).astype(np.float32)).to(DEV)
    xs = torch.from_numpy(np.exp(np.random.default_rng(1).normal(0, 0.5, size=(64,))).astype(np.float32)).to(DEV)
    again_small = _static(*small)
    scaled = _static(*big, ws=ws, xs=xs, xc=1)
    torch.cuda.synchronize()
    assert torch.equal(again_small[1:4], got_small[1:4])       # rows 0 and 4 are NaN guards
    hdr, d_blob, x = big
    want = ecf8.ecf8_gemm_fp8_splitk(hdr, d_blob, x, ecf8.gemm_splitk_workspace(hdr.rows, hdr.cols, 64, DEV), ws, xs)
    torch.cuda.synchronize()
    assert torch.equal(scaled[1:65], want)


def test_static_scratch_shapes_that_do_not_split_and_argument_errors():
    hdr, d_blob, x = _case(4096, 256, 5, 3)     # blocks enough: falls through to the plain kernels, like the workspace call
    got = _static(hdr, d_blob, x)
    want = ecf8.ecf8_gemm_fp8(hdr, d_blob, x)
    torch.cuda.synchronize()
    assert torch.equal(got[1:6], want)
    y = torch.zeros((5, 4096), dtype=torch.float32, device=DEV)
    rc = ecf8._lib.ecf8_gemm_fp8_splitk_static(ctypes.byref(hdr), d_blob.data_ptr(), x.data_ptr(), 65, None, None, 0, y.data_ptr(), None)
    assert rc == ecf8.E_ARG
    rc = ecf8._lib.ecf8_gemm_fp8_splitk_static(ctypes.byref(hdr), None, x.data_ptr(), 5, None, None, 0, y.data_ptr(), None)
    assert rc == ecf8.E_ARG

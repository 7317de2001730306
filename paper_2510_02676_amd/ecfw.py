"""Thin Python binding of the wide-alphabet calls (``include/ecfw.h``): E5M2 and BF16.

Argument marshalling only; every step of the decode path runs inside ``libecf8.so``
(importing this module fails loudly when the library is not built).
"""
import ctypes

import numpy as np
import torch

from . import ecf8 as _e

_lib = _e._lib
FMT_E5M2, FMT_BF16 = 1, 2
ELEM_BYTES = {FMT_E5M2: 1, FMT_BF16: 2}


class WHeader(ctypes.Structure):
    """struct ecfw_header: the first 256 bytes of a wide-alphabet blob."""
    _fields_ = [("magic", ctypes.c_uint32), ("version", ctypes.c_uint32),
                ("total_size", ctypes.c_uint64), ("n_elem", ctypes.c_uint64),
                ("rows", ctypes.c_uint64), ("cols", ctypes.c_uint64),
                ("fmt", ctypes.c_uint32), ("lane_syms", ctypes.c_uint32),
                ("group_chunks", ctypes.c_uint32), ("max_code_len", ctypes.c_uint32),
                ("n_alphabet", ctypes.c_uint32), ("n_symbols", ctypes.c_uint32),
                ("n_chunks", ctypes.c_uint64), ("stream_bits", ctypes.c_uint64),
                ("off_code_len", ctypes.c_uint64), ("off_freq", ctypes.c_uint64),
                ("off_chunk_bit", ctypes.c_uint64), ("off_lane_bits", ctypes.c_uint64),
                ("off_stream", ctypes.c_uint64), ("off_plane", ctypes.c_uint64), ("off_sign", ctypes.c_uint64),
                ("stream_bytes", ctypes.c_uint64), ("plane_bytes", ctypes.c_uint64), ("sign_bytes", ctypes.c_uint64),
                ("reserved", ctypes.c_uint8 * 96)]


class WEncodeOpts(ctypes.Structure):
    _fields_ = [("fmt", ctypes.c_uint32), ("lane_syms", ctypes.c_uint32), ("n_threads", ctypes.c_uint32),
                ("group_chunks", ctypes.c_uint32), ("max_code_len", ctypes.c_uint32),
                ("reserved", ctypes.c_uint32 * 3)]


assert ctypes.sizeof(WHeader) == 256

_vp, _u64, _u32 = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32
_lib.ecfw_encode.argtypes = [_vp, _u64, _u64, ctypes.POINTER(WEncodeOpts), ctypes.POINTER(_vp)]
_lib.ecfw_encode_bound.argtypes = [_u64, _u64, ctypes.POINTER(WEncodeOpts), ctypes.POINTER(_u64)]
_lib.ecfw_encode_gpu.argtypes = [_vp, _u64, _u64, ctypes.POINTER(WEncodeOpts), _vp, _u64, ctypes.POINTER(WHeader), _vp]
_lib.ecfw_blob_describe.argtypes = [_vp, _u64, ctypes.POINTER(WHeader)]
_lib.ecfw_blob_validate.argtypes = [_vp, _u64]
_lib.ecfw_decode.argtypes = [_vp, ctypes.POINTER(WHeader), _vp, _u64, _u32, _vp]


def _host_elems(fmt, x):
    if isinstance(x, torch.Tensor):
        x = x.cpu().contiguous()
        x = x.view(torch.uint8).numpy() if fmt == FMT_E5M2 else x.view(torch.int16).numpy().view(np.uint16)
    x = np.ascontiguousarray(x)
    want = np.uint8 if fmt == FMT_E5M2 else np.uint16
    if x.dtype != want:
        raise TypeError("expected raw %s bit patterns" % ("E5M2 (uint8)" if fmt == FMT_E5M2 else "BF16 (uint16)"))
    return x


class WBlob:
    """Host object owning one encoded wide-alphabet container."""

    def __init__(self, handle):
        self._h = handle
        self.size = int(_lib.ecf8_blob_size(handle))
        self._ptr = _lib.ecf8_blob_data(handle)
        self.header = blob_describe(self._ptr, self.size)

    def numpy(self):
        buf = (ctypes.c_uint8 * self.size).from_address(self._ptr)
        buf._owner = self
        return np.frombuffer(buf, dtype=np.uint8)

    def to(self, device):
        return torch.from_numpy(self.numpy()).to(device)

    def code_len(self):
        h = self.header
        return self.numpy()[h.off_code_len:h.off_code_len + h.n_alphabet].copy()

    def __del__(self, _free=_lib.ecf8_blob_free):
        if getattr(self, "_h", None):
            _free(self._h)
            self._h = None


def ecfw_encode(fmt, x, rows=None, cols=None, lane_syms=0, n_threads=0, group_chunks=0, max_code_len=0):
    """CPU encoder: raw E5M2 bytes / BF16 words (host tensor or array) -> WBlob."""
    if fmt not in ELEM_BYTES:
        raise _e.Ecf8Error("ecfw_encode", _e.E_ARG)
    x = _host_elems(fmt, x)
    if rows is None:
        rows, cols = (x.shape if x.ndim == 2 else (1, x.size))
    if rows * cols != x.size:
        raise _e.Ecf8Error("ecfw_encode", _e.E_ARG)
    opts = WEncodeOpts(fmt, lane_syms, n_threads, group_chunks, max_code_len)
    h = _vp()
    _e._check("ecfw_encode", _lib.ecfw_encode(x.ctypes.data, rows, cols, ctypes.byref(opts), ctypes.byref(h)))
    return WBlob(h)


def ecfw_encode_gpu(fmt, d_x, rows=None, cols=None, lane_syms=0, group_chunks=0, max_code_len=0, d_blob=None, stream=None):
    """GPU encoder: device tensor of raw E5M2 bytes (uint8) or BF16 words (bfloat16 / int16) -> (WHeader, uint8
    device tensor holding the blob).  Same options and same bytes as ecfw_encode."""
    if rows is None:
        rows, cols = (d_x.shape if d_x.dim() == 2 else (1, d_x.numel()))
    if (fmt not in ELEM_BYTES or rows * cols != d_x.numel() or d_x.element_size() != ELEM_BYTES[fmt]
            or not d_x.is_contiguous() or d_x.device.type != "cuda"):
        raise _e.Ecf8Error("ecfw_encode_gpu", _e.E_ARG)
    opts = WEncodeOpts(fmt, lane_syms, 0, group_chunks, max_code_len)
    if d_blob is None:
        bound = _u64(0)
        _e._check("ecfw_encode_bound", _lib.ecfw_encode_bound(rows, cols, ctypes.byref(opts), ctypes.byref(bound)))
        d_blob = torch.empty(int(bound.value), dtype=torch.uint8, device=d_x.device)
    hdr = WHeader()
    _e._check("ecfw_encode_gpu", _lib.ecfw_encode_gpu(d_x.data_ptr(), rows, cols, ctypes.byref(opts), d_blob.data_ptr(),
                                                      d_blob.numel(), ctypes.byref(hdr), _e._stream_ptr(stream)))
    return hdr, d_blob[:hdr.total_size]


def blob_describe(ptr_or_array, size=None):
    if isinstance(ptr_or_array, np.ndarray):
        size = ptr_or_array.size
        ptr_or_array = ptr_or_array.ctypes.data
    hdr = WHeader()
    _e._check("ecfw_blob_describe", _lib.ecfw_blob_describe(ptr_or_array, size, ctypes.byref(hdr)))
    return hdr


def blob_validate(arr):
    arr = np.ascontiguousarray(arr, dtype=np.uint8)
    _e._check("ecfw_blob_validate", _lib.ecfw_blob_validate(arr.ctypes.data, arr.size))


def ecfw_decode(d_blob, hdr, d_out=None, max_workgroups=0, stream=None):
    """GPU decoder: uint8 device tensor holding the blob -> uint8 (E5M2) / int16-viewed-as-bfloat16 (BF16) tensor.
    d_out, when given, is a contiguous device tensor of at least n_elem elements' bytes."""
    if d_blob.device.type != "cuda":
        raise _e.Ecf8Error("ecfw_decode", _e.E_ARG)
    if d_out is None:
        d_out = torch.empty(hdr.n_elem, dtype=torch.uint8 if hdr.fmt == FMT_E5M2 else torch.bfloat16, device=d_blob.device)
    _e._check("ecfw_decode", _lib.ecfw_decode(d_blob.data_ptr(), ctypes.byref(hdr), d_out.data_ptr(),
                                              d_out.numel() * d_out.element_size(), max_workgroups,
                                              _e._stream_ptr(stream)))
    return d_out


class WBatchItem(ctypes.Structure):
    _fields_ = [("d_blob", _u64), ("d_out", _u64), ("n_elem", _u64), ("n_chunks", _u64), ("first_chunk", _u64),
                ("stream_bytes", _u64), ("off_code_len", _u64), ("off_chunk_bit", _u64), ("off_lane_bits", _u64),
                ("off_stream", _u64), ("off_plane", _u64), ("off_sign", _u64), ("group_chunks", _u64),
                ("reserved", _u64 * 3)]


class WBatchInfo(ctypes.Structure):
    _fields_ = [("total_chunks", _u64), ("fmt", _u32), ("lane_syms", _u32), ("max_code_len", _u32),
                ("max_workgroups", _u32), ("reserved", _u64)]


assert ctypes.sizeof(WBatchItem) == 128 and ctypes.sizeof(WBatchInfo) == 32
_lib.ecfw_batch_prepare.argtypes = [ctypes.POINTER(WHeader), ctypes.POINTER(_vp), ctypes.POINTER(_vp),
                                    ctypes.POINTER(_u64), _u32, ctypes.POINTER(WBatchItem), ctypes.POINTER(WBatchInfo)]
_lib.ecfw_decode_batched.argtypes = [_vp, _u32, ctypes.POINTER(WBatchInfo), _vp]


_lib.ecfw_jit_layer_prepare.argtypes = [_vp, _u32, ctypes.POINTER(WHeader), ctypes.POINTER(_vp), _u32,
                                        ctypes.POINTER(WBatchItem), ctypes.POINTER(_u64)]
_lib.ecfw_jit_layer_commit.argtypes = [_vp, _u32, _vp]


class WBatch:
    """Device-resident item table for ecfw_decode_batched (built once, reused)."""

    def __init__(self, hdrs, d_blobs, d_outs):
        n = len(hdrs)
        H = (WHeader * n)(*hdrs)
        B = (_vp * n)(*[t.data_ptr() for t in d_blobs])
        O = (_vp * n)(*[t.data_ptr() for t in d_outs])
        C = (_u64 * n)(*[t.numel() * t.element_size() for t in d_outs])
        items = (WBatchItem * n)()
        self.info = WBatchInfo()
        _e._check("ecfw_batch_prepare", _lib.ecfw_batch_prepare(H, B, O, C, n, items, ctypes.byref(self.info)))
        self.d_items = torch.from_numpy(np.frombuffer(items, dtype=np.uint8).copy()).to(d_blobs[0].device)
        self.n = n
        self._keep = (list(d_blobs), list(d_outs))


def ecfw_decode_batched(batch, stream=None):
    _e._check("ecfw_decode_batched", _lib.ecfw_decode_batched(batch.d_items.data_ptr(), batch.n,
                                                              ctypes.byref(batch.info), _e._stream_ptr(stream)))

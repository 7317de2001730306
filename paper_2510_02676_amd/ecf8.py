"""Thin Python binding of the ECF8 C-ABI library (argument marshalling only).

Names follow ``include/ecf8.h``.  PyTorch appears here only as the owner of
device memory and of the current HIP stream; every step of the decode path
runs inside ``libecf8.so``.  Importing this module fails loudly when the
library has not been built (``python -m paper_2510_02676_amd.build``).
"""
import ctypes
import os

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libecf8.so")

if not os.path.exists(LIB_PATH):
    raise ImportError("libecf8.so is not built: run `python -m paper_2510_02676_amd.build` "
                      "(or __graft_entry__.build()) first; there is no fallback path")
_lib = ctypes.CDLL(LIB_PATH)

OK, E_ARG, E_FORMAT, E_CAPACITY, E_ALIGN, E_HIP, E_NOMEM = 0, -1, -2, -3, -4, -5, -6


class Header(ctypes.Structure):
    """struct ecf8_header: the first 256 bytes of a blob."""
    _fields_ = [("magic", ctypes.c_uint32), ("version", ctypes.c_uint32),
                ("total_size", ctypes.c_uint64), ("n_elem", ctypes.c_uint64),
                ("rows", ctypes.c_uint64), ("cols", ctypes.c_uint64),
                ("lane_syms", ctypes.c_uint32), ("table_bits", ctypes.c_uint16), ("group_chunks", ctypes.c_uint8), ("tile_rows", ctypes.c_uint8),
                ("n_chunks", ctypes.c_uint64), ("stream_bits", ctypes.c_uint64),
                ("code_len", ctypes.c_uint8 * 16),
                ("off_chunk_bit", ctypes.c_uint64), ("off_lane_bits", ctypes.c_uint64),
                ("off_stream", ctypes.c_uint64), ("off_plane", ctypes.c_uint64),
                ("stream_bytes", ctypes.c_uint64), ("plane_bytes", ctypes.c_uint64),
                ("freq", ctypes.c_uint64 * 16)]


class EncodeOpts(ctypes.Structure):
    _fields_ = [("lane_syms", ctypes.c_uint32), ("n_threads", ctypes.c_uint32),
                ("table_mode", ctypes.c_uint32), ("group_chunks", ctypes.c_uint32),
                ("max_code_len", ctypes.c_uint32), ("tile_rows", ctypes.c_uint32),
                ("reserved", ctypes.c_uint32 * 2)]


class Stats(ctypes.Structure):
    _fields_ = [("entropy_bits", ctypes.c_double), ("avg_code_bits", ctypes.c_double),
                ("bits_per_weight", ctypes.c_double), ("ratio", ctypes.c_double),
                ("max_code_len", ctypes.c_uint32), ("n_symbols", ctypes.c_uint32)]


class BatchItem(ctypes.Structure):
    _fields_ = [("d_blob", ctypes.c_uint64), ("d_out", ctypes.c_uint64), ("n_elem", ctypes.c_uint64),
                ("n_chunks", ctypes.c_uint64), ("first_chunk", ctypes.c_uint64),
                ("off_chunk_bit", ctypes.c_uint64), ("off_lane_bits", ctypes.c_uint64),
                ("off_stream", ctypes.c_uint64), ("off_plane", ctypes.c_uint64),
                ("stream_bytes", ctypes.c_uint64), ("code_len", ctypes.c_uint8 * 16),
                ("off_table", ctypes.c_uint64), ("group_chunks", ctypes.c_uint64),
                ("tile_cols", ctypes.c_uint64), ("reserved", ctypes.c_uint64 * 1)]


class BatchInfo(ctypes.Structure):
    _fields_ = [("total_chunks", ctypes.c_uint64), ("lane_syms", ctypes.c_uint32),
                ("max_code_len", ctypes.c_uint32), ("max_workgroups", ctypes.c_uint32),
                ("row_tiled", ctypes.c_uint32)]


class GemmGroupDesc(ctypes.Structure):
    _fields_ = [("hdr", ctypes.POINTER(Header)), ("d_w", ctypes.c_void_p), ("rows", ctypes.c_uint64),
                ("cols", ctypes.c_uint64), ("d_x", ctypes.c_void_p), ("d_y", ctypes.c_void_p),
                ("d_w_scale", ctypes.c_void_p), ("d_x_scale", ctypes.c_void_p), ("x_scale_cols", ctypes.c_uint32),
                ("M", ctypes.c_uint32)]


class GemmGroupItem(ctypes.Structure):
    _fields_ = [("opaque", ctypes.c_uint64 * 32)]


class GemmGroupInfo(ctypes.Structure):
    _fields_ = [("total_work", ctypes.c_uint64), ("n_items", ctypes.c_uint32), ("max_M", ctypes.c_uint32),
                ("scale_mode", ctypes.c_uint32), ("raw", ctypes.c_uint32)]


assert ctypes.sizeof(Header) == 256 and ctypes.sizeof(BatchItem) == 128 and ctypes.sizeof(GemmGroupItem) == 256

_vp, _u64, _u32 = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32
_lib.ecf8_encode.argtypes = [_vp, _u64, _u64, ctypes.POINTER(EncodeOpts), ctypes.POINTER(_vp)]
_lib.ecf8_encode_bound.argtypes = [_u64, _u64, ctypes.POINTER(EncodeOpts), ctypes.POINTER(_u64)]
_lib.ecf8_encode_gpu.argtypes = [_vp, _u64, _u64, ctypes.POINTER(EncodeOpts), _vp, _u64, ctypes.POINTER(Header), _vp]
_lib.ecf8_blob_free.argtypes = [_vp]
_lib.ecf8_blob_free.restype = None
_lib.ecf8_blob_data.argtypes = [_vp]
_lib.ecf8_blob_data.restype = _vp
_lib.ecf8_blob_size.argtypes = [_vp]
_lib.ecf8_blob_size.restype = _u64
_lib.ecf8_blob_describe.argtypes = [_vp, _u64, ctypes.POINTER(Header)]
_lib.ecf8_blob_validate.argtypes = [_vp, _u64]
_lib.ecf8_blob_stats.argtypes = [ctypes.POINTER(Header), ctypes.POINTER(Stats)]
_lib.ecf8_decode.argtypes = [ctypes.POINTER(Header), _vp, _vp, _u64, _vp]
_lib.ecf8_batch_prepare.argtypes = [ctypes.POINTER(Header), ctypes.POINTER(_vp), ctypes.POINTER(_vp),
                                    ctypes.POINTER(_u64), _u32, ctypes.POINTER(BatchItem),
                                    ctypes.POINTER(BatchInfo)]
_lib.ecf8_decode_batched.argtypes = [_vp, _u32, ctypes.POINTER(BatchInfo), _vp]
_lib.ecf8_gemm_fp8.argtypes = [ctypes.POINTER(Header), _vp, _vp, _u32, _vp, _vp]
_lib.ecf8_gemm_fp8_raw.argtypes = [_vp, _u64, _u64, _vp, _u32, _vp, _vp]
_lib.ecf8_gemm_fp8_scaled.argtypes = [ctypes.POINTER(Header), _vp, _vp, _u32, _vp, _vp, _u32, _vp, _vp]
_lib.ecf8_gemm_fp8_raw_scaled.argtypes = [_vp, _u64, _u64, _vp, _u32, _vp, _vp, _u32, _vp, _vp]
_lib.ecf8_gemm_splitk_plan.argtypes = [_u64, _u64, _u32, _u32, ctypes.POINTER(_u32), ctypes.POINTER(_u64)]
_lib.ecf8_gemm_splitk_slices.argtypes = [_u64, _u64]
_lib.ecf8_gemm_splitk_slices.restype = _u32
_lib.ecf8_gemm_splitk_workspace_bytes.argtypes = [_u64, _u64, _u32]
_lib.ecf8_gemm_splitk_workspace_bytes.restype = _u64
_lib.ecf8_gemm_splitk_workspace_init.argtypes = [_vp, _u64, _vp]
_lib.ecf8_gemm_fp8_splitk.argtypes = [ctypes.POINTER(Header), _vp, _vp, _u32, _vp, _vp, _u32, _vp, _vp, _u64, _vp]
_lib.ecf8_gemm_fp8_raw_splitk.argtypes = [_vp, _u64, _u64, _vp, _u32, _vp, _vp, _u32, _vp, _vp, _u64, _vp]
_lib.ecf8_gemm_fp8_splitk_static.argtypes = [ctypes.POINTER(Header), _vp, _vp, _u32, _vp, _vp, _u32, _vp, _vp]
_lib.ecf8_gemm_fp8_exact.argtypes = [ctypes.POINTER(Header), _vp, _vp, _u32, _vp, _vp, _u32, _vp, _vp]
_lib.ecf8_gemm_fp8_raw_exact.argtypes = [_vp, _u64, _u64, _vp, _u32, _vp, _vp, _u32, _vp, _vp]
_lib.ecf8_gemm_group_prepare.argtypes = [ctypes.POINTER(GemmGroupDesc), _u32, ctypes.POINTER(GemmGroupItem),
                                         ctypes.POINTER(GemmGroupInfo)]
_lib.ecf8_gemm_fp8_grouped.argtypes = [_vp, ctypes.POINTER(GemmGroupInfo), _vp]
_lib.ecf8_jit_create.argtypes = [_u32, _u32, ctypes.POINTER(_vp), _u64, ctypes.POINTER(_vp)]
_lib.ecf8_jit_destroy.argtypes = [_vp]
_lib.ecf8_jit_destroy.restype = None
_lib.ecf8_jit_layer_prepare.argtypes = [_vp, _u32, ctypes.POINTER(Header), ctypes.POINTER(_vp), _u32,
                                        ctypes.POINTER(BatchItem), ctypes.POINTER(_u64)]
_lib.ecf8_jit_layer_commit.argtypes = [_vp, _u32, _vp]
_lib.ecf8_jit_prefetch.argtypes = [_vp, _u32]
_lib.ecf8_jit_set_decode_workgroups.argtypes = [_vp, _u32]
_lib.ecf8_jit_acquire.argtypes = [_vp, _u32, _vp, ctypes.POINTER(_vp)]
_lib.ecf8_jit_release.argtypes = [_vp, _u32, _vp]
_lib.ecf8_strerror.argtypes = [ctypes.c_int]
_lib.ecf8_strerror.restype = ctypes.c_char_p
_lib.ecf8_version.restype = _u32


class Ecf8Error(RuntimeError):
    def __init__(self, fn, code):
        self.code = code
        super().__init__("%s: %s (%d)" % (fn, _lib.ecf8_strerror(code).decode(), code))


def _check(fn, rc):
    if rc != OK:
        raise Ecf8Error(fn, rc)


def _host_u8(x):
    if isinstance(x, torch.Tensor):
        if x.device.type != "cpu":
            x = x.cpu()
        if x.dtype != torch.uint8:
            x = x.view(torch.uint8)
        x = x.contiguous().numpy()
    x = np.ascontiguousarray(x)
    if x.dtype != np.uint8:
        raise TypeError("expected raw FP8 bytes (uint8)")
    return x


class Blob:
    """Host object owning one encoded container (an ``ecf8_blob``)."""

    def __init__(self, handle):
        self._h = handle
        self.size = int(_lib.ecf8_blob_size(handle))
        self._ptr = _lib.ecf8_blob_data(handle)
        self.header = blob_describe(self._ptr, self.size)

    def numpy(self):
        """Zero-copy uint8 view of the container bytes; the view keeps this object alive."""
        buf = (ctypes.c_uint8 * self.size).from_address(self._ptr)
        buf._owner = self
        return np.frombuffer(buf, dtype=np.uint8)

    def to(self, device):
        """Copy of the container in device memory (a uint8 tensor the caller owns)."""
        return torch.from_numpy(self.numpy()).to(device)

    def stats(self):
        return blob_stats(self.header)

    def __del__(self, _free=_lib.ecf8_blob_free):
        if getattr(self, "_h", None):
            _free(self._h)
            self._h = None


def ecf8_encode(fp8, rows=None, cols=None, lane_syms=0, n_threads=0, table_mode=0, group_chunks=0,
                max_code_len=0, tile_rows=0):
    """CPU encoder: raw E4M3 bytes (host tensor / array) -> Blob.
    table_mode: 0 embed the decode table for tensors of >= 2^22 weights, 1 always, 2 never.
    group_chunks: chunks interleaved per group (0 = default 32; 1 = chunk-major, what the fused GEMM needs).
    max_code_len: cap on the code length (0 = default 7; 15 = plain Huffman).
    tile_rows: 0 = linear layout; 16 = row-tiled layout (what ecf8_gemm_fp8 needs, with lane_syms=64)."""
    x = _host_u8(fp8)
    if rows is None:
        rows, cols = (x.shape if x.ndim == 2 else (1, x.size))
    if rows * cols != x.size:
        raise Ecf8Error("ecf8_encode", E_ARG)
    opts = EncodeOpts(lane_syms, n_threads, table_mode, group_chunks, max_code_len, tile_rows)
    h = _vp()
    _check("ecf8_encode", _lib.ecf8_encode(x.ctypes.data, rows, cols, ctypes.byref(opts), ctypes.byref(h)))
    return Blob(h)


def ecf8_encode_gpu(d_fp8, rows=None, cols=None, lane_syms=0, table_mode=0, group_chunks=0, max_code_len=0,
                    tile_rows=0, d_blob=None, stream=None):
    """GPU encoder: uint8 device tensor of raw E4M3 bytes -> (Header, uint8 device tensor holding the blob).
    Same options and same bytes as ecf8_encode."""
    if rows is None:
        rows, cols = (d_fp8.shape if d_fp8.dim() == 2 else (1, d_fp8.numel()))
    if rows * cols != d_fp8.numel() or d_fp8.dtype != torch.uint8 or not d_fp8.is_contiguous():
        raise Ecf8Error("ecf8_encode_gpu", E_ARG)
    opts = EncodeOpts(lane_syms, 0, table_mode, group_chunks, max_code_len, tile_rows)
    if d_blob is None:
        bound = _u64(0)
        _check("ecf8_encode_bound", _lib.ecf8_encode_bound(rows, cols, ctypes.byref(opts), ctypes.byref(bound)))
        d_blob = torch.empty(int(bound.value), dtype=torch.uint8, device=d_fp8.device)
    hdr = Header()
    _check("ecf8_encode_gpu", _lib.ecf8_encode_gpu(d_fp8.data_ptr(), rows, cols, ctypes.byref(opts), d_blob.data_ptr(),
                                                   d_blob.numel(), ctypes.byref(hdr), _stream_ptr(stream)))
    return hdr, d_blob[:hdr.total_size]


def blob_describe(ptr_or_array, size=None):
    if isinstance(ptr_or_array, np.ndarray):
        size = ptr_or_array.size
        ptr_or_array = ptr_or_array.ctypes.data
    hdr = Header()
    _check("ecf8_blob_describe", _lib.ecf8_blob_describe(ptr_or_array, size, ctypes.byref(hdr)))
    return hdr


def blob_validate(arr):
    arr = np.ascontiguousarray(arr, dtype=np.uint8)
    _check("ecf8_blob_validate", _lib.ecf8_blob_validate(arr.ctypes.data, arr.size))


def save_blob(path, blob):
    """Writes a container (Blob or uint8 array) to a file as is: the format is position independent."""
    arr = blob.numpy() if isinstance(blob, Blob) else np.ascontiguousarray(blob, dtype=np.uint8)
    blob_validate(arr)
    with open(path, "wb") as f:
        f.write(arr.tobytes())


def load_blob(path):
    """Reads a container file; returns (Header, uint8 array) after the full host-side check."""
    arr = np.fromfile(path, dtype=np.uint8)
    blob_validate(arr)
    return blob_describe(arr), arr


def blob_stats(hdr):
    st = Stats()
    _check("ecf8_blob_stats", _lib.ecf8_blob_stats(ctypes.byref(hdr), ctypes.byref(st)))
    return {k: getattr(st, k) for k, _ in Stats._fields_}


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def ecf8_decode(hdr, d_blob, d_out=None, stream=None):
    """GPU decode of one tensor.  d_blob: uint8 device tensor holding the blob."""
    if d_out is None:
        d_out = torch.empty((hdr.rows, hdr.cols), dtype=torch.uint8, device=d_blob.device)
    _check("ecf8_decode", _lib.ecf8_decode(ctypes.byref(hdr), d_blob.data_ptr(), d_out.data_ptr(),
                                           d_out.numel(), _stream_ptr(stream)))
    return d_out


class Batch:
    """Device-resident item table for ecf8_decode_batched (built once, reused)."""

    def __init__(self, hdrs, d_blobs, d_outs):
        n = len(hdrs)
        H = (Header * n)(*hdrs)
        B = (_vp * n)(*[t.data_ptr() for t in d_blobs])
        O = (_vp * n)(*[t.data_ptr() for t in d_outs])
        C = (_u64 * n)(*[t.numel() for t in d_outs])
        items = (BatchItem * n)()
        self.info = BatchInfo()
        _check("ecf8_batch_prepare", _lib.ecf8_batch_prepare(H, B, O, C, n, items, ctypes.byref(self.info)))
        host = np.frombuffer(items, dtype=np.uint8).copy()
        self.d_items = torch.from_numpy(host).to(d_blobs[0].device)
        self.n = n
        self.total_chunks = int(self.info.total_chunks)
        self.lane_syms = int(self.info.lane_syms)
        self.max_code_len = int(self.info.max_code_len)
        self._keep = (list(d_blobs), list(d_outs))


def ecf8_decode_batched(batch, stream=None):
    _check("ecf8_decode_batched", _lib.ecf8_decode_batched(batch.d_items.data_ptr(), batch.n,
                                                           ctypes.byref(batch.info), _stream_ptr(stream)))


class Jit:
    """Just-in-time layer decode over shared buffers (ecf8_jit_*): layers = list of (headers, device
    blobs); layer l decodes into buffer l % n_buffers.  prefetch(l) queues the decode on the
    manager's own stream, acquire(l) orders the caller's stream behind it and returns the layer's
    tensors (views into the buffer), release(l) lets the buffer be reused.  A layer's headers are either
    all ecf8 headers (FP8) or all wide-alphabet headers (E5M2 / BF16, see ecfw.py)."""

    def __init__(self, layers, n_buffers=2, buffer_bytes=None):
        dev = layers[0][1][0].device

        def nbytes(h):
            return h.n_elem * (2 if getattr(h, "fmt", 0) == 2 else 1)
        need = max(sum((nbytes(h) + 255) // 256 * 256 for h in hdrs) for hdrs, _ in layers)
        self.buffer_bytes = buffer_bytes if buffer_bytes is not None else need
        self.buffers = [torch.empty(self.buffer_bytes, dtype=torch.uint8, device=dev) for _ in range(n_buffers)]
        B = (_vp * n_buffers)(*[b.data_ptr() for b in self.buffers])
        self._h = _vp()
        _check("ecf8_jit_create", _lib.ecf8_jit_create(len(layers), n_buffers, B, self.buffer_bytes,
                                                       ctypes.byref(self._h)))
        self._keep, self._views = [], []
        for l, (hdrs, d_blobs) in enumerate(layers):
            n = len(hdrs)
            P = (_vp * n)(*[t.data_ptr() for t in d_blobs])
            offs = (_u64 * n)()
            wide = hasattr(hdrs[0], "fmt")
            if wide:
                from . import ecfw
                H = (ecfw.WHeader * n)(*hdrs)
                items = (ecfw.WBatchItem * n)()
                _check("ecfw_jit_layer_prepare", _lib.ecfw_jit_layer_prepare(self._h, l, H, P, n, items, offs))
            else:
                H = (Header * n)(*hdrs)
                items = (BatchItem * n)()
                _check("ecf8_jit_layer_prepare", _lib.ecf8_jit_layer_prepare(self._h, l, H, P, n, items, offs))
            d_items = torch.from_numpy(np.frombuffer(items, dtype=np.uint8).copy()).to(dev)
            if wide:
                _check("ecfw_jit_layer_commit", _lib.ecfw_jit_layer_commit(self._h, l, d_items.data_ptr()))
            else:
                _check("ecf8_jit_layer_commit", _lib.ecf8_jit_layer_commit(self._h, l, d_items.data_ptr()))
            self._keep.append((d_items, list(d_blobs)))
            buf = self.buffers[l % n_buffers]
            views = []
            for o, h in zip(offs, hdrs):
                v = buf[int(o):int(o) + nbytes(h)]
                if getattr(h, "fmt", 0) == 2:
                    v = v.view(torch.bfloat16)
                views.append(v.view(h.rows, h.cols))
            self._views.append(views)

    def set_decode_workgroups(self, max_workgroups):
        _check("ecf8_jit_set_decode_workgroups", _lib.ecf8_jit_set_decode_workgroups(self._h, max_workgroups))

    def prefetch(self, layer):
        _check("ecf8_jit_prefetch", _lib.ecf8_jit_prefetch(self._h, layer))

    def acquire(self, layer, stream=None):
        base = _vp()
        _check("ecf8_jit_acquire", _lib.ecf8_jit_acquire(self._h, layer, _stream_ptr(stream), ctypes.byref(base)))
        assert base.value == self.buffers[layer % len(self.buffers)].data_ptr()
        return self._views[layer]

    def release(self, layer, stream=None):
        _check("ecf8_jit_release", _lib.ecf8_jit_release(self._h, layer, _stream_ptr(stream)))

    def close(self, _destroy=_lib.ecf8_jit_destroy):
        if getattr(self, "_h", None):
            _destroy(self._h)
            self._h = None

    __del__ = close


def ecf8_gemm_fp8(hdr, d_blob, d_x, d_y=None, stream=None):
    """Y = X @ W.T with W decoded on the fly from its blob.  d_x: (M, cols) uint8 E4M3 on the device."""
    M = d_x.shape[0]
    if d_y is None:
        d_y = torch.empty((M, hdr.rows), dtype=torch.float32, device=d_x.device)
    _check("ecf8_gemm_fp8", _lib.ecf8_gemm_fp8(ctypes.byref(hdr), d_blob.data_ptr(), d_x.data_ptr(), M,
                                               d_y.data_ptr(), _stream_ptr(stream)))
    return d_y


def ecf8_gemm_fp8_raw(d_w, d_x, d_y=None, stream=None):
    """The same GEMM on uncompressed weights d_w: (rows, cols) uint8 E4M3 on the device."""
    M = d_x.shape[0]
    rows, cols = d_w.shape
    if d_y is None:
        d_y = torch.empty((M, rows), dtype=torch.float32, device=d_x.device)
    _check("ecf8_gemm_fp8_raw", _lib.ecf8_gemm_fp8_raw(d_w.data_ptr(), rows, cols, d_x.data_ptr(), M,
                                                       d_y.data_ptr(), _stream_ptr(stream)))
    return d_y


def _scale_ptrs(fn, rows, cols, M, w_scale, x_scale):
    if (w_scale.dtype != torch.float32 or not w_scale.is_contiguous()
            or tuple(w_scale.shape) != ((rows + 127) // 128, cols // 128)):
        raise Ecf8Error(fn, E_ARG)
    xs_cols = 0
    if x_scale is not None:
        if x_scale.dtype != torch.float32 or not x_scale.is_contiguous():
            raise Ecf8Error(fn, E_ARG)
        if tuple(x_scale.shape) == (M,):
            xs_cols = 1
        elif tuple(x_scale.shape) == (M, cols // 128):
            xs_cols = cols // 128
        else:
            raise Ecf8Error(fn, E_ARG)
    return w_scale.data_ptr(), (x_scale.data_ptr() if x_scale is not None else None), xs_cols


def ecf8_gemm_fp8_scaled(hdr, d_blob, d_x, w_scale, x_scale=None, d_y=None, stream=None):
    """Y = (x_scale X) @ (w_scale W).T: w_scale fp32 (ceil(rows/128), cols/128); x_scale fp32 (M,) for one scale
    per row of X, (M, cols/128) for one per row and 128 columns, or None."""
    M = d_x.shape[0]
    ws, xs, xc = _scale_ptrs("ecf8_gemm_fp8_scaled", hdr.rows, hdr.cols, M, w_scale, x_scale)
    if d_y is None:
        d_y = torch.empty((M, hdr.rows), dtype=torch.float32, device=d_x.device)
    _check("ecf8_gemm_fp8_scaled", _lib.ecf8_gemm_fp8_scaled(ctypes.byref(hdr), d_blob.data_ptr(), d_x.data_ptr(), M,
                                                             ws, xs, xc, d_y.data_ptr(), _stream_ptr(stream)))
    return d_y


def ecf8_gemm_fp8_raw_scaled(d_w, d_x, w_scale, x_scale=None, d_y=None, stream=None):
    M = d_x.shape[0]
    rows, cols = d_w.shape
    ws, xs, xc = _scale_ptrs("ecf8_gemm_fp8_raw_scaled", rows, cols, M, w_scale, x_scale)
    if d_y is None:
        d_y = torch.empty((M, rows), dtype=torch.float32, device=d_x.device)
    _check("ecf8_gemm_fp8_raw_scaled", _lib.ecf8_gemm_fp8_raw_scaled(d_w.data_ptr(), rows, cols, d_x.data_ptr(), M,
                                                                     ws, xs, xc, d_y.data_ptr(), _stream_ptr(stream)))
    return d_y


def gemm_splitk_slices(rows, cols):
    """Workgroups per block of 16 rows the split-K calls use for this shape on the current device (1 = no split)."""
    return int(_lib.ecf8_gemm_splitk_slices(rows, cols))


def gemm_splitk_plan(rows, cols, M, compute_units=0):
    """(slices, workspace bytes) of the split-K calls for this shape on a device of that many compute units
    (0 = the current device)."""
    sl, nb = _u32(), _u64()
    _check("ecf8_gemm_splitk_plan", _lib.ecf8_gemm_splitk_plan(rows, cols, M, compute_units, ctypes.byref(sl), ctypes.byref(nb)))
    return int(sl.value), int(nb.value)


def gemm_splitk_workspace(rows, cols, M, device, stream=None):
    """A zeroed workspace for the split-K calls on a rows x cols matrix with up to M rows of X (uint8 tensor; it may
    be reused for any later call it is large enough for, one call at a time)."""
    n = int(_lib.ecf8_gemm_splitk_workspace_bytes(rows, cols, M))
    ws = torch.empty((max(n, 16),), dtype=torch.uint8, device=device)
    _check("ecf8_gemm_splitk_workspace_init", _lib.ecf8_gemm_splitk_workspace_init(ws.data_ptr(), ws.numel(), _stream_ptr(stream)))
    return ws


def _opt_scale_ptrs(fn, rows, cols, M, w_scale, x_scale):
    if w_scale is None and x_scale is None:
        return None, None, 0
    if w_scale is None:
        raise Ecf8Error(fn, E_ARG)
    return _scale_ptrs(fn, rows, cols, M, w_scale, x_scale)


def ecf8_gemm_fp8_splitk(hdr, d_blob, d_x, workspace, w_scale=None, x_scale=None, d_y=None, stream=None):
    """ecf8_gemm_fp8 / ecf8_gemm_fp8_scaled with K split among workgroups (matrices of few rows)."""
    M = d_x.shape[0]
    ws, xs, xc = _opt_scale_ptrs("ecf8_gemm_fp8_splitk", hdr.rows, hdr.cols, M, w_scale, x_scale)
    if d_y is None:
        d_y = torch.empty((M, hdr.rows), dtype=torch.float32, device=d_x.device)
    _check("ecf8_gemm_fp8_splitk", _lib.ecf8_gemm_fp8_splitk(ctypes.byref(hdr), d_blob.data_ptr(), d_x.data_ptr(), M, ws, xs, xc,
                                                             d_y.data_ptr(), workspace.data_ptr(), workspace.numel(),
                                                             _stream_ptr(stream)))
    return d_y


def ecf8_gemm_fp8_raw_splitk(d_w, d_x, workspace, w_scale=None, x_scale=None, d_y=None, stream=None):
    M = d_x.shape[0]
    rows, cols = d_w.shape
    ws, xs, xc = _opt_scale_ptrs("ecf8_gemm_fp8_raw_splitk", rows, cols, M, w_scale, x_scale)
    if d_y is None:
        d_y = torch.empty((M, rows), dtype=torch.float32, device=d_x.device)
    _check("ecf8_gemm_fp8_raw_splitk", _lib.ecf8_gemm_fp8_raw_splitk(d_w.data_ptr(), rows, cols, d_x.data_ptr(), M, ws, xs, xc,
                                                                     d_y.data_ptr(), workspace.data_ptr(), workspace.numel(),
                                                                     _stream_ptr(stream)))
    return d_y


def ecf8_gemm_fp8_splitk_static(hdr, d_blob, d_x, w_scale=None, x_scale=None, d_y=None, stream=None):
    """ecf8_gemm_fp8_splitk with the workspace inside the library (nothing to allocate; one call at a time per GPU)."""
    M = d_x.shape[0]
    ws, xs, xc = _opt_scale_ptrs("ecf8_gemm_fp8_splitk_static", hdr.rows, hdr.cols, M, w_scale, x_scale)
    if d_y is None:
        d_y = torch.empty((M, hdr.rows), dtype=torch.float32, device=d_x.device)
    _check("ecf8_gemm_fp8_splitk_static", _lib.ecf8_gemm_fp8_splitk_static(ctypes.byref(hdr), d_blob.data_ptr(), d_x.data_ptr(), M,
                                                                           ws, xs, xc, d_y.data_ptr(), _stream_ptr(stream)))
    return d_y


def ecf8_gemm_fp8_exact(hdr, d_blob, d_x, w_scale=None, x_scale=None, d_y=None, stream=None):
    """ecf8_gemm_fp8 / _scaled on the F16 matrix cores: exact products, fp32 sums."""
    M = d_x.shape[0]
    ws, xs, xc = _opt_scale_ptrs("ecf8_gemm_fp8_exact", hdr.rows, hdr.cols, M, w_scale, x_scale)
    if d_y is None:
        d_y = torch.empty((M, hdr.rows), dtype=torch.float32, device=d_x.device)
    _check("ecf8_gemm_fp8_exact", _lib.ecf8_gemm_fp8_exact(ctypes.byref(hdr), d_blob.data_ptr(), d_x.data_ptr(), M, ws, xs, xc,
                                                           d_y.data_ptr(), _stream_ptr(stream)))
    return d_y


def ecf8_gemm_fp8_raw_exact(d_w, d_x, w_scale=None, x_scale=None, d_y=None, stream=None):
    M = d_x.shape[0]
    rows, cols = d_w.shape
    ws, xs, xc = _opt_scale_ptrs("ecf8_gemm_fp8_raw_exact", rows, cols, M, w_scale, x_scale)
    if d_y is None:
        d_y = torch.empty((M, rows), dtype=torch.float32, device=d_x.device)
    _check("ecf8_gemm_fp8_raw_exact", _lib.ecf8_gemm_fp8_raw_exact(d_w.data_ptr(), rows, cols, d_x.data_ptr(), M, ws, xs, xc,
                                                                   d_y.data_ptr(), _stream_ptr(stream)))
    return d_y


class GemmGroup:
    """Device-resident item table for ecf8_gemm_fp8_grouped (built once, reused).  members: a list of dicts with
    either hdr + blob (compressed W) or w (uncompressed (rows, cols) uint8 tensor), x ((M, cols) uint8), optional
    w_scale / x_scale as for ecf8_gemm_fp8_scaled, optional y ((M, rows) fp32, allocated when absent).
    self.y holds the outputs in order."""

    def __init__(self, members):
        n = len(members)
        descs = (GemmGroupDesc * n)()
        self.y, self._keep = [], []
        for d, m in zip(descs, members):
            x = m["x"]
            M = x.shape[0]
            if "hdr" in m:
                hdr, rows, cols, w = m["hdr"], m["hdr"].rows, m["hdr"].cols, m["blob"]
                d.hdr = ctypes.pointer(hdr)
            else:
                w = m["w"]
                rows, cols = w.shape
                d.rows, d.cols = rows, cols
            y = m.get("y")
            if y is None:
                y = torch.empty((M, rows), dtype=torch.float32, device=x.device)
            ws, xs, xc = _opt_scale_ptrs("ecf8_gemm_group_prepare", rows, cols, M, m.get("w_scale"), m.get("x_scale"))
            d.d_w, d.d_x, d.d_y, d.M = w.data_ptr(), x.data_ptr(), y.data_ptr(), M
            d.d_w_scale, d.d_x_scale, d.x_scale_cols = ws, xs, xc
            self.y.append(y)
            self._keep.append((w, x, m.get("w_scale"), m.get("x_scale"), m.get("hdr")))
        items = (GemmGroupItem * n)()
        self.info = GemmGroupInfo()
        _check("ecf8_gemm_group_prepare", _lib.ecf8_gemm_group_prepare(descs, n, items, ctypes.byref(self.info)))
        self.d_items = torch.from_numpy(np.frombuffer(items, dtype=np.uint8).copy()).to(members[0]["x"].device)


def ecf8_gemm_fp8_grouped(group, stream=None):
    """All products of a GemmGroup in one launch; returns group.y."""
    _check("ecf8_gemm_fp8_grouped", _lib.ecf8_gemm_fp8_grouped(group.d_items.data_ptr(), ctypes.byref(group.info),
                                                               _stream_ptr(stream)))
    return group.y


def version():
    return int(_lib.ecf8_version())

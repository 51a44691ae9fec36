"""Thin ctypes binding over the C-ABI library (include/apgemv.h): argument marshalling only.

PyTorch is used for device memory and streams; every step of the path runs in the HIP library.
If the library has not been built the import of this module fails loudly - there is no fallback.
"""
import ctypes
import os

import numpy as np

try:  # torch first: the library must bind to the HIP runtime that torch has already loaded
    import torch
except Exception:  # pragma: no cover - torch is part of the image
    torch = None

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libapgemv.so")

AP_OK = 0
STATUS_NAMES = {0: "AP_OK", 1: "AP_ERR_INVALID_ARG", 2: "AP_ERR_SHAPE", 3: "AP_ERR_BITS",
                4: "AP_ERR_INDEX_RANGE", 5: "AP_ERR_BUFFER_TOO_SMALL", 6: "AP_ERR_BATCH",
                7: "AP_ERR_HIP", 8: "AP_ERR_NO_MEMORY"}

EXPORTS = ["ap_packed_size", "ap_pack_host", "ap_unpack_host", "ap_blob_lut_entry",
           "ap_read_extent", "ap_pack", "ap_attach", "ap_set_option", "ap_unpack", "ap_gemv", "ap_gemv_multi", "ap_gemv_list", "ap_gemv_list_batch", "ap_dequantize",
           "ap_gemm_workspace_size", "ap_gemm", "ap_gemm_static", "ap_quantize", "ap_probe_read", "ap_probe_issue", "ap_matrix_info",
           "ap_free", "ap_strerror"]


OPTIONS = {"waves": 0, "row_groups": 1, "mfma_min_batch": 2, "variant": 3}
VARIANT_AUTO, VARIANT_NO_EXCHANGE, VARIANT_EXCHANGE, VARIANT_BANK_PER_LANE = 0, 1, 3, 5
VARIANT_PAIR, VARIANT_NO_PAIR = 7, 8
VARIANT_TILE, VARIANT_TILE2 = 9, 10


class ApError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s: %s (%s)" % (where, STATUS_NAMES.get(status, status), strerror(status)))


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError("libapgemv.so is not built: run `python -m paper_2402_10517_amd.build` "
                          "or __graft_entry__.build()")
    L = ctypes.CDLL(LIB_PATH)
    vp, ci, cu, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_uint, ctypes.c_size_t
    psz = ctypes.POINTER(ctypes.c_size_t)
    L.ap_packed_size.argtypes = [ci, ci, ci, cu, psz]
    L.ap_pack_host.argtypes = [vp, ci, ci, ci, vp, vp, sz]
    L.ap_unpack_host.argtypes = [vp, sz, vp]
    L.ap_blob_lut_entry.argtypes = [vp, sz, ci, ci, ci, ctypes.POINTER(ctypes.c_uint16)]
    L.ap_read_extent.argtypes = [ci, ci, ci, cu, ci, psz, psz, psz, psz]
    L.ap_pack.argtypes = [vp, ci, ci, ci, vp, vp, sz, vp, ctypes.POINTER(vp)]
    L.ap_attach.argtypes = [vp, sz, vp, ctypes.POINTER(vp)]
    L.ap_set_option.argtypes = [vp, ci, ci]
    L.ap_unpack.argtypes = [vp, vp, vp]
    L.ap_gemv.argtypes = [vp, ci, vp, vp, ci, vp]
    L.ap_gemv_multi.argtypes = [vp, ci, ci, ci, vp]
    L.ap_gemv_list.argtypes = [vp, ci, vp]
    L.ap_gemv_list_batch.argtypes = [vp, ci, ci, vp]
    L.ap_dequantize.argtypes = [vp, ci, vp, vp]
    L.ap_gemm_workspace_size.argtypes = [vp, psz]
    L.ap_gemm.argtypes = [vp, ci, vp, vp, ci, vp, sz, vp]
    L.ap_gemm_static.argtypes = [vp, ci, vp, vp, ci, vp]
    L.ap_quantize.argtypes = [vp, vp, ci, ci, ci, ci, ci, vp, vp]
    L.ap_probe_read.argtypes = [vp, sz, vp]
    L.ap_probe_issue.argtypes = [ctypes.c_int, ctypes.c_int, vp]
    L.ap_matrix_info.argtypes = [vp, ctypes.POINTER(ci), ctypes.POINTER(ci), ctypes.POINTER(ci),
                                 ctypes.POINTER(cu)]
    L.ap_free.argtypes = [vp]
    L.ap_free.restype = None
    L.ap_strerror.argtypes = [ci]
    L.ap_strerror.restype = ctypes.c_char_p
    for name in EXPORTS:
        if name not in ("ap_free", "ap_strerror"):
            getattr(L, name).restype = ci
    return L


lib = _load()


def strerror(status):
    return lib.ap_strerror(int(status)).decode()


def _check(status, where):
    if status != AP_OK:
        raise ApError(status, where)


def _lut_array(luts):
    """luts: {b: (M, 2**b) float16/uint16 array} -> (ctypes array of 9 pointers, keep-alive list)."""
    arr = (ctypes.c_void_p * 9)()
    keep = []
    for b, t in luts.items():
        t = np.ascontiguousarray(t)
        if t.dtype == np.float16:
            t = t.view(np.uint16)
        assert t.dtype == np.uint16 and 0 <= b <= 8
        keep.append(t)
        arr[b] = t.ctypes.data
    return arr, keep


def lut_mask(bit_widths):
    m = 0
    for b in bit_widths:
        m |= 1 << b
    return m


def ap_packed_size(M, K, n, mask):
    out = ctypes.c_size_t(0)
    _check(lib.ap_packed_size(M, K, n, mask, ctypes.byref(out)), "ap_packed_size")
    return out.value


def ap_pack_host(idx, luts, n=8):
    """Pack on the host; returns the blob as a uint8 numpy array."""
    idx = np.ascontiguousarray(idx, dtype=np.uint8)
    M, K = idx.shape
    size = ap_packed_size(M, K, n, lut_mask(luts.keys()))
    blob = np.empty(size, dtype=np.uint8)
    arr, keep = _lut_array(luts)
    _check(lib.ap_pack_host(idx.ctypes.data, M, K, n, arr, blob.ctypes.data, size), "ap_pack_host")
    return blob


def ap_unpack_host(blob, M, K):
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    out = np.empty((M, K), dtype=np.uint8)
    _check(lib.ap_unpack_host(blob.ctypes.data, blob.size, out.ctypes.data), "ap_unpack_host")
    return out


def ap_read_extent(M, K, n, mask, b):
    v = [ctypes.c_size_t(0) for _ in range(4)]
    _check(lib.ap_read_extent(M, K, n, mask, b, *[ctypes.byref(a) for a in v]), "ap_read_extent")
    return tuple(a.value for a in v)


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream), stream


class PackedMatrix:
    """Owns the torch device buffer and the library handle of one packed matrix."""

    def __init__(self, handle, buf, M, K, n, mask):
        self.handle, self.buf = handle, buf
        self.M, self.K, self.n, self.mask = M, K, n, mask

    def close(self):
        if self.handle:
            lib.ap_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_options(self, **opts):
        """Kernel-selection overrides (tests, A/B runs): waves, row_groups, mfma_min_batch, variant."""
        for name, value in opts.items():
            _check(lib.ap_set_option(self.handle, OPTIONS[name], int(value)), "ap_set_option(%s)" % name)
        return self

    def clone(self):
        """Device-to-device copy of the blob, adopted through ap_attach (distinct addresses)."""
        buf = self.buf.clone()
        h = ctypes.c_void_p()
        sp, _ = _stream_ptr(None)
        _check(lib.ap_attach(buf.data_ptr(), buf.numel(), sp, ctypes.byref(h)), "ap_attach")
        return PackedMatrix(h, buf, self.M, self.K, self.n, self.mask)


def ap_pack(idx, luts, n=8, device="cuda:0", stream=None):
    idx = np.ascontiguousarray(idx, dtype=np.uint8)
    M, K = idx.shape
    mask = lut_mask(luts.keys())
    size = ap_packed_size(M, K, n, mask)
    buf = torch.empty(size, dtype=torch.uint8, device=device)
    arr, keep = _lut_array(luts)
    h = ctypes.c_void_p()
    sp, _ = _stream_ptr(stream)
    _check(lib.ap_pack(idx.ctypes.data, M, K, n, arr, buf.data_ptr(), size, sp, ctypes.byref(h)),
           "ap_pack")
    return PackedMatrix(h, buf, M, K, n, mask)


def ap_unpack(pm, stream=None):
    out = np.empty((pm.M, pm.K), dtype=np.uint8)
    sp, _ = _stream_ptr(stream)
    _check(lib.ap_unpack(pm.handle, out.ctypes.data, sp), "ap_unpack")
    return out


def ap_gemv(pm, b, x, y=None, stream=None):
    """x: (batch, K) float16 device tensor; returns y: (batch, M) float16 device tensor."""
    assert x.dtype == torch.float16 and x.is_cuda and x.is_contiguous()
    batch = 1 if x.dim() == 1 else x.shape[0]
    if y is None:
        y = torch.empty((batch, pm.M), dtype=torch.float16, device=x.device)
    sp, _ = _stream_ptr(stream)
    _check(lib.ap_gemv(pm.handle, int(b), x.data_ptr(), y.data_ptr(), batch, sp), "ap_gemv")
    return y


class GemvItem(ctypes.Structure):
    _fields_ = [("h", ctypes.c_void_p), ("x_dev", ctypes.c_void_p), ("y_dev", ctypes.c_void_p)]


def make_items(triples):
    """[(PackedMatrix, x tensor, y tensor), ...] -> ctypes array for ap_gemv_multi."""
    arr = (GemvItem * len(triples))()
    for i, (pm, x, y) in enumerate(triples):
        arr[i].h = pm.handle.value if isinstance(pm.handle, ctypes.c_void_p) else pm.handle
        arr[i].x_dev = x.data_ptr()
        arr[i].y_dev = y.data_ptr()
    return arr


class GemvListItem(ctypes.Structure):
    _fields_ = [("h", ctypes.c_void_p), ("b", ctypes.c_int), ("x_dev", ctypes.c_void_p), ("y_dev", ctypes.c_void_p)]


def make_list(quads):
    """[(PackedMatrix, b, x tensor, y tensor), ...] -> ctypes array for ap_gemv_list."""
    arr = (GemvListItem * len(quads))()
    for i, (pm, b, x, y) in enumerate(quads):
        arr[i].h = pm.handle.value if isinstance(pm.handle, ctypes.c_void_p) else pm.handle
        arr[i].b = int(b)
        arr[i].x_dev = x.data_ptr()
        arr[i].y_dev = y.data_ptr()
    return arr


def ap_gemv_list(quads, stream=None):
    """Batch-1 work list, one bit-width per item: quads = [(PackedMatrix, b, x, y), ...]; fills the y's."""
    arr = make_list(quads)
    sp, _ = _stream_ptr(stream)
    _check(lib.ap_gemv_list(arr, len(quads), sp), "ap_gemv_list")
    return [q[3] for q in quads]


def ap_gemv_list_batch(quads, batch, stream=None):
    """Work list for `batch` activation rows per item: quads = [(PackedMatrix, b, x (batch, K), y (batch, M)), ...]."""
    arr = make_list(quads)
    sp, _ = _stream_ptr(stream)
    _check(lib.ap_gemv_list_batch(arr, len(quads), int(batch), sp), "ap_gemv_list_batch")
    return [q[3] for q in quads]


def ap_gemv_multi(triples, b, stream=None):
    """One launch for several matrices of equal K: triples = [(PackedMatrix, x, y), ...]; fills the y's."""
    batch = 1 if triples[0][1].dim() == 1 else triples[0][1].shape[0]
    arr = make_items(triples)
    sp, _ = _stream_ptr(stream)
    _check(lib.ap_gemv_multi(arr, len(triples), int(b), batch, sp), "ap_gemv_multi")
    return [t[2] for t in triples]


def ap_dequantize(pm, b, w=None, stream=None):
    """Dense (M, K) float16 device tensor of the b-bit model's weights."""
    if w is None:
        w = torch.empty((pm.M, pm.K), dtype=torch.float16, device=pm.buf.device)
    sp, _ = _stream_ptr(stream)
    _check(lib.ap_dequantize(pm.handle, int(b), w.data_ptr(), sp), "ap_dequantize")
    return w


def ap_gemm(pm, b, x, work=None, y=None, stream=None):
    """Large-batch path: x (batch, K) float16 -> y (batch, M) float16 via dequantise + dense GEMM."""
    assert x.dtype == torch.float16 and x.is_cuda and x.is_contiguous() and x.dim() == 2
    batch = x.shape[0]
    size = ctypes.c_size_t(0)
    _check(lib.ap_gemm_workspace_size(pm.handle, ctypes.byref(size)), "ap_gemm_workspace_size")
    if work is None:
        work = torch.empty(size.value, dtype=torch.uint8, device=x.device)
    if y is None:
        y = torch.empty((batch, pm.M), dtype=torch.float16, device=x.device)
    sp, _ = _stream_ptr(stream)
    _check(lib.ap_gemm(pm.handle, int(b), x.data_ptr(), y.data_ptr(), batch, work.data_ptr(),
                       work.numel(), sp), "ap_gemm")
    return y


def ap_quantize(w, sens=None, n_seed=3, n=8, iters=20):
    """Incremental-upscaling quantiser on the host: returns (idx uint8 (M, K), {b: float16 (M, 2**b)})."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    M, K = w.shape
    if sens is not None:
        sens = np.ascontiguousarray(sens, dtype=np.float32)
        assert sens.shape == w.shape
    idx = np.empty((M, K), dtype=np.uint8)
    luts = {b: np.empty((M, 1 << b), dtype=np.uint16) for b in range(max(n_seed, 0), min(n, 8) + 1)}
    arr = (ctypes.c_void_p * 9)()
    for b, t in luts.items():
        arr[b] = t.ctypes.data
    _check(lib.ap_quantize(w.ctypes.data, None if sens is None else sens.ctypes.data, M, K, n_seed, n, iters,
                           idx.ctypes.data, arr), "ap_quantize")
    return idx, {b: t.view(np.float16) for b, t in luts.items()}


def ap_gemv_raw(handle, b, x_ptr, y_ptr, batch, stream_ptr):
    """Unchecked call for timing loops: returns the status code."""
    return lib.ap_gemv(handle, b, x_ptr, y_ptr, batch, stream_ptr)

"""Thin ctypes binding of librtoss.so: same names as the C ABI, argument marshalling only.

Pointers are passed as integers (torch `tensor.data_ptr()` or any device address); the
stream is a raw hipStream_t handle (torch `torch.cuda.current_stream().cuda_stream`).
Every function raises RtossError on a non-zero status.  There is no CPU fallback: if the
library has not been built, loading fails.
"""
import ctypes
import os

import numpy as np

OK, EINVAL, ESHAPE, EDTYPE, ELAYOUT, ENOSPACE, EHIP = range(7)
F32, F16, BF16 = 0, 1, 2
NCHW, NHWC = 0, 1
RULE_ALL, RULE_ANYPAIR4, RULE_CONNECTED4, RULE_CONNECTED8 = 0, 1, 2, 3

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "librtoss.so")
_lib = None


class RtossError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("rtoss status %d: %s" % (status, message))
        self.status = status


class WDesc(ctypes.Structure):
    _fields_ = [("Co", ctypes.c_int), ("Ci", ctypes.c_int), ("ksize", ctypes.c_int), ("k", ctypes.c_int),
                ("dt", ctypes.c_int)]


class CDesc(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int), ("H", ctypes.c_int), ("W", ctypes.c_int), ("stride", ctypes.c_int),
                ("pad", ctypes.c_int), ("layout", ctypes.c_int), ("out_dt", ctypes.c_int),
                ("fuse_relu", ctypes.c_int)]


ACT_NONE, ACT_RELU, ACT_SILU = 0, 1, 2


class EpilogueDesc(ctypes.Structure):
    _fields_ = [("scale_dev", ctypes.c_void_p), ("bias_dev", ctypes.c_void_p), ("act", ctypes.c_int),
                ("residual_dev", ctypes.c_void_p), ("y_ld", ctypes.c_int), ("residual_ld", ctypes.c_int)]


class PackItemDesc(ctypes.Structure):
    _fields_ = [("desc", WDesc), ("w_dev", ctypes.c_void_p), ("idx_dev", ctypes.c_void_p), ("packed_dev", ctypes.c_void_p),
                ("packed_bytes", ctypes.c_size_t)]


class SelectItem(ctypes.Structure):
    _fields_ = [("w_dev", ctypes.c_void_p), ("n_elems", ctypes.c_int64), ("idx_dev", ctypes.c_void_p)]


EXPORTS = ["rtoss_pattern_dict", "rtoss_select_patterns", "rtoss_select_patterns_batch", "rtoss_pattern_histogram", "rtoss_reduce_dict",
           "rtoss_pack_size", "rtoss_pack", "rtoss_pack_batch", "rtoss_conv2d_pattern", "rtoss_conv2d_pattern_fused",
           "rtoss_pack_size_coherent", "rtoss_pack_coherent", "rtoss_conv2d_pattern_coherent", "rtoss_last_error"]


def lib():
    """Load librtoss.so (built in-tree by build.py / __graft_entry__.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError("librtoss.so is not built: run `python -m paper_2303_02191_amd.build` "
                              "(there is no fallback path)")
        # torch owns the device memory and the streams handed to this library, so the
        # library must bind to the HIP runtime torch has loaded: import torch first.
        import torch  # noqa: F401
        L = ctypes.CDLL(_LIB_PATH)
        vp, i, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        u16p = ctypes.POINTER(ctypes.c_uint16)
        szp = ctypes.POINTER(ctypes.c_size_t)
        L.rtoss_last_error.restype = ctypes.c_char_p
        L.rtoss_last_error.argtypes = []
        L.rtoss_pattern_dict.restype = i
        L.rtoss_pattern_dict.argtypes = [i, i, u16p, i, ctypes.POINTER(i)]
        L.rtoss_select_patterns.restype = i
        L.rtoss_select_patterns.argtypes = [vp, i, i64, u16p, i, vp, vp]
        L.rtoss_select_patterns_batch.restype = i
        L.rtoss_select_patterns_batch.argtypes = [ctypes.POINTER(SelectItem), i, i, u16p, i, vp]
        L.rtoss_pattern_histogram.restype = i
        L.rtoss_pattern_histogram.argtypes = [vp, i64, i, vp, vp]
        L.rtoss_reduce_dict.restype = i
        L.rtoss_reduce_dict.argtypes = [u16p, i, ctypes.POINTER(ctypes.c_uint32), i, u16p, ctypes.POINTER(ctypes.c_uint8)]
        L.rtoss_pack_size.restype = i
        L.rtoss_pack_size.argtypes = [ctypes.POINTER(WDesc), u16p, i, szp, szp]
        L.rtoss_pack.restype = i
        L.rtoss_pack.argtypes = [ctypes.POINTER(WDesc), vp, vp, u16p, i, vp, ctypes.c_size_t, vp, ctypes.c_size_t, vp]
        L.rtoss_conv2d_pattern.restype = i
        L.rtoss_conv2d_pattern.argtypes = [ctypes.POINTER(WDesc), ctypes.POINTER(CDesc), u16p, i, vp, vp, vp, vp]
        L.rtoss_pack_batch.restype = i
        L.rtoss_pack_batch.argtypes = [ctypes.POINTER(PackItemDesc), i, u16p, i, vp]
        L.rtoss_conv2d_pattern_fused.restype = i
        L.rtoss_conv2d_pattern_fused.argtypes = [ctypes.POINTER(WDesc), ctypes.POINTER(CDesc), ctypes.POINTER(EpilogueDesc),
                                                 u16p, i, vp, vp, vp, vp]
        L.rtoss_pack_size_coherent.restype = i
        L.rtoss_pack_size_coherent.argtypes = [ctypes.POINTER(WDesc), u16p, i, szp, szp]
        L.rtoss_pack_coherent.restype = i
        L.rtoss_pack_coherent.argtypes = [ctypes.POINTER(WDesc), vp, vp, u16p, i, vp, ctypes.c_size_t, vp]
        L.rtoss_conv2d_pattern_coherent.restype = i
        L.rtoss_conv2d_pattern_coherent.argtypes = [ctypes.POINTER(WDesc), ctypes.POINTER(CDesc), ctypes.POINTER(EpilogueDesc),
                                                    u16p, i, vp, vp, vp, vp]
        _lib = L
    return _lib


def _check(st):
    if st != OK:
        raise RtossError(st, lib().rtoss_last_error().decode())


def _masks_arg(masks):
    if masks is None:
        return None, 0, None
    m = np.ascontiguousarray(masks, dtype=np.uint16)
    return m.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), int(m.size), m


def rtoss_last_error():
    return lib().rtoss_last_error().decode()


def rtoss_pattern_dict(k, rule=RULE_CONNECTED4):
    """Host-side dictionary: uint16 masks of the k-entry patterns that pass `rule`."""
    P = ctypes.c_int(0)
    _check(lib().rtoss_pattern_dict(int(k), int(rule), None, 0, ctypes.byref(P)))
    masks = np.zeros(P.value, dtype=np.uint16)
    _check(lib().rtoss_pattern_dict(int(k), int(rule), masks.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)),
                                    P.value, ctypes.byref(P)))
    return masks


def rtoss_select_patterns(w_ptr, dt, n_elems, masks, idx_ptr, stream=0):
    mp, P, _keep = _masks_arg(masks)
    _check(lib().rtoss_select_patterns(w_ptr, int(dt), int(n_elems), mp, P, idx_ptr, stream))


def rtoss_select_patterns_batch(items, dt, masks, stream=0):
    """items: sequence of (w_ptr, n_elems, idx_ptr)."""
    mp, P, _keep = _masks_arg(masks)
    if items is None:
        _check(lib().rtoss_select_patterns_batch(None, 1, int(dt), mp, P, stream))
        return
    arr = (SelectItem * max(len(items), 1))()
    for i, (w_ptr, n, idx_ptr) in enumerate(items):
        arr[i] = SelectItem(w_ptr, int(n), idx_ptr)
    _check(lib().rtoss_select_patterns_batch(arr, len(items), int(dt), mp, P, stream))


def rtoss_pattern_histogram(idx_ptr, G, P, hist_ptr, stream=0):
    _check(lib().rtoss_pattern_histogram(idx_ptr, int(G), int(P), hist_ptr, stream))


def rtoss_reduce_dict(masks, hist, M):
    """Host only: the M most used patterns in dictionary order, and their original indices."""
    mp, P, _keep = _masks_arg(masks)
    h = None if hist is None else np.ascontiguousarray(hist, dtype=np.uint32)
    n = max(int(M), 1) if M is not None else 1
    out = np.zeros(n, dtype=np.uint16)
    kept = np.zeros(n, dtype=np.uint8)
    _check(lib().rtoss_reduce_dict(mp, P, None if h is None else h.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)), int(M),
                                   out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)),
                                   kept.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))))
    return out, kept


def rtoss_pack_size(wdesc, masks):
    mp, P, _keep = _masks_arg(masks)
    a, b = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(lib().rtoss_pack_size(ctypes.byref(wdesc) if wdesc is not None else None, mp, P, ctypes.byref(a),
                                 ctypes.byref(b)))
    return a.value, b.value


def rtoss_pack(wdesc, w_ptr, idx_ptr, masks, packed_ptr, packed_bytes, workspace_ptr=0, workspace_bytes=0, stream=0):
    mp, P, _keep = _masks_arg(masks)
    _check(lib().rtoss_pack(ctypes.byref(wdesc) if wdesc is not None else None, w_ptr, idx_ptr, mp, P, packed_ptr,
                            packed_bytes, workspace_ptr, workspace_bytes, stream))


def rtoss_conv2d_pattern(wdesc, cdesc, masks, packed_ptr, x_ptr, y_ptr, stream=0):
    mp, P, _keep = _masks_arg(masks)
    _check(lib().rtoss_conv2d_pattern(ctypes.byref(wdesc) if wdesc is not None else None,
                                      ctypes.byref(cdesc) if cdesc is not None else None, mp, P, packed_ptr, x_ptr,
                                      y_ptr, stream))


def rtoss_conv2d_pattern_fused(wdesc, cdesc, epilogue, masks, packed_ptr, x_ptr, y_ptr, stream=0):
    """epilogue: EpilogueDesc (scale, bias, activation, residual)."""
    mp, P, _keep = _masks_arg(masks)
    _check(lib().rtoss_conv2d_pattern_fused(ctypes.byref(wdesc) if wdesc is not None else None,
                                            ctypes.byref(cdesc) if cdesc is not None else None,
                                            ctypes.byref(epilogue) if epilogue is not None else None, mp, P,
                                            packed_ptr, x_ptr, y_ptr, stream))


def rtoss_pack_size_coherent(wdesc, masks):
    """(packed bytes, byte offset of the per-(stage, channel block) step records)."""
    mp, P, _keep = _masks_arg(masks)
    a, b = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(lib().rtoss_pack_size_coherent(ctypes.byref(wdesc) if wdesc is not None else None, mp, P, ctypes.byref(a),
                                          ctypes.byref(b)))
    return a.value, b.value


def rtoss_pack_coherent(wdesc, w_ptr, idx_ptr, masks, packed_ptr, packed_bytes, stream=0):
    mp, P, _keep = _masks_arg(masks)
    _check(lib().rtoss_pack_coherent(ctypes.byref(wdesc) if wdesc is not None else None, w_ptr, idx_ptr, mp, P, packed_ptr,
                                     packed_bytes, stream))


def rtoss_conv2d_pattern_coherent(wdesc, cdesc, epilogue, masks, packed_ptr, x_ptr, y_ptr, stream=0):
    mp, P, _keep = _masks_arg(masks)
    _check(lib().rtoss_conv2d_pattern_coherent(ctypes.byref(wdesc) if wdesc is not None else None,
                                               ctypes.byref(cdesc) if cdesc is not None else None,
                                               ctypes.byref(epilogue) if epilogue is not None else None, mp, P,
                                               packed_ptr, x_ptr, y_ptr, stream))


def rtoss_pack_batch(items, masks, stream=0):
    """items: sequence of (wdesc, w_ptr, idx_ptr, packed_ptr, packed_bytes)."""
    mp, P, _keep = _masks_arg(masks)
    if items is None:
        _check(lib().rtoss_pack_batch(None, 1, mp, P, stream))
        return
    arr = (PackItemDesc * max(len(items), 1))()
    for i, (wd, w_ptr, idx_ptr, packed_ptr, packed_bytes) in enumerate(items):
        arr[i] = PackItemDesc(wd, w_ptr, idx_ptr, packed_ptr, int(packed_bytes))
    _check(lib().rtoss_pack_batch(arr, len(items), mp, P, stream))


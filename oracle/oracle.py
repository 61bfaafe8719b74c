"""ctypes loader for rtoss_oracle.c (test infrastructure; see that file's header).

Every function takes and returns numpy float64 / integer arrays in the logical layouts of
the paper's tensors: weights [Co][Ci][ks][ks], activations [N][C][H][W].
"""
import ctypes
import os
import subprocess

import numpy as np

RULE_ALL, RULE_ANYPAIR4, RULE_CONNECTED4, RULE_CONNECTED8 = 0, 1, 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rtoss_oracle.c")
_LIB = os.path.join(_HERE, "librtoss_oracle.so")
_lib = None


def build(force=False):
    """Compile the C oracle with gcc (no fast-math, no FMA contraction, OpenMP over outputs)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
             "-Wall", "-Wextra", "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        c_dp = ctypes.POINTER(ctypes.c_double)
        c_u16p = ctypes.POINTER(ctypes.c_uint16)
        c_u8p = ctypes.POINTER(ctypes.c_uint8)
        c_i32p = ctypes.POINTER(ctypes.c_int32)
        i, i64 = ctypes.c_int, ctypes.c_int64
        lib.rtoss_oracle_pattern_dict.argtypes = [i, i, c_u16p, i]
        lib.rtoss_oracle_pattern_dict.restype = i
        lib.rtoss_oracle_select.argtypes = [c_dp, i64, c_u16p, i, c_u8p]
        lib.rtoss_oracle_select.restype = None
        lib.rtoss_oracle_mask.argtypes = [c_dp, i64, c_u16p, c_u8p, c_dp]
        lib.rtoss_oracle_mask.restype = None
        lib.rtoss_oracle_conv2d.argtypes = [c_dp, c_dp, c_dp, i, i, i, i, i, i, i, i, i]
        lib.rtoss_oracle_conv2d.restype = None
        lib.rtoss_oracle_conv2d_points.argtypes = [c_dp, c_dp, c_i32p, i64, c_dp, i, i, i, i, i, i, i]
        lib.rtoss_oracle_conv2d_points.restype = None
        lib.rtoss_oracle_conv2d_live3x3.argtypes = [c_dp, c_dp, c_u16p, c_u8p, c_dp, i, i, i, i, i, i, i]
        lib.rtoss_oracle_conv2d_live3x3.restype = None
        lib.rtoss_oracle_threads.argtypes = []
        lib.rtoss_oracle_threads.restype = i
        _lib = lib
    return _lib


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _u16(a):
    a = np.ascontiguousarray(a, dtype=np.uint16)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def _u8(a):
    a = np.ascontiguousarray(a, dtype=np.uint8)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8))


def threads():
    return int(_load().rtoss_oracle_threads())


def pattern_dict(k, rule=RULE_CONNECTED4):
    """Section IV.B: bit masks (uint16, bit t = tap t) of the k-entry patterns that pass `rule`."""
    lib = _load()
    n = lib.rtoss_oracle_pattern_dict(int(k), int(rule), None, 0)
    if n < 0:
        raise ValueError("bad k or rule")
    masks = np.zeros(n, dtype=np.uint16)
    lib.rtoss_oracle_pattern_dict(int(k), int(rule), masks.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)), n)
    return masks


def select(w, masks):
    """Section IV.C / IV.D: best pattern index per group of 9 contiguous weights of w.ravel()."""
    w, wp = _f64(np.asarray(w).reshape(-1))
    masks, mp = _u16(masks)
    idx = np.zeros(w.size // 9, dtype=np.uint8)
    _load().rtoss_oracle_select(wp, w.size, mp, masks.size, idx.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)))
    return idx


def mask(w, masks, idx):
    """W (.) mask[idx] on the flat view, tail (size % 9 elements) zeroed; same shape as w."""
    shape = np.asarray(w).shape
    w, wp = _f64(np.asarray(w).reshape(-1))
    masks, mp = _u16(masks)
    idx, ip = _u8(idx)
    assert idx.size == w.size // 9
    out = np.empty_like(w)
    _load().rtoss_oracle_mask(wp, w.size, mp, ip, out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    return out.reshape(shape)


def _out_hw(H, W, ks, stride, pad):
    return (H + 2 * pad - ks) // stride + 1, (W + 2 * pad - ks) // stride + 1


def conv2d(x, w, stride=1, pad=None, relu=False):
    """Direct fp64 cross-correlation. x [N,Ci,H,W], w [Co,Ci,ks,ks] (already masked) -> y [N,Co,Ho,Wo]."""
    x, xp = _f64(x)
    w, wp = _f64(w)
    N, Ci, H, W = x.shape
    Co, Ci2, ks, ks2 = w.shape
    assert Ci == Ci2 and ks == ks2
    if pad is None:
        pad = ks // 2
    Ho, Wo = _out_hw(H, W, ks, stride, pad)
    y = np.empty((N, Co, Ho, Wo), dtype=np.float64)
    _load().rtoss_oracle_conv2d(xp, wp, y.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), N, Ci, H, W, Co, ks,
                                int(stride), int(pad), int(bool(relu)))
    return y


def conv2d_points(x, w, pts, stride=1, pad=None, relu=False):
    """The same sum as conv2d for a list of output coordinates pts[i] = (n, co, oh, ow)."""
    x, xp = _f64(x)
    w, wp = _f64(w)
    N, Ci, H, W = x.shape
    Co, Ci2, ks, _ = w.shape
    assert Ci == Ci2
    if pad is None:
        pad = ks // 2
    pts = np.ascontiguousarray(pts, dtype=np.int32).reshape(-1, 4)
    Ho, Wo = _out_hw(H, W, ks, stride, pad)
    assert (pts >= 0).all() and (pts[:, 0] < N).all() and (pts[:, 1] < Co).all()
    assert (pts[:, 2] < Ho).all() and (pts[:, 3] < Wo).all()
    out = np.empty(pts.shape[0], dtype=np.float64)
    _load().rtoss_oracle_conv2d_points(xp, wp, pts.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), pts.shape[0],
                                       out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), Ci, H, W, ks,
                                       int(stride), int(pad), int(bool(relu)))
    return out


def conv2d_live3x3(x, w, masks, idx, stride=1, relu=False):
    """3x3 pad-1 conv that visits only the live taps of each kernel; w is the UNMASKED tensor."""
    x, xp = _f64(x)
    w, wp = _f64(w)
    masks, mp = _u16(masks)
    idx, ip = _u8(idx)
    N, Ci, H, W = x.shape
    Co = w.shape[0]
    assert w.shape == (Co, Ci, 3, 3) and idx.size == Co * Ci
    Ho, Wo = _out_hw(H, W, 3, stride, 1)
    y = np.empty((N, Co, Ho, Wo), dtype=np.float64)
    _load().rtoss_oracle_conv2d_live3x3(xp, wp, mp, ip, y.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), N, Ci, H,
                                        W, Co, int(stride), int(bool(relu)))
    return y


def histogram(idx, P):
    """Section IV.B, second narrowing criterion: how often each of the P patterns was selected.
    Plain count; indices >= P are ignored."""
    idx = np.asarray(idx).reshape(-1).astype(np.int64)
    counts = np.zeros(P, dtype=np.int64)
    for p in range(P):
        counts[p] = int(np.count_nonzero(idx == p))
    return counts


def reduce_dict(masks, counts, M):
    """Section IV.B, second narrowing criterion: the M most used patterns.  Ranking: higher count first,
    lower index first among equal counts; the kept patterns stay in their original order.
    Returns (masks[kept], kept)."""
    masks = np.asarray(masks)
    counts = np.asarray(counts)
    assert 1 <= M <= len(masks) == len(counts)
    ranked = sorted(range(len(masks)), key=lambda p: (-int(counts[p]), p))
    kept = np.array(sorted(ranked[:M]), dtype=np.int64)
    return masks[kept], kept


ACT_NONE, ACT_RELU, ACT_SILU = 0, 1, 2


def conv2d_fused(x, w, stride=1, pad=None, scale=None, bias=None, act=ACT_NONE, residual=None):
    """Convolution followed by the output stage of a detector block, written out term by term:
        y = act(scale[co] * conv(x, w) + bias[co]) + residual
    act: none, ReLU max(v, 0), or SiLU v * sigmoid(v) = v / (1 + exp(-v)).  All in float64."""
    y = conv2d(x, w, stride=stride, pad=pad, relu=False)
    Co = y.shape[1]
    if scale is not None:
        y = y * np.asarray(scale, dtype=np.float64).reshape(1, Co, 1, 1)
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64).reshape(1, Co, 1, 1)
    if act == ACT_RELU:
        y = np.maximum(y, 0.0)
    elif act == ACT_SILU:
        y = y / (1.0 + np.exp(-y))
    elif act != ACT_NONE:
        raise ValueError("unknown activation")
    if residual is not None:
        y = y + np.asarray(residual, dtype=np.float64)
    return y


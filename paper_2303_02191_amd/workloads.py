"""Seeded synthetic workloads and dtype plumbing shared by the tests and the benchmark.

This module holds no arithmetic of the method: it only draws random tensors of the shapes
the five configurations name, rounds them once to the configured dtype, and converts
between storage bits and exact float64 values.  Both the CPU oracle's tests and the GPU
path's tests take their inputs from here, so the two sides see identical bits.

Shapes follow the paper's setting (Section V.A: 640x640 frames, YOLOv5s and RetinaNet) but
every tensor is random: no dataset record and no trained weight is reproduced.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

F32, F16, BF16 = 0, 1, 2
DTYPE_NAMES = {F32: "f32", F16: "f16", BF16: "bf16"}
ELEM_BYTES = {F32: 4, F16: 2, BF16: 2}


# --------------------------------------------------------------------------------------
# dtype plumbing: float64 <-> storage bits.  bfloat16 has no numpy type, so it travels as
# uint16 bit patterns.
# --------------------------------------------------------------------------------------
def round_to_dtype(a64, dt):
    """Round a float64 array once (round-to-nearest-even) to `dt`; returns the storage array
    (float32, float16, or uint16 holding bfloat16 bits)."""
    a64 = np.asarray(a64, dtype=np.float64)
    if dt == F32:
        return a64.astype(np.float32)
    if dt == F16:
        return a64.astype(np.float16)
    if dt == BF16:
        f32 = a64.astype(np.float32)  # double rounding is avoided below by working on the f32 bits
        # float64 -> float32 -> bfloat16 could double-round; redo from float64 where the
        # float32 value is not exactly the float64 value and sits on a bfloat16 tie.
        bits = f32.view(np.uint32).astype(np.uint64)
        lower = bits & 0xFFFF
        tie = lower == 0x8000
        inexact = f32.astype(np.float64) != a64
        rounded = (bits + 0x7FFF + ((bits >> 16) & 1)) >> 16
        if np.any(tie & inexact):
            # break the tie by the sign of the float32 rounding error
            up = np.abs(a64) > np.abs(f32.astype(np.float64))
            fix = tie & inexact
            rounded = np.where(fix, (bits >> 16) + up.astype(np.uint64), rounded)
        nan = np.isnan(a64)
        rounded = np.where(nan, 0x7FC0, rounded)
        return rounded.astype(np.uint16)
    raise ValueError("unknown dtype %r" % (dt,))


def to_f64(store, dt):
    """Exact float64 value of a storage array produced by round_to_dtype."""
    if dt == BF16:
        s = np.asarray(store, dtype=np.uint16)
        return (s.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return np.asarray(store).astype(np.float64)


def nchw_to_nhwc(a):
    return np.ascontiguousarray(np.transpose(a, (0, 2, 3, 1)))


def nhwc_to_nchw(a):
    return np.ascontiguousarray(np.transpose(a, (0, 3, 1, 2)))


# --------------------------------------------------------------------------------------
# configurations
# --------------------------------------------------------------------------------------
@dataclass
class Layer:
    Ci: int
    Co: int
    H: int  # input height
    W: int  # input width
    ksize: int  # 1 or 3
    stride: int  # 1 or 2
    relu: bool = False

    @property
    def pad(self):
        return self.ksize // 2

    @property
    def Ho(self):
        return (self.H + 2 * self.pad - self.ksize) // self.stride + 1

    @property
    def Wo(self):
        return (self.W + 2 * self.pad - self.ksize) // self.stride + 1

    @property
    def n_weights(self):
        return self.Co * self.Ci * self.ksize * self.ksize

    @property
    def groups(self):
        return self.n_weights // 9


@dataclass
class Config:
    name: str
    N: int
    dtype: int
    k: int
    seed: int
    x_dist: str  # "normal" or "uniform"
    w_std: float
    layers: List[Layer] = field(default_factory=list)
    chained: bool = False  # layer l+1 consumes layer l's output instead of a fresh draw

    def nonzero_macs(self):
        return sum(self.N * L.Ho * L.Wo * self.k * L.groups for L in self.layers)

    def dense_macs(self):
        return sum(self.N * L.Ho * L.Wo * L.n_weights for L in self.layers)

    def algorithmic_bytes(self):
        """Input once + output once + k values and one index byte per group, per layer."""
        eb = ELEM_BYTES[self.dtype]
        tot = 0
        for L in self.layers:
            tot += self.N * L.Ci * L.H * L.W * eb + self.N * L.Co * L.Ho * L.Wo * eb
            tot += L.groups * (self.k * eb + 1)
        return tot


def _yolo5s_shaped_layers():
    """57 conv layers, 18 of them 3x3 and 39 of them 1x1 (68.42 %, the share Section III
    quotes for YOLOv5), widths 32..512 at a 640x640 frame.  (Ci, Co, H_in, ksize, stride)."""
    t = []

    def add(ci, co, h, ks, s, times=1):
        for _ in range(times):
            t.append(Layer(ci, co, h, h, ks, s))

    def block(cin, mid, h, reps, cout):
        add(cin, mid, h, 1, 1, 2)
        for _ in range(reps):
            add(mid, mid, h, 1, 1)
            add(mid, mid, h, 3, 1)
        add(cout, cout, h, 1, 1)

    add(3, 32, 640, 3, 2)
    add(32, 64, 320, 3, 2)
    block(64, 32, 160, 1, 64)
    add(64, 128, 160, 3, 2)
    block(128, 64, 80, 2, 128)
    add(128, 256, 80, 3, 2)
    block(256, 128, 40, 3, 256)
    add(256, 512, 40, 3, 2)
    block(512, 256, 20, 1, 512)
    add(512, 256, 20, 1, 1)
    add(1024, 512, 20, 1, 1)
    add(512, 256, 20, 1, 1)
    block(512, 128, 40, 1, 256)
    add(256, 128, 40, 1, 1)
    block(256, 64, 80, 1, 128)
    add(128, 128, 80, 3, 2)
    block(256, 128, 40, 1, 256)
    add(256, 256, 40, 3, 2)
    block(512, 256, 20, 1, 512)
    return t


def get_config(i: int) -> Config:
    """The five configurations (1-based)."""
    if i == 1:
        return Config("cfg1_single3x3_f32_4EP", 1, F32, 4, 0, "normal", 0.05, [Layer(64, 64, 56, 56, 3, 1)])
    if i == 2:
        chans = [(3, 32, 640), (32, 64, 320), (64, 128, 160), (128, 256, 80), (256, 512, 40)]
        return Config("cfg2_yolo5s_backbone3x3_f16_3EP", 1, F16, 3, 2, "normal", 0.02,
                      [Layer(ci, co, h, h, 3, 2) for ci, co, h in chans])
    if i == 3:
        return Config("cfg3_1x1_f16_2EP", 8, F16, 2, 3, "uniform", 0.03, [Layer(256, 256, 80, 80, 1, 1)])
    if i == 4:
        layers = [Layer(256, 256, 100, 168, 3, 1, relu=(j < 3)) for j in range(4)]
        return Config("cfg4_retinanet_head_bf16_3EP", 4, BF16, 3, 4, "normal", 0.01, layers, chained=True)
    if i == 5:
        return Config("cfg5_yolo5s_convset_f16_2EP", 16, F16, 2, 5, "normal", 0.02, _yolo5s_shaped_layers())
    raise ValueError("config index must be 1..5")


def draw_x(rng, cfg: Config, L: Layer, N: Optional[int] = None):
    """Activation tensor [N, Ci, H, W] as (storage array in cfg.dtype, exact float64 values)."""
    n = cfg.N if N is None else N
    shape = (n, L.Ci, L.H, L.W)
    a = rng.standard_normal(shape) if cfg.x_dist == "normal" else rng.uniform(-1.0, 1.0, shape)
    s = round_to_dtype(a, cfg.dtype)
    return s, to_f64(s, cfg.dtype)


def draw_w(rng, cfg: Config, L: Layer):
    """Weight tensor [Co, Ci, ks, ks] as (storage array in cfg.dtype, exact float64 values)."""
    a = rng.standard_normal((L.Co, L.Ci, L.ksize, L.ksize)) * cfg.w_std
    s = round_to_dtype(a, cfg.dtype)
    return s, to_f64(s, cfg.dtype)


def draw_random_kernels(seed, n_kernels, dtype):
    """n_kernels 3x3 kernels with iid U[-1, 1] weights (the random kernels of Section IV.B's usage
    count), rounded once to dtype: (storage array [n, 9], exact float64 values)."""
    a = np.random.default_rng(seed).uniform(-1.0, 1.0, (n_kernels, 9))
    s = round_to_dtype(a, dtype)
    return s, to_f64(s, dtype)


def make_rng(cfg: Config):
    return np.random.default_rng(cfg.seed)

"""GPU parity: rtoss_conv2d_pattern vs the oracle's direct fp64 convolution.

Tolerances: fp32 tensors  max|y - ref| <= 1e-5 * max|ref|;
            fp16 / bf16 tensors with fp32 output  max|y - ref| <= 2e-3 * rms(ref);
            16-bit output must equal the fp32 output rounded once to nearest-even.
"""
import numpy as np
import pytest

import oracle
from paper_2303_02191_amd import binding as B
from paper_2303_02191_amd import workloads as wl

from gpu_util import GpuLayer, decode_live_section

pytestmark = pytest.mark.gpu


def check(y, ref, dt):
    y = np.asarray(y, dtype=np.float64)
    err = np.max(np.abs(y - ref))
    if dt == wl.F32:
        bound = 1e-5 * np.max(np.abs(ref))
    else:
        bound = 2e-3 * np.sqrt(np.mean(ref ** 2))
    assert err <= bound, "max err %.3e > bound %.3e" % (err, bound)


def run_case(dt, N, Ci, Co, H, W, ks, stride, k, relu, seed, x_dist="normal", w_std=0.05, rule=B.RULE_CONNECTED4):
    rng = np.random.default_rng(seed)
    masks = B.rtoss_pattern_dict(k, rule)
    xa = rng.standard_normal((N, Ci, H, W)) if x_dist == "normal" else rng.uniform(-1, 1, (N, Ci, H, W))
    xs = wl.round_to_dtype(xa, dt)
    ws = wl.round_to_dtype(rng.standard_normal((Co, Ci, ks, ks)) * w_std, dt)
    xv, wv = wl.to_f64(xs, dt), wl.to_f64(ws, dt)
    idx = oracle.select(wv, masks)
    ref = oracle.conv2d(xv, oracle.mask(wv, masks, idx), stride=stride, relu=relu)
    g = GpuLayer(ws, dt, masks, k)
    assert np.array_equal(g.idx_host(), idx)
    y32 = g.conv_nchw(xs, stride=stride, relu=relu, out_dt=wl.F32)
    assert y32.shape == ref.shape and y32.dtype == np.float32
    check(y32, ref, dt)
    if dt != wl.F32:
        y16 = g.conv_nchw(xs, stride=stride, relu=relu)
        assert np.array_equal(y16, wl.round_to_dtype(y32.astype(np.float64), dt))
    return y32, ref


SMALL = [
    # N, Ci, Co, H,  W, ks, stride, k, relu
    (1, 3, 32, 20, 20, 3, 2, 3, False),
    (2, 16, 40, 9, 13, 3, 1, 2, True),
    (1, 64, 64, 17, 23, 3, 1, 3, False),
    (1, 64, 64, 17, 23, 3, 2, 3, True),
    (3, 5, 7, 8, 8, 3, 1, 4, False),
    (1, 1, 1, 1, 1, 3, 1, 2, False),
    (1, 8, 8, 1, 5, 3, 2, 3, False),
    (2, 32, 48, 10, 12, 1, 1, 2, False),
    (1, 13, 7, 5, 6, 1, 1, 3, True),
    (1, 256, 64, 6, 6, 1, 1, 2, False),
    (1, 2, 2, 3, 3, 1, 1, 2, False),  # fewer than 9 weights: everything is tail, output is zero
]


@pytest.mark.parametrize("dt", [wl.F32, wl.F16, wl.BF16])
@pytest.mark.parametrize("case", SMALL)
def test_conv_small_shapes(dt, case):
    N, Ci, Co, H, W, ks, stride, k, relu = case
    run_case(dt, N, Ci, Co, H, W, ks, stride, k, relu, seed=hash(case) % 10000 + dt)


MATRIX_CORE = [
    # shapes that take the matrix-core path (Ci % 32 == 0, Co % 16 == 0, 16-bit types):
    # ragged tiles, several channel blocks, odd extents, batch > 1
    # N, Ci, Co,  H,  W, stride, k, relu
    (1, 32, 16, 4, 4, 1, 3, False),
    (1, 32, 16, 5, 7, 1, 2, True),
    (2, 96, 48, 19, 21, 1, 3, False),
    (1, 64, 144, 33, 18, 1, 2, False),
    (1, 32, 272, 16, 16, 1, 3, True),
    (3, 64, 128, 16, 35, 1, 3, False),
    (1, 256, 256, 20, 24, 1, 3, False),
    (1, 32, 16, 7, 9, 2, 3, False),
    (2, 64, 80, 37, 41, 2, 2, True),
    (1, 128, 256, 40, 40, 2, 3, False),
    (1, 32, 32, 1, 1, 1, 3, False),
    (1, 32, 32, 2, 70, 2, 2, False),
    # enough 16x16 tiles for two rounds over the compute units but one round of 20x16 tiles: the
    # launcher takes the tall tile (5 position blocks per wave), here with ragged rows and columns
    (43, 128, 48, 37, 30, 1, 3, True),
    (130, 160, 16, 21, 16, 1, 2, False),
    # the pipelined kernel (more than 64 channels in and out, at least 200 tiles of 16x16 positions x 128
    # channels): 20x16 tiles with ragged rows and columns and a partial group of 64 output channels ...
    (43, 128, 80, 37, 30, 1, 3, True),
    # ... and 16x16 tiles, three stages, two channel blocks of which the second is mostly padding
    (13, 96, 144, 64, 50, 1, 2, False),
]


@pytest.mark.parametrize("dt", [wl.F16, wl.BF16])
@pytest.mark.parametrize("case", MATRIX_CORE)
def test_conv3x3_matrix_core_shapes(dt, case):
    N, Ci, Co, H, W, stride, k, relu = case
    run_case(dt, N, Ci, Co, H, W, 3, stride, k, relu, seed=hash(case) % 10000 + dt, w_std=0.02)


DENSE_MODE = [
    # dictionaries with three corners or three edge midpoints in one pattern: dense mode on the matrix
    # cores (every tap a dense step, pruned weights explicit zeros)
    # N, Ci, Co,  H,  W, stride, k, rule, relu
    (1, 32, 16, 4, 4, 1, 4, B.RULE_CONNECTED4, False),
    (2, 96, 48, 19, 21, 1, 4, B.RULE_CONNECTED4, True),
    (1, 64, 144, 33, 18, 1, 5, B.RULE_CONNECTED4, False),
    (3, 64, 128, 16, 35, 1, 3, B.RULE_ALL, False),
    (1, 256, 256, 20, 24, 1, 4, B.RULE_CONNECTED8, True),
    (1, 32, 16, 7, 9, 2, 4, B.RULE_CONNECTED4, False),
    (2, 64, 80, 37, 41, 2, 5, B.RULE_CONNECTED4, True),
    (1, 128, 256, 40, 40, 2, 4, B.RULE_CONNECTED4, False),
    (1, 32, 32, 1, 1, 1, 8, B.RULE_CONNECTED4, False),
]


@pytest.mark.parametrize("dt", [wl.F16, wl.BF16])
@pytest.mark.parametrize("case", DENSE_MODE)
def test_conv3x3_dense_mode_shapes(dt, case):
    N, Ci, Co, H, W, stride, k, rule, relu = case
    run_case(dt, N, Ci, Co, H, W, 3, stride, k, relu, seed=hash(case) % 10000 + dt, w_std=0.02, rule=rule)


THREE_GROUP_LAYOUT = [
    # 4-entry edge-connected patterns: the T shapes keep three edge midpoints, so the corner / edge-midpoint split
    # does not fit them; the taps are laid out as three 2-of-4 groups {0,4,8}, {1,5,6}, {2,3,7} instead (6 sparse
    # steps per 32 channels, no dense step).  Shapes for every tile variant of that path.
    # N, Ci, Co,  H,  W, stride, relu
    (1, 32, 16, 5, 7, 1, True),
    (2, 64, 144, 33, 18, 1, False),
    (3, 128, 128, 16, 35, 1, False),
    (2, 256, 256, 40, 40, 1, True),
    (1, 32, 64, 33, 37, 2, False),
    (2, 64, 80, 37, 41, 2, True),
    (2, 256, 272, 20, 24, 2, False),
]


@pytest.mark.parametrize("dt", [wl.F16, wl.BF16])
@pytest.mark.parametrize("case", THREE_GROUP_LAYOUT)
def test_conv3x3_four_entry_patterns_on_the_sparse_instruction(dt, case):
    N, Ci, Co, H, W, stride, relu = case
    masks = B.rtoss_pattern_dict(4)
    # the packed blob must be the compressed format (6 fragments + 3 index words per tile), not the 9 dense ones
    nbytes, _ = B.rtoss_pack_size(B.WDesc(Co, Ci, 3, 4, dt), masks)
    tiles = (Ci // 32) * (((Co + 15) // 16 + 7) // 8 * 8)
    assert nbytes < tiles * 7200 + Co * Ci * 9 + 8192
    run_case(dt, N, Ci, Co, H, W, 3, stride, 4, relu, seed=hash(case) % 10000 + dt, w_std=0.02)


FP32_MATRIX_CORE = [
    # fp32 tensors with Ci % 16 == 0 and Co % 16 == 0: dense mode on the fp32 matrix instruction, small
    # launches (16 channels x 4x16 positions per workgroup) and large ones (64 channels x 16x16)
    # N, Ci, Co,  H,  W, stride, k, relu
    (1, 16, 16, 4, 4, 1, 3, False),
    (1, 64, 64, 56, 56, 1, 4, False),
    (2, 48, 80, 19, 21, 1, 2, True),
    (1, 32, 48, 33, 18, 2, 3, False),
    (16, 16, 64, 64, 64, 1, 3, True),
    (20, 16, 32, 63, 65, 2, 2, False),
]


@pytest.mark.parametrize("case", FP32_MATRIX_CORE)
def test_conv3x3_fp32_matrix_core_shapes(case):
    N, Ci, Co, H, W, stride, k, relu = case
    run_case(wl.F32, N, Ci, Co, H, W, 3, stride, k, relu, seed=hash(case) % 10000, w_std=0.05)


def test_conv3x3_matrix_core_dictionaries():
    # every pair of taps (36 patterns): still at most 2 corners and 2 edge midpoints -> sparse path
    run_case(wl.F16, 1, 64, 64, 12, 12, 3, 1, 2, False, seed=31, rule=B.RULE_ALL)
    # single-tap patterns
    run_case(wl.BF16, 1, 32, 32, 9, 9, 3, 1, 1, False, seed=32)
    # 4-entry connected patterns include a T shape with 3 edge midpoints -> dense mode
    run_case(wl.F16, 1, 64, 64, 12, 12, 3, 1, 4, False, seed=33)
    # identical weights in every kernel: every kernel picks pattern 0 (ties) -> coherent tiles
    masks = B.rtoss_pattern_dict(3)
    ws = np.full((32, 32, 3, 3), 0.25, dtype=np.float16)
    xs = wl.round_to_dtype(np.random.default_rng(34).standard_normal((1, 32, 8, 8)), wl.F16)
    g = GpuLayer(ws, wl.F16, masks, 3)
    assert (g.idx_host() == 0).all()
    ref = oracle.conv2d(wl.to_f64(xs, wl.F16), oracle.mask(wl.to_f64(ws, wl.F16), masks, g.idx_host()))
    check(g.conv_nchw(xs, out_dt=wl.F32), ref, wl.F16)


MATRIX_CORE_1X1 = [
    # 1x1 shapes on the matrix-core path (Ci % 32 == 0, Co % 16 == 0): ragged position tiles,
    # one / several channel blocks, groups of 9 that straddle rows (Ci % 9 != 0), deep K
    # N, Ci, Co,  H,  W, k, relu
    (1, 32, 16, 1, 1, 2, False),
    (1, 32, 32, 9, 13, 2, True),
    (2, 64, 48, 11, 12, 3, False),
    (1, 128, 144, 16, 8, 2, False),
    (3, 256, 272, 7, 19, 2, True),
    (1, 1024, 512, 5, 5, 2, False),
    (2, 512, 128, 20, 20, 2, False),
    (1, 288, 64, 6, 7, 3, False),  # Ci % 9 == 0: groups never straddle rows
    (1, 96, 32, 13, 11, 2, True),  # Ci / 32 not a power of two: ring kernel with weights in LDS
    # streaming kernel (Ci = 32 * 2^n): every (depth, wave split) variant, many buffers per workgroup,
    # ragged last buffer, channel counts that do not fill the workgroup's channel span
    (4, 64, 32, 40, 37, 2, False),
    (2, 32, 64, 50, 33, 2, True),
    (1, 32, 256, 30, 30, 3, False),
    (2, 64, 112, 17, 23, 2, False),
    (2, 128, 128, 33, 31, 2, True),
    (2, 128, 64, 33, 31, 3, False),
    (3, 256, 128, 29, 23, 2, False),
    (2, 256, 256, 31, 33, 2, True),
    (1, 256, 64, 40, 40, 2, False),
    (1, 512, 256, 20, 21, 2, False),
    (1, 512, 48, 9, 9, 2, True),
    (1, 1024, 80, 7, 9, 2, False),
]


@pytest.mark.parametrize("dt", [wl.F16, wl.BF16])
@pytest.mark.parametrize("case", MATRIX_CORE_1X1)
def test_conv1x1_matrix_core_shapes(dt, case):
    N, Ci, Co, H, W, k, relu = case
    run_case(dt, N, Ci, Co, H, W, 1, 1, k, relu, seed=hash(case) % 10000 + dt, x_dist="uniform", w_std=0.03)


STEM = [
    # <= 3 input channels (image stem): N, Ci, Co, H, W, stride, k, relu
    (1, 3, 32, 64, 64, 2, 2, False),
    (2, 3, 16, 37, 45, 2, 3, True),
    (1, 3, 64, 19, 70, 1, 2, False),
    (1, 1, 32, 9, 9, 1, 3, False),
    (2, 2, 48, 33, 17, 2, 2, True),
    (1, 3, 32, 1, 1, 1, 2, False),
]


@pytest.mark.parametrize("dt", [wl.F16, wl.BF16])
@pytest.mark.parametrize("case", STEM)
def test_conv3x3_stem_shapes(dt, case):
    N, Ci, Co, H, W, stride, k, relu = case
    run_case(dt, N, Ci, Co, H, W, 3, stride, k, relu, seed=hash(case) % 10000 + dt, w_std=0.1)


@pytest.mark.parametrize("ks,Ci,Co,H", [(3, 64, 32, 12), (1, 64, 48, 9), (3, 8, 8, 7)])
def test_child_layer_reuses_parent_patterns(ks, Ci, Co, H):
    # Section IV.A / IV.C: layers of one group share the kernel patterns of the group's parent layer.
    # The child is pruned and packed with the parent's index tensor (no selection of its own) and its
    # convolution is compared with the oracle's masked convolution under the same indices.
    dt, k = wl.F16, 3
    masks = B.rtoss_pattern_dict(k)
    rng = np.random.default_rng(900 + ks + Ci)
    w_parent = wl.round_to_dtype(rng.standard_normal((Co, Ci, ks, ks)) * 0.05, dt)
    w_child = wl.round_to_dtype(rng.standard_normal((Co, Ci, ks, ks)) * 0.05, dt)
    xs = wl.round_to_dtype(rng.standard_normal((2, Ci, H, H)), dt)
    parent = GpuLayer(w_parent, dt, masks, k)
    child = GpuLayer(w_child, dt, masks, k, idx=parent.idx)
    idx = parent.idx_host()
    assert np.array_equal(idx, oracle.select(wl.to_f64(w_parent, dt), masks))
    pruned_child = oracle.mask(wl.to_f64(w_child, dt), masks, idx)
    dec, dec_idx = decode_live_section(child.blob_host(), Co, Ci, ks, k, dt, masks)
    assert np.array_equal(dec_idx, idx)
    assert np.array_equal(wl.to_f64(dec, dt), pruned_child)
    check(child.conv_nchw(xs, out_dt=wl.F32), oracle.conv2d(wl.to_f64(xs, dt), pruned_child), dt)


def test_conv_all_ones_pattern_is_dense():
    # k = 9: one pattern that keeps every tap -> ordinary dense convolution
    run_case(wl.F16, 1, 16, 16, 9, 9, 3, 1, 9, False, seed=1, rule=B.RULE_ALL)
    run_case(wl.F32, 1, 8, 8, 7, 7, 3, 2, 9, False, seed=2, rule=B.RULE_ALL)


def test_conv_other_dictionaries():
    run_case(wl.F16, 1, 32, 32, 12, 12, 3, 1, 3, False, seed=3, rule=B.RULE_ALL)        # 84 patterns
    run_case(wl.BF16, 1, 32, 32, 12, 12, 3, 1, 4, True, seed=4, rule=B.RULE_CONNECTED8)  # 85 patterns
    run_case(wl.F16, 1, 32, 32, 12, 12, 3, 2, 5, False, seed=5)


def test_cfg1_full():
    cfg = wl.get_config(1)
    L = cfg.layers[0]
    rng = wl.make_rng(cfg)
    xs, xv = wl.draw_x(rng, cfg, L)
    ws, wv = wl.draw_w(rng, cfg, L)
    masks = B.rtoss_pattern_dict(cfg.k)
    assert masks.size == 36
    idx = oracle.select(wv, masks)
    ref = oracle.conv2d(xv, oracle.mask(wv, masks, idx), stride=1)
    g = GpuLayer(ws, cfg.dtype, masks, cfg.k)
    assert np.array_equal(g.idx_host(), idx)
    check(g.conv_nchw(xs, stride=1), ref, wl.F32)


def _sample_points(rng, N, Co, Ho, Wo, n):
    pts = np.stack([rng.integers(0, N, n), rng.integers(0, Co, n), rng.integers(0, Ho, n), rng.integers(0, Wo, n)], 1)
    # always include the four corners and an edge midpoint (padding paths)
    extra = [[0, 0, 0, 0], [N - 1, Co - 1, Ho - 1, Wo - 1], [0, Co - 1, 0, Wo - 1], [N - 1, 0, Ho - 1, 0],
             [0, Co // 2, Ho // 2, 0]]
    return np.concatenate([pts, np.array(extra)]).astype(np.int32)


# The oracle's direct loop does about 1.4 G multiply-adds per second and core; a layer whose whole output
# would take it longer than this (on the cores it has) is checked on sampled outputs instead.
ORACLE_BUDGET_S = 20.0


def _oracle_seconds(N, L):
    return N * L.Ho * L.Wo * L.Co * L.Ci * L.ksize * L.ksize / (1.2e9 * max(1, oracle.threads()))


def _check_layer_full(cfg, L, xs, xv, ws, wv, masks, relu, seed, npts=4000):
    """Full-size layer in the benchmarked launch shape: selection bit-exact; EVERY output element compared
    with the oracle's direct convolution (sampled outputs only when the whole tensor would exceed
    ORACLE_BUDGET_S of oracle time)."""
    idx = oracle.select(wv, masks)
    wm = oracle.mask(wv, masks, idx)
    g = GpuLayer(ws, cfg.dtype, masks, cfg.k)
    assert np.array_equal(g.idx_host(), idx)
    y32 = g.conv_nchw(xs, stride=L.stride, relu=relu, out_dt=wl.F32)
    assert np.isfinite(y32).all()
    if _oracle_seconds(xs.shape[0], L) <= ORACLE_BUDGET_S:
        ref = oracle.conv2d(xv, wm, stride=L.stride, relu=relu)
        assert y32.shape == ref.shape
        check(y32, ref, cfg.dtype)
    else:
        pts = _sample_points(np.random.default_rng(seed), xs.shape[0], L.Co, L.Ho, L.Wo, npts)
        ref = oracle.conv2d_points(xv, wm, pts, stride=L.stride, relu=relu)
        check(y32[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]], ref, cfg.dtype)
    return g, y32


@pytest.mark.parametrize("dt", [wl.F16, wl.BF16])
def test_pipelined_kernel_many_tiles_per_workgroup(dt):
    """About seven tiles per persistent workgroup (176 strips of 84 rows x 2 channel blocks on 256 compute units):
    every workgroup walks several tall tiles and then short ones, each tile's last stage working out the next
    tile's copy sources.  Sampled outputs against the oracle; stored 16-bit output against the fp32 output."""
    N, Ci, Co, H, W, k = 44, 96, 256, 84, 64, 3
    rng = np.random.default_rng(4242 + dt)
    masks = B.rtoss_pattern_dict(k)
    xs = wl.round_to_dtype(rng.standard_normal((N, Ci, H, W)), dt)
    ws = wl.round_to_dtype(rng.standard_normal((Co, Ci, 3, 3)) * 0.05, dt)
    xv, wv = wl.to_f64(xs, dt), wl.to_f64(ws, dt)
    idx = oracle.select(wv, masks)
    g = GpuLayer(ws, dt, masks, k)
    assert np.array_equal(g.idx_host(), idx)
    y32 = g.conv_nchw(xs, relu=True, out_dt=wl.F32)
    y16 = g.conv_nchw(xs, relu=True)
    assert np.array_equal(y16, wl.round_to_dtype(y32.astype(np.float64), dt))
    pts = _sample_points(rng, N, Co, H, W, 6000)
    ref = oracle.conv2d_points(xv, oracle.mask(wv, masks, idx), pts, relu=True)
    check(y32[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]], ref, dt)


def test_cfg2_full_layers():
    cfg = wl.get_config(2)
    rng = wl.make_rng(cfg)
    masks = B.rtoss_pattern_dict(cfg.k)
    assert masks.size == 22
    for i, L in enumerate(cfg.layers):
        xs, xv = wl.draw_x(rng, cfg, L)
        ws, wv = wl.draw_w(rng, cfg, L)
        assert _oracle_seconds(cfg.N, L) <= ORACLE_BUDGET_S  # whole tensors
        g, y32 = _check_layer_full(cfg, L, xs, xv, ws, wv, masks, False, seed=i)
        y16 = g.conv_nchw(xs, stride=L.stride)
        assert np.array_equal(y16, wl.round_to_dtype(y32.astype(np.float64), cfg.dtype))


def test_cfg3_full():
    cfg = wl.get_config(3)
    L = cfg.layers[0]
    rng = wl.make_rng(cfg)
    masks = B.rtoss_pattern_dict(cfg.k)
    assert masks.size == 12
    xs, xv = wl.draw_x(rng, cfg, L)
    ws, wv = wl.draw_w(rng, cfg, L)
    assert _oracle_seconds(cfg.N, L) <= ORACLE_BUDGET_S  # whole tensor
    g, y32 = _check_layer_full(cfg, L, xs, xv, ws, wv, masks, False, seed=3)
    y16 = g.conv_nchw(xs)
    assert np.array_equal(y16, wl.round_to_dtype(y32.astype(np.float64), cfg.dtype))


def test_cfg4_full_chain():
    """Four stacked 3x3 layers with ReLU between; every output element of each layer is checked against the
    oracle fed with the GPU's own stored (bf16) output of the previous layer."""
    cfg = wl.get_config(4)
    rng = wl.make_rng(cfg)
    masks = B.rtoss_pattern_dict(cfg.k)
    xs, xv = wl.draw_x(rng, cfg, cfg.layers[0])
    weights = [wl.draw_w(rng, cfg, L) for L in cfg.layers]
    for i, L in enumerate(cfg.layers):
        ws, wv = weights[i]
        assert _oracle_seconds(cfg.N, L) <= ORACLE_BUDGET_S  # whole tensors
        g, y32 = _check_layer_full(cfg, L, xs, xv, ws, wv, masks, L.relu, seed=40 + i)
        y16 = g.conv_nchw(xs, stride=1, relu=L.relu)
        assert np.array_equal(y16, wl.round_to_dtype(y32.astype(np.float64), cfg.dtype))
        xs, xv = y16, wl.to_f64(y16, cfg.dtype)


def test_cfg5_all_layers_batch16():
    """All 57 layers of the YOLOv5s-shaped set at batch 16, the benchmarked launch shape: whole output tensors
    against the oracle (every layer fits the oracle budget on the test machine's cores; the helper falls back
    to sampled outputs where one would not)."""
    cfg = wl.get_config(5)
    masks = B.rtoss_pattern_dict(cfg.k)
    rng = wl.make_rng(cfg)
    sampled = []
    for i, L in enumerate(cfg.layers):
        xs, xv = wl.draw_x(rng, cfg, L)
        ws, wv = wl.draw_w(rng, cfg, L)
        if _oracle_seconds(cfg.N, L) > ORACLE_BUDGET_S:
            sampled.append(i)
        _check_layer_full(cfg, L, xs, xv, ws, wv, masks, i % 2 == 0, seed=500 + i)
        print("cfg5 layer %d (%d->%d @%d %dx%d s%d) ok" % (i, L.Ci, L.Co, L.H, L.ksize, L.ksize, L.stride), flush=True)
    assert len(sampled) <= 4, "layers checked on samples only: %r" % (sampled,)


NCHW_CASES = [
    # dt, N, Ci, Co, H, W, ks, stride, k, relu: shapes that take the matrix-core kernels when channels-last,
    # and shapes of the element-wise kernel
    (wl.F16, 2, 64, 64, 17, 23, 3, 1, 3, False),
    (wl.BF16, 1, 128, 144, 20, 24, 3, 2, 2, True),
    (wl.F16, 2, 256, 64, 9, 11, 1, 1, 2, False),
    (wl.F32, 1, 16, 24, 14, 15, 3, 1, 4, True),
    (wl.F16, 1, 3, 32, 20, 20, 3, 2, 3, False),
    (wl.BF16, 3, 5, 7, 8, 8, 1, 1, 2, False),
]


@pytest.mark.parametrize("case", NCHW_CASES)
def test_conv_nchw_layout(case):
    """RTOSS_NCHW activations ([N][C][H][W] in and out): same results as the oracle, and for 16-bit tensors
    exactly the channels-last call's output, transposed."""
    import torch
    from paper_2303_02191_amd import pipeline as pl
    dt, N, Ci, Co, H, W, ks, stride, k, relu = case
    rng = np.random.default_rng(7000 + Ci + Co + ks)
    masks = B.rtoss_pattern_dict(k)
    xs = wl.round_to_dtype(rng.standard_normal((N, Ci, H, W)), dt)
    ws = wl.round_to_dtype(rng.standard_normal((Co, Ci, ks, ks)) * 0.05, dt)
    g = GpuLayer(ws, dt, masks, k)
    ref = oracle.conv2d(wl.to_f64(xs, dt), oracle.mask(wl.to_f64(ws, dt), masks, g.idx_host()), stride=stride, relu=relu)
    x_nchw = pl.to_device(np.ascontiguousarray(xs), dt)
    y32 = g.layer.conv(x_nchw, stride=stride, relu=relu, out_dt=wl.F32, layout=B.NCHW)
    torch.cuda.synchronize()
    assert tuple(y32.shape) == ref.shape
    check(pl.to_host(y32), ref, dt)
    if dt != wl.F32:
        y16 = g.layer.conv(x_nchw, stride=stride, relu=relu, layout=B.NCHW)
        torch.cuda.synchronize()
        assert np.array_equal(pl.to_host(y16), wl.round_to_dtype(pl.to_host(y32).astype(np.float64), dt))

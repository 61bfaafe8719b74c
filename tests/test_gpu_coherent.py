"""GPU parity of the coherent path (rtoss_pack_coherent / rtoss_conv2d_pattern_coherent): live taps of
block-shared patterns gathered onto the dense matrix instruction.  Section IV.A / IV.C: the layers of a group
share the kernel patterns of the group's parent.  The path must be exact for ANY index tensor; the packer's
detection result (dense steps per stage and channel block) is checked where the sharing structure fixes it."""
import numpy as np
import pytest
import torch

import oracle
from paper_2303_02191_amd import binding as B
from paper_2303_02191_amd import pipeline as pl
from paper_2303_02191_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _indices(kind, rng, Co, Ci, P, w_parent64, masks):
    if kind == "run":       # one pattern per run of 8 input channels, shared by all output channels
        return np.repeat(rng.integers(0, P, Ci // 8), 8)[None, :].repeat(Co, 0)
    if kind == "block":     # one pattern per (64 output channels, 8 input channels) block
        blocks = rng.integers(0, P, ((Co + 63) // 64, Ci // 8))
        return np.repeat(np.repeat(blocks, 64, 0)[:Co], 8, 1)
    if kind == "filter":    # one pattern per output channel (not coherent in the sense of the kernel: up to 9 steps)
        return rng.integers(0, P, Co)[:, None].repeat(Ci, 1)
    if kind == "uneven":    # even blocks of 64 output channels share per run, odd blocks have independent patterns
        idx = np.repeat(rng.integers(0, P, Ci // 8), 8)[None, :].repeat(Co, 0)
        for b0 in range(64, Co, 128):
            idx[b0:b0 + 64] = rng.integers(0, P, idx[b0:b0 + 64].shape)
        return idx
    if kind == "parent":    # the parent layer's own selection, kernel by kernel (independent patterns)
        return oracle.select(w_parent64, masks).reshape(Co, Ci)
    raise ValueError(kind)


CASES = [
    # dt, N, Ci, Co, H, W, stride, k, relu
    (wl.F16, 2, 64, 64, 17, 23, 1, 3, False),
    (wl.BF16, 1, 128, 80, 33, 18, 1, 2, True),
    (wl.F16, 1, 256, 144, 20, 24, 1, 3, False),
    (wl.BF16, 2, 64, 128, 37, 41, 2, 3, True),
    (wl.F16, 1, 32, 16, 5, 7, 2, 4, False),
    # large stride-1 layers: the pipelined kernel (tall and short tiles, ragged last strip, a channel-block pair
    # without its second block; independent patterns run past the steps it keeps in LDS)
    (wl.BF16, 13, 96, 144, 50, 64, 1, 3, True),
    (wl.F16, 10, 160, 128, 52, 70, 1, 2, False),
]


@pytest.mark.parametrize("kind", ["run", "block", "filter", "parent", "uneven"])
@pytest.mark.parametrize("case", CASES, ids=lambda c: "dt%d_%d-%d_%dx%d_s%d_k%d" % (c[0], c[2], c[3], c[4], c[5], c[6], c[7]))
def test_coherent_path_matches_the_oracle(case, kind):
    dt, N, Ci, Co, H, W, stride, k, relu = case
    rng = np.random.default_rng(1000 * Ci + Co + 7 * k + len(kind))
    masks = B.rtoss_pattern_dict(k)
    P = len(masks)
    w_parent = wl.round_to_dtype(rng.standard_normal((Co, Ci, 3, 3)) * 0.05, dt)
    ws = wl.round_to_dtype(rng.standard_normal((Co, Ci, 3, 3)) * 0.05, dt)  # the child layer's own weights
    xs = wl.round_to_dtype(rng.standard_normal((N, Ci, H, W)), dt)
    idx = _indices(kind, rng, Co, Ci, P, wl.to_f64(w_parent, dt), masks).astype(np.uint8).reshape(-1)
    ref = oracle.conv2d(wl.to_f64(xs, dt), oracle.mask(wl.to_f64(ws, dt), masks, idx), stride=stride, relu=relu)
    lay = pl.CoherentLayer(Co, Ci, k, dt, masks).pack(pl.to_device(ws, dt), torch.from_numpy(idx).cuda())
    steps = lay.steps()
    assert steps.shape == (Ci // 32, (Co + 63) // 64)
    if kind in ("run", "block"):
        assert (steps == k).all(), steps  # every block keeps exactly its pattern's k taps
    else:
        assert (steps >= k).all() and (steps <= 9).all()
    x_dev = pl.to_device(wl.nchw_to_nhwc(xs), dt)
    y32 = lay.conv(x_dev, stride=stride, relu=relu, out_dt=wl.F32)
    y16 = lay.conv(x_dev, stride=stride, relu=relu)
    torch.cuda.synchronize()
    got = wl.nhwc_to_nchw(pl.to_host(y32)).astype(np.float64)
    assert got.shape == ref.shape
    assert np.max(np.abs(got - ref)) <= 2e-3 * np.sqrt(np.mean(ref ** 2))
    assert np.array_equal(wl.nhwc_to_nchw(pl.to_host(y16)), wl.round_to_dtype(got, dt))
    # the blob's public section is the same as rtoss_pack's
    plain = pl.PackedLayer(Co, Ci, 3, k, dt, masks).pack(pl.to_device(ws, dt), torch.from_numpy(idx).cuda())
    torch.cuda.synchronize()
    n0 = (Co * Ci * k * 2 + 255) // 256 * 256 + Co * Ci
    assert torch.equal(lay.blob[:n0], plain.blob[:n0])


def test_coherent_and_two_of_four_paths_agree_bit_for_bit_on_shared_patterns():
    # same products, same fp32 accumulation per K-slot order?  Not the same order: compare within the tolerance,
    # and the stored 16-bit outputs against each path's own fp32 output (done above); here: both against the oracle
    dt, k, Ci, Co = wl.BF16, 3, 256, 256
    rng = np.random.default_rng(5)
    masks = B.rtoss_pattern_dict(k)
    ws = wl.round_to_dtype(rng.standard_normal((Co, Ci, 3, 3)) * 0.01, dt)
    xs = wl.round_to_dtype(rng.standard_normal((1, Ci, 40, 48)), dt)
    idx = np.repeat(rng.integers(0, len(masks), Ci // 8), 8)[None, :].repeat(Co, 0).astype(np.uint8).reshape(-1)
    ref = oracle.conv2d(wl.to_f64(xs, dt), oracle.mask(wl.to_f64(ws, dt), masks, idx))
    w_dev, idx_dev, x_dev = pl.to_device(ws, dt), torch.from_numpy(idx).cuda(), pl.to_device(wl.nchw_to_nhwc(xs), dt)
    a = pl.CoherentLayer(Co, Ci, k, dt, masks).pack(w_dev, idx_dev).conv(x_dev, out_dt=wl.F32)
    b = pl.PackedLayer(Co, Ci, 3, k, dt, masks).pack(w_dev, idx_dev).conv(x_dev, out_dt=wl.F32)
    torch.cuda.synchronize()
    tol = 2e-3 * np.sqrt(np.mean(ref ** 2))
    for y in (a, b):
        assert np.max(np.abs(wl.nhwc_to_nchw(pl.to_host(y)).astype(np.float64) - ref)) <= tol


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_pipelined_kernel_every_step_count(k):
    """The pipelined kernel has one branch-free stage body per step count 1..5: patterns shared per run of 8 input
    channels give exactly k steps in every stage, on a shape that takes that kernel (tall and short tiles, a ragged
    last strip, an unpaired last channel block that takes the general body)."""
    dt, N, Ci, Co, H, W = wl.F16, 13, 96, 144, 50, 64
    rng = np.random.default_rng(900 + k)
    masks = B.rtoss_pattern_dict(k)
    ws = wl.round_to_dtype(rng.standard_normal((Co, Ci, 3, 3)) * 0.05, dt)
    xs = wl.round_to_dtype(rng.standard_normal((N, Ci, H, W)), dt)
    idx = _indices("run", rng, Co, Ci, len(masks), None, masks).astype(np.uint8).reshape(-1)
    ref = oracle.conv2d(wl.to_f64(xs, dt), oracle.mask(wl.to_f64(ws, dt), masks, idx), relu=True)
    lay = pl.CoherentLayer(Co, Ci, k, dt, masks).pack(pl.to_device(ws, dt), torch.from_numpy(idx).cuda())
    assert (lay.steps() == k).all()
    x_dev = pl.to_device(wl.nchw_to_nhwc(xs), dt)
    y16 = lay.conv(x_dev, relu=True)                    # the pipelined kernel
    y32 = lay.conv(x_dev, relu=True, out_dt=wl.F32)     # the simple kernel
    torch.cuda.synchronize()
    got = wl.nhwc_to_nchw(pl.to_host(y32)).astype(np.float64)
    assert np.max(np.abs(got - ref)) <= 2e-3 * np.sqrt(np.mean(ref ** 2))
    assert np.array_equal(wl.nhwc_to_nchw(pl.to_host(y16)), wl.round_to_dtype(got, dt))


def test_pipelined_kernel_at_the_largest_channel_count():
    """Ci = 2048 is 64 stages, the most the header tables hold (one table entry per thread): outputs sampled, each
    checked against the oracle; the 16-bit output of the pipelined kernel against the simple kernel's fp32 output."""
    dt, N, Ci, Co, H, W, k = wl.BF16, 50, 2048, 128, 17, 18, 3
    rng = np.random.default_rng(77)
    masks = B.rtoss_pattern_dict(k)
    ws = wl.round_to_dtype(rng.standard_normal((Co, Ci, 3, 3)) * 0.02, dt)
    xs = wl.round_to_dtype(rng.standard_normal((N, Ci, H, W)), dt)
    idx = _indices("run", rng, Co, Ci, len(masks), None, masks).astype(np.uint8).reshape(-1)
    lay = pl.CoherentLayer(Co, Ci, k, dt, masks).pack(pl.to_device(ws, dt), torch.from_numpy(idx).cuda())
    assert lay.steps().shape == (64, 2) and (lay.steps() == k).all()
    x_dev = pl.to_device(wl.nchw_to_nhwc(xs), dt)
    y16 = lay.conv(x_dev)
    y32 = lay.conv(x_dev, out_dt=wl.F32)
    torch.cuda.synchronize()
    got32 = wl.nhwc_to_nchw(pl.to_host(y32)).astype(np.float64)
    assert np.array_equal(wl.nhwc_to_nchw(pl.to_host(y16)), wl.round_to_dtype(got32, dt))
    pts = np.stack([rng.integers(0, N, 3000), rng.integers(0, Co, 3000), rng.integers(0, H, 3000), rng.integers(0, W, 3000)], 1)
    pts[:8] = [[0, 0, 0, 0], [N - 1, Co - 1, H - 1, W - 1], [0, 64, 15, 15], [1, 63, 16, 16], [2, 127, 16, 17], [3, 1, 0, 17],
               [4, 65, 8, 0], [49, 5, 16, 0]]
    ref = oracle.conv2d_points(wl.to_f64(xs, dt), oracle.mask(wl.to_f64(ws, dt), masks, idx), pts)
    vals = got32[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]]
    assert np.max(np.abs(vals - ref)) <= 2e-3 * np.sqrt(np.mean(ref ** 2))


def test_pipelined_kernel_many_tiles_per_workgroup():
    """Four rounds of tiles and more per persistent workgroup (tall after tall, short after short): each tile's last
    stage works out the next tile's copy sources between its matrix instructions."""
    dt, N, Ci, Co, H, W, k = wl.BF16, 44, 96, 256, 84, 64, 3
    rng = np.random.default_rng(78)
    masks = B.rtoss_pattern_dict(k)
    ws = wl.round_to_dtype(rng.standard_normal((Co, Ci, 3, 3)) * 0.05, dt)
    xs = wl.round_to_dtype(rng.standard_normal((N, Ci, H, W)), dt)
    idx = _indices("run", rng, Co, Ci, len(masks), None, masks).astype(np.uint8).reshape(-1)
    lay = pl.CoherentLayer(Co, Ci, k, dt, masks).pack(pl.to_device(ws, dt), torch.from_numpy(idx).cuda())
    assert (lay.steps() == k).all()
    x_dev = pl.to_device(wl.nchw_to_nhwc(xs), dt)
    y16 = lay.conv(x_dev, relu=True)
    y32 = lay.conv(x_dev, relu=True, out_dt=wl.F32)
    torch.cuda.synchronize()
    got32 = wl.nhwc_to_nchw(pl.to_host(y32)).astype(np.float64)
    assert np.array_equal(wl.nhwc_to_nchw(pl.to_host(y16)), wl.round_to_dtype(got32, dt))
    pts = np.stack([rng.integers(0, N, 4000), rng.integers(0, Co, 4000), rng.integers(0, H, 4000), rng.integers(0, W, 4000)], 1)
    pts[:4] = [[0, 0, 0, 0], [N - 1, Co - 1, H - 1, W - 1], [N - 1, 128, 83, 0], [7, 255, 40, 63]]
    ref = oracle.conv2d_points(wl.to_f64(xs, dt), oracle.mask(wl.to_f64(ws, dt), masks, idx), pts, relu=True)
    vals = got32[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]]
    assert np.max(np.abs(vals - ref)) <= 2e-3 * np.sqrt(np.mean(ref ** 2))

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

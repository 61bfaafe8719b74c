"""GPU parity of the fused output stage: y = act(scale[co] * conv + bias[co]) + residual, for every
convolution kernel family, against the oracle's term-by-term definition."""
import zlib

import numpy as np
import pytest
import torch

import oracle
from paper_2303_02191_amd import binding as B
from paper_2303_02191_amd import pipeline as pl
from paper_2303_02191_amd import workloads as wl

from gpu_util import GpuLayer

pytestmark = pytest.mark.gpu

# dt, N, Ci, Co, H, W, ks, stride, k, rule: one case per kernel family and shape class
CASES = [
    (wl.BF16, 13, 128, 128, 52, 50, 3, 1, 3, B.RULE_CONNECTED4),  # pipelined sparse kernel (>= 200 tiles of 16x16 x 128 channels)
    (wl.F16, 7, 256, 272, 33, 49, 3, 1, 2, B.RULE_CONNECTED4),    # ... ragged tiles, padded channel block
    (wl.BF16, 1, 128, 128, 20, 24, 3, 1, 3, B.RULE_CONNECTED4),   # single-buffered sparse kernel, deep layer
    (wl.F16, 2, 64, 48, 19, 21, 3, 1, 3, B.RULE_CONNECTED4),      # single-buffered sparse kernel, stride 1
    (wl.BF16, 1, 128, 144, 37, 41, 3, 2, 2, B.RULE_CONNECTED4),   # ... stride 2
    (wl.F16, 1, 64, 80, 18, 20, 3, 1, 4, B.RULE_CONNECTED4),      # dense mode
    (wl.BF16, 1, 96, 64, 21, 9, 3, 2, 5, B.RULE_CONNECTED4),      # dense mode, stride 2
    (wl.F16, 2, 3, 32, 33, 35, 3, 2, 2, B.RULE_CONNECTED4),       # stem
    (wl.F16, 3, 64, 32, 23, 17, 1, 1, 2, B.RULE_CONNECTED4),      # 1x1 streaming kernel, waves over positions
    (wl.BF16, 2, 256, 256, 15, 13, 1, 1, 2, B.RULE_CONNECTED4),   # ... waves over channels
    (wl.F16, 1, 512, 128, 11, 10, 1, 1, 3, B.RULE_CONNECTED4),    # ... two fragments per wave
    (wl.F16, 1, 1024, 80, 7, 9, 1, 1, 2, B.RULE_CONNECTED4),      # ... one fragment per wave, padded channels
    (wl.BF16, 1, 96, 48, 13, 11, 1, 1, 2, B.RULE_CONNECTED4),     # 1x1 ring kernel
    (wl.F32, 1, 16, 24, 14, 15, 3, 1, 4, B.RULE_CONNECTED4),      # direct kernel, fp32
    (wl.F16, 1, 24, 40, 9, 10, 3, 2, 3, B.RULE_CONNECTED4),       # direct kernel, odd channel counts
    (wl.F32, 2, 40, 24, 8, 9, 1, 1, 2, B.RULE_CONNECTED4),        # direct kernel, 1x1
]
STAGES = [
    dict(scale=True, bias=True, act=B.ACT_SILU, residual=True),
    dict(scale=False, bias=True, act=B.ACT_RELU, residual=False),
    dict(scale=True, bias=False, act=B.ACT_NONE, residual=False),
    dict(scale=False, bias=False, act=B.ACT_NONE, residual=True),
    dict(scale=False, bias=False, act=B.ACT_SILU, residual=False),
]


def _tolerance(ref, dt, out_dt):
    if dt == wl.F32:
        return 1e-5 * np.max(np.abs(ref))
    tol = 2e-3 * np.sqrt(np.mean(ref ** 2))
    if out_dt != wl.F32:  # one rounding of the stored value on top
        tol = tol + np.max(np.abs(ref)) * (2.0 ** -8 if out_dt == wl.BF16 else 2.0 ** -11)
    return tol


@pytest.mark.parametrize("stage", STAGES, ids=lambda s: "%s%s%d%s" % ("s" if s["scale"] else "-", "b" if s["bias"] else "-",
                                                                      s["act"], "r" if s["residual"] else "-"))
@pytest.mark.parametrize("case", CASES, ids=lambda c: "dt%d_%dx%d_k%d_s%d_%d-%d" % (c[0], c[6], c[6], c[8], c[7], c[2], c[3]))
def test_fused_output_stage(case, stage):
    dt, N, Ci, Co, H, W, ks, stride, k, rule = case
    rng = np.random.default_rng(zlib.crc32(repr((case, sorted(stage.items()))).encode()))  # the same inputs in every process
    masks = B.rtoss_pattern_dict(k, rule)
    xs = wl.round_to_dtype(rng.standard_normal((N, Ci, H, W)), dt)
    ws = wl.round_to_dtype(rng.standard_normal((Co, Ci, ks, ks)) * (0.4 / np.sqrt(Ci)), dt)
    xv, wv = wl.to_f64(xs, dt), wl.to_f64(ws, dt)
    scale = rng.uniform(0.5, 1.5, Co).astype(np.float32) if stage["scale"] else None
    bias = rng.standard_normal(Co).astype(np.float32) if stage["bias"] else None
    g = GpuLayer(ws, dt, masks, k)
    pruned = oracle.mask(wv, masks, g.idx_host())
    x_dev = pl.to_device(wl.nchw_to_nhwc(xs), dt)
    sc_dev = torch.from_numpy(scale).cuda() if scale is not None else None
    bi_dev = torch.from_numpy(bias).cuda() if bias is not None else None
    for out_dt in ([wl.F32] if dt == wl.F32 else [wl.F32, dt]):
        ref0 = oracle.conv2d(xv, pruned, stride=stride)
        res_store = res_vals = res_dev = None
        if stage["residual"]:
            res_store = wl.round_to_dtype(rng.standard_normal(ref0.shape), out_dt)
            res_vals = wl.to_f64(res_store, out_dt)
            res_dev = pl.to_device(wl.nchw_to_nhwc(res_store), out_dt)
        ref = oracle.conv2d_fused(xv, pruned, stride=stride, scale=scale, bias=bias, act=stage["act"], residual=res_vals)
        y = g.layer.conv_fused(x_dev, stride=stride, scale=sc_dev, bias=bi_dev, act=stage["act"], residual=res_dev,
                               out_dt=out_dt)
        torch.cuda.synchronize()
        got = wl.to_f64(wl.nhwc_to_nchw(pl.to_host(y)), out_dt)
        assert got.shape == ref.shape
        err = np.max(np.abs(got - ref))
        assert err <= _tolerance(ref, dt, out_dt), (err, _tolerance(ref, dt, out_dt), out_dt)


def test_fused_relu_equals_the_plain_call_bit_for_bit():
    # act = ReLU through the fused entry point and fuse_relu through the plain one are the same arithmetic
    dt, k = wl.BF16, 3
    rng = np.random.default_rng(4)
    masks = B.rtoss_pattern_dict(k)
    for Ci, Co, ks, stride in [(128, 128, 3, 1), (64, 64, 3, 2), (256, 64, 1, 1)]:
        ws = wl.round_to_dtype(rng.standard_normal((Co, Ci, ks, ks)) * 0.05, dt)
        xs = wl.round_to_dtype(rng.standard_normal((2, Ci, 18, 22)), dt)
        g = GpuLayer(ws, dt, masks, k)
        x_dev = pl.to_device(wl.nchw_to_nhwc(xs), dt)
        a = g.layer.conv(x_dev, stride=stride, relu=True)
        b = g.layer.conv_fused(x_dev, stride=stride, act=B.ACT_RELU)
        torch.cuda.synchronize()
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


# dt, N, Ci, Co_a, Co_b, H, W, ks, stride, k: two layers over one input write the two channel slices of one buffer
CONCAT_CASES = [
    (wl.BF16, 13, 128, 128, 64, 52, 50, 3, 1, 3),   # pipelined sparse kernel + single-buffered sparse kernel
    (wl.F16, 2, 64, 48, 16, 19, 21, 3, 1, 3),       # single-buffered sparse kernel, stride 1
    (wl.BF16, 1, 128, 144, 32, 37, 41, 3, 2, 2),    # ... stride 2
    (wl.F16, 1, 64, 80, 48, 18, 20, 3, 1, 4),       # dense mode
    (wl.F16, 2, 3, 32, 16, 33, 35, 3, 2, 2),        # stem
    (wl.F16, 3, 64, 32, 64, 23, 17, 1, 1, 2),       # 1x1 streaming kernel
    (wl.BF16, 2, 256, 256, 128, 15, 13, 1, 1, 2),   # ... waves over channels
    (wl.BF16, 1, 96, 48, 16, 13, 11, 1, 1, 2),      # 1x1 ring kernel
    (wl.F32, 1, 16, 24, 8, 14, 15, 3, 1, 4),        # direct kernel, fp32
    (wl.F16, 1, 24, 40, 8, 9, 10, 3, 2, 3),         # direct kernel, odd channel counts
]


@pytest.mark.parametrize("case", CONCAT_CASES, ids=lambda c: "dt%d_%dx%d_s%d_%d-%d+%d" % (c[0], c[7], c[7], c[8], c[2], c[3], c[4]))
def test_two_layers_write_one_concatenation(case):
    """Section V.C times whole detectors, whose blocks concatenate branch outputs along channels: two
    convolutions write their channel slices of one channels-last buffer (y_ld = the buffer's channel count),
    the second adding a shortcut read from a slice of another wide buffer (residual_ld).  Both slices are
    compared with the oracle and the channels between and around them must keep their sentinel."""
    dt, N, Ci, Ca, Cb, H, W, ks, stride, k = case
    rng = np.random.default_rng(zlib.crc32(repr(case).encode()))
    masks = B.rtoss_pattern_dict(k)
    xs = wl.round_to_dtype(rng.standard_normal((N, Ci, H, W)), dt)
    xv = wl.to_f64(xs, dt)
    x_dev = pl.to_device(wl.nchw_to_nhwc(xs), dt)
    layers, pruned = [], []
    for Co in (Ca, Cb):
        ws = wl.round_to_dtype(rng.standard_normal((Co, Ci, ks, ks)) * (0.4 / np.sqrt(Ci)), dt)
        g = GpuLayer(ws, dt, masks, k)
        layers.append(g)
        pruned.append(oracle.mask(wl.to_f64(ws, dt), masks, g.idx_host()))
    bias = rng.standard_normal(Cb).astype(np.float32)
    ref_a = oracle.conv2d_fused(xv, pruned[0], stride=stride, act=B.ACT_RELU)
    gap = 8  # untouched channels between the two slices
    for out_dt in ([wl.F32] if dt == wl.F32 else [wl.F32, dt]):
        tdt = pl.TORCH_DTYPE[out_dt]
        _, _, Ho, Wo = ref_a.shape
        res_store = wl.round_to_dtype(rng.standard_normal((N, Cb, Ho, Wo)), out_dt)
        res_wide = torch.full((N, Ho, Wo, Cb + 24), 7.0, dtype=tdt, device="cuda")
        res_wide[..., 16:16 + Cb] = pl.to_device(wl.nchw_to_nhwc(res_store), out_dt)
        ref_b = oracle.conv2d_fused(xv, pruned[1], stride=stride, bias=bias, act=B.ACT_SILU,
                                    residual=wl.to_f64(res_store, out_dt))
        total = Ca + gap + Cb + 8
        buf = torch.full((N, Ho, Wo, total), -3.0, dtype=tdt, device="cuda")
        ya, yb = buf[..., :Ca], buf[..., Ca + gap: Ca + gap + Cb]
        layers[0].layer.conv_fused(x_dev, stride=stride, act=B.ACT_RELU, out_dt=out_dt, y=ya)
        layers[1].layer.conv_fused(x_dev, stride=stride, bias=torch.from_numpy(bias).cuda(), act=B.ACT_SILU,
                                   residual=res_wide[..., 16:16 + Cb], out_dt=out_dt, y=yb)
        torch.cuda.synchronize()
        host = buf.cpu()
        assert bool((host[..., Ca:Ca + gap] == -3.0).all()) and bool((host[..., Ca + gap + Cb:] == -3.0).all())
        for ysl, ref in ((host[..., :Ca], ref_a), (host[..., Ca + gap: Ca + gap + Cb], ref_b)):
            got = wl.to_f64(wl.nhwc_to_nchw(pl.to_host(ysl.contiguous())), out_dt)
            err = np.max(np.abs(got - ref))
            assert err <= _tolerance(ref, dt, out_dt), (err, _tolerance(ref, dt, out_dt), out_dt)

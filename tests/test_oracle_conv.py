"""Pins for the oracle's convolution: library routine, impulses, matmul, linearity."""
import numpy as np
import pytest
import torch

import oracle


def _rng(seed):
    return np.random.default_rng(seed)


def _torch_conv(x, w, stride, pad):
    return torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(w), stride=stride, padding=pad).numpy()


@pytest.mark.parametrize("stride", [1, 2])
@pytest.mark.parametrize("H,W", [(9, 7), (12, 12), (5, 16)])
def test_all_ones_pattern_is_dense_conv(stride, H, W):
    # k = 9: the only pattern keeps every tap, so the masked conv is the dense conv,
    # checked against the library's float64 conv2d.
    masks = oracle.pattern_dict(9, oracle.RULE_ALL)
    x = _rng(1).standard_normal((2, 5, H, W))
    w = _rng(2).standard_normal((4, 5, 3, 3))
    idx = oracle.select(w, masks)
    assert (idx == 0).all()
    wm = oracle.mask(w, masks, idx)
    assert np.array_equal(wm, w)
    y = oracle.conv2d(x, wm, stride=stride)
    ref = _torch_conv(x, w, stride, 1)
    assert y.shape == ref.shape
    assert np.max(np.abs(y - ref)) <= 1e-12 * np.max(np.abs(ref))


@pytest.mark.parametrize("k,stride", [(2, 1), (3, 2), (4, 1)])
def test_sparse_conv_is_library_conv_on_masked_weights(k, stride):
    masks = oracle.pattern_dict(k)
    x = _rng(3).standard_normal((2, 6, 11, 13))
    w = _rng(4).standard_normal((7, 6, 3, 3))
    idx = oracle.select(w, masks)
    wm = oracle.mask(w, masks, idx)
    y = oracle.conv2d(x, wm, stride=stride, relu=True)
    ref = np.maximum(_torch_conv(x, wm, stride, 1), 0.0)
    assert np.max(np.abs(y - ref)) <= 1e-12 * np.max(np.abs(ref))
    # the loop over live taps only gives the identical float64 sums
    y2 = oracle.conv2d_live3x3(x, w, masks, idx, stride=stride, relu=True)
    assert np.array_equal(y, y2)


@pytest.mark.parametrize("stride", [1, 2])
def test_unit_impulse_returns_the_kernel(stride):
    # One 1 at (ih, iw) in channel ci: output (co, oh, ow) must be w[co, ci, ih-oh*s+1, iw-ow*s+1].
    Ci, Co, H, W = 3, 2, 8, 9
    w = _rng(5).standard_normal((Co, Ci, 3, 3))
    for ci, ih, iw in [(0, 0, 0), (1, 4, 5), (2, 7, 8), (1, 3, 0)]:
        x = np.zeros((1, Ci, H, W))
        x[0, ci, ih, iw] = 1.0
        y = oracle.conv2d(x, w, stride=stride)
        Ho, Wo = y.shape[2:]
        for co in range(Co):
            for oh in range(Ho):
                for ow in range(Wo):
                    kh, kw = ih - oh * stride + 1, iw - ow * stride + 1
                    want = w[co, ci, kh, kw] if 0 <= kh < 3 and 0 <= kw < 3 else 0.0
                    assert y[0, co, oh, ow] == want


def test_output_extent():
    x = np.zeros((1, 1, 640, 640))
    assert oracle.conv2d(x[:, :, :20, :20], np.zeros((1, 1, 3, 3)), stride=2).shape == (1, 1, 10, 10)
    assert oracle.conv2d(x[:, :, :7, :9], np.zeros((1, 1, 3, 3)), stride=2).shape == (1, 1, 4, 5)
    assert oracle.conv2d(x[:, :, :7, :9], np.zeros((1, 1, 1, 1)), stride=1).shape == (1, 1, 7, 9)


def test_1x1_is_matmul():
    x = _rng(6).standard_normal((3, 10, 4, 5))
    w = _rng(7).standard_normal((8, 10, 1, 1))
    y = oracle.conv2d(x, w)
    ref = np.einsum("oc,nchw->nohw", w[:, :, 0, 0], x)
    assert np.max(np.abs(y - ref)) <= 1e-12 * np.max(np.abs(ref))


def test_linearity():
    x1, x2 = _rng(8).standard_normal((2, 1, 4, 6, 6))
    w1, w2 = _rng(9).standard_normal((2, 3, 4, 3, 3))
    a = oracle.conv2d(x1 + 2 * x2, w1)
    b = oracle.conv2d(x1, w1) + 2 * oracle.conv2d(x2, w1)
    assert np.max(np.abs(a - b)) < 1e-12
    c = oracle.conv2d(x1, w1 - 3 * w2)
    d = oracle.conv2d(x1, w1) - 3 * oracle.conv2d(x1, w2)
    assert np.max(np.abs(c - d)) < 1e-12


def test_points_match_full():
    x = _rng(10).standard_normal((2, 4, 9, 9))
    w = _rng(11).standard_normal((5, 4, 3, 3))
    y = oracle.conv2d(x, w, stride=2, relu=True)
    pts = np.array([[0, 0, 0, 0], [1, 4, 4, 4], [0, 2, 3, 1], [1, 1, 0, 4]], dtype=np.int32)
    got = oracle.conv2d_points(x, w, pts, stride=2, relu=True)
    assert np.array_equal(got, y[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]])


def test_fused_output_stage_against_library_and_closed_form():
    # y = act(scale * conv + bias) + residual, against torch's float64 CPU routines ...
    import torch
    import torch.nn.functional as F
    rng = np.random.default_rng(77)
    x = rng.standard_normal((2, 5, 9, 8))
    w = rng.standard_normal((7, 5, 3, 3)) * 0.3
    scale, bias = rng.uniform(0.5, 1.5, 7), rng.standard_normal(7)
    for stride in (1, 2):
        base = F.conv2d(torch.from_numpy(x), torch.from_numpy(w), stride=stride, padding=1)
        res = rng.standard_normal(tuple(base.shape))
        lin = base * torch.from_numpy(scale).view(1, 7, 1, 1) + torch.from_numpy(bias).view(1, 7, 1, 1)
        for act, f in [(oracle.ACT_NONE, lambda t: t), (oracle.ACT_RELU, F.relu), (oracle.ACT_SILU, F.silu)]:
            want = (f(lin) + torch.from_numpy(res)).numpy()
            got = oracle.conv2d_fused(x, w, stride=stride, scale=scale, bias=bias, act=act, residual=res)
            assert np.max(np.abs(got - want)) < 1e-12
    # ... and a closed form: a 1x1 identity convolution leaves silu(s * x + b) + r
    x = np.array([[[[0.0, 1.0, -2.0]]]])
    got = oracle.conv2d_fused(x, np.ones((1, 1, 1, 1)), scale=[2.0], bias=[0.0], act=oracle.ACT_SILU, residual=np.full((1, 1, 1, 3), 0.5))
    want = np.array([0.0, 2.0 / (1.0 + np.exp(-2.0)), -4.0 / (1.0 + np.exp(4.0))]) + 0.5
    assert np.allclose(got.reshape(-1), want, rtol=0, atol=1e-15)
    # without any stage it is the plain convolution
    assert np.array_equal(oracle.conv2d_fused(x, np.ones((1, 1, 1, 1))), oracle.conv2d(x, np.ones((1, 1, 1, 1))))


"""Shape pins for the synthetic workloads (Section III layer share, Section V.A sizes)."""
import os

import numpy as np

from paper_2303_02191_amd import workloads as wl


def test_yolo5s_shaped_table_matches_printed_share(golden_dir):
    vals = dict(line.split() for line in open(os.path.join(golden_dir, "section3_layer_share.txt"))
                if line.strip() and not line.startswith("#"))
    cfg = wl.get_config(5)
    n1 = sum(L.ksize == 1 for L in cfg.layers)
    assert len(cfg.layers) == 57 and n1 == 39
    assert round(100.0 * n1 / len(cfg.layers), 2) == float(vals["share_1x1_percent"])
    params = sum(L.n_weights for L in cfg.layers) / 1e6
    assert abs(params - float(vals["params_millions"])) / float(vals["params_millions"]) < 0.01
    # every 3x3 layer's channel pair chains: widths 32..512
    assert {L.Co for L in cfg.layers} <= {32, 64, 128, 256, 512}


def test_group_counts():
    assert wl.get_config(1).layers[0].groups == 4096
    assert [L.groups for L in wl.get_config(2).layers] == [96, 2048, 8192, 32768, 131072]
    assert wl.get_config(3).layers[0].groups == 7281
    assert sum(L.groups for L in wl.get_config(4).layers) == 262144


def test_rounding_is_exact_and_once():
    rng = np.random.default_rng(0)
    a = rng.standard_normal(10000)
    for dt in (wl.F32, wl.F16, wl.BF16):
        s = wl.round_to_dtype(a, dt)
        v = wl.to_f64(s, dt)
        assert np.array_equal(wl.round_to_dtype(v, dt), s)  # idempotent
        ulp = {wl.F32: 2.0 ** -24, wl.F16: 2.0 ** -11, wl.BF16: 2.0 ** -8}[dt]
        assert np.all(np.abs(v - a) <= ulp * np.maximum(np.abs(a), 1e-3))
    # bfloat16 ties round to even
    assert wl.round_to_dtype(np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8]), wl.BF16).tolist() == [0x3F80, 0x3F82]


def test_seeded_draws_repeat():
    cfg = wl.get_config(1)
    a = wl.draw_x(wl.make_rng(cfg), cfg, cfg.layers[0])[0]
    b = wl.draw_x(wl.make_rng(cfg), cfg, cfg.layers[0])[0]
    assert np.array_equal(a, b) and a.dtype == np.float32 and a.shape == (1, 64, 56, 56)

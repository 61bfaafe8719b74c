"""The library's launches must replay correctly from a captured HIP graph: it allocates
nothing and records no memset, so select, pack and conv capture as plain kernel nodes.
Every replay is checked against the eager result, with eager work and synchronisations
between the replays."""
import numpy as np
import pytest
import torch

from paper_2303_02191_amd import binding as B
from paper_2303_02191_amd import pipeline as pl
from paper_2303_02191_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("ks,Ci,Co,stride,dt", [(3, 64, 128, 1, wl.BF16), (3, 32, 32, 2, wl.F16), (1, 128, 64, 1, wl.F16),
                                                 (3, 3, 32, 2, wl.F16), (3, 16, 16, 1, wl.F32)])
def test_graph_replays_match_eager(ks, Ci, Co, stride, dt):
    k = 3 if dt == wl.BF16 else 2
    masks = B.rtoss_pattern_dict(k)
    rng = np.random.default_rng(Ci + Co + ks)
    ws = wl.round_to_dtype(rng.standard_normal((Co, Ci, ks, ks)) * 0.05, dt)
    w = pl.to_device(ws, dt)
    xs_host = [wl.round_to_dtype(rng.standard_normal((2, 21, 19, Ci)), dt) for _ in range(3)]
    x = pl.to_device(xs_host[0], dt)
    idx = torch.zeros(max(w.numel() // 9, 1), dtype=torch.uint8, device="cuda")
    layer = pl.PackedLayer(Co, Ci, ks, k, dt, masks)
    y = torch.zeros(layer.out_shape(x.shape, stride), dtype=pl.TORCH_DTYPE[dt], device="cuda")

    def run():
        B.rtoss_select_patterns(w.data_ptr(), dt, w.numel(), masks, idx.data_ptr(), torch.cuda.current_stream().cuda_stream)
        layer.pack(w, idx)
        layer.conv(x, stride=stride, relu=True, y=y)

    eager = []
    for xh in xs_host:  # eager results for three different inputs (also warms up kernel attributes)
        x.copy_(pl.to_device(xh, dt))
        run()
        torch.cuda.synchronize()
        eager.append(pl.to_host(y).copy())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run()
    for rep in range(6):
        i = rep % 3
        x.copy_(pl.to_device(xs_host[i], dt))  # eager work between replays
        y.zero_()
        layer.blob.zero_()
        idx.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(pl.to_host(y), eager[i]), "replay %d differs from the eager result" % rep

"""GPU parity: rtoss_pack's live-weight section vs the oracle's mask step, bit-exact."""
import numpy as np
import pytest
import torch

import oracle
from paper_2303_02191_amd import binding as B
from paper_2303_02191_amd import pipeline as pl
from paper_2303_02191_amd import workloads as wl

from gpu_util import GpuLayer, decode_live_section

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dt", [wl.F32, wl.F16, wl.BF16])
@pytest.mark.parametrize("Co,Ci,ks,k", [(64, 64, 3, 3), (5, 7, 3, 2), (32, 3, 3, 4), (256, 256, 1, 2), (7, 11, 1, 3),
                                        (2, 4, 1, 2), (130, 70, 3, 5)])
def test_pack_live_section(dt, Co, Ci, ks, k):
    masks = B.rtoss_pattern_dict(k)
    a = np.random.default_rng(Co * 31 + Ci + k).standard_normal((Co, Ci, ks, ks)) * 0.05
    store = wl.round_to_dtype(a, dt)
    vals = wl.to_f64(store, dt)
    g = GpuLayer(store, dt, masks, k)
    idx_want = oracle.select(vals, masks)
    assert np.array_equal(g.idx_host(), idx_want)
    wm, idx_blob = decode_live_section(g.blob_host(), Co, Ci, ks, k, dt, masks)
    assert np.array_equal(idx_blob, idx_want)
    want = oracle.mask(vals, masks, idx_want)
    got = wl.to_f64(wm, dt)
    assert np.array_equal(got, want)  # survivors bit-identical, everything else (and the tail) zero
    tail = (Co * Ci * ks * ks) % 9
    if tail:
        assert (got.reshape(-1)[-tail:] == 0).all()


def test_batched_pack_equals_single_packs():
    # layers of every blob format (and more of one format than a launch table holds): the batched call must
    # write exactly the bytes the per-layer call writes
    import torch
    from paper_2303_02191_amd import pipeline as pl
    dt, k = wl.F16, 2
    masks = B.rtoss_pattern_dict(k)
    shapes = [(64, 64, 3), (32, 3, 3), (48, 96, 1), (40, 24, 3), (128, 256, 1)] + [(32 + 16 * (i % 3), 64, 1) for i in range(30)] \
        + [(16 * (1 + i % 4), 32 * (1 + i % 2), 3) for i in range(27)]
    rng = np.random.default_rng(5)
    ws, idxs, single, batched = [], [], [], []
    for Co, Ci, ks in shapes:
        w = pl.to_device(wl.round_to_dtype(rng.standard_normal((Co, Ci, ks, ks)) * 0.05, dt), dt)
        ws.append(w)
        idxs.append(pl.select_patterns(w, dt, masks))
        single.append(pl.PackedLayer(Co, Ci, ks, k, dt, masks))
        batched.append(pl.PackedLayer(Co, Ci, ks, k, dt, masks))
        single[-1].blob.zero_()
        batched[-1].blob.zero_()
    for lay, w, idx in zip(single, ws, idxs):
        lay.pack(w, idx)
    pl.pack_layers(batched, ws, idxs)
    torch.cuda.synchronize()
    for (Co, Ci, ks), a, b in zip(shapes, single, batched):
        assert torch.equal(a.blob, b.blob), (Co, Ci, ks)



def test_sparse_pack_of_tensors_aligned_to_their_element_only():
    """Weights one element, indices one byte into their allocations: the blob equals the aligned one's."""
    dt, k = wl.F16, 3
    Co, Ci = 48, 64
    masks = B.rtoss_pattern_dict(k)
    rng = np.random.default_rng(12)
    ws = wl.round_to_dtype(rng.standard_normal((Co, Ci, 3, 3)) * 0.05, dt)
    w = pl.to_device(ws, dt)
    idx = pl.select_patterns(w, dt, masks)
    ref = pl.PackedLayer(Co, Ci, 3, k, dt, masks).pack(w, idx)
    wbuf = torch.empty(w.numel() + 1, dtype=w.dtype, device="cuda")
    wbuf[1:] = w.reshape(-1)
    ibuf = torch.empty(idx.numel() + 1, dtype=torch.uint8, device="cuda")
    ibuf[1:] = idx
    w2, idx2 = wbuf[1:].reshape(w.shape), ibuf[1:]
    assert w2.data_ptr() % 16 != 0 and idx2.data_ptr() % 16 != 0
    got = pl.PackedLayer(Co, Ci, 3, k, dt, masks).pack(w2, idx2)
    torch.cuda.synchronize()
    assert torch.equal(got.blob, ref.blob)

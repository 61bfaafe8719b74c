"""Helpers for the GPU parity tests: run the HIP path through the C ABI on tensors drawn by
the workload module and hand back numpy arrays in the oracle's logical layouts."""
import numpy as np
import torch

from paper_2303_02191_amd import binding as B
from paper_2303_02191_amd import pipeline as pl
from paper_2303_02191_amd import workloads as wl


def gpu_select(w_store, dt, masks):
    w = pl.to_device(np.ascontiguousarray(w_store), dt)
    idx = pl.select_patterns(w, dt, masks)
    torch.cuda.synchronize()
    return idx.cpu().numpy()


def decode_live_section(blob, Co, Ci, ksize, k, dt, masks):
    """Rebuild the pruned weight tensor from section 0 of a packed blob (documented layout)."""
    n = Co * Ci * ksize * ksize
    G = n // 9
    eb = wl.ELEM_BYTES[dt]
    raw = blob[: G * k * eb]
    np_t = {wl.F32: np.float32, wl.F16: np.float16, wl.BF16: np.uint16}[dt]
    live = raw.view(np_t).reshape(G, k)
    idx_off = (G * k * eb + 255) // 256 * 256
    idx = blob[idx_off: idx_off + G]
    out = np.zeros(n, dtype=np_t)
    for j in range(k):
        # j-th live tap of each group's pattern
        taps = np.array([[t for t in range(9) if m >> t & 1][j] for m in masks.tolist()], dtype=np.int64)
        out[np.arange(G) * 9 + taps[idx]] = live[:, j]
    return out.reshape(Co, Ci, ksize, ksize), idx


class GpuLayer:
    """select -> pack -> conv for one layer, on storage arrays in the logical layouts."""

    def __init__(self, w_store, dt, masks, k, idx=None):
        """idx: pattern indices to prune with (a cuda uint8 tensor, e.g. another layer's) instead of selecting."""
        Co, Ci, ks, _ = w_store.shape
        self.dt, self.masks, self.k = dt, masks, k
        self.w = pl.to_device(np.ascontiguousarray(w_store), dt)
        self.idx = pl.select_patterns(self.w, dt, masks) if idx is None else idx
        self.layer = pl.PackedLayer(Co, Ci, ks, k, dt, masks).pack(self.w, self.idx)

    def idx_host(self):
        torch.cuda.synchronize()
        return self.idx.cpu().numpy()

    def blob_host(self):
        torch.cuda.synchronize()
        return self.layer.blob.cpu().numpy()

    def conv_nchw(self, x_store_nchw, stride=1, relu=False, out_dt=None):
        """x as [N, Ci, H, W] storage array -> y as [N, Co, Ho, Wo] storage array."""
        x = pl.to_device(wl.nchw_to_nhwc(x_store_nchw), self.dt)
        y = self.layer.conv(x, stride=stride, relu=relu, out_dt=out_dt)
        torch.cuda.synchronize()
        return wl.nhwc_to_nchw(pl.to_host(y))

"""Convenience wrappers that hold torch device buffers and call the C ABI in order.

No arithmetic happens here: torch is used for device memory and the current stream only;
selection, packing and convolution all run in librtoss.so.
"""
import torch

from . import binding as B

TORCH_DTYPE = {B.F32: torch.float32, B.F16: torch.float16, B.BF16: torch.bfloat16}


def _stream():
    return torch.cuda.current_stream().cuda_stream


def to_device(store, dt):
    """numpy storage array (float32 / float16 / uint16 bfloat16 bits) -> torch cuda tensor of dtype dt."""
    t = torch.from_numpy(store)
    if dt == B.BF16:
        t = t.view(torch.bfloat16)
    return t.cuda()


def to_host(t):
    """torch tensor -> numpy storage array (bfloat16 comes back as uint16 bits)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.uint16).numpy()
    return t.numpy()


def select_patterns(w, dt, masks):
    """w: contiguous cuda tensor of weights (any shape). Returns uint8 cuda tensor [numel // 9]."""
    assert w.is_cuda and w.is_contiguous()
    idx = torch.empty(max(w.numel() // 9, 1), dtype=torch.uint8, device=w.device)
    B.rtoss_select_patterns(w.data_ptr(), dt, w.numel(), masks, idx.data_ptr(), _stream())
    return idx[: w.numel() // 9]


def select_patterns_batch(ws, dt, masks, idxs=None, stream=None):
    """Selection for several weight tensors (contiguous cuda tensors of one dtype) in one call.
    Returns the list of uint8 index tensors (idxs, if given, are filled in place)."""
    if idxs is None:
        idxs = [torch.empty(max(w.numel() // 9, 1), dtype=torch.uint8, device=w.device) for w in ws]
    items = []
    for w, idx in zip(ws, idxs):
        assert w.is_cuda and w.is_contiguous() and idx.is_cuda and idx.numel() >= w.numel() // 9
        items.append((w.data_ptr(), w.numel(), idx.data_ptr()))
    B.rtoss_select_patterns_batch(items, dt, masks, _stream() if stream is None else stream)
    return [idx[: w.numel() // 9] for w, idx in zip(ws, idxs)]


def pack_layers(layers, ws, idxs, stream=None):
    """Pack several PackedLayer objects (one dictionary) from their weight and index tensors in one call."""
    if not layers:
        return layers
    items = []
    for lay, w, idx in zip(layers, ws, idxs):
        assert w.is_cuda and w.is_contiguous() and idx.is_cuda
        items.append((lay.wdesc, w.data_ptr(), idx.data_ptr(), lay.blob.data_ptr(), lay.packed_bytes))
    B.rtoss_pack_batch(items, layers[0].masks, _stream() if stream is None else stream)
    return layers


def pattern_histogram(idx, P, hist=None):
    """Adds the usage counts of idx (uint8 cuda tensor) to hist (uint32 counts as an int32 cuda tensor [P])."""
    assert idx.is_cuda and idx.dtype == torch.uint8 and idx.is_contiguous()
    if hist is None:
        hist = torch.zeros(P, dtype=torch.int32, device=idx.device)
    B.rtoss_pattern_histogram(idx.data_ptr(), idx.numel(), P, hist.data_ptr(), _stream())
    return hist


def reduce_dictionary(masks, w_random, dt, M):
    """Section IV.B, second criterion: select over the random kernels in w_random (cuda tensor, numel % 9 == 0),
    count the winners and keep the M most used patterns.  Returns (reduced masks, kept indices, counts)."""
    idx = select_patterns(w_random, dt, masks)
    hist = pattern_histogram(idx, len(masks))
    counts = hist.cpu().numpy().astype("uint32")
    out, kept = B.rtoss_reduce_dict(masks, counts, M)
    return out, kept, counts


class CoherentLayer:
    """A 3x3 layer packed for the dense-instruction gather path (block-shared patterns)."""

    def __init__(self, Co, Ci, k, dt, masks, device="cuda"):
        self.wdesc = B.WDesc(Co, Ci, 3, k, dt)
        self.masks, self.dt = masks, dt
        self.packed_bytes, self.steps_offset = B.rtoss_pack_size_coherent(self.wdesc, masks)
        self.blob = torch.empty(self.packed_bytes, dtype=torch.uint8, device=device)

    def pack(self, w, idx):
        assert w.is_cuda and w.is_contiguous() and idx.is_cuda
        B.rtoss_pack_coherent(self.wdesc, w.data_ptr(), idx.data_ptr(), self.masks, self.blob.data_ptr(), self.packed_bytes,
                              _stream())
        return self

    def steps(self):
        """Detection result: dense steps per (stage, block of 64 output channels), as a numpy array [stages, blocks]."""
        stages, blocks = self.wdesc.Ci // 32, (self.wdesc.Co + 63) // 64
        torch.cuda.synchronize()
        rec = self.blob[self.steps_offset: self.steps_offset + stages * blocks * 64].cpu().numpy().reshape(stages, blocks, 64)
        return rec[:, :, :4].copy().view("<u4").reshape(stages, blocks)

    def conv(self, x, stride=1, relu=False, out_dt=None, y=None):
        assert x.is_cuda and x.is_contiguous() and x.shape[3] == self.wdesc.Ci
        out_dt = self.dt if out_dt is None else out_dt
        N, H, W, _ = x.shape
        if y is None:
            y = torch.empty((N, (H - 1) // stride + 1, (W - 1) // stride + 1, self.wdesc.Co), dtype=TORCH_DTYPE[out_dt],
                            device=x.device)
        cdesc = B.CDesc(N, H, W, stride, 1, B.NHWC, out_dt, int(bool(relu)))
        B.rtoss_conv2d_pattern_coherent(self.wdesc, cdesc, None, self.masks, self.blob.data_ptr(), x.data_ptr(), y.data_ptr(),
                                        _stream())
        return y


class PackedLayer:
    """One layer's packed blob plus the descriptors the convolution call needs."""

    def __init__(self, Co, Ci, ksize, k, dt, masks, device="cuda"):
        self.wdesc = B.WDesc(Co, Ci, ksize, k, dt)
        self.masks = masks
        self.dt = dt
        self.packed_bytes, self.workspace_bytes = B.rtoss_pack_size(self.wdesc, masks)
        # torch's caching allocator returns 512-byte aligned blocks
        self.blob = torch.empty(self.packed_bytes, dtype=torch.uint8, device=device)
        self.workspace = torch.empty(max(self.workspace_bytes, 1), dtype=torch.uint8, device=device)

    def pack(self, w, idx, stream=None):
        """stream: raw HIP stream handle (default: torch's current stream)."""
        assert w.is_cuda and w.is_contiguous() and idx.is_cuda
        B.rtoss_pack(self.wdesc, w.data_ptr(), idx.data_ptr(), self.masks, self.blob.data_ptr(), self.packed_bytes,
                     self.workspace.data_ptr(), self.workspace_bytes, _stream() if stream is None else stream)
        return self

    def out_shape(self, x_shape, stride):
        N, H, W, _ = x_shape
        ks = self.wdesc.ksize
        pad = ks // 2
        return (N, (H + 2 * pad - ks) // stride + 1, (W + 2 * pad - ks) // stride + 1, self.wdesc.Co)

    def conv(self, x, stride=1, relu=False, out_dt=None, y=None, layout=B.NHWC):
        """x: cuda tensor of the layer's dtype, channels-last [N, H, W, Ci] (or [N, Ci, H, W] with layout=B.NCHW).
        Returns y [N, Ho, Wo, Co] (or [N, Co, Ho, Wo])."""
        assert x.is_cuda and x.is_contiguous()
        out_dt = self.dt if out_dt is None else out_dt
        if layout == B.NCHW:
            N, C, H, W = x.shape
            shape = self.out_shape((N, H, W, C), stride)
            shape = (shape[0], shape[3], shape[1], shape[2])
        else:
            N, H, W, C = x.shape
            shape = self.out_shape(x.shape, stride)
        assert C == self.wdesc.Ci
        if y is None:
            y = torch.empty(shape, dtype=TORCH_DTYPE[out_dt], device=x.device)
        cdesc = B.CDesc(N, H, W, stride, self.wdesc.ksize // 2, layout, out_dt, int(bool(relu)))
        B.rtoss_conv2d_pattern(self.wdesc, cdesc, self.masks, self.blob.data_ptr(), x.data_ptr(), y.data_ptr(),
                               _stream())
        return y

    def conv_fused(self, x, stride=1, scale=None, bias=None, act=B.ACT_NONE, residual=None, out_dt=None, y=None):
        """y = act(scale[co] * conv + bias[co]) + residual.  scale/bias: float32 cuda tensors [Co] or None;
        residual: cuda tensor of y's dtype and shape or None.  y and residual may be channel slices
        buf[..., c0:c0+Co] of wider channels-last buffers (a concatenation the layer writes its part of)."""
        assert x.is_cuda and x.is_contiguous() and x.shape[3] == self.wdesc.Ci
        out_dt = self.dt if out_dt is None else out_dt
        if y is None:
            y = torch.empty(self.out_shape(x.shape, stride), dtype=TORCH_DTYPE[out_dt], device=x.device)
        for t in (scale, bias):
            assert t is None or (t.is_cuda and t.dtype == torch.float32 and t.numel() == self.wdesc.Co)

        def pitch(t):  # position pitch of a channels-last tensor or channel slice of one (0: plain)
            n, h, w, c = t.shape
            ld = t.stride(2)
            assert t.stride(3) == 1 and t.stride(1) == w * ld and t.stride(0) == h * w * ld, "not a channel slice"
            return 0 if ld == c else ld

        assert tuple(y.shape) == self.out_shape(x.shape, stride) and y.dtype == TORCH_DTYPE[out_dt]
        assert residual is None or (residual.is_cuda and residual.shape == y.shape and residual.dtype == y.dtype)
        N, H, W, _ = x.shape
        cdesc = B.CDesc(N, H, W, stride, self.wdesc.ksize // 2, B.NHWC, out_dt, 0)
        ep = B.EpilogueDesc(scale.data_ptr() if scale is not None else None, bias.data_ptr() if bias is not None else None,
                            int(act), residual.data_ptr() if residual is not None else None,
                            pitch(y), pitch(residual) if residual is not None else 0)
        B.rtoss_conv2d_pattern_fused(self.wdesc, cdesc, ep, self.masks, self.blob.data_ptr(), x.data_ptr(), y.data_ptr(),
                                     _stream())
        return y


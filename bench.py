#!/usr/bin/env python3
"""Benchmark of the R-TOSS hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: pattern selection
over every weight tensor of the workload, packing of every layer, and the pattern-sparse
convolution of every layer.  Inputs are resident in HBM before the timed region starts.
Prints ONE JSON line.  `value` is effective TFLOP/s counted on non-zero MACs only
(2 * N*Ho*Wo*k*groups / time), whole step; `roofline` describes the dominant kernel (the
convolution) from HIP-event timings taken inside the timed region (on every --event-every-th
step: the records themselves cost stream time); `cpu_baseline` is the
fp64 CPU oracle timed on a bounded sample of the same workload.

The run proves what it prints: the convolutions of the oracle's sample are repeated with fp32
output and compared with the oracle (max |y - ref| <= 2e-3 * rms(ref) for 16-bit tensors,
1e-5 * max |ref| for fp32 tensors), and every stored 16-bit output of the timed step must equal
the fp32 output rounded once to nearest-even.  A violation is reported in the JSON line
("parity": {"ok": false, ...}) and the exit status is 1.

The default run (cfg4, the metric's "effective TFLOP/s" half) also times the YOLOv5s-shaped
conv set (cfg5) replayed from HIP graphs and reports it under "yolo5s_forward" (the metric's
"ms per YOLOv5s-shaped forward" half); --no-forward skips that.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_MFMA_16BIT_TFLOPS = 2500.0   # MI355X dense fp16/bf16 matrix peak
PEAK_FP32_VECTOR_TFLOPS = 157.3   # MI355X fp32 vector peak
PEAK_HBM_GBS = 8000.0             # MI355X HBM3E peak

WORKLOADS = {"cfg1": 1, "cfg2": 2, "cfg3": 3, "cfg4": 4, "cfg5": 5}

TOL_16BIT_OVER_RMS = 2e-3  # fp16 / bf16 tensors, fp32 output: max |y - ref| <= 2e-3 * rms(ref)
TOL_FP32_OVER_MAX = 1e-5   # fp32 tensors: max |y - ref| <= 1e-5 * max |ref|


def measured_traffic(summary_name):
    """HBM bytes per launch from the committed counter summary, or None.

    The summary (profiles/) records FETCH_SIZE + WRITE_SIZE of the convolution kernel, scaled by what the same
    counters read for a copy of known size, and a hash of the kernel's sources at the time of the counter
    runs; once the sources differ the figure no longer describes this kernel and is dropped.
    """
    import hashlib
    here = os.path.dirname(os.path.abspath(__file__))
    path = os.path.join(here, "profiles", summary_name)
    if not os.path.exists(path):
        return None
    fields = {}
    for line in open(path):
        if ":" in line:
            k, v = line.split(":", 1)
            fields[k.strip()] = v.strip()
    try:
        h = hashlib.sha256()
        for f in ("conv3x3_rows.hip", "sparse_frag.h", "mma.h", "dtypes.h", "common.h", "epilogue.h"):
            h.update(open(os.path.join(here, "paper_2303_02191_amd", "csrc", f), "rb").read())
        if h.hexdigest() != fields.get("kernel_source_sha256"):
            return None
        return int(fields["traffic_bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        return None


def conv_error(got32, ref, is_fp32_tensor):
    """(error, bound) of an fp32-output convolution against the oracle, both as multiples of the
    reference's scale: rms(ref) for 16-bit tensors, max |ref| for fp32 tensors."""
    got32 = np.asarray(got32, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if got32.shape != ref.shape:
        return float("inf"), 0.0
    err = float(np.max(np.abs(got32 - ref))) if ref.size else 0.0
    if not np.isfinite(err):
        return float("inf"), 0.0
    if is_fp32_tensor:
        scale = float(np.max(np.abs(ref))) or 1.0
        return err / scale, TOL_FP32_OVER_MAX
    scale = float(np.sqrt(np.mean(ref ** 2))) or 1.0
    return err / scale, TOL_16BIT_OVER_RMS


class Parity:
    """Accumulates the parity evidence of one run."""

    def __init__(self, is_fp32_tensor):
        self.is_fp32 = is_fp32_tensor
        self.worst = 0.0        # fp32-output error / scale
        self.bound = TOL_FP32_OVER_MAX if is_fp32_tensor else TOL_16BIT_OVER_RMS
        self.worst_stored = 0.0  # stored-output error / scale (includes the output's own rounding)
        self.n_oracle = 0
        self.rne_checked = 0
        self.rne_equal = True
        self.failures = []

    def add_oracle(self, what, got32, got_stored64, ref):
        e, b = conv_error(got32, ref, self.is_fp32)
        self.worst = max(self.worst, e)
        self.n_oracle += 1
        if not e <= b:
            self.failures.append("%s: fp32-output error %.3e exceeds %.1e of the reference scale" % (what, e, b))
        es, _ = conv_error(got_stored64, ref, self.is_fp32)
        self.worst_stored = max(self.worst_stored, es)

    def add_rne(self, what, equal):
        self.rne_checked += 1
        if not equal:
            self.rne_equal = False
            self.failures.append("%s: stored 16-bit output differs from the fp32 output rounded to nearest-even" % what)

    def ok(self):
        return not self.failures

    def report(self):
        return {"ok": self.ok(), "fp32_out_max_err": self.worst, "bound": self.bound,
                "scale": "max|ref|" if self.is_fp32 else "rms(ref)",
                "convolutions_vs_oracle": self.n_oracle,
                "stored_equals_rne_of_fp32_out": (self.rne_equal if self.rne_checked else None),
                "layers_rne_checked": self.rne_checked,
                "stored_out_max_err": self.worst_stored, "failures": self.failures[:4]}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=300,
                    help="untimed steps in front of the timed ones.  The chip needs tens of milliseconds of load to reach "
                         "its steady clocks: the first steps after an idle phase run about 15 %% slower than the rest")
    ap.add_argument("--event-every", type=int, default=10,
                    help="record the HIP events that time the three phases on every Nth timed step only: an event "
                         "record costs about 3 us of stream time (kernels on either side of it do not overlap), "
                         "and four per step took 6 %% off the throughput of a 0.2 ms step")
    ap.add_argument("--prewarm-ms", type=float, default=100.0,
                    help="besides the warm-up steps: keep running untimed steps until this much wall time has passed, so "
                         "that a small --warmup still measures steady clocks (0: off)")
    ap.add_argument("--workload", choices=sorted(WORKLOADS), default="cfg4",
                    help="cfg4 (RetinaNet-shaped head, the largest shapes) is the headline workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense torch conv2d comparator")
    ap.add_argument("--no-forward", action="store_true",
                    help="skip the YOLOv5s-shaped forward (cfg5) that the default run reports next to cfg4")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="target wall time of the oracle sample")
    ap.add_argument("--graph", choices=["auto", "on", "off"], default="auto",
                    help="replay the step from three captured HIP graphs (select, pack, conv) instead of enqueueing "
                         "every call from Python; auto: when the workload has more than 8 layers, where the host "
                         "time per launch exceeds the kernels' (a graph launch itself costs about 10 us)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 256 MiB device copy (a reference dispatch of known traffic for "
                         "scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--k", type=int, default=0,
                    help="entries kept per kernel instead of the workload's own (the axis of the sensitivity study, "
                         "Table 3)")
    ap.add_argument("--dict-top", type=int, default=0,
                    help="reduce the dictionary to its M most used patterns first (Section IV.B, second criterion: "
                         "winners counted over 2^20 random kernels in [-1, 1]) and run the step with that")
    ap.add_argument("--per-layer", action="store_true", help="after the timed region, time every layer's conv alone (stderr)")
    return ap.parse_args()


class Workload:
    """Device-resident tensors of one configuration and the three phases of a step."""

    prewarm_ms = 100.0  # see --prewarm-ms
    event_every = 10    # see --event-every

    def __init__(self, cfg, dev, dict_top=0):
        import torch
        from paper_2303_02191_amd import binding as B
        from paper_2303_02191_amd import pipeline as pl
        from paper_2303_02191_amd import workloads as wl
        self.torch, self.B, self.pl, self.wl = torch, B, pl, wl
        self.cfg = cfg
        self.masks = B.rtoss_pattern_dict(cfg.k)
        self.tdt = pl.TORCH_DTYPE[cfg.dtype]
        self.dict_counts = None
        if dict_top:
            g = torch.Generator(device=dev)
            g.manual_seed(cfg.seed + 1000)
            w_rand = (torch.rand((1 << 20) * 9, generator=g, device=dev, dtype=torch.float32) * 2 - 1).to(self.tdt)
            self.masks, kept, counts = pl.reduce_dictionary(self.masks, w_rand, cfg.dtype, dict_top)
            self.dict_counts = {"kept": [int(i) for i in kept], "wins": [int(c) for c in counts]}
            del w_rand
        # ---- inputs: weights drawn on the host (seeded numpy), activations on the device (seeded torch) ----
        rng = np.random.default_rng(cfg.seed)
        gen = torch.Generator(device=dev)
        gen.manual_seed(cfg.seed)
        self.w_host = [wl.draw_w(rng, cfg, L) for L in cfg.layers]
        # all 3x3 tensors live in one contiguous buffer so that one select item covers them
        self.n3 = sum(L.n_weights for L in cfg.layers if L.ksize == 3)
        self.w3_all = torch.empty(max(self.n3, 1), dtype=self.tdt, device=dev)
        self.idx3_all = torch.empty(max(self.n3 // 9, 1), dtype=torch.uint8, device=dev)
        self.w_dev, self.idx_dev, off = [], [], 0
        for L, (ws, _) in zip(cfg.layers, self.w_host):
            if L.ksize == 3:
                view = self.w3_all[off: off + L.n_weights]
                view.copy_(pl.to_device(ws.reshape(-1), cfg.dtype))
                self.w_dev.append(view)
                self.idx_dev.append(self.idx3_all[off // 9: (off + L.n_weights) // 9])
                off += L.n_weights
            else:
                self.w_dev.append(pl.to_device(ws.reshape(-1), cfg.dtype))
                self.idx_dev.append(torch.empty(max(L.groups, 1), dtype=torch.uint8, device=dev))

        def draw_act(L):
            shape = (cfg.N, L.H, L.W, L.Ci)  # channels-last
            if cfg.x_dist == "normal":
                a = torch.randn(shape, generator=gen, device=dev, dtype=torch.float32)
            else:
                a = torch.rand(shape, generator=gen, device=dev, dtype=torch.float32) * 2 - 1
            return a.to(self.tdt)

        self.xs, self.ys = [], []
        for i, L in enumerate(cfg.layers):
            self.xs.append(self.ys[i - 1] if cfg.chained and i > 0 else draw_act(L))
            self.ys.append(torch.empty((cfg.N, L.Ho, L.Wo, L.Co), dtype=self.tdt, device=dev))
        self.layers = [pl.PackedLayer(L.Co, L.Ci, L.ksize, cfg.k, cfg.dtype, self.masks) for L in cfg.layers]
        torch.cuda.synchronize()

    def do_select(self):
        # one batched call: all 3x3 kernels as one tensor, every 1x1 tensor as an item of its own
        items = []
        if self.n3:
            items.append((self.w3_all.data_ptr(), self.n3, self.idx3_all.data_ptr()))
        for L, w, idx in zip(self.cfg.layers, self.w_dev, self.idx_dev):
            if L.ksize == 1:
                items.append((w.data_ptr(), L.n_weights, idx.data_ptr()))
        self.B.rtoss_select_patterns_batch(items, self.cfg.dtype, self.masks, self.torch.cuda.current_stream().cuda_stream)

    def do_pack(self):
        self.pl.pack_layers(self.layers, self.w_dev, self.idx_dev)  # a launch per (format, dtype) group of layers

    def do_conv(self):
        for L, lay, x, y in zip(self.cfg.layers, self.layers, self.xs, self.ys):
            lay.conv(x, stride=L.stride, relu=L.relu, y=y)

    def time_steps(self, steps, warmup, use_graph, before_warmup=None):
        """Returns (ms_per_step, select_ms, pack_ms, conv_ms): wall clock around `steps` steps, and HIP-event
        means of the three phases inside them."""
        torch = self.torch
        phases = [self.do_select, self.do_pack, self.do_conv]
        for f in phases:  # first launches also set kernel attributes: must happen outside capture
            f()
        torch.cuda.synchronize()
        if use_graph:
            # The library allocates nothing and records no memset, so its launches capture as plain
            # kernel nodes; three graphs so that the phases can still be timed apart.
            graphs = []
            for f in phases:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    f()
                graphs.append(g)
            self._graphs = graphs
            phases = [g.replay for g in graphs]
        ev = lambda: torch.cuda.Event(enable_timing=True)

        def step(events=None):
            for i, f in enumerate(phases):
                if events:
                    events[i].record()
                f()
            if events:
                events[3].record()

        t_start_warm = time.perf_counter()
        if before_warmup:
            before_warmup()
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        t_end = time.perf_counter() + self.prewarm_ms * 1e-3 - (time.perf_counter() - t_start_warm)
        while time.perf_counter() < t_end:  # (untimed: brings the clocks to their steady state)
            for _ in range(10):
                step()
            torch.cuda.synchronize()
        every = max(1, min(self.event_every, steps))
        all_events = [[ev() for _ in range(4)] for _ in range((steps + every - 1) // every)]
        t0 = time.perf_counter()
        for s in range(steps):
            step(all_events[s // every] if s % every == 0 else None)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms = (t1 - t0) * 1e3 / steps
        sel = float(np.mean([e[0].elapsed_time(e[1]) for e in all_events]))
        pack = float(np.mean([e[1].elapsed_time(e[2]) for e in all_events]))
        conv = float(np.mean([e[2].elapsed_time(e[3]) for e in all_events]))
        return ms, sel, pack, conv

    def check_rne(self, parity):
        """Every layer once more with fp32 output: the stored 16-bit output of the timed step must be that
        result rounded once to nearest-even (bit for bit).  Returns the fp32 outputs of the layers in `keep`."""
        torch, cfg = self.torch, self.cfg
        if cfg.dtype == self.wl.F32:
            return
        for i, (L, lay, x, y) in enumerate(zip(cfg.layers, self.layers, self.xs, self.ys)):
            y32 = lay.conv(x, stride=L.stride, relu=L.relu, out_dt=self.wl.F32)
            same = torch.equal(y32.to(self.tdt).view(torch.int16), y.view(torch.int16))
            parity.add_rne("layer %d" % i, bool(same))
            del y32
        torch.cuda.synchronize()

    def oracle_sample(self, parity, seconds):
        """The oracle over whole (layer, batch item) convolutions, in layer-major order until `seconds` of
        oracle conv time are used; each is compared with what the GPU computed.  Returns the cpu_baseline dict."""
        import oracle
        cfg, wl, pl = self.cfg, self.wl, self.pl
        t_sel = time.perf_counter()
        masked = []
        for L, (ws, wv) in zip(cfg.layers, self.w_host):
            masked.append(oracle.mask(wv, self.masks, oracle.select(wv, self.masks)))
        t_sel = time.perf_counter() - t_sel
        done_macs, t_conv, n_done = 0.0, 0.0, 0
        for li, L in enumerate(cfg.layers):
            if t_conv >= seconds:
                break
            y32 = None
            for n in range(cfg.N):
                if t_conv >= seconds:
                    break
                if y32 is None:  # the same convolution with fp32 output: what the tolerance is stated for
                    y32 = self.layers[li].conv(self.xs[li], stride=L.stride, relu=L.relu, out_dt=wl.F32)
                    self.torch.cuda.synchronize()
                x0 = pl.to_host(self.xs[li][n:n + 1]).copy()  # [1, H, W, Ci] storage, as the GPU saw it
                xv = wl.to_f64(wl.nhwc_to_nchw(x0), cfg.dtype)
                t_a = time.perf_counter()
                ref = oracle.conv2d(xv, masked[li], stride=L.stride, relu=L.relu)
                t_conv += time.perf_counter() - t_a
                got32 = wl.nhwc_to_nchw(pl.to_host(y32[n:n + 1])).astype(np.float64)
                got = wl.to_f64(wl.nhwc_to_nchw(pl.to_host(self.ys[li][n:n + 1])), cfg.dtype)
                parity.add_oracle("layer %d item %d" % (li, n), got32, got, ref)
                done_macs += L.Ho * L.Wo * cfg.k * L.groups
                n_done += 1
            del y32
        return {"value": 2.0 * done_macs / max(t_conv, 1e-9) / 1e12, "unit": "TFLOP/s", "cores": oracle.threads(),
                "kind": "oracle",
                "sample": "%d whole (layer, batch item) convolutions of %s in layer-major order, %.2f s of oracle "
                          "conv time; select+mask of all %d groups took %.3f s" % (
                              n_done, cfg.name, t_conv, sum(L.groups for L in cfg.layers), t_sel)}


def roofline_of(cfg, wl, workload, conv_ms, k_override):
    n_conv = len(cfg.layers)
    conv_launch_s = conv_ms * 1e-3 / n_conv
    nz_flops = 2.0 * cfg.nonzero_macs()
    if workload in ("cfg2", "cfg3", "cfg5"):
        alg_bytes = cfg.algorithmic_bytes() / n_conv
        achieved = alg_bytes / conv_launch_s / 1e9
        r = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
             "frac": achieved / PEAK_HBM_GBS, "traffic": None}
    elif cfg.dtype == wl.F32:
        achieved = nz_flops / n_conv / conv_launch_s / 1e12
        # fp32 3x3 layers run on the fp32 matrix instruction, whose dense peak equals the vector peak (157.3)
        r = {"bound": "mfma", "achieved": achieved, "peak": PEAK_FP32_VECTOR_TFLOPS, "unit": "TFLOP/s",
             "frac": achieved / PEAK_FP32_VECTOR_TFLOPS, "traffic": None}
    else:
        achieved = nz_flops / n_conv / conv_launch_s / 1e12
        r = {"bound": "mfma", "achieved": achieved, "peak": PEAK_MFMA_16BIT_TFLOPS, "unit": "TFLOP/s",
             "frac": achieved / PEAK_MFMA_16BIT_TFLOPS, "traffic": None}
    if workload == "cfg4" and not k_override:
        r["traffic"] = measured_traffic("conv3x3_rows_cfg4_hbm_traffic.txt")
    r["kernel"] = "rtoss_conv2d_pattern"
    r["avg_launch_us"] = conv_launch_s * 1e6
    r["launches_per_step"] = n_conv
    return r


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: one GPU only; --gpus %d is not supported (the path would shard by batch, with no "
              "collective; this program measures a single device)" % args.gpus, file=sys.stderr)
        return 2

    import torch
    from paper_2303_02191_amd import binding as B
    from paper_2303_02191_amd import pipeline as pl
    from paper_2303_02191_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    B.lib()  # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    cfg = wl.get_config(WORKLOADS[args.workload])
    if args.k:
        import dataclasses
        cfg = dataclasses.replace(cfg, k=args.k, name="%s_k%d" % (cfg.name, args.k))
    eb = wl.ELEM_BYTES[cfg.dtype]
    Workload.prewarm_ms = args.prewarm_ms
    Workload.event_every = args.event_every
    work = Workload(cfg, dev, args.dict_top)
    masks, dict_counts = work.masks, work.dict_counts
    ev = lambda: torch.cuda.Event(enable_timing=True)
    use_graph = args.graph == "on" or (args.graph == "auto" and len(cfg.layers) > 8)

    def copy_probe():
        if args.copy_probe:
            src = torch.zeros(64 << 20, dtype=torch.float32, device=dev)
            dst = torch.empty_like(src)
            torch.add(src, 1.0, out=dst)  # one elementwise kernel: reads 256 MiB, writes 256 MiB
            torch.cuda.synchronize()

    def time_call(fn, iters=20):
        """Mean ms per call of fn at steady clocks: untimed calls for at least 60 ms (and at least 5), then `iters`."""
        t0 = time.perf_counter()
        n = 0
        while n < 5 or time.perf_counter() - t0 < 0.06:
            fn()
            n += 1
            if n % 5 == 0:
                torch.cuda.synchronize()
        torch.cuda.synchronize()
        a, b = ev(), ev()
        a.record()
        for _ in range(iters):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / iters

    ms_per_step, sel_ms, pack_ms, conv_ms = work.time_steps(args.steps, args.warmup, use_graph, copy_probe)
    nz_flops = 2.0 * cfg.nonzero_macs()
    value = nz_flops / (ms_per_step * 1e-3) / 1e12
    roofline = roofline_of(cfg, wl, args.workload, conv_ms, args.k)
    layers, xs, ys, w_dev, w_host = work.layers, work.xs, work.ys, work.w_dev, work.w_host

    if args.per_layer:
        print("layer  Ci   Co    H  ks s   conv_us  hbm_ideal_us  mfma_ideal_us(nz)", file=sys.stderr)
        for i, (L, lay, x, y) in enumerate(zip(cfg.layers, layers, xs, ys)):
            t_layer = time_call(lambda: lay.conv(x, stride=L.stride, relu=L.relu, y=y))
            byts = cfg.N * (L.Ci * L.H * L.W + L.Co * L.Ho * L.Wo) * eb + L.groups * (cfg.k * eb + 1)
            nz = 2.0 * cfg.N * L.Ho * L.Wo * cfg.k * L.groups
            print("%3d %5d %4d %4d  %d %d  %8.1f  %8.2f  %8.2f" % (i, L.Ci, L.Co, L.H, L.ksize, L.stride,
                  t_layer * 1e3, byts / PEAK_HBM_GBS / 1e3, nz / PEAK_MFMA_16BIT_TFLOPS / 1e6), file=sys.stderr)

    # ---- parity of what was just timed ----
    parity = Parity(cfg.dtype == wl.F32)
    work.check_rne(parity)
    cpu = None
    if not args.no_cpu_baseline:
        cpu = work.oracle_sample(parity, args.cpu_seconds)

    # ---- dense comparator: torch conv2d (MIOpen / hipBLASLt) on the same shapes, bench only ----
    dense_ms = None
    if not args.no_dense:
        try:
            dense_ms = 0.0
            for L, (ws, _), x in zip(cfg.layers, w_host, xs):
                wt = pl.to_device(ws, cfg.dtype).contiguous(memory_format=torch.channels_last)
                xt = x.permute(0, 3, 1, 2)  # NCHW view of channels-last storage
                dense_ms += time_call(lambda: torch.nn.functional.conv2d(xt, wt, stride=L.stride, padding=L.pad))
        except Exception as e:  # comparator only
            dense_ms = None
            print("dense comparator failed: %r" % (e,), file=sys.stderr)

    # ---- dense comparator 2: this library's own kernels in dense mode (the all-ones pattern keeps every
    # weight; the matrix-core kernels then run with nothing to skip) on the same tensors.  (The 1x1 kernels
    # multiply zero-filled fragments either way: for 1x1 layers this is the same launch as the pruned one.) ----
    dense_own_ms = None
    if not args.no_dense:
        masks9 = B.rtoss_pattern_dict(9)
        dense_own_ms = 0.0
        for L, w, x, y in zip(cfg.layers, w_dev, xs, ys):
            # (a flattened 1x1 tensor's tail of < 9 weights is pruned by definition; the rest is dense)
            idx9 = torch.zeros(max(L.n_weights // 9, 1), dtype=torch.uint8, device=dev)
            lay9 = pl.PackedLayer(L.Co, L.Ci, L.ksize, 9, cfg.dtype, masks9).pack(w, idx9)
            yd = torch.empty_like(y)
            t9 = time_call(lambda: lay9.conv(x, stride=L.stride, relu=L.relu, y=yd))
            dense_own_ms += t9
            if args.per_layer:
                print("dense mode, own kernel: Ci %4d Co %4d H %3d ks %d s %d  %8.1f us" %
                      (L.Ci, L.Co, L.H, L.ksize, L.stride, t9 * 1e3), file=sys.stderr)
            del lay9, yd

    # ---- block-shared patterns (layers that take over a parent's patterns, shared per run of 8 input channels):
    # the same layers with such indices through the gather path on the dense instruction and through the
    # 2-of-4 path, for comparison (bench only; not part of the timed step) ----
    coherent = None
    if not args.no_dense and cfg.dtype != wl.F32 and all(L.ksize == 3 and L.Ci % 32 == 0 and L.Co % 16 == 0 for L in cfg.layers):
        rngc = np.random.default_rng(cfg.seed + 100)
        t_gather = t_sparse = 0.0
        steps_seen = set()
        for L, w, x, y in zip(cfg.layers, w_dev, xs, ys):
            idxc = np.repeat(rngc.integers(0, len(masks), L.Ci // 8), 8)[None, :].repeat(L.Co, 0).astype(np.uint8).reshape(-1)
            idxc = torch.from_numpy(idxc).to(dev)
            layc = pl.CoherentLayer(L.Co, L.Ci, cfg.k, cfg.dtype, masks).pack(w, idxc)
            lays = pl.PackedLayer(L.Co, L.Ci, 3, cfg.k, cfg.dtype, masks).pack(w, idxc)
            steps_seen |= set(np.unique(layc.steps()).tolist())
            yd = torch.empty_like(y)
            t_gather += time_call(lambda: layc.conv(x, stride=L.stride, relu=L.relu, y=yd))
            t_sparse += time_call(lambda: lays.conv(x, stride=L.stride, relu=L.relu, y=yd))
            del layc, lays, yd
        coherent = {"patterns": "one per run of 8 input channels, shared by all output channels",
                    "dense_steps_per_stage": sorted(int(v) for v in steps_seen),
                    "gather_path_conv_ms": t_gather, "two_of_four_path_conv_ms": t_sparse,
                    "gather_path_frac_of_peak": nz_flops / (t_gather * 1e-3) / 1e12 / PEAK_MFMA_16BIT_TFLOPS}

    # ---- the metric's second half: ms per YOLOv5s-shaped forward (cfg5), replayed from HIP graphs ----
    forward = None
    ok = parity.ok()
    if args.workload == "cfg4" and not args.k and not args.no_forward:
        del work, layers, xs, ys, w_dev
        torch.cuda.empty_cache()
        cfg5 = wl.get_config(5)
        w5 = Workload(cfg5, dev)
        f_ms, f_sel, f_pack, f_conv = w5.time_steps(args.steps, args.warmup, True)
        p5 = Parity(False)
        w5.check_rne(p5)
        if not args.no_cpu_baseline:
            w5.oracle_sample(p5, min(3.0, args.cpu_seconds))
        r5 = roofline_of(cfg5, wl, "cfg5", f_conv, 0)
        forward = {"workload": cfg5.name, "ms_per_forward": f_ms, "launch": "hip_graph", "steps": args.steps,
                   "batch": cfg5.N, "layers": len(cfg5.layers), "dtype": wl.DTYPE_NAMES[cfg5.dtype],
                   "breakdown_ms": {"select": f_sel, "pack": f_pack, "conv": f_conv},
                   "effective_tflops": 2.0 * cfg5.nonzero_macs() / (f_ms * 1e-3) / 1e12,
                   "roofline": r5, "parity": p5.report()}
        ok = ok and p5.ok()

    out = {
        "metric": "effective TFLOP/s on non-zero MACs, select+pack+pattern-sparse conv",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "prewarm_ms": args.prewarm_ms, "phase_events_every": args.event_every, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.DTYPE_NAMES[cfg.dtype], "data": "synthetic",
        "launch": "hip_graph" if use_graph else "eager",
        "config": {"workload": cfg.name, "batch": cfg.N, "layers": len(cfg.layers), "k": cfg.k,
                   "patterns": int(masks.size), "nonzero_gflop_per_step": nz_flops / 1e9,
                   "dense_gflop_per_step": 2.0 * cfg.dense_macs() / 1e9},
        "breakdown_ms": {"select": sel_ms, "pack": pack_ms, "conv": conv_ms,
                         "dense_torch_conv2d": dense_ms, "dense_own_kernels": dense_own_ms},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "parity": parity.report(),
        "coherent_patterns": coherent,
        "yolo5s_forward": forward,
    }
    if dict_counts:
        out["config"]["dictionary_reduction"] = dict_counts
    print(json.dumps(out))
    if not ok:
        print("bench.py: PARITY FAILED: the numbers above describe a wrong result", file=sys.stderr)
        return 1
    return 0


if __name__ == "__main__":
    sys.exit(main())

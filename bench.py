"""Benchmark of the access-pattern hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

The default workload is the ResNet-18-shaped stack at batch 64, the largest of the five
configurations and the only one that passes through every step of the hot path.  The other
workloads time one step of the path each (conv3x3, im2col_gather, maxpool, reduce, dense, mlp,
mlp_scaled), HBM-bound ones in GB/s of algorithmic bytes.

A step is one pass of the workload's whole call sequence over one batch of synthetic input that
is already resident in HBM.  Steps are captured once into HIP graphs (one per rotating buffer
set, so that consecutive steps do not find their inputs in cache) and replayed; the timed region
is exactly K steps between two device synchronisations.  Prints one JSON line.
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import torch  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_I8_TOPS = 5000.0         # MI355X dense int8 MFMA
PEAK_F8_TFLOPS = 5000.0       # MI355X dense fp8 MFMA
PEAK_HBM_GBS = 8000.0
ROTATE_BYTES = 512 << 20      # rotate over enough buffer sets to exceed the last-level cache
DOM_BATCH = 20                # launches of the dominant kernel per timing graph

# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (each
# scaled by the same counter's reading for a plain copy of known size; see profiles/).  A reading
# only counts for the kernel sources it was taken with: their hash is stored beside it and the
# bench reports null once the sources differ.
KERNEL_SOURCES = {
    "conv": ("conv4_kernel.h", "conv_kernels.h", "conv3_inst.hip", "conv.hip", "common.h"),
    "windows": ("windows.hip", "common.h"),
    "reduce": ("reduce.hip", "common.h"),
    "move": ("move.hip", "common.h"),
    "gemm": ("gemm.hip", "common.h"),
    "depthwise": ("depthwise.hip", "common.h"),
}
# workload -> (fetch + write bytes per launch of its dominant kernel, source group, digest of the
# sources the counters were taken with)
TRAFFIC = {
    "resnet18": (26.75e6 + 25.69e6, "conv", "f4748cc2caa3c2531990a0702814e011d54d0b5a9e9a12edc92d73cba98f0991"),       # the stage-1 convolution measured on its own (conv3x3_b64), without the residual every second launch reads
    "conv3x3": (13.90e6 + 12.85e6, "conv", "f4748cc2caa3c2531990a0702814e011d54d0b5a9e9a12edc92d73cba98f0991"),
    "conv3x3_b64": (26.75e6 + 25.69e6, "conv", "f4748cc2caa3c2531990a0702814e011d54d0b5a9e9a12edc92d73cba98f0991"),
    "im2col_gather": (12.97e6 + 115.65e6, "windows", "28be54f8a8d040349c57db5f9820cda36bffe90e20b1b9dee462b12e92a66d8b"),
    "maxpool": (103.00e6 + 25.69e6, "reduce", "b45ea8b2d26f14f5a55128314b01ed29d77f86f18a0cd19592276c47d9523874"),
    "reduce": (268.44e6 + 0.52e6, "reduce", "b45ea8b2d26f14f5a55128314b01ed29d77f86f18a0cd19592276c47d9523874"),
    "transpose": (25.82e6 + 25.70e6, "move", "3f71ed284b450b94c97176cd729f28061f8fef2f40f28ca8a27bfbf72e4a3d62"),
    "dense_blocked": (50.63e6 + 16.78e6, "gemm", "26fb4e7e86e567072c495a5931bb5d3a671db0d4bbb0683e7d6380e858d29ee1"),
    "dense": (1611.42e6 + 281.85e6, "gemm", "26fb4e7e86e567072c495a5931bb5d3a671db0d4bbb0683e7d6380e858d29ee1"),
    "mlp_scaled": (28.91e6 + 16.78e6, "gemm", "26fb4e7e86e567072c495a5931bb5d3a671db0d4bbb0683e7d6380e858d29ee1"),
    "conv3x3_i8": (7.15e6 + 25.69e6, "conv", "f4748cc2caa3c2531990a0702814e011d54d0b5a9e9a12edc92d73cba98f0991"),
    "dense_i8": (805.93e6 + 287.46e6, "gemm", "26fb4e7e86e567072c495a5931bb5d3a671db0d4bbb0683e7d6380e858d29ee1"),
    "dense_fp8": (806.21e6 + 134.22e6, "gemm", "26fb4e7e86e567072c495a5931bb5d3a671db0d4bbb0683e7d6380e858d29ee1"),
    "depthwise": (103.03e6 + 102.76e6, "depthwise", "c9515252f603786f310d6a9178342e1244cdadaa9101f1a1d8b67c2f26904071"),
}


def _sources_digest(group):
    import hashlib
    h = hashlib.sha256()
    for f in KERNEL_SOURCES[group]:
        with open(os.path.join(ROOT, "paper_2105_09377_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def _traffic(workload):
    t = TRAFFIC.get(workload)
    return t[0] if t and t[2] == _sources_digest(t[1]) else None


def _graph_of(fn, stream):
    """Capture fn() (already warmed up) into a HIP graph on `stream`."""
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=stream):
        fn()
    return g


def _time_region(launchers, steps, stream):
    """Run `steps` launches (launcher i % len) and return (wall seconds, event milliseconds)."""
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    with torch.cuda.stream(stream):
        start.record(stream)
        for i in range(steps):
            launchers[i % len(launchers)]()
        stop.record(stream)
    torch.cuda.synchronize()
    return time.perf_counter() - t0, start.elapsed_time(stop)


def _max_rel_err(got, ref):
    """max |got - ref| / max |ref|: the timed buffers against the oracle's values (fp64 / int64),
    relative to the largest magnitude of the reference (the measure the whole-stack parity test
    bounds by 1e-2); 0.0 means bit-exact integers."""
    import numpy as np
    g = got.detach().cpu()
    g = g.to(torch.float64).numpy() if g.dtype.is_floating_point else g.numpy().astype(np.int64)
    r = np.asarray(ref)
    assert g.shape == r.shape, (g.shape, r.shape)
    if r.size == 0:
        return 0.0
    r = r.astype(np.float64)
    finite = np.isfinite(r)
    if not np.array_equal(np.isfinite(g), finite) or not np.array_equal(g[~finite], r[~finite]):
        return float("inf")
    return float(np.abs(g[finite] - r[finite]).max() / max(np.abs(r[finite]).max(), 1e-30)) if finite.any() else 0.0


def _bf16_to_f64(t):
    """Exact float64 values of a CPU bfloat16 tensor (for the CPU baseline's oracle)."""
    import numpy as np
    from oracle import numerics
    return numerics.bf16_bits_to_f64(t.contiguous().view(torch.int16).numpy().view(np.uint16))


class Conv3x3:
    """ResNet-style 3x3 convolution: N=32, C=64, 56x56 -> 64 channels, stride 1, pad 1, bf16."""

    batch = 32
    in_dtype = "bf16"
    dominant = "conv_direct4_kernel"
    name = property(lambda self: f"resnet-style 3x3 conv N={self.batch} C=64 H=W=56 O=64 s1 p1, " +
                                 ("bf16 in/out, fp32 accumulate" if self.in_dtype == "bf16" else "int8 in, int32 out"))

    def __init__(self, dev):
        from paper_2105_09377_amd import binding as gs, synth
        self.gs = gs
        cfg = synth.resnet_conv3x3(self.in_dtype, self.batch)
        self.cfg = cfg
        x, w = cfg["x"], cfg["w"]
        self.flops = 2.0 * self.batch * 56 * 56 * 64 * 64 * 9
        set_bytes = x.numel() * x.element_size() + x.numel() * (2 if self.in_dtype == "bf16" else 4)
        self.nsets = max(2, min(48, -(-ROTATE_BYTES // set_bytes)))
        self.w = w.to(dev)
        self.xs = [x.to(dev).clone() for _ in range(self.nsets)]
        out_dtype = torch.bfloat16 if self.in_dtype == "bf16" else torch.int32
        self.outs = [torch.empty((self.batch, 64, 56, 56), dtype=out_dtype, device=dev) for _ in range(self.nsets)]
        self.ws = torch.empty(gs.conv2d_workspace(self.xs[0], self.w, (1, 1), (1, 1)), dtype=torch.uint8, device=dev)
        self.packed = gs.conv2d_pack_weights(self.w)

    def step(self, i):
        """The public entry point as a user calls it: weight packing + convolution."""
        self.gs.conv2d_direct(self.xs[i], self.w, (1, 1), (1, 1), out=self.outs[i], workspace=self.ws)

    def dominant_launch(self, i):
        """The convolution kernel alone (weights packed beforehand)."""
        self.gs.conv2d_direct_packed(self.xs[i], self.w, self.packed, (1, 1), (1, 1), out=self.outs[i])

    dominant_flops = property(lambda self: self.flops)

    def cpu_baseline(self):
        import numpy as np
        from oracle import brute, numerics
        n = 32              # images of the workload that the oracle is timed on
        x = self.cfg["x"][:n].contiguous()
        xo = numerics.bf16_bits_to_f64(x.view(torch.int16).numpy().view(np.uint16))
        wo = numerics.bf16_bits_to_f64(self.cfg["w"].view(torch.int16).numpy().view(np.uint16))
        brute.conv2d(xo[:1], wo, (1, 1), (1, 1))
        t0 = time.perf_counter()
        ref = brute.conv2d(xo, wo, (1, 1), (1, 1))
        dt = time.perf_counter() - t0
        return {"value": self.flops * n / self.batch / dt / 1e12, "unit": "TFLOP/s", "cores": brute.num_threads(),
                "kind": "oracle", "sample": f"brute-force C loops (fp64, OpenMP) on {n} images of the workload, {dt:.2f} s",
                "max_rel_err": _max_rel_err(self.outs[0][:n], ref)}


class Conv3x3Int8(Conv3x3):
    """The same convolution with int8 inputs and exact int32 results."""

    in_dtype = "i8"
    dtype = "i8"
    bound, unit, peak = "mfma", "TOP/s", PEAK_I8_TOPS

    def cpu_baseline(self):
        import numpy as np
        from oracle import brute
        n = 32
        xo = self.cfg["x"][:n].numpy().astype(np.int64)
        wo = self.cfg["w"].numpy().astype(np.int64)
        brute.conv2d(xo[:1], wo, (1, 1), (1, 1))
        t0 = time.perf_counter()
        ref = brute.conv2d(xo, wo, (1, 1), (1, 1))
        dt = time.perf_counter() - t0
        return {"value": self.flops * n / self.batch / dt / 1e12, "unit": "TOP/s", "cores": brute.num_threads(),
                "kind": "oracle", "sample": f"brute-force C loops (int64, OpenMP) on {n} images of the workload, {dt:.2f} s",
                "max_rel_err": _max_rel_err(self.outs[0][:n], ref)}


class Conv3x3Batch64(Conv3x3):
    """The same convolution at batch 64: the stack's stage-1 layer (its dominant kernel) on its own."""

    batch = 64


class ResNet18:
    """ResNet-18-shaped stack forward at batch 64 (the largest of the five workloads): 7x7 stem
    convolution, max pooling, sixteen 3x3 convolutions (direct form) and three 1x1 stride-2
    projections (im2col form) with fused residual / ReLU, global average, classifier."""

    name = "resnet18-shaped conv stack forward, batch 64, 3x224x224, bf16 in/out, fp32 accumulate"
    dominant = "conv_direct4_kernel (stage 1: N=64 C=64 56x56 -> 64, 3x3 s1 p1; 4 of the 20 convolutions)"

    def __init__(self, dev):
        from paper_2105_09377_amd import binding as gs, synth
        from paper_2105_09377_amd.resnet import ResNet18Stack
        self.gs = gs
        self.cfg = synth.resnet18_stack(batch=64, image=224)
        self.nsets = 2                       # one step touches > 600 MB: two sets defeat every cache
        self.nets = [ResNet18Stack(self.cfg["weights"], 64, 224, dev) for _ in range(self.nsets)]
        for net in self.nets:
            net.x.copy_(self.cfg["x"])
        hw, flops = 224, 0.0
        for name, cin, cout, k, s, p in synth.RESNET18_CONVS:
            if name == "conv1":
                hin = hw
                hw = (hw + 2 * p - k) // s + 1
                out_hw = hw
                hw = (hw + 2 - 3) // 2 + 1          # max pooling
            elif name.endswith("c1"):
                hin = hw
                hw = (hw + 2 * p - k) // s + 1
                out_hw = hw
            else:
                out_hw = hw
            flops += 2.0 * 64 * out_hw * out_hw * cout * cin * k * k
        flops += 2.0 * 64 * 512 * 1000
        self.flops = flops
        self.dominant_flops = 2.0 * 64 * 56 * 56 * 64 * 64 * 9
        # The dominant kernel on its own: the stage-1 convolution on rotating inputs and outputs
        # that together exceed the last-level cache, so every launch reads its input from HBM.
        act_bytes = 64 * 64 * 56 * 56 * 2
        self.dom_sets = -(-ROTATE_BYTES // (2 * act_bytes))
        self.dom_x = [synth.normal_bf16((64, 64, 56, 56), 1.0, 7700).to(dev).clamp_(min=0) for _ in range(self.dom_sets)]
        self.dom_out = [torch.empty((64, 64, 56, 56), dtype=torch.bfloat16, device=dev) for _ in range(self.dom_sets)]

    def step(self, i):
        self.nets[i].forward()

    def dominant_launch(self, i):
        net, j = self.nets[0], i % self.dom_sets
        self.gs.conv2d_direct_packed(self.dom_x[j], net.w["s1b1c1"], net.packed["s1b1c1"], (1, 1), (1, 1),
                                     act=self.gs.GS_ACT_RELU, out=self.dom_out[j])

    def per_layer(self):
        """(name, call, work, unit) for every library call of one forward pass of buffer set 0."""
        from paper_2105_09377_amd import synth
        net, rows = self.nets[0], []
        spec = {name: (cin, cout, k) for name, cin, cout, k, _s, _p in synth.RESNET18_CONVS}
        for name, call in net.steps:
            if name in spec:
                cin, cout, k = spec[name]
                o = net.bufs[name]
                rows.append((name, call, 2.0 * o.shape[0] * o.shape[2] * o.shape[3] * cout * cin * k * k, "TFLOP/s"))
            elif name == "pool":
                rows.append((name, call, (net.bufs["conv1"].numel() + net.bufs["pool"].numel()) * 2.0, "GB/s"))
            elif name == "avg":
                rows.append((name, call, net.bufs["s4b2c2"].numel() * 2.0, "GB/s"))
            else:
                rows.append((name, call, 2.0 * 64 * 512 * net.logits.shape[1], "TFLOP/s"))
        return rows

    def cpu_baseline(self):
        from oracle import brute, resnet as oresnet
        from paper_2105_09377_amd import synth
        n = 64
        x = _bf16_to_f64(self.cfg["x"][:n])
        w = {k: _bf16_to_f64(v) for k, v in self.cfg["weights"].items()}
        t0 = time.perf_counter()
        ref = oresnet.forward(x, w, synth.RESNET18_CONVS)
        dt = time.perf_counter() - t0
        # the logits left in the timed buffers by the last timed step, all 64 images, against the
        # oracle's end-to-end logits (every layer's bfloat16 rounding compounds: the tests bound it by 1e-2)
        err = max(_max_rel_err(net.logits, ref["fc"]) for net in self.nets)
        return {"value": self.flops * n / 64 / dt / 1e12, "unit": "TFLOP/s", "cores": brute.num_threads(),
                "kind": "oracle", "sample": f"the stack oracle (fp64 C loops, OpenMP) on {n} of the 64 images, {dt:.1f} s",
                "max_rel_err": err}


class _Simple:
    """One library call per step on rotating buffer sets; the call is also the dominant kernel."""

    bound = "hbm"
    unit = "GB/s"
    peak = PEAK_HBM_GBS

    def dominant_launch(self, i):
        self.step(i)

    def _sets(self, set_bytes, cap=32):
        return max(2, min(cap, -(-ROTATE_BYTES // set_bytes)))


class Im2colGather(_Simple):
    """access_windows on the 3x3 workload: (32,64,56,56) bf16 -> the [100352, 576] im2col matrix."""

    name = "access_windows (im2col gather) N=32 C=64 H=W=56, window (64,3,3) s1 p1, bf16"
    dominant = "windows_chw_kernel"

    def __init__(self, dev):
        from paper_2105_09377_amd import binding as gs, synth
        self.gs, self.cfg = gs, synth.resnet_conv3x3("bf16", 32)
        x = self.cfg["x"]
        self.work = x.numel() * 2 + 32 * 56 * 56 * 576 * 2          # |in| + M*K*elt bytes
        self.nsets = self._sets(self.work, 6)
        self.xs = [x.to(dev).clone() for _ in range(self.nsets)]
        self.outs = [torch.empty((32, 1, 56, 56, 64, 3, 3), dtype=torch.bfloat16, device=dev) for _ in range(self.nsets)]

    def step(self, i):
        self.gs.access_windows(self.xs[i], 1, (64, 3, 3), (1, 1, 1), (0, 1, 1), (0, 1, 1), out=self.outs[i])

    def cpu_baseline(self):
        from oracle import access_pattern as ap
        x = _bf16_to_f64(self.cfg["x"][:4])
        t0 = time.perf_counter()
        ref = ap.windows(ap.access(ap.pad(ap.pad(ap.tensor(x), 2, 1, 1, 0.0), 3, 1, 1, 0.0), 1), (64, 3, 3), (1, 1, 1)).materialize()
        dt = time.perf_counter() - t0
        return {"value": self.work * 4 / 32 / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                "sample": f"access-pattern interpreter (numpy gather) on 4 of the 32 images, {dt:.2f} s",
                "max_rel_err": _max_rel_err(self.outs[0][:4], ref)}


class MaxPool(_Simple):
    """windows + reduceMax of the stack: (64,64,112,112) bf16, 3x3 stride 2 pad 1."""

    name = "windows + compute reduceMax (max-pool) (64,64,112,112) bf16, 3x3 s2 p1"
    dominant = "pool2d_vec_kernel"

    def __init__(self, dev):
        from paper_2105_09377_amd import binding as gs, synth
        self.gs = gs
        self.x = synth.normal_bf16((64, 64, 112, 112), 1.0, 7101)
        self.work = self.x.numel() * 2 + 64 * 64 * 56 * 56 * 2
        self.nsets = self._sets(self.work, 6)
        self.xs = [self.x.to(dev).clone() for _ in range(self.nsets)]
        self.outs = [torch.empty((64, 64, 56, 56), dtype=torch.bfloat16, device=dev) for _ in range(self.nsets)]

    def step(self, i):
        self.gs.windows_reduce(self.xs[i], 2, (3, 3), (2, 2), (1, 1), (1, 1), self.gs.GS_MAX, out=self.outs[i])

    def cpu_baseline(self):
        import numpy as np
        from oracle import brute
        x = _bf16_to_f64(self.x)
        t0 = time.perf_counter()
        ref = brute.max_pool2d(x, (3, 3), (2, 2), (1, 1), -np.inf)
        dt = time.perf_counter() - t0
        return {"value": self.work / dt / 1e9, "unit": "GB/s", "cores": brute.num_threads(), "kind": "oracle",
                "sample": f"brute-force C loops (fp64, OpenMP) on the whole tensor, {dt:.2f} s",
                "max_rel_err": _max_rel_err(self.outs[0], ref)}


class Depthwise(_Simple):
    """Depth-wise windows: (32,128,112,112) bf16, one 3x3 filter per channel, stride 1, pad 1."""

    name = "depth-wise 3x3 s1 p1 on (32,128,112,112) bf16 -> bf16 (one filter per channel)"
    dominant = "depthwise_kernel"

    def __init__(self, dev):
        from paper_2105_09377_amd import binding as gs, synth
        self.gs = gs
        self.x = synth.normal_bf16((32, 128, 112, 112), 1.0, 7601)
        self.w = synth.normal_bf16((128, 3, 3), 1.0 / 3.0, 7602)
        self.work = 2 * self.x.numel() * 2 + self.w.numel() * 2
        self.nsets = self._sets(self.work, 6)
        self.xs = [self.x.to(dev).clone() for _ in range(self.nsets)]
        self.wd = self.w.to(dev)
        self.outs = [torch.empty((32, 128, 112, 112), dtype=torch.bfloat16, device=dev) for _ in range(self.nsets)]

    def step(self, i):
        self.gs.depthwise_conv2d(self.xs[i], self.wd, (1, 1), (1, 1), out=self.outs[i])

    def cpu_baseline(self):
        import numpy as np
        from oracle import brute
        n = 8
        x, w = _bf16_to_f64(self.x[:n]), _bf16_to_f64(self.w)
        t0 = time.perf_counter()
        ref = []
        for c in range(128):       # channel c against filter c: the one-channel program of Fig. 2a
            ref.append(brute.conv2d(np.ascontiguousarray(x[:, c:c + 1]), np.ascontiguousarray(w[c:c + 1, None]), (1, 1), (1, 1)))
        dt = time.perf_counter() - t0
        return {"value": self.work * n / 32 / dt / 1e9, "unit": "GB/s", "cores": brute.num_threads(), "kind": "oracle",
                "sample": f"brute-force C loops (fp64, OpenMP), channel by channel, on {n} of the 32 images, {dt:.2f} s",
                "max_rel_err": _max_rel_err(self.outs[0][:n], np.concatenate(ref, axis=1))}


class Transpose(_Simple):
    """transpose (0 3 1 2): the (N,H',W',O) -> (N,O,H',W') tail of the im2col convolution listing,
    at the size of the stack's stage-1 result (batch 64), bf16."""

    name = "transpose (0 3 1 2) of ((64),(56,56,64)) bf16 -> (64,64,56,56)"
    dominant = "move_transpose_kernel"

    def __init__(self, dev):
        from paper_2105_09377_amd import binding as gs, synth
        self.gs = gs
        self.x = synth.normal_bf16((64, 56, 56, 64), 1.0, 7301)
        self.work = 2 * self.x.numel() * 2
        self.nsets = self._sets(self.work, 6)
        self.xs = [self.x.to(dev).clone() for _ in range(self.nsets)]
        self.outs = [torch.empty((64, 64, 56, 56), dtype=torch.bfloat16, device=dev) for _ in range(self.nsets)]

    def step(self, i):
        self.gs.transpose(self.xs[i], 1, (0, 3, 1, 2), out=self.outs[i])

    def cpu_baseline(self):
        from oracle import access_pattern as ap
        x = _bf16_to_f64(self.x[:8])
        t0 = time.perf_counter()
        ref = ap.transpose(ap.access(ap.tensor(x), 1), (0, 3, 1, 2)).materialize()
        dt = time.perf_counter() - t0
        return {"value": self.work / 8 / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                "sample": f"the access-pattern interpreter (numpy gather, fp64) on 8 of the 64 images, {dt:.2f} s",
                "max_rel_err": _max_rel_err(self.outs[0][:8], ref)}


class RowReduce(_Simple):
    """compute reduceSum over ((65536),(1024)) fp32."""

    name = "compute reduceSum ((65536),(1024)) f32"
    dominant = "reduce_rows_vec_kernel"
    dtype = "f32"

    def __init__(self, dev):
        from paper_2105_09377_amd import binding as gs, synth
        self.gs = gs
        self.x = synth.normal_f32((65536, 1024), 1.0, 7201)
        self.work = self.x.numel() * 4 + 65536 * 4
        self.nsets = 3
        self.xs = [self.x.to(dev).clone() for _ in range(self.nsets)]
        self.outs = [torch.empty((65536,), dtype=torch.float32, device=dev) for _ in range(self.nsets)]

    def step(self, i):
        self.gs.reduce(self.xs[i], 1, self.gs.GS_SUM, out=self.outs[i])

    def cpu_baseline(self):
        from oracle import brute
        x = self.x.numpy().astype("float64")
        t0 = time.perf_counter()
        ref = brute.row_reduce(x, False)
        dt = time.perf_counter() - t0
        return {"value": self.work / dt / 1e9, "unit": "GB/s", "cores": brute.num_threads(), "kind": "oracle",
                "sample": f"brute-force C loops (fp64, OpenMP) on the whole tensor, {dt:.2f} s",
                "max_rel_err": _max_rel_err(self.outs[0], ref)}


class DenseBig(_Simple):
    """compute dotProd (cartProd a0 a1) at a size that fills the chip: 8192 x 8192 x 8192 bf16."""

    name = "cartesian_dot ((8192),(8192)) x ((8192),(8192)) bf16 -> f32"
    dominant = "gemm_nt_dma_kernel"
    bound, unit, peak = "mfma", "TFLOP/s", PEAK_BF16_TFLOPS

    def __init__(self, dev):
        from paper_2105_09377_amd import binding as gs, synth
        self.gs = gs
        self.a = synth.normal_bf16((8192, 8192), 1.0, 7301)
        self.b = synth.normal_bf16((8192, 8192), 8192 ** -0.5, 7302)
        self.work = 2.0 * 8192 ** 3
        self.nsets = 2
        self.as_ = [self.a.to(dev).clone() for _ in range(self.nsets)]
        self.bs = [self.b.to(dev).clone() for _ in range(self.nsets)]
        self.outs = [torch.empty((8192, 8192), dtype=torch.float32, device=dev) for _ in range(self.nsets)]

    def step(self, i):
        self.gs.cartesian_dot(self.as_[i], self.bs[i], out=self.outs[i])

    def cpu_baseline(self):
        from oracle import brute
        a, b = _bf16_to_f64(self.a[:256]), _bf16_to_f64(self.b[:512])
        t0 = time.perf_counter()
        ref = brute.matmul(a, b.T)
        dt = time.perf_counter() - t0
        return {"value": 2.0 * 256 * 512 * 8192 / dt / 1e12, "unit": "TFLOP/s", "cores": brute.num_threads(),
                "kind": "oracle", "sample": f"brute-force C loops (fp64, OpenMP) on a 256 x 512 block of the result, {dt:.2f} s",
                "max_rel_err": _max_rel_err(self.outs[0][:256, :512], ref)}


class DenseInt8(DenseBig):
    """The same product on int8 operands (the int8 datapath of the paper's accelerators), int32 result."""

    name = "cartesian_dot ((8192),(8192)) x ((8192),(8192)) int8 -> int32"
    dtype = "i8"
    bound, unit, peak = "mfma", "TOP/s", PEAK_I8_TOPS

    def __init__(self, dev):
        from paper_2105_09377_amd import binding as gs, synth
        self.gs = gs
        self.a = synth.uniform_int8((8192, 8192), -127, 127, 7311)
        self.b = synth.uniform_int8((8192, 8192), -127, 127, 7312)
        self.work = 2.0 * 8192 ** 3
        self.nsets = 2
        self.as_ = [self.a.to(dev).clone() for _ in range(self.nsets)]
        self.bs = [self.b.to(dev).clone() for _ in range(self.nsets)]
        self.outs = [torch.empty((8192, 8192), dtype=torch.int32, device=dev) for _ in range(self.nsets)]

    def cpu_baseline(self):
        from oracle import brute
        a, b = self.a[:256].numpy().astype("int64"), self.b[:512].numpy().astype("int64")
        t0 = time.perf_counter()
        ref = brute.matmul(a, b.T)
        dt = time.perf_counter() - t0
        return {"value": 2.0 * 256 * 512 * 8192 / dt / 1e12, "unit": "TOP/s", "cores": brute.num_threads(),
                "kind": "oracle", "sample": f"brute-force C loops (int64, OpenMP) on a 256 x 512 block of the result, {dt:.2f} s",
                "max_rel_err": _max_rel_err(self.outs[0][:256, :512], ref)}


class DenseFp8(DenseBig):
    """The same product on 8-bit float operands (OCP e4m3), fp32 accumulate, bf16 result."""

    name = "cartesian_dot ((8192),(8192)) x ((8192),(8192)) fp8 e4m3 -> bf16"
    dtype = "f8"
    bound, unit, peak = "mfma", "TFLOP/s", PEAK_F8_TFLOPS

    def __init__(self, dev):
        from paper_2105_09377_amd import binding as gs, synth
        self.gs = gs
        self.a = synth.normal_fp8((8192, 8192), 1.0, 7321)
        self.b = synth.normal_fp8((8192, 8192), 8192 ** -0.5, 7322)
        self.work = 2.0 * 8192 ** 3
        self.nsets = 2
        self.as_ = [self.a.to(dev).clone() for _ in range(self.nsets)]
        self.bs = [self.b.to(dev).clone() for _ in range(self.nsets)]
        self.outs = [torch.empty((8192, 8192), dtype=torch.bfloat16, device=dev) for _ in range(self.nsets)]

    def cpu_baseline(self):
        import numpy as np
        from oracle import brute, numerics
        a = numerics.e4m3_bits_to_f64(self.a[:256].view(torch.uint8).numpy())
        b = numerics.e4m3_bits_to_f64(self.b[:512].view(torch.uint8).numpy())
        t0 = time.perf_counter()
        ref = brute.matmul(a, np.ascontiguousarray(b.T))
        dt = time.perf_counter() - t0
        return {"value": 2.0 * 256 * 512 * 8192 / dt / 1e12, "unit": "TFLOP/s", "cores": brute.num_threads(),
                "kind": "oracle", "sample": f"brute-force C loops (fp64, OpenMP) on a 256 x 512 block of the result, {dt:.2f} s",
                "max_rel_err": _max_rel_err(self.outs[0][:256, :512], ref)}


class DenseBlocked(_Simple):
    """The blocked form of the product (slice / dotProd / pair + reduceSum / concat) on
    2048 x 2048 x 2048 bf16 with cubic blocks of TILE, one launch whose workgroups stay inside
    blocks and fold the K slices in order: the tile-shape sweep of the paper's systolic-array
    sizes.  TILE = 2048 is the unblocked product."""

    TILE = 512
    dominant = "gemm_nt_dma_kernel (tiles confined to blocks)"
    bound, unit, peak = "mfma", "TFLOP/s", PEAK_BF16_TFLOPS
    name = property(lambda self: f"cartesian_dot_blocked 2048^3 bf16 -> f32, blocks of {self.TILE}^3 "
                                 f"({(2048 // self.TILE) ** 3} block products per step, one launch)")

    def __init__(self, dev):
        from paper_2105_09377_amd import binding as gs, synth
        self.gs = gs
        self.a = synth.normal_bf16((2048, 2048), 1.0, 7401)
        self.b = synth.normal_bf16((2048, 2048), 2048 ** -0.5, 7402)
        self.work = 2.0 * 2048 ** 3
        self.nsets = 4
        self.as_ = [self.a.to(dev).clone() for _ in range(self.nsets)]
        self.bs = [self.b.to(dev).clone() for _ in range(self.nsets)]
        self.outs = [torch.empty((2048, 2048), dtype=torch.float32, device=dev) for _ in range(self.nsets)]

    def step(self, i):
        t = self.TILE
        self.gs.cartesian_dot_blocked(self.as_[i], self.bs[i], t, t, t, out=self.outs[i])

    def cpu_baseline(self):
        from oracle import brute
        a, b = _bf16_to_f64(self.a[:512]), _bf16_to_f64(self.b[:512])
        t0 = time.perf_counter()
        ref = brute.matmul(a, b.T)
        dt = time.perf_counter() - t0
        return {"value": 2.0 * 512 * 512 * 2048 / dt / 1e12, "unit": "TFLOP/s", "cores": brute.num_threads(),
                "kind": "oracle", "sample": f"brute-force C loops (fp64, OpenMP) on a 512 x 512 block of the result, {dt:.2f} s",
                "max_rel_err": _max_rel_err(self.outs[0][:512, :512], ref)}


class Mlp(_Simple):
    """The dense MLP workload (batch 256, 784-512-512-10, ReLU) as three cartesian_dot calls."""

    name = "MLP 784-512-512-10, batch 256, bf16 in / fp32 accumulate, ReLU fused"
    dominant = "gemm_nt_* (layer 1: 256 x 512 x 784)"
    bound, unit, peak = "mfma", "TFLOP/s", PEAK_BF16_TFLOPS
    batch = 256

    def __init__(self, dev):
        from paper_2105_09377_amd import binding as gs, synth
        self.gs = gs
        self.cfg = synth.mlp_bf16(self.batch)
        dims = (784, 512, 512, 10)
        self.work = sum(2.0 * self.batch * dims[i] * dims[i + 1] for i in range(3))
        self.dominant_work = 2.0 * self.batch * 784 * 512
        self.nsets = 8
        self.xs = [self.cfg["x"].to(dev).clone() for _ in range(self.nsets)]
        self.ws = [[w.to(dev).clone() for w in self.cfg["weights"]] for _ in range(self.nsets)]
        self.h = [[torch.empty((self.batch, d), dtype=torch.bfloat16 if j < 2 else torch.float32, device=dev)
                   for j, d in enumerate(dims[1:])] for _ in range(self.nsets)]

    def step(self, i):
        gs, h = self.gs, self.xs[i]
        for j, w in enumerate(self.ws[i]):
            h = gs.cartesian_dot(h, w, act=gs.GS_ACT_RELU if j < 2 else gs.GS_ACT_NONE, out=self.h[i][j])

    def dominant_launch(self, i):
        self.gs.cartesian_dot(self.xs[i], self.ws[i][0], act=self.gs.GS_ACT_RELU, out=self.h[i][0])

    def cpu_baseline(self):
        import numpy as np
        from oracle import brute, numerics
        h = _bf16_to_f64(self.cfg["x"])
        ws = [_bf16_to_f64(w) for w in self.cfg["weights"]]
        t0 = time.perf_counter()
        for j, w in enumerate(ws):
            h = brute.matmul(h, w.T)
            if j < 2:
                h = numerics.round_to_bf16_value(np.maximum(h, 0))
        dt = time.perf_counter() - t0
        return {"value": self.work / dt / 1e12, "unit": "TFLOP/s", "cores": brute.num_threads(), "kind": "oracle",
                "sample": f"brute-force C loops (fp64, OpenMP), the whole batch, {dt:.2f} s",
                "max_rel_err": _max_rel_err(self.h[0][2], h)}


class MlpScaled(Mlp):
    """The same layers at batch 16384 (a labelled scaled variant: batch 256 is launch-bound)."""

    name = "MLP 784-512-512-10 at batch 16384 (scaled variant of the batch-256 workload)"
    dominant = "gemm_nt_dma_kernel (layer 1: 16384 x 512 x 784)"
    batch = 16384

    def cpu_baseline(self):
        return None


WORKLOADS = {"conv3x3": Conv3x3, "conv3x3_b64": Conv3x3Batch64, "conv3x3_i8": Conv3x3Int8, "resnet18": ResNet18, "im2col_gather": Im2colGather, "maxpool": MaxPool,
             "reduce": RowReduce, "transpose": Transpose, "depthwise": Depthwise, "dense": DenseBig, "dense_i8": DenseInt8, "dense_fp8": DenseFp8, "dense_blocked": DenseBlocked, "mlp": Mlp, "mlp_scaled": MlpScaled}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="resnet18", choices=sorted(WORKLOADS))
    ap.add_argument("--tile", type=int, default=None,
                    help="dense_blocked only: edge of the cubic blocks (a divisor of 2048, at least 64; default 512)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--batches", type=int, default=5,
                    help="timed batches of --steps steps each; the reported time is the median batch")
    ap.add_argument("--per-layer", action="store_true",
                    help="resnet18 only: add a per_layer table (every library call of the forward pass timed "
                         "on its own, back to back on one buffer set, i.e. with its input warm in cache)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run a plain 256 MiB -> 256 MiB elementwise copy 10 times and exit (reference "
                         "reading for the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.calibrate_copy:
        src = torch.ones(64 << 20, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(10):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": {"launches": 10, "read_bytes": src.numel() * 4,
                                             "write_bytes": dst.numel() * 4}}))
        return
    if args.tile is not None:
        if args.workload != "dense_blocked" or args.tile < 64 or 2048 % args.tile:
            sys.exit("--tile needs --workload dense_blocked and a divisor of 2048 that is at least 64")
        DenseBlocked.TILE = args.tile
    wl = WORKLOADS[args.workload](dev)
    stream = torch.cuda.Stream(device=dev)

    dom_sets = getattr(wl, "dom_sets", wl.nsets)
    with torch.cuda.stream(stream):
        for i in range(wl.nsets):           # first calls set kernel attributes: not capturable
            wl.step(i)
        for i in range(dom_sets):
            wl.dominant_launch(i)
    torch.cuda.synchronize()
    step_graphs = [_graph_of(lambda i=i: wl.step(i), stream) for i in range(wl.nsets)]
    # The dominant kernel is timed back to back inside one graph (DOM_BATCH launches cycling
    # through the buffer sets), so that the gap between graph launches -- several microseconds,
    # not part of any kernel -- does not count as kernel time.
    dom_batch = max(DOM_BATCH, dom_sets)

    def dom_body():
        for k in range(dom_batch):
            wl.dominant_launch(k % dom_sets)

    dom_graph = _graph_of(dom_body, stream)
    step_launch = [g.replay for g in step_graphs]
    dom_launch = [dom_graph.replay]

    # W warm-up steps, then `batches` timed regions of exactly K steps each, every region bracketed
    # by a device synchronisation on both sides; the median region is the one reported.
    _time_region(step_launch, args.warmup, stream)
    regions = sorted(_time_region(step_launch, args.steps, stream) for _ in range(max(1, args.batches)))
    wall, ev_ms = regions[len(regions) // 2]
    ms_per_step = wall * 1e3 / args.steps

    dom_replays = max(1, -(-args.steps // dom_batch))
    _time_region(dom_launch, 1, stream)
    dom_regions = sorted(_time_region(dom_launch, dom_replays, stream)[1] for _ in range(max(1, args.batches)))
    dom_s = dom_regions[len(dom_regions) // 2] * 1e-3 / (dom_replays * dom_batch)
    # Work per step / per dominant launch in the workload's own unit: FLOP for MFMA-bound
    # workloads, algorithmic bytes for HBM-bound ones.
    bound = getattr(wl, "bound", "mfma")
    unit = getattr(wl, "unit", "TFLOP/s")
    peak = getattr(wl, "peak", PEAK_BF16_TFLOPS)
    scale = 1e12 if unit in ("TFLOP/s", "TOP/s") else 1e9
    work = getattr(wl, "work", None) or wl.flops
    dom_work = getattr(wl, "dominant_work", None) or getattr(wl, "dominant_flops", None) or work
    achieved = dom_work / dom_s / scale

    out = {
        "metric": "conv2d/matmul TFLOP/s + % MFMA peak; im2col/reduce GB/s + % HBM peak",
        "value": work / (ms_per_step * 1e-3) / scale,
        "unit": unit,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": getattr(wl, "dtype", "bf16"), "data": "synthetic",
        "config": {"workload": wl.name, "buffer_sets": wl.nsets, "launch": "hip graph replay",
                   "dominant_kernel_buffer_sets": dom_sets},
        "event_ms_per_step": ev_ms / args.steps,
        "batches": len(regions), "batches_ms_per_step": [w * 1e3 / args.steps for w, _ in regions],
        "roofline": {"bound": bound, "kernel": wl.dominant, "achieved": achieved,
                     "peak": peak, "unit": unit, "frac": achieved / peak,
                     "us_per_launch": dom_s * 1e6, "traffic": None if args.tile not in (None, 512) else _traffic(args.workload)},   # counters were taken at the default tile
    }
    if args.per_layer:
        if not hasattr(wl, "per_layer"):
            sys.exit("--per-layer needs --workload resnet18")
        table = []
        for name, call, lwork, lunit in wl.per_layer():
            def body(call=call):
                for _ in range(DOM_BATCH):
                    call()
            g = _graph_of(body, stream)
            _time_region([g.replay], 1, stream)
            ms = sorted(_time_region([g.replay], 5, stream)[1] for _ in range(3))[1]
            us = ms * 1e3 / (5 * DOM_BATCH)
            table.append({"layer": name, "us": round(us, 2),
                          "rate": round(lwork / (us * 1e-6) / (1e12 if lunit == "TFLOP/s" else 1e9), 1), "unit": lunit})
        out["per_layer"] = table
        out["per_layer_sum_us"] = round(sum(r["us"] for r in table), 1)
    if not args.no_cpu_baseline:
        base = wl.cpu_baseline()
        if base is not None:
            out["cpu_baseline"] = base
    print(json.dumps(out))


if __name__ == "__main__":
    main()

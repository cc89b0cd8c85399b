#!/usr/bin/env python3
"""Benchmark of the memory-bound CNN hot path on one MI355X.

One "step" is one pass of the whole hot path -- layout transform in both
directions, max- and average-pooling in both layouts, fused softmax -- each on
the largest tensor the benchmark configurations give that kernel:

  transform : N=128, C=96, 55x55 fp32 (config 2), NCHW->CHWN then CHWN->NCHW
  pool      : N=64, C=64, 224x224 fp32, 2x2 / stride 2 (config 4), max and avg,
              in NCHW and in CHWN
  softmax   : 4096 x 21841 fp32 logits with planted +50 outliers (config 5)

Inputs are synthetic (seeded) and already resident in HBM when timing starts.
Every launch goes through the C ABI on torch's current stream and is bracketed
by HIP events on that stream; buffers rotate so that no launch finds its input
in the 256 MB last-level cache.  The printed JSON line carries the whole-step
throughput (algorithmic bytes / wall time), the roofline of the dominant
kernel, every kernel's own figures, and the CPU oracle timed on the same
inputs (one pass of the full workload).
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


WORKLOADS = {
    "largest": "each kernel on its largest configured tensor (the headline run)",
    "table1": "every pooling and classifier layer of the paper's Table 1",
    "softmax_sweep": "softmax over batch size x categories (Fig. 13's range)",
    "layouts": "changes between the named storage orders (NCHW, NHWC, CHWN, HWCN) on the config 2 tensor, a VGG "
               "tensor and an RGB input batch (Section I, IV.A)",
    "backward": "backward passes: pooling 2x2/s2 on 64x64x224x224 and 3x3/s2 on 128x96x55x55 (both layouts, max and "
                "avg), softmax on 4096x21841",
    "shapes": "layer shapes beyond the paper's networks: small and awkward batches, padded / stride-1 / 5x5 / global "
              "pooling, very short and very long softmax rows; with --compare-torch also PyTorch's own kernel per launch",
    "access_patterns": "what the memory system makes of the transform's access order: pattern-only kernels (the "
                       "addresses of a tiled transpose without LDS, barrier or transposition) and copies in scattered "
                       "chunk order, beside the library's transform and copy on the config 2 tensor",
    "configs": "every tensor of the five benchmark configurations, one launch each (the default run reports the "
               "same launches, timed back to back, under per_config)",
    "layout_policy": "the three AlexNet pooling layers of config 3 under both layout policies: pool where the "
                     "data is (NCHW) against transform + pool in CHWN + transform back (Section IV.B, IV.D)",
}
WORKLOAD_TEXT = {
    "largest": "largest tensor per kernel: transform 128x96x55x55 both directions (config 2), "
               "max+avg pool 2x2/s2 on 64x64x224x224 in NCHW and CHWN (config 4), softmax 4096x21841 (config 5)",
    "table1": "Table 1 of the paper: max-pool PL1..PL10 in NCHW and CHWN, softmax CLASS1..CLASS5",
    "softmax_sweep": "softmax, batch 32..256 x categories 10..10000 (the range of Fig. 13)",
    "layouts": "storage-order changes among NCHW / NHWC / CHWN / HWCN on 128x96x55x55, 64x64x112x112 and 64x3x224x224",
    "backward": "backward of max/avg pooling (64x64x224x224 2x2/s2, 128x96x55x55 3x3/s2; NCHW and CHWN) and of softmax (4096x21841)",
    "access_patterns": "transform 128x96x55x55 both ways, a copy of the same bytes, pattern-only kernels and scattered-chunk copies",
    "configs": "all five configurations: pooling in NCHW and CHWN, transforms both ways, softmax, on every tensor they name",
    "layout_policy": "config 3 (AlexNet, N=128) max-pool 3x3/s2 x3: NCHW in place vs NCHW->CHWN + pool + CHWN->NCHW",
    "shapes": "general shapes: transform at batches 1..100, pooling 3x3/s2/p1, 3x3/s1/p1, 5x5/s3/p2, global 7x7 (NCHW and "
              "CHWN, max and avg), softmax 1048576x10 and 512x128256",
}


def parse_args():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--only", default="", help="comma list of op names to run (profiling aid)")
    ap.add_argument("--workload", choices=sorted(WORKLOADS), default="largest",
                    help="; ".join(f"{k}: {v}" for k, v in sorted(WORKLOADS.items())))
    ap.add_argument("--dtype", choices=["f32", "f16", "bf16"], default="f32",
                    help="storage format of the tensors of the headline workload (arithmetic is fp32 in every case)")
    ap.add_argument("--graph", action="store_true",
                    help="also capture the step into a HIP graph and time its replays (removes the host's launch "
                         "cost, which dominates workloads of very small tensors)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the warm-cache and same-bytes-copy yardsticks measured after the timed region")
    ap.add_argument("--compare-torch", action="store_true",
                    help="workload 'shapes': also time PyTorch's own kernel for the same operation (context only)")
    ap.add_argument("--verbose", action="store_true")
    return ap.parse_args()



class Op:
    """One launch of the hot path with its rotating buffer sets."""

    def __init__(self, name, kind, alg_bytes, units, unit_name, launch, nsets):
        self.name, self.kind, self.alg_bytes = name, kind, alg_bytes
        self.units, self.unit_name = units, unit_name
        self.launch, self.nsets = launch, nsets
        self.ms = []


def build_ops(torch, cm, wl, rl, only, dtype="f32"):
    dev = torch.device("cuda:0")
    ops = []
    host = {}
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[dtype]
    tag = {"f32": cm.F32, "f16": cm.F16, "bf16": cm.BF16}[dtype]
    scale = 1 if dtype == "f32" else 2                       # bytes per element: 4 / scale

    def rotating(t, n):
        return [t] + [t.clone() for _ in range(n - 1)]

    def want(name):
        return not only or name in only

    # ---- transform: config 2 tensor --------------------------------------------------
    t = wl.config(2).transforms[0]
    if want("transform_nchw_to_chwn") or want("transform_chwn_to_nchw"):
        host["transform"] = wl.make_tensor(t, wl.rng_for(2))
        x = torch.from_numpy(host["transform"]).to(dev).to(tdt)
        nset = 4 * scale                                     # 4 x (149 + 149) MB > 1 GB
        xs = rotating(x, nset)
        cs = [torch.empty((t.C, t.H, t.W, t.N), dtype=tdt, device=dev) for _ in range(nset)]
        bs = [torch.empty((t.N, t.C, t.H, t.W), dtype=tdt, device=dev) for _ in range(nset)]
        for i in range(nset):
            cm.transform(xs[i], t.N, t.C, t.H, t.W, cm.NCHW, cm.CHWN, out=cs[i])
        tb = rl.transform_bytes(t.N, t.C, t.H, t.W) // scale
        if want("transform_nchw_to_chwn"):
            ops.append(Op("transform_nchw_to_chwn", "transform", tb, t.numel, "elements",
                          lambda i: cm.cnnmem_transform_dtype(xs[i], cs[i], t.N, t.C, t.H, t.W, cm.NCHW, cm.CHWN, tag),
                          nset))
        if want("transform_chwn_to_nchw"):
            ops.append(Op("transform_chwn_to_nchw", "transform", tb, t.numel, "elements",
                          lambda i: cm.cnnmem_transform_dtype(cs[i], bs[i], t.N, t.C, t.H, t.W, cm.CHWN, cm.NCHW, tag),
                          nset))

    # ---- pooling: config 4, first tensor ----------------------------------------------
    p = wl.config(4).pools[0].tensor
    pool_names = ["pool_max_nchw", "pool_max_chwn", "pool_avg_nchw", "pool_avg_chwn"]
    if any(want(n) for n in pool_names):
        host["pool"] = wl.make_tensor(p, wl.rng_for(4, 0))
        x = torch.from_numpy(host["pool"]).to(dev).to(tdt)
        nset = 2 * scale                                     # 2 x (822 + 206) MB
        st, Ho, Wo = cm.cnnmem_pool_out_dims(p.H, p.W, 2, 2, 2, 2, 0, 0)
        assert st == 0
        pb = rl.pool_bytes(p.N, p.C, p.H, p.W, 2, 2, 2, 2) // scale
        xn = rotating(x, nset)
        xc = [cm.transform(xn[i], p.N, p.C, p.H, p.W, cm.NCHW, cm.CHWN) for i in range(nset)]
        on = [torch.empty((p.N, p.C, Ho, Wo), dtype=tdt, device=dev) for _ in range(nset)]
        oc = [torch.empty((p.C, Ho, Wo, p.N), dtype=tdt, device=dev) for _ in range(nset)]

        def pool_launch(src, dst, layout, mode):
            return lambda i: cm.cnnmem_pool_dtype(src[i], dst[i], p.N, p.C, p.H, p.W, layout, mode, 2, 2, 2, 2, 0, 0,
                                                  tag)

        table = {"pool_max_nchw": (xn, on, cm.NCHW, cm.POOL_MAX), "pool_max_chwn": (xc, oc, cm.CHWN, cm.POOL_MAX),
                 "pool_avg_nchw": (xn, on, cm.NCHW, cm.POOL_AVG), "pool_avg_chwn": (xc, oc, cm.CHWN, cm.POOL_AVG)}
        for name in pool_names:
            if want(name):
                ops.append(Op(name, "pool", pb, p.numel, "input elements", pool_launch(*table[name]), nset))

    # ---- softmax: config 5 ---------------------------------------------------------------
    s = wl.config(5).softmaxes[0]
    if want("softmax"):
        host["softmax"] = wl.make_logits(s, wl.rng_for(5, 0))
        z = torch.from_numpy(host["softmax"]).to(dev).to(tdt)
        nset = 2 * scale                                     # 2 x (358 + 358) MB
        zs = rotating(z, nset)
        ps = [torch.empty_like(z) for _ in range(nset)]
        ops.append(Op("softmax", "softmax", rl.softmax_bytes(s.N, s.classes) // scale, s.N * s.classes, "elements",
                      lambda i: cm.cnnmem_softmax_dtype(zs[i], ps[i], s.N, s.classes, tag), nset))
    # ---- optional: plain copy of known size, the yardstick the traffic counters are scaled by ----
    if "copy_calibration" in only:
        n = t.numel
        nset = 4
        a = [torch.zeros(n, dtype=torch.float32, device=dev) for _ in range(nset)]
        b = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(nset)]
        ops.append(Op("copy_calibration", "copy", 2 * 4 * n, n, "elements",
                      lambda i: cm.cnnmem_transform(a[i], b[i], t.N, t.C, t.H, t.W, cm.NCHW, cm.NCHW), nset))
    torch.cuda.synchronize()
    return ops, host


def build_table1_ops(torch, cm, wl, rl, only):
    """Second workload: max-pooling of PL1..PL10 in both layouts and softmax of CLASS1..CLASS5 (Table 1)."""
    dev = torch.device("cuda:0")
    ops = []
    gen = torch.Generator(device="cuda").manual_seed(1610)

    nsets_for = _nsets_for
    for (name, N, hw, k, C, s) in wl.TABLE1_POOLS:
        st, Ho, Wo = cm.cnnmem_pool_out_dims(hw, hw, k, k, s, s, 0, 0)
        n_in, n_out = N * C * hw * hw, N * C * Ho * Wo
        ns = nsets_for(4 * (n_in + n_out))
        pb = rl.pool_bytes(N, C, hw, hw, k, k, s, s)
        for layout, tag in ((cm.NCHW, "nchw"), (cm.CHWN, "chwn")):
            opname = f"{name.lower()}_max_{tag}"
            if only and opname not in only:
                continue
            xs = [torch.randn(n_in, device=dev, generator=gen).relu_() for _ in range(ns)]
            ys = [torch.empty(n_out, dtype=torch.float32, device=dev) for _ in range(ns)]
            ops.append(Op(opname, "pool", pb, n_in, "input elements",
                          (lambda xs, ys, N, C, hw, layout, k, s:
                           lambda i: cm.cnnmem_pool(xs[i], ys[i], N, C, hw, hw, layout, cm.POOL_MAX, k, k, s, s, 0, 0))(
                              xs, ys, N, C, hw, layout, k, s), ns))
    for (name, n, c) in wl.TABLE1_CLASSIFIERS:
        opname = f"{name.lower()}_softmax"
        if only and opname not in only:
            continue
        ns = 16
        zs = [torch.randn((n, c), device=dev, generator=gen) * 3 for _ in range(ns)]
        ps = [torch.empty_like(zs[0]) for _ in range(ns)]
        ops.append(Op(opname, "softmax", rl.softmax_bytes(n, c), n * c, "elements",
                      (lambda zs, ps, n, c: lambda i: cm.cnnmem_softmax(zs[i], ps[i], n, c))(zs, ps, n, c), ns))
    torch.cuda.synchronize()
    return ops, {}


def _nsets_for(nbytes):
    return int(min(16, max(2, (1 << 30) // nbytes + 1)))


def build_softmax_sweep_ops(torch, cm, wl, rl, only):
    """Softmax over a batch x categories grid (the range Fig. 13 covers)."""
    dev = torch.device("cuda:0")
    gen = torch.Generator(device="cuda").manual_seed(1613)
    ops = []
    for (n, c) in wl.SOFTMAX_SWEEP:
        opname = f"softmax_{n}x{c}"
        if only and opname not in only:
            continue
        ns = _nsets_for(8 * n * c)
        zs = [torch.randn((n, c), device=dev, generator=gen) * 3 for _ in range(ns)]
        ps = [torch.empty_like(zs[0]) for _ in range(ns)]
        ops.append(Op(opname, "softmax", rl.softmax_bytes(n, c), n * c, "elements",
                      (lambda zs, ps, n, c: lambda i: cm.cnnmem_softmax(zs[i], ps[i], n, c))(zs, ps, n, c), ns))
    torch.cuda.synchronize()
    return ops, {}


SHAPES_TRANSFORM = [(1, 64, 224, 224), (4, 64, 224, 224), (8, 64, 112, 112), (32, 512, 28, 28), (100, 64, 57, 57)]
SHAPES_POOL = [  # N, C, H, W, window, stride, pad
    (256, 64, 112, 112, 3, 2, 1),       # ResNet stem
    (64, 256, 56, 56, 3, 1, 1),         # Inception branch
    (64, 64, 150, 150, 5, 3, 2),
    (128, 2048, 7, 7, 7, 7, 0),         # global pooling
]
SHAPES_SOFTMAX = [(1048576, 10), (512, 128256)]


def build_shapes_ops(torch, cm, wl, rl, only):
    """Layer shapes outside the paper's networks (Section III.A lists LeNet, Cifar, AlexNet, ZFNet, VGG)."""
    import torch.nn.functional as F
    dev = torch.device("cuda:0")
    gen = torch.Generator(device="cuda").manual_seed(1617)
    ops = []

    def add(name, kind, nbytes, units, unit_name, launch, ns, torch_launch):
        if only and name not in only:
            return
        op = Op(name, kind, nbytes, units, unit_name, launch, ns)
        op.torch_launch = torch_launch
        ops.append(op)

    for (N, C, H, W) in SHAPES_TRANSFORM:
        n = N * C * H * W
        ns = _nsets_for(8 * n)
        a = [torch.randn((N, C, H, W), device=dev, generator=gen) for _ in range(ns)]
        b = [torch.empty((C, H, W, N), dtype=torch.float32, device=dev) for _ in range(ns)]
        c = [torch.empty((N, C, H, W), dtype=torch.float32, device=dev) for _ in range(ns)]
        for i in range(ns):
            cm.transform(a[i], N, C, H, W, cm.NCHW, cm.CHWN, out=b[i])
        tag = f"{N}x{C}x{H}x{W}"
        add(f"transform_nchw_to_chwn_{tag}", "transform", rl.transform_bytes(N, C, H, W), n, "elements",
            (lambda a, b, N, C, H, W: lambda i: cm.cnnmem_transform(a[i], b[i], N, C, H, W, cm.NCHW, cm.CHWN))(a, b, N, C, H, W),
            ns, (lambda a, b: lambda i: b[i].copy_(a[i].permute(1, 2, 3, 0)))(a, b))
        add(f"transform_chwn_to_nchw_{tag}", "transform", rl.transform_bytes(N, C, H, W), n, "elements",
            (lambda b, c, N, C, H, W: lambda i: cm.cnnmem_transform(b[i], c[i], N, C, H, W, cm.CHWN, cm.NCHW))(b, c, N, C, H, W),
            ns, (lambda b, c: lambda i: c[i].copy_(b[i].permute(3, 0, 1, 2)))(b, c))
    for (N, C, H, W, k, s, p) in SHAPES_POOL:
        st, Ho, Wo = cm.cnnmem_pool_out_dims(H, W, k, k, s, s, p, p)
        n_in, n_out = N * C * H * W, N * C * Ho * Wo
        ns = _nsets_for(4 * (n_in + n_out))
        x = [torch.randn((N, C, H, W), device=dev, generator=gen).relu_() for _ in range(ns)]
        xc = [cm.transform(t, N, C, H, W, cm.NCHW, cm.CHWN) for t in x]
        y = [torch.empty(n_out, dtype=torch.float32, device=dev) for _ in range(ns)]
        pb = rl.pool_bytes(N, C, H, W, k, k, s, s, p, p)
        tag = f"{N}x{C}x{H}x{W}_k{k}s{s}p{p}"
        for mode, mname in ((cm.POOL_MAX, "max"), (cm.POOL_AVG, "avg")):
            tl = ((lambda x, k, s, p: lambda i: F.max_pool2d(x[i], k, s, p))(x, k, s, p) if mode == cm.POOL_MAX else
                  (lambda x, k, s, p: lambda i: F.avg_pool2d(x[i], k, s, p))(x, k, s, p))
            for layout, src, lname in ((cm.NCHW, x, "nchw"), (cm.CHWN, xc, "chwn")):
                add(f"pool_{mname}_{lname}_{tag}", "pool", pb, n_in, "input elements",
                    (lambda src, y, N, C, H, W, layout, mode, k, s, p:
                     lambda i: cm.cnnmem_pool(src[i], y[i], N, C, H, W, layout, mode, k, k, s, s, p, p))(
                         src, y, N, C, H, W, layout, mode, k, s, p), ns, tl if layout == cm.NCHW else None)
    for (n, c) in SHAPES_SOFTMAX:
        ns = _nsets_for(8 * n * c)
        zs = [torch.randn((n, c), device=dev, generator=gen) * 3 for _ in range(ns)]
        ps = [torch.empty_like(zs[0]) for _ in range(ns)]
        add(f"softmax_{n}x{c}", "softmax", rl.softmax_bytes(n, c), n * c, "elements",
            (lambda zs, ps, n, c: lambda i: cm.cnnmem_softmax(zs[i], ps[i], n, c))(zs, ps, n, c), ns,
            (lambda zs: lambda i: torch.softmax(zs[i], dim=1))(zs))
    torch.cuda.synchronize()
    return ops, {}


def measure_torch(torch, ops, iters=20):
    """PyTorch's own kernel for the same operation, as context: median of `iters` launches on rotating inputs."""
    out = {}
    for op in ops:
        fn = getattr(op, "torch_launch", None)
        if fn is None:
            continue
        for i in range(3):
            fn(i % op.nsets)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(ev):
            a.record()
            fn(i % op.nsets)
            b.record()
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) for a, b in ev)
        out[op.name] = ms[len(ms) // 2]
    return out


def build_layouts_ops(torch, cm, wl, rl, only):
    """Changes between the storage orders the paper names, on three tensor shapes."""
    dev = torch.device("cuda:0")
    gen = torch.Generator(device="cuda").manual_seed(1615)
    pairs = [("NCHW", "NHWC"), ("NHWC", "NCHW"), ("NCHW", "CHWN"), ("CHWN", "NCHW"), ("CHWN", "HWCN"),
             ("HWCN", "CHWN"), ("NCHW", "HWCN"), ("HWCN", "NCHW")]
    ops = []
    for (N, C, H, W) in [(128, 96, 55, 55), (64, 64, 112, 112), (64, 3, 224, 224)]:
        n = N * C * H * W
        ns = _nsets_for(8 * n)
        a = [torch.randn(n, device=dev, generator=gen) for _ in range(ns)]
        b = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(ns)]
        for (s_, d_) in pairs:
            name = f"{N}x{C}x{H}x{W}:{s_}>{d_}"
            if only and name not in only:
                continue
            ops.append(Op(name, "transform", rl.transform_bytes(N, C, H, W), n, "elements",
                          (lambda a, b, N, C, H, W, s_, d_: lambda i: cm.cnnmem_relayout(a[i], b[i], N, C, H, W, s_, d_))(
                              a, b, N, C, H, W, s_, d_), ns))
    torch.cuda.synchronize()
    return ops, {}


def build_backward_ops(torch, cm, wl, rl, only):
    """Backward passes on the headline tensors."""
    dev = torch.device("cuda:0")
    gen = torch.Generator(device="cuda").manual_seed(1616)
    ops = []
    for (N, C, H, W, k, s_) in [(64, 64, 224, 224, 2, 2), (128, 96, 55, 55, 3, 2)]:
        st, Ho, Wo = cm.cnnmem_pool_out_dims(H, W, k, k, s_, s_, 0, 0)
        n_in, n_out = N * C * H * W, N * C * Ho * Wo
        ns = _nsets_for(4 * (2 * n_in + n_out))
        x = [torch.randn(n_in, device=dev, generator=gen).relu_() for _ in range(ns)]
        dy = [torch.randn(n_out, device=dev, generator=gen) for _ in range(ns)]
        dx = [torch.empty(n_in, dtype=torch.float32, device=dev) for _ in range(ns)]
        for layout, ltag in ((cm.NCHW, "nchw"), (cm.CHWN, "chwn")):
            for mode, mtag in ((cm.POOL_MAX, "max"), (cm.POOL_AVG, "avg")):
                name = f"pool_bwd_{mtag}_{ltag}_{C}x{H}x{W}"
                if only and name not in only:
                    continue
                b = rl.pool_backward_bytes(N, C, H, W, k, k, s_, s_, needs_input=(mode == cm.POOL_MAX))
                ops.append(Op(name, "pool", b, n_in, "input elements",
                              (lambda x, dy, dx, N, C, H, W, layout, mode, k, s_:
                               lambda i: cm.cnnmem_pool_backward(x[i], dy[i], dx[i], N, C, H, W, layout, mode, k, k, s_, s_, 0, 0))(
                                  x, dy, dx, N, C, H, W, layout, mode, k, s_), ns))
    n, c = 4096, 21841
    if not only or "softmax_bwd" in only:
        ns = 2
        p = [torch.softmax(torch.randn((n, c), device=dev, generator=gen) * 3, dim=1) for _ in range(ns)]
        dp = [torch.randn((n, c), device=dev, generator=gen) for _ in range(ns)]
        dz = [torch.empty((n, c), dtype=torch.float32, device=dev) for _ in range(ns)]
        ops.append(Op("softmax_bwd", "softmax", rl.softmax_backward_bytes(n, c), n * c, "elements",
                      lambda i: cm.cnnmem_softmax_backward(p[i], dp[i], dz[i], n, c), ns))
    torch.cuda.synchronize()
    return ops, {}


def build_layout_policy_ops(torch, cm, wl, rl, only):
    """Config 3's three pooling layers, data arriving and leaving in NCHW (what the neighbouring
    convolutions of AlexNet prefer at N = 128, C >= 96 under Section IV.A's rule): either pool in NCHW, or follow
    the always-CHWN rule for pooling and pay a transform before and after."""
    dev = torch.device("cuda:0")
    gen = torch.Generator(device="cuda").manual_seed(1614)
    ops = []
    for li, pc in enumerate(wl.config(3).pools):
        t = pc.tensor
        st, Ho, Wo = cm.cnnmem_pool_out_dims(t.H, t.W, pc.k, pc.k, pc.s, pc.s, 0, 0)
        n_in, n_out = t.numel, t.N * t.C * Ho * Wo
        ns = _nsets_for(8 * (n_in + n_out))
        x = [torch.randn(n_in, device=dev, generator=gen).relu_() for _ in range(ns)]
        xc = [torch.empty(n_in, dtype=torch.float32, device=dev) for _ in range(ns)]
        y = [torch.empty(n_out, dtype=torch.float32, device=dev) for _ in range(ns)]
        yc = [torch.empty(n_out, dtype=torch.float32, device=dev) for _ in range(ns)]
        pb = rl.pool_bytes(t.N, t.C, t.H, t.W, pc.k, pc.k, pc.s, pc.s)
        N, C, H, W, k, s_ = t.N, t.C, t.H, t.W, pc.k, pc.s
        tag = f"l{li + 1}_{C}x{H}x{W}"
        mk = [
            (f"{tag}:keep:pool_nchw", "pool", pb,
             lambda i, x=x, y=y, N=N, C=C, H=H, W=W, k=k, s_=s_:
                 cm.cnnmem_pool(x[i], y[i], N, C, H, W, cm.NCHW, cm.POOL_MAX, k, k, s_, s_, 0, 0)),
            (f"{tag}:chwn:transform_in", "transform", rl.transform_bytes(N, C, H, W),
             lambda i, x=x, xc=xc, N=N, C=C, H=H, W=W: cm.cnnmem_transform(x[i], xc[i], N, C, H, W, cm.NCHW, cm.CHWN)),
            (f"{tag}:chwn:pool_chwn", "pool", pb,
             lambda i, xc=xc, yc=yc, N=N, C=C, H=H, W=W, k=k, s_=s_:
                 cm.cnnmem_pool(xc[i], yc[i], N, C, H, W, cm.CHWN, cm.POOL_MAX, k, k, s_, s_, 0, 0)),
            (f"{tag}:chwn:transform_out", "transform", rl.transform_bytes(N, C, Ho, Wo),
             lambda i, yc=yc, y=y, N=N, C=C, Ho=Ho, Wo=Wo: cm.cnnmem_transform(yc[i], y[i], N, C, Ho, Wo, cm.CHWN, cm.NCHW)),
        ]
        for name, kind, b, fn in mk:
            if only and name not in only:
                continue
            ops.append(Op(name, kind, b, n_in, "input elements", fn, ns))
    torch.cuda.synchronize()
    return ops, {}


def layout_policy_summary(kernels):
    """Per layer: microseconds for pooling in place (NCHW) against transform + CHWN pooling + transform."""
    layers = {}
    for k in kernels:
        tag, policy, _ = k["name"].split(":")
        layers.setdefault(tag, {"keep_layout_us": 0.0, "always_chwn_us": 0.0})
        layers[tag]["keep_layout_us" if policy == "keep" else "always_chwn_us"] += k["median_ms"] * 1e3
    for v in layers.values():
        v["keep_layout_us"] = round(v["keep_layout_us"], 2)
        v["always_chwn_us"] = round(v["always_chwn_us"], 2)
        v["ratio"] = round(v["always_chwn_us"] / v["keep_layout_us"], 3) if v["keep_layout_us"] else None
    return layers


def measure_extras(torch, cm, ops, tev, iters=20):
    """Two yardsticks beside every launch, measured after the timed region:

    warm -- the same launch repeated on one buffer set (the last-level cache may serve it);
    copy -- the library's plain copy kernel moving the same number of bytes (half read, half
            written) between rotating buffers: the practical ceiling of this memory system;
    back to back -- the launch, and the copy, repeated ``iters`` times on rotating buffer sets between ONE
            pair of events: the time per launch without the 2-5 us that an event after every launch adds,
            which is most of what a launch of a few microseconds measures otherwise.
    """
    dev = torch.device("cuda:0")
    out = {}
    copy_cache = {}

    # a launch of a millisecond or so that goes first, so that the host has queued every timed launch
    # before the GPU reaches it and the events bracket GPU time only
    pa = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
    pb = torch.empty_like(pa)

    def timed(fn, n):
        for i in range(3):
            fn(i)
        ev = [tev.create(2) for _ in range(n)]
        torch.cuda.synchronize()
        for _ in range(3):
            cm.cnnmem_transform(pa, pb, 1, 1, 1, pa.numel(), cm.NCHW, cm.NCHW)
        for i, (a, b) in enumerate(ev):
            tev.record(a)
            fn(i)
            tev.record(b)
        torch.cuda.synchronize()
        ms = sorted(tev.elapsed_ms(a, b) for a, b in ev)
        tev.destroy_all()
        return ms[len(ms) // 2]

    def train(fn, n):
        for i in range(3):
            fn(i)
        a, b = tev.create(2)
        torch.cuda.synchronize()
        for _ in range(3):
            cm.cnnmem_transform(pa, pb, 1, 1, 1, pa.numel(), cm.NCHW, cm.NCHW)
        tev.record(a)
        for i in range(n):
            fn(i)
        tev.record(b)
        torch.cuda.synchronize()
        ms = tev.elapsed_ms(a, b) / n
        tev.destroy_all()
        return ms

    for op in ops:
        warm_ms = timed(lambda i, op=op: op.launch(0), iters)
        b2b_ms = train(lambda i, op=op: op.launch(i % op.nsets), iters)
        if op.alg_bytes not in copy_cache:
            n = max(4, (op.alg_bytes // 8) // 4 * 4)           # floats each way
            ns = _nsets_for(8 * n)
            a = [torch.zeros(n, dtype=torch.float32, device=dev) for _ in range(ns)]
            b = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(ns)]
            fn = lambda i, a=a, b=b, n=n, ns=ns: cm.cnnmem_transform(a[i % ns], b[i % ns], 1, 1, 1, n, cm.NCHW, cm.NCHW)
            copy_cache[op.alg_bytes] = (timed(fn, iters), train(fn, iters))
            del a, b
        out[op.name] = (warm_ms, copy_cache[op.alg_bytes][0], b2b_ms, copy_cache[op.alg_bytes][1])
    return out


def build_access_pattern_ops(torch, cm, wl, rl, only):
    """Section IV.C's transform beside kernels that only reproduce its memory accesses (no LDS, no barrier, data
    not transposed) and beside copies whose chunks are read or written in a scattered order."""
    import ctypes
    from paper_1610_03618_amd import build as hip_build
    probes = ctypes.CDLL(hip_build.PROBES_LIB_PATH)
    p, i, ll = ctypes.c_void_p, ctypes.c_int, ctypes.c_longlong
    probes.cnnmem_probe_tile_pattern.argtypes = [p, p, ll, ll, i, i, i, i, p]
    probes.cnnmem_probe_chunk_copy.argtypes = [p, p, ll, i, i, p]
    dev = torch.device("cuda:0")
    t = wl.config(2).transforms[0]
    N, C, H, W = t.N, t.C, t.H, t.W
    M, n = C * H * W, t.numel
    ns = 4
    a = [torch.randn(n, device=dev) for _ in range(ns)]
    b = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(ns)]
    ops = []

    def stream():
        return torch.cuda.current_stream().cuda_stream or None

    def add(name, nbytes, fn):
        if not only or name in only:
            ops.append(Op(name, "transform", nbytes, n, "elements", fn, ns))

    full = rl.transform_bytes(N, C, H, W)
    add("copy", full, lambda k: cm.cnnmem_transform(a[k], b[k], 1, 1, 1, n, cm.NCHW, cm.NCHW))
    add("transform_nchw_to_chwn", full, lambda k: cm.cnnmem_transform(a[k], b[k], N, C, H, W, cm.NCHW, cm.CHWN))
    add("transform_chwn_to_nchw", full, lambda k: cm.cnnmem_transform(a[k], b[k], N, C, H, W, cm.CHWN, cm.NCHW))
    for (TR, NS, r_fastest) in ((32, 128, 0), (128, 32, 0), (128, 32, 1), (256, 32, 1), (512, 32, 1)):
        covered = 2 * 4 * (M // TR) * TR * N
        tag = f"{TR}x{NS}" + ("_image_groups_slowest" if r_fastest else "")
        add(f"pattern_chwn_to_nchw_{tag}", covered,
            lambda k, TR=TR, NS=NS, rf=r_fastest: probes.cnnmem_probe_tile_pattern(
                a[k].data_ptr(), b[k].data_ptr(), M, N, TR, NS, 1, rf, stream()))
        add(f"pattern_nchw_to_chwn_{tag}", covered,
            lambda k, TR=TR, NS=NS, rf=r_fastest: probes.cnnmem_probe_tile_pattern(
                a[k].data_ptr(), b[k].data_ptr(), M, N, TR, NS, 0, rf, stream()))
    for chunk in (128, 4096, 65536, 1048576):
        whole = (4 * n // chunk) * chunk // 4
        for scatter, sname in ((1, "reads"), (2, "writes"), (3, "both")):
            add(f"copy_chunks_{chunk}B_scattered_{sname}", 2 * 4 * whole,
                lambda k, chunk=chunk, scatter=scatter, whole=whole: probes.cnnmem_probe_chunk_copy(
                    a[k].data_ptr(), b[k].data_ptr(), whole, chunk, scatter, stream()))
    torch.cuda.synchronize()
    return ops, {}


def build_config_ops(torch, cm, wl, rl, only):
    """Every tensor the five benchmark configurations name, one launch each: the pooling layers in both layouts
    (config 4: max and avg), the transforms in both directions (config 3: on the pooled shapes too), the
    classifiers.  Tensors are filled on the device with seeded values of the configuration's distribution."""
    dev = torch.device("cuda:0")
    gen = torch.Generator(device="cuda").manual_seed(161003618)
    ops = []
    names = set()
    chosen = set(only) - {"copy_calibration"}               # "copy_calibration" alone adds the copy to every launch

    def values(spec_values, shape):
        if spec_values == "uniform":
            return torch.rand(shape, device=dev, generator=gen) * 2 - 1
        return torch.randn(shape, device=dev, generator=gen).relu_()

    def wanted(cfg, name):
        if (cfg, name) in names or (chosen and name not in chosen):   # config 3: a pooled shape that is also an input
            return False
        names.add((cfg, name))
        return True

    def add(cfg, name, kind, nbytes, units, fn, ns):
        op = Op(name, kind, nbytes, units, "elements", fn, ns)
        op.config = cfg
        ops.append(op)

    def transforms(cfg, N, C, H, W, vals):
        n = N * C * H * W
        tag = f"{N}x{C}x{H}x{W}"
        todo = [d for d in ("nchw_to_chwn", "chwn_to_nchw") if wanted(cfg, f"transform_{d}_{tag}")]
        if not todo:
            return
        ns = _nsets_for(8 * n)
        a = [values(vals, (N, C, H, W)) for _ in range(ns)]
        b = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(ns)]
        for d in todo:
            s_, d_ = (cm.NCHW, cm.CHWN) if d == "nchw_to_chwn" else (cm.CHWN, cm.NCHW)
            add(cfg, f"transform_{d}_{tag}", "transform", rl.transform_bytes(N, C, H, W), n,
                lambda i, s_=s_, d_=d_: cm.cnnmem_transform(a[i], b[i], N, C, H, W, s_, d_), ns)

    def pools(cfg, N, C, H, W, k, s_, modes, vals):
        st, Ho, Wo = cm.cnnmem_pool_out_dims(H, W, k, k, s_, s_, 0, 0)
        n_in, n_out = N * C * H * W, N * C * Ho * Wo
        todo = []
        for mode in modes:
            for layout, lname in ((cm.NCHW, "nchw"), (cm.CHWN, "chwn")):
                name = f"pool_{'max' if mode == cm.POOL_MAX else 'avg'}_{lname}_{N}x{C}x{H}x{W}_k{k}s{s_}"
                if wanted(cfg, name):
                    todo.append((name, mode, layout))
        if todo:
            ns = _nsets_for(4 * (n_in + n_out))
            x = [values(vals, (n_in,)) for _ in range(ns)]
            y = [torch.empty(n_out, dtype=torch.float32, device=dev) for _ in range(ns)]
            pb = rl.pool_bytes(N, C, H, W, k, k, s_, s_)
            for name, mode, layout in todo:
                add(cfg, name, "pool", pb, n_in,
                    lambda i, layout=layout, mode=mode: cm.cnnmem_pool(x[i], y[i], N, C, H, W, layout, mode,
                                                                       k, k, s_, s_, 0, 0), ns)
        return Ho, Wo

    def softmax(cfg, n, c, sigma):
        if not wanted(cfg, f"softmax_{n}x{c}"):
            return
        ns = _nsets_for(8 * n * c)
        z = [torch.randn((n, c), device=dev, generator=gen) * sigma for _ in range(ns)]
        pr = [torch.empty_like(z[0]) for _ in range(ns)]
        add(cfg, f"softmax_{n}x{c}", "softmax", rl.softmax_bytes(n, c), n * c,
            lambda i: cm.cnnmem_softmax(z[i], pr[i], n, c), ns)

    for k in (1, 2, 3, 4, 5):
        cfg = wl.config(k)
        seen = set()
        for pc in cfg.pools:
            t = pc.tensor
            if t.name in seen:
                continue
            seen.add(t.name)
            modes = sorted({q.mode for q in cfg.pools if q.tensor is t})
            Ho, Wo = pools(k, t.N, t.C, t.H, t.W, pc.k, pc.s, modes, t.values)
            if k == 3:                                       # the transforms between the layers: pooled shapes too
                transforms(k, t.N, t.C, Ho, Wo, t.values)
        for t in cfg.transforms:
            transforms(k, t.N, t.C, t.H, t.W, t.values)
        for sm in cfg.softmaxes:
            softmax(k, sm.N, sm.classes, sm.sigma)
    if "copy_calibration" in only:
        n = 128 * 96 * 55 * 55
        ca = [torch.zeros(n, dtype=torch.float32, device=dev) for _ in range(4)]
        cb = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(4)]
        add(0, "copy_calibration", "copy", 2 * 4 * n, n,
            lambda i: cm.cnnmem_transform(ca[i], cb[i], 1, 1, 1, n, cm.NCHW, cm.NCHW), 4)
    torch.cuda.synchronize()
    return ops, {}


def measure_configs(torch, cm, wl, rl, tev, iters=20):
    """The launches of ``build_config_ops``, each timed back to back: ``iters`` launches on rotating buffer
    sets (together larger than the last-level cache), replayed as one HIP graph between one pair of events after
    three untimed launches.  Several of these tensors take a few microseconds, less than the host needs to
    issue a launch from Python, hence the graph.  Nothing here is checked against the oracle (the parity tests
    run the same tensors through it)."""
    from paper_1610_03618_amd.timing import graph_train_ms
    ops, _ = build_config_ops(torch, cm, wl, rl, set())
    dev = torch.device("cuda:0")
    out = []
    copy_ms = {}
    for op in ops:
        ms = graph_train_ms(torch, tev, op.launch, op.nsets, iters, replays=1)
        if op.alg_bytes not in copy_ms:
            # yardstick: the library's plain copy moving the same number of bytes (half read, half written)
            n = max(4, (op.alg_bytes // 8) // 4 * 4)
            ns = _nsets_for(8 * n)
            a = [torch.zeros(n, dtype=torch.float32, device=dev) for _ in range(ns)]
            b = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(ns)]
            copy_ms[op.alg_bytes] = graph_train_ms(
                torch, tev, lambda i: cm.cnnmem_transform(a[i], b[i], 1, 1, 1, n, cm.NCHW, cm.NCHW), ns, iters, replays=1)
            del a, b
        gbps = op.alg_bytes / (ms * 1e-3) / 1e9
        out.append({"config": op.config, "name": op.name, "alg_bytes": op.alg_bytes, "back_to_back_ms": round(ms, 5),
                    "achieved": round(gbps, 1), "frac": round(gbps / rl.PEAK_HBM_GBPS, 4),
                    "copy_same_bytes_ms": round(copy_ms[op.alg_bytes], 5),
                    "frac_of_copy": round(copy_ms[op.alg_bytes] / ms, 4)})
    del ops
    torch.cuda.empty_cache()
    return out


def cpu_baseline(wl, rl, host, reps=3):
    """The oracle, as it stands, timed on the same inputs (host copies): best of ``reps`` passes over
    the full workload on all host threads, and one pass on one thread over an eighth of every tensor."""
    import oracle
    t = wl.config(2).transforms[0]
    p = wl.config(4).pools[0].tensor
    s = wl.config(5).softmaxes[0]
    t_start = time.perf_counter()
    xpc = None
    if "pool" in host:                                           # input prep, not timed
        xpc = oracle.transform(host["pool"], p.N, p.C, p.H, p.W, oracle.NCHW, oracle.CHWN)

    def one_pass(frac):
        """Times one pass over the first 1/frac of every tensor (whole images / whole rows)."""
        parts = {}
        if "transform" in host:
            n = t.N // frac
            x = host["transform"][:n]
            t0 = time.perf_counter()
            xtc = oracle.transform(x, n, t.C, t.H, t.W, oracle.NCHW, oracle.CHWN)
            oracle.transform(xtc, n, t.C, t.H, t.W, oracle.CHWN, oracle.NCHW)
            parts["transform"] = (2 * rl.transform_bytes(n, t.C, t.H, t.W), time.perf_counter() - t0)
        if "pool" in host:
            c = p.C // frac                                     # CHWN slices along C stay contiguous
            xn, xc = host["pool"][:, :c], xpc[:c]
            if frac > 1:
                import numpy as np
                xn = np.ascontiguousarray(xn)
            t0 = time.perf_counter()
            for mode in (oracle.POOL_MAX, oracle.POOL_AVG):
                oracle.pool(xn, p.N, c, p.H, p.W, oracle.NCHW, mode, 2, 2, 2, 2)
                oracle.pool(xc, p.N, c, p.H, p.W, oracle.CHWN, mode, 2, 2, 2, 2)
            parts["pool"] = (4 * rl.pool_bytes(p.N, c, p.H, p.W, 2, 2, 2, 2), time.perf_counter() - t0)
        if "softmax" in host:
            n = s.N // frac
            t0 = time.perf_counter()
            oracle.softmax(host["softmax"][:n])
            parts["softmax"] = (rl.softmax_bytes(n, s.classes), time.perf_counter() - t0)
        return parts

    best = None
    for _ in range(reps):
        parts = one_pass(1)
        if best is None or sum(d for _, d in parts.values()) < sum(d for _, d in best.values()):
            best = parts
    cores = oracle.threads()
    oracle.set_threads(1)
    single = one_pass(8)
    oracle.set_threads(cores)
    total_bytes = sum(b for b, _ in best.values())
    dt = sum(d for _, d in best.values())
    sb, sd = sum(b for b, _ in single.values()), sum(d for _, d in single.values())
    return {"value": round(total_bytes / dt / 1e9, 3), "unit": "GB/s", "cores": cores,
            "kind": "oracle", "seconds": round(dt, 3),
            "per_layer": {k: round(b / d / 1e9, 3) for k, (b, d) in best.items()},
            "single_thread": {"value": round(sb / sd / 1e9, 3), "unit": "GB/s", "seconds": round(sd, 3),
                              "sample": "one pass over the first eighth of every tensor on one thread"},
            "sample": f"best of {reps} passes of the same launches over the full workload "
                      f"({total_bytes / 1e6:.0f} MB algorithmic per pass; {time.perf_counter() - t_start:.1f} s wall "
                      f"including untimed input preparation and the single-thread pass)"}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this hot path has no multi-GPU leg in this build "
              "(run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_1610_03618_amd as cm
    from paper_1610_03618_amd import counters
    from paper_1610_03618_amd.timing import TimingEvents
    from paper_1610_03618_amd import roofline as rl
    from paper_1610_03618_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU (there is no CPU fallback for the hot path)", file=sys.stderr)
        sys.exit(2)
    cm.library()                                  # fails loudly if the HIP library is not built
    torch.cuda.set_device(0)
    only = set(filter(None, args.only.split(",")))
    builders = {"largest": build_ops, "table1": build_table1_ops, "softmax_sweep": build_softmax_sweep_ops,
                "layout_policy": build_layout_policy_ops, "layouts": build_layouts_ops,
                "backward": build_backward_ops, "shapes": build_shapes_ops, "configs": build_config_ops,
                "access_patterns": build_access_pattern_ops}
    if args.workload == "largest":
        ops, host_inputs = build_ops(torch, cm, wl, rl, only, args.dtype)
    else:
        if args.dtype != "f32":
            print("--dtype applies to the headline workload only", file=sys.stderr)
            sys.exit(2)
        # "copy_calibration" in --only adds the yardstick copy below; alone, it adds it to every launch of the workload
        chosen = only if args.workload == "configs" else only - {"copy_calibration"}
        ops, host_inputs = builders[args.workload](torch, cm, wl, rl, chosen)
    if "copy_calibration" in only and not any(op.name == "copy_calibration" for op in ops):
        # a plain copy of known size, the yardstick the traffic counters are scaled by (any workload)
        n_cal = 128 * 96 * 55 * 55
        cal_a = [torch.zeros(n_cal, dtype=torch.float32, device="cuda") for _ in range(4)]
        cal_b = [torch.empty(n_cal, dtype=torch.float32, device="cuda") for _ in range(4)]
        ops.append(Op("copy_calibration", "copy", 2 * 4 * n_cal, n_cal, "elements",
                      lambda i: cm.cnnmem_transform(cal_a[i], cal_b[i], 1, 1, 1, n_cal, cm.NCHW, cm.NCHW), 4))
    if args.workload != "largest" or args.dtype != "f32":
        args.no_cpu_baseline = True                # the oracle baseline is reported for the headline workload
    if not ops:
        print("no op selected", file=sys.stderr)
        sys.exit(2)

    # One event before the first launch of a step and one after every launch: launch k of a step lasted
    # from event k to event k + 1 (the launches of a step run back to back on one stream).
    tev = TimingEvents(torch)

    def one_step(step, events=None):
        if events is not None:
            tev.record(events[0])
        for k, op in enumerate(ops):
            # launch k of a step takes buffer set step + k: launches that share tensors (both pooling modes
            # on one input, a transform and its inverse) never touch a set the previous launch just used,
            # so the last-level cache cannot serve one launch with what its neighbour left there
            st = op.launch((step + k) % op.nsets)
            if events is not None:
                tev.record(events[k + 1])
            if st != 0:
                raise RuntimeError(f"{op.name}: status {st}")

    for w in range(args.warmup):
        one_step(w)
    torch.cuda.synchronize()

    # Two timed regions of K steps each, both between synchronisations.  The first has nothing on the stream
    # but the launches and gives `value`; the second repeats the same steps with the events in place and
    # gives the per-launch durations (its own wall time is reported as `ms_per_step_with_events`).
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        one_step(args.warmup + s)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    all_events = [tev.create(len(ops) + 1) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        one_step(args.warmup + s, all_events[s])
    torch.cuda.synchronize()
    wall_events = time.perf_counter() - t0

    for s in range(args.steps):
        for k, op in enumerate(ops):
            op.ms.append(tev.elapsed_ms(all_events[s][k], all_events[s][k + 1]))

    graph_info = None
    if args.graph:
        # One graph holds as many consecutive steps as the deepest buffer rotation, so replays keep
        # cycling through the buffer sets exactly like the eager loop.
        per_graph = max(op.nsets for op in ops)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for s in range(per_graph):
                one_step(s)
        graph.replay()
        torch.cuda.synchronize()
        reps = max(1, -(-args.steps // per_graph))
        t0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        gwall = (time.perf_counter() - t0) / (reps * per_graph)
        graph_info = {"steps_per_graph": per_graph, "replays": reps, "ms_per_step": round(gwall * 1e3, 4),
                      "value": round(sum(op.alg_bytes for op in ops) / gwall / 1e9, 1), "unit": "GB/s"}

    tev.destroy_all()
    extras = {} if args.no_extras else measure_extras(torch, cm, ops, tev)
    # the driver's default run also times every other tensor of the five configurations
    per_config = None
    if args.workload == "largest" and args.dtype == "f32" and not only and not args.no_extras:
        per_config = measure_configs(torch, cm, wl, rl, tev)
    torch_ms = measure_torch(torch, ops) if args.compare_torch else {}
    step_bytes = sum(op.alg_bytes for op in ops)
    ms_per_step = wall / args.steps * 1e3
    value = step_bytes / (wall / args.steps) / 1e9
    # HBM bytes per launch from the committed rocprofv3 counter summary; only while that summary was measured on
    # the kernel sources this run uses (a digest of csrc/ and include/), otherwise null
    digest = counters.sources_digest()
    traffic_file = {"largest": "hbm_traffic_largest_configs.json", "configs": "hbm_traffic_all_configs.json"}
    traffic_path = os.path.join(ROOT, "profiles", traffic_file.get(args.workload, "none"))
    traffic_table = counters.load_for(traffic_path, digest)
    kernels = []
    for op in ops:
        avg_ms = sum(op.ms) / len(op.ms)
        med_ms = sorted(op.ms)[len(op.ms) // 2]
        gbps = op.alg_bytes / (avg_ms * 1e-3) / 1e9
        kernels.append({"name": op.name, "kind": op.kind, "avg_ms": round(avg_ms, 5), "median_ms": round(med_ms, 5),
                        "min_ms": round(min(op.ms), 5), "alg_bytes": op.alg_bytes,
                        "achieved": round(gbps, 1), "frac": round(gbps / rl.PEAK_HBM_GBPS, 4),
                        "traffic": (traffic_table["ops"].get(op.name, {}).get("traffic")
                                    if traffic_table and args.dtype == "f32" else None)})
        if op.name in extras:
            warm_ms, copy_ms, b2b_ms, copy_b2b_ms = extras[op.name]
            kernels[-1]["warm_median_ms"] = round(warm_ms, 5)
            kernels[-1]["copy_same_bytes_median_ms"] = round(copy_ms, 5)
            kernels[-1]["frac_of_copy"] = round(copy_ms / med_ms, 4)
            kernels[-1]["back_to_back_ms"] = round(b2b_ms, 5)
            kernels[-1]["back_to_back_frac"] = round(op.alg_bytes / (b2b_ms * 1e-3) / 1e9 / rl.PEAK_HBM_GBPS, 4)
            kernels[-1]["copy_back_to_back_ms"] = round(copy_b2b_ms, 5)
        if op.name in torch_ms:
            kernels[-1]["torch_median_ms"] = round(torch_ms[op.name], 5)
    dominant = max(kernels, key=lambda k: k["avg_ms"])
    roofline = {"bound": "hbm", "kernel": dominant["name"], "achieved": dominant["achieved"],
                "peak": rl.PEAK_HBM_GBPS, "unit": "GB/s", "frac": dominant["frac"],
                "traffic": dominant["traffic"],
                "traffic_source": (f"profiles/{traffic_file.get(args.workload)} (rocprofv3 FETCH_SIZE / WRITE_SIZE on "
                                   "these kernel sources)" if traffic_table else
                                   "none: no counter summary for the kernel sources of this run"),
                "alg_bytes_per_launch": dominant["alg_bytes"], "avg_ms": dominant["avg_ms"]}
    if "back_to_back_ms" in dominant:
        # the same launch repeated between one pair of events: no event after every launch, so this is the
        # figure that agrees with the profiler's kernel duration
        roofline["back_to_back"] = {"avg_ms": dominant["back_to_back_ms"],
                                    "achieved": round(dominant["alg_bytes"] / (dominant["back_to_back_ms"] * 1e-3) / 1e9, 1),
                                    "frac": dominant["back_to_back_frac"]}
    per_kind = {}
    for kind in ("transform", "pool", "softmax"):
        ks = [k for k in kernels if k["kind"] == kind]
        if ks:
            b = sum(k["alg_bytes"] for k in ks)
            t = sum(k["avg_ms"] for k in ks) * 1e-3
            per_kind[kind] = {"achieved": round(b / t / 1e9, 1), "frac": round(b / t / 1e9 / rl.PEAK_HBM_GBPS, 4)}

    per_kind_b2b = {}
    for kind in ("transform", "pool", "softmax"):
        ks = [k for k in kernels if k["kind"] == kind and "back_to_back_ms" in k]
        if ks:
            b = sum(k["alg_bytes"] for k in ks)
            t = sum(k["back_to_back_ms"] for k in ks) * 1e-3
            per_kind_b2b[kind] = {"achieved": round(b / t / 1e9, 1), "frac": round(b / t / 1e9 / rl.PEAK_HBM_GBPS, 4)}

    out = {
        "metric": "achieved HBM GB/s (and % of peak) per layer: transform, pool, softmax",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "ms_per_step_with_events": round(wall_events / args.steps * 1e3, 4),
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": args.dtype, "data": "synthetic", "sources_digest": digest,
        "config": {"workload": WORKLOAD_TEXT[args.workload] + ("" if args.dtype == "f32" else f", tensors stored as {args.dtype}"),
                   "launches_per_step": len(ops), "alg_bytes_per_step": step_bytes,
                   "cache_control": "rotating buffer sets, each larger than the 256 MB last-level cache"},
        "per_layer": per_kind,
        "per_layer_back_to_back": per_kind_b2b,
        "roofline": roofline,
        "kernels": kernels,
    }
    if per_config is not None:
        out["per_config"] = per_config
    if graph_info:
        out["graph"] = graph_info
    if args.workload == "layout_policy":
        out["layout_policy"] = layout_policy_summary(kernels)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, rl, host_inputs)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()

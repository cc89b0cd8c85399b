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


def parse_args():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--only", default="", help="comma list of op names to run (profiling aid)")
    ap.add_argument("--workload", choices=["largest", "table1"], default="largest",
                    help="largest: each kernel on its largest configured tensor (the headline run); "
                         "table1: every pooling and classifier layer of the paper's Table 1")
    ap.add_argument("--verbose", action="store_true")
    return ap.parse_args()


class Op:
    """One launch of the hot path with its rotating buffer sets."""

    def __init__(self, name, kind, alg_bytes, units, unit_name, launch, nsets):
        self.name, self.kind, self.alg_bytes = name, kind, alg_bytes
        self.units, self.unit_name = units, unit_name
        self.launch, self.nsets = launch, nsets
        self.ms = []


def build_ops(torch, cm, wl, rl, only):
    dev = torch.device("cuda:0")
    ops = []
    host = {}

    def rotating(t, n):
        return [t] + [t.clone() for _ in range(n - 1)]

    def want(name):
        return not only or name in only

    # ---- transform: config 2 tensor --------------------------------------------------
    t = wl.config(2).transforms[0]
    if want("transform_nchw_to_chwn") or want("transform_chwn_to_nchw"):
        host["transform"] = wl.make_tensor(t, wl.rng_for(2))
        x = torch.from_numpy(host["transform"]).to(dev)
        nset = 4                                             # 4 x (149 + 149) MB > 1 GB
        xs = rotating(x, nset)
        cs = [torch.empty((t.C, t.H, t.W, t.N), dtype=torch.float32, device=dev) for _ in range(nset)]
        bs = [torch.empty((t.N, t.C, t.H, t.W), dtype=torch.float32, device=dev) for _ in range(nset)]
        for i in range(nset):
            cm.transform(xs[i], t.N, t.C, t.H, t.W, cm.NCHW, cm.CHWN, out=cs[i])
        tb = rl.transform_bytes(t.N, t.C, t.H, t.W)
        if want("transform_nchw_to_chwn"):
            ops.append(Op("transform_nchw_to_chwn", "transform", tb, t.numel, "elements",
                          lambda i: cm.cnnmem_transform(xs[i], cs[i], t.N, t.C, t.H, t.W, cm.NCHW, cm.CHWN), nset))
        if want("transform_chwn_to_nchw"):
            ops.append(Op("transform_chwn_to_nchw", "transform", tb, t.numel, "elements",
                          lambda i: cm.cnnmem_transform(cs[i], bs[i], t.N, t.C, t.H, t.W, cm.CHWN, cm.NCHW), nset))

    # ---- pooling: config 4, first tensor ----------------------------------------------
    p = wl.config(4).pools[0].tensor
    pool_names = ["pool_max_nchw", "pool_max_chwn", "pool_avg_nchw", "pool_avg_chwn"]
    if any(want(n) for n in pool_names):
        host["pool"] = wl.make_tensor(p, wl.rng_for(4, 0))
        x = torch.from_numpy(host["pool"]).to(dev)
        nset = 2                                             # 2 x (822 + 206) MB
        st, Ho, Wo = cm.cnnmem_pool_out_dims(p.H, p.W, 2, 2, 2, 2, 0, 0)
        assert st == 0
        pb = rl.pool_bytes(p.N, p.C, p.H, p.W, 2, 2, 2, 2)
        xn = rotating(x, nset)
        xc = [cm.transform(xn[i], p.N, p.C, p.H, p.W, cm.NCHW, cm.CHWN) for i in range(nset)]
        on = [torch.empty((p.N, p.C, Ho, Wo), dtype=torch.float32, device=dev) for _ in range(nset)]
        oc = [torch.empty((p.C, Ho, Wo, p.N), dtype=torch.float32, device=dev) for _ in range(nset)]

        def pool_launch(src, dst, layout, mode):
            return lambda i: cm.cnnmem_pool(src[i], dst[i], p.N, p.C, p.H, p.W, layout, mode, 2, 2, 2, 2, 0, 0)

        table = {"pool_max_nchw": (xn, on, cm.NCHW, cm.POOL_MAX), "pool_max_chwn": (xc, oc, cm.CHWN, cm.POOL_MAX),
                 "pool_avg_nchw": (xn, on, cm.NCHW, cm.POOL_AVG), "pool_avg_chwn": (xc, oc, cm.CHWN, cm.POOL_AVG)}
        for name in pool_names:
            if want(name):
                ops.append(Op(name, "pool", pb, p.numel, "input elements", pool_launch(*table[name]), nset))

    # ---- softmax: config 5 ---------------------------------------------------------------
    s = wl.config(5).softmaxes[0]
    if want("softmax"):
        host["softmax"] = wl.make_logits(s, wl.rng_for(5, 0))
        z = torch.from_numpy(host["softmax"]).to(dev)
        nset = 2                                             # 2 x (358 + 358) MB
        zs = rotating(z, nset)
        ps = [torch.empty_like(z) for _ in range(nset)]
        ops.append(Op("softmax", "softmax", rl.softmax_bytes(s.N, s.classes), s.N * s.classes, "elements",
                      lambda i: cm.cnnmem_softmax(zs[i], ps[i], s.N, s.classes), nset))
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

    def nsets_for(nbytes):
        return int(min(16, max(2, (1 << 30) // nbytes + 1)))

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


def cpu_baseline(wl, rl, host):
    """The oracle, as it stands, timed on one pass over the same inputs (host copies)."""
    import oracle
    t = wl.config(2).transforms[0]
    p = wl.config(4).pools[0].tensor
    s = wl.config(5).softmaxes[0]
    total_bytes, parts = 0, {}
    t_start = time.perf_counter()
    if "transform" in host:
        t0 = time.perf_counter()
        xtc = oracle.transform(host["transform"], t.N, t.C, t.H, t.W, oracle.NCHW, oracle.CHWN)
        oracle.transform(xtc, t.N, t.C, t.H, t.W, oracle.CHWN, oracle.NCHW)
        parts["transform"] = (2 * rl.transform_bytes(t.N, t.C, t.H, t.W), time.perf_counter() - t0)
        del xtc
    if "pool" in host:
        xp = host["pool"]
        xpc = oracle.transform(xp, p.N, p.C, p.H, p.W, oracle.NCHW, oracle.CHWN)   # input prep, not timed
        t0 = time.perf_counter()
        for mode in (oracle.POOL_MAX, oracle.POOL_AVG):
            oracle.pool(xp, p.N, p.C, p.H, p.W, oracle.NCHW, mode, 2, 2, 2, 2)
            oracle.pool(xpc, p.N, p.C, p.H, p.W, oracle.CHWN, mode, 2, 2, 2, 2)
        parts["pool"] = (4 * rl.pool_bytes(p.N, p.C, p.H, p.W, 2, 2, 2, 2), time.perf_counter() - t0)
        del xpc
    if "softmax" in host:
        t0 = time.perf_counter()
        oracle.softmax(host["softmax"])
        parts["softmax"] = (rl.softmax_bytes(s.N, s.classes), time.perf_counter() - t0)
    total_bytes = sum(b for b, _ in parts.values())
    dt = sum(d for _, d in parts.values())
    return {"value": round(total_bytes / dt / 1e9, 3), "unit": "GB/s", "cores": oracle.threads(),
            "kind": "oracle", "seconds": round(dt, 3),
            "per_layer": {k: round(b / d / 1e9, 3) for k, (b, d) in parts.items()},
            "sample": f"one pass of the same launches over the full workload "
                      f"({total_bytes / 1e6:.0f} MB algorithmic, {time.perf_counter() - t_start:.1f} s wall "
                      f"including untimed input preparation)"}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this hot path has no multi-GPU leg in this build "
              "(run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_1610_03618_amd as cm
    from paper_1610_03618_amd import roofline as rl
    from paper_1610_03618_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU (there is no CPU fallback for the hot path)", file=sys.stderr)
        sys.exit(2)
    cm.library()                                  # fails loudly if the HIP library is not built
    torch.cuda.set_device(0)
    only = set(filter(None, args.only.split(",")))
    if args.workload == "table1":
        ops, host_inputs = build_table1_ops(torch, cm, wl, rl, only)
        args.no_cpu_baseline = True                # the oracle baseline is reported for the headline workload
    else:
        ops, host_inputs = build_ops(torch, cm, wl, rl, only)
    if not ops:
        print("no op selected", file=sys.stderr)
        sys.exit(2)

    def one_step(step, events=None):
        for k, op in enumerate(ops):
            if events is not None:
                events[k][0].record()
            st = op.launch(step % op.nsets)
            if events is not None:
                events[k][1].record()
            if st != 0:
                raise RuntimeError(f"{op.name}: status {st}")

    for w in range(args.warmup):
        one_step(w)
    torch.cuda.synchronize()

    all_events = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in ops]
                  for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        one_step(args.warmup + s, all_events[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    for s in range(args.steps):
        for k, op in enumerate(ops):
            op.ms.append(all_events[s][k][0].elapsed_time(all_events[s][k][1]))

    step_bytes = sum(op.alg_bytes for op in ops)
    ms_per_step = wall / args.steps * 1e3
    value = step_bytes / (wall / args.steps) / 1e9
    kernels = []
    for op in ops:
        avg_ms = sum(op.ms) / len(op.ms)
        med_ms = sorted(op.ms)[len(op.ms) // 2]
        gbps = op.alg_bytes / (avg_ms * 1e-3) / 1e9
        kernels.append({"name": op.name, "kind": op.kind, "avg_ms": round(avg_ms, 5), "median_ms": round(med_ms, 5),
                        "min_ms": round(min(op.ms), 5), "alg_bytes": op.alg_bytes,
                        "achieved": round(gbps, 1), "frac": round(gbps / rl.PEAK_HBM_GBPS, 4),
                        "traffic": rl.MEASURED_TRAFFIC.get(op.name)})
    dominant = max(kernels, key=lambda k: k["avg_ms"])
    roofline = {"bound": "hbm", "kernel": dominant["name"], "achieved": dominant["achieved"],
                "peak": rl.PEAK_HBM_GBPS, "unit": "GB/s", "frac": dominant["frac"],
                "traffic": rl.MEASURED_TRAFFIC.get(dominant["name"]),
                "alg_bytes_per_launch": dominant["alg_bytes"], "avg_ms": dominant["avg_ms"]}
    per_kind = {}
    for kind in ("transform", "pool", "softmax"):
        ks = [k for k in kernels if k["kind"] == kind]
        if ks:
            b = sum(k["alg_bytes"] for k in ks)
            t = sum(k["avg_ms"] for k in ks) * 1e-3
            per_kind[kind] = {"achieved": round(b / t / 1e9, 1), "frac": round(b / t / 1e9 / rl.PEAK_HBM_GBPS, 4)}

    out = {
        "metric": "achieved HBM GB/s (and % of peak) per layer: transform, pool, softmax",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": ("largest tensor per kernel: transform 128x96x55x55 both directions (config 2), "
                                "max+avg pool 2x2/s2 on 64x64x224x224 in NCHW and CHWN (config 4), "
                                "softmax 4096x21841 (config 5)") if args.workload == "largest" else
                               "Table 1 of the paper: max-pool PL1..PL10 in NCHW and CHWN, softmax CLASS1..CLASS5",
                   "launches_per_step": len(ops), "alg_bytes_per_step": step_bytes,
                   "cache_control": "rotating buffer sets, each larger than the 256 MB last-level cache"},
        "per_layer": per_kind,
        "roofline": roofline,
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, rl, host_inputs)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()

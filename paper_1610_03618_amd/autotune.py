"""Pooling auto-tuner (Section V.A of the paper).

The paper expands the number of outputs a thread computes ("working set
expansion") along both image directions and searches the two factors by hill
climbing: start at 2, keep adding 1 while the kernel gets faster, stop at the
first step that does not help (more registers, less parallelism).  Here the same
search runs over the fields of :class:`PoolTuning` — output rows and columns per
lane for the CHWN kernel — followed by a short scan of the choices this GPU adds
(occupancy cap; for NCHW the kernel and its lanes per LDS slab).

Timing is done on the GPU: a train of launches on rotating buffers (so that the
last-level cache cannot serve the input) is replayed as one HIP graph between a
pair of HIP events on torch's current stream.  The search only
measures; results of a pooling call never depend on the tuning.

Command line::

    python -m paper_1610_03618_amd.autotune --layout chwn --N 128 --C 96 --H 55 --W 55 --k 3 --s 2
    python -m paper_1610_03618_amd.autotune --table1 --out pool_tuning.json
"""
from __future__ import annotations

import argparse
import json
import sys
from typing import Callable, Dict, List, Optional, Tuple

NCHW, CHWN = 0, 1
POOL_MAX, POOL_AVG = 0, 1
NOISE = 0.02        # a candidate has to be this much faster to replace the current choice


def hill_climb(cost: Callable[[int], float], lo: int, hi: int, start: int = 2,
               margin: float = 0.0) -> Tuple[int, Dict[int, float]]:
    """The paper's search along one direction.

    ``cost(f)`` is the measured time with expansion factor ``f``.  The factor
    ``lo`` (no expansion) is the baseline; ``start`` is tried next and the factor
    then grows by one while the time keeps improving, up to ``hi``.  Returns the
    best factor and everything that was measured.  ``margin``: the fraction by which a step has to be
    faster to count (measured times carry noise; 0 is the paper's plain rule).
    """
    seen = {lo: cost(lo)}
    best = lo
    f = max(start, lo + 1)
    while f <= hi:
        seen[f] = cost(f)
        if seen[f] < seen[best] * (1.0 - margin):
            best = f
            f += 1
        else:
            break
    return best, seen


def _time_launch(launch: Callable[[int], int], nsets: int, iters: int) -> float:
    """Milliseconds per launch: a train of ``iters`` launches on rotating buffers, replayed as one HIP graph
    between one pair of events (best of seven replays).  An event pair around every launch, the clock this
    tuner used first, costs more than the 6-10 us launches of the small layers take, and the winner changed
    from run to run."""
    import torch

    from .timing import TimingEvents, graph_train_ms
    global _events
    if _events is None:
        _events = TimingEvents(torch)
    return graph_train_ms(torch, _events, launch, nsets, iters, replays=7)


_events = None


def tune_pool(N: int, C: int, H: int, W: int, layout: int, mode: int, k: int, s: int, p: int = 0,
              iters: int = 30, log: Optional[Callable[[str], None]] = None) -> Tuple[dict, List[dict]]:
    """Searches the pooling launch shape for one layer; returns (best tuning, history).

    The history lists every configuration that was timed with its milliseconds
    and GB/s (algorithmic bytes / time).
    """
    import torch

    from . import binding as cm
    from . import roofline as rl

    st, Ho, Wo = cm.cnnmem_pool_out_dims(H, W, k, k, s, s, p, p)
    if st != 0:
        raise ValueError("invalid pooling geometry")
    n_in, n_out = N * C * H * W, N * C * Ho * Wo
    alg_bytes = rl.pool_bytes(N, C, H, W, k, k, s, s, p, p)
    nsets = int(min(16, max(2, (1 << 30) // (4 * (n_in + n_out)) + 1)))
    gen = torch.Generator(device="cuda").manual_seed(1610)
    xs = [torch.randn(n_in, device="cuda", generator=gen).relu_() for _ in range(nsets)]
    ys = [torch.empty(n_out, dtype=torch.float32, device="cuda") for _ in range(nsets)]
    history: List[dict] = []

    def timed(tuning: dict) -> float:
        t = cm.PoolTuning(**tuning)
        ms = _time_launch(lambda i: cm.cnnmem_pool_tuned(xs[i], ys[i], N, C, H, W, layout, mode, k, k, s, s, p, p, t),
                          nsets, iters)
        entry = dict(tuning=dict(tuning), ms=round(ms, 5), gbps=round(alg_bytes / ms / 1e6, 1))
        history.append(entry)
        if log:
            log(f"  {tuning} -> {ms * 1e3:.1f} us, {entry['gbps']:.0f} GB/s")
        return ms

    best: dict = {}
    if layout == CHWN:
        rows, _ = hill_climb(lambda f: timed({**best, "rows_per_lane": f}), 1, 4, margin=NOISE)
        best["rows_per_lane"] = rows
        cols, _ = hill_climb(lambda f: timed({**best, "cols_per_lane": f}), 1, 2, margin=NOISE)
        best["cols_per_lane"] = cols
    else:
        # the library's own choice first (row pairs, the rows kernel or the slab kernel), then the slab kernel by size
        candidates = [dict()] + [dict(nchw_kernel=2, slab_lanes=lanes) for lanes in (512, 256, 1024)]
        times = [(timed(c), c) for c in candidates]
        # the library's default kernel (first candidate) stays unless another beats it by more than the noise
        first_ms = times[0][0]
        win_ms, win = min(times, key=lambda tc: tc[0])
        best = dict(win if win_ms < first_ms * (1.0 - NOISE) else times[0][1])
    # occupancy cap: none, then tighter while it helps
    base = timed({**best, "workgroups_per_cu": -1})
    cap_best, cap_ms = -1, base
    for cap in (6, 4, 3, 2):
        ms = timed({**best, "workgroups_per_cu": cap})
        if ms < cap_ms * (1.0 - NOISE):
            cap_best, cap_ms = cap, ms
        else:
            break
    best["workgroups_per_cu"] = cap_best
    return best, history


def load_table(path: str) -> Dict[tuple, dict]:
    """Reads a table written by ``--out`` and keys it by shape:
    (N, C, H, W, k, s, p, layout, mode) -> dict of :class:`PoolTuning` fields."""
    with open(path) as f:
        raw = json.load(f)
    table = {}
    for entry in raw.values():
        sh = entry["shape"]
        key = (sh["N"], sh["C"], sh["H"], sh["W"], sh["k"], sh["s"], sh["p"], sh["layout"], sh["mode"])
        table[key] = dict(entry["tuning"])
    return table


def lookup(table: Dict[tuple, dict], N: int, C: int, H: int, W: int, k: int, s: int, p: int, layout: int,
           mode: int) -> Optional[dict]:
    """The cached tuning of a layer, or None (= library defaults) when the shape was never tuned.
    Pass the result as ``tuning=`` to :func:`paper_1610_03618_amd.pool`."""
    return table.get((N, C, H, W, k, s, p, layout, mode))


def _table1_layers():
    from . import workloads as wl
    return [(name, N, C, hw, hw, k, s) for (name, N, hw, k, C, s) in wl.TABLE1_POOLS]


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--layout", choices=["nchw", "chwn", "both"], default="both")
    ap.add_argument("--mode", choices=["max", "avg"], default="max")
    ap.add_argument("--N", type=int)
    ap.add_argument("--C", type=int)
    ap.add_argument("--H", type=int)
    ap.add_argument("--W", type=int)
    ap.add_argument("--k", type=int, default=3)
    ap.add_argument("--s", type=int, default=2)
    ap.add_argument("--p", type=int, default=0)
    ap.add_argument("--iters", type=int, default=30)
    ap.add_argument("--table1", action="store_true", help="tune the ten pooling layers of Table 1")
    ap.add_argument("--out", help="write the shape -> tuning table here as JSON")
    args = ap.parse_args(argv)

    import torch
    if not torch.cuda.is_available():
        print("the auto-tuner measures on the GPU; none is visible", file=sys.stderr)
        return 2
    if args.table1:
        layers = _table1_layers()
    else:
        if None in (args.N, args.C, args.H, args.W):
            ap.error("give --N --C --H --W or --table1")
        layers = [("layer", args.N, args.C, args.H, args.W, args.k, args.s)]
    layouts = {"nchw": [NCHW], "chwn": [CHWN], "both": [NCHW, CHWN]}[args.layout]
    mode = POOL_MAX if args.mode == "max" else POOL_AVG
    table = {}
    for (name, N, C, H, W, k, s) in layers:
        for layout in layouts:
            tag = f"{name} N={N} C={C} {H}x{W} k{k}/s{s} {'NCHW' if layout == NCHW else 'CHWN'} {args.mode}"
            print(tag, flush=True)
            best, hist = tune_pool(N, C, H, W, layout, mode, k, s, args.p, args.iters, log=lambda m: print(m, flush=True))
            top = min(hist, key=lambda h: h["ms"])
            print(f"  best {best}: {top['gbps']:.0f} GB/s (first point of the search {hist[0]['gbps']:.0f} GB/s)",
                  flush=True)
            table[tag] = dict(shape=dict(N=N, C=C, H=H, W=W, k=k, s=s, p=args.p, layout=layout, mode=mode),
                              tuning=best, gbps=top["gbps"])
    if args.out:
        with open(args.out, "w") as f:
            json.dump(table, f, indent=1)
    return 0


if __name__ == "__main__":
    sys.exit(main())

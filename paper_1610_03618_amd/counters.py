"""HBM traffic per launch from rocprofv3 counter runs of ``bench.py`` (measurement support, not the hot path).

``FETCH_SIZE`` and ``WRITE_SIZE`` are collected in two separate runs of the same ``bench.py`` command with
``--no-extras --only <ops>,copy_calibration``; the last ``steps x launches`` library dispatches of such a run are
the event-timed steps, one dispatch per launch in the order of the JSON line's ``kernels``.  Each counter is
scaled by what it reads for ``copy_calibration``, a plain copy of known size.  The result is written as a JSON
file that records the digest of the kernel sources it was measured on; ``bench.py`` prints a ``traffic`` figure
only while that digest still matches the sources it runs.

    python3 -m paper_1610_03618_amd.counters --fetch DIR --write DIR --bench-line FILE --out profiles/NAME.json
"""
from __future__ import annotations

import argparse
import csv
import glob
import hashlib
import json
import os
import re
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def sources_digest() -> str:
    """SHA-256 over the kernel sources and the public header (names and contents, sorted)."""
    h = hashlib.sha256()
    for folder in (os.path.join(HERE, "csrc"), os.path.join(ROOT, "include")):
        for name in sorted(os.listdir(folder)):
            path = os.path.join(folder, name)
            if os.path.isfile(path):
                h.update(name.encode())
                with open(path, "rb") as f:
                    h.update(f.read())
    return h.hexdigest()[:16]


def _short(kernel: str) -> str:
    k = re.sub(r"cnnmem::\(anonymous namespace\)::", "", kernel)
    k = re.sub(r"^void ", "", k)
    return k.split("(")[0]


def library_dispatches(folder: str, counter: str):
    """[(dispatch id, kernel, value)] of the library's own kernels in a rocprofv3 counter-collection run."""
    files = glob.glob(os.path.join(folder, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise FileNotFoundError(f"no counter_collection.csv under {folder}")
    per_dispatch = {}
    for path in files:
        with open(path) as f:
            for row in csv.DictReader(f):
                if row["Counter_Name"] != counter or "cnnmem::" not in row["Kernel_Name"]:
                    continue
                key = int(row["Dispatch_Id"])
                name, value = per_dispatch.get(key, (row["Kernel_Name"], 0.0))
                per_dispatch[key] = (name, value + float(row["Counter_Value"]))   # one row per XCD on some versions
    return [(k, _short(n), v) for k, (n, v) in sorted(per_dispatch.items())]


def per_op(folder: str, counter: str, names, steps: int):
    """Average counter value per launch name over the event-timed steps (the run's last dispatches)."""
    rows = library_dispatches(folder, counter)
    need = steps * len(names)
    if len(rows) < need:
        raise ValueError(f"{folder}: {len(rows)} library dispatches, expected at least {need}")
    tail = rows[-need:]
    out = {}
    for i, name in enumerate(names):
        mine = tail[i::len(names)]
        kernels = {k for _, k, _ in mine}
        if len(kernels) != 1:
            raise ValueError(f"{name}: dispatches of several kernels {sorted(kernels)}; is one launch one kernel?")
        out[name] = {"kernel": kernels.pop(), "value": sum(v for _, _, v in mine) / len(mine)}
    return out


def summarise(fetch_dir: str, write_dir: str, bench_line: dict) -> dict:
    kernels = bench_line["kernels"]
    names = [k["name"] for k in kernels]
    alg = {k["name"]: k["alg_bytes"] for k in kernels}
    if "copy_calibration" not in names:
        raise ValueError("the counter runs need --only ...,copy_calibration")
    steps = bench_line["steps"]
    fetch = per_op(fetch_dir, "FETCH_SIZE", names, steps)
    write = per_op(write_dir, "WRITE_SIZE", names, steps)
    copy_kib = alg["copy_calibration"] / 2 / 1024.0           # read = written = half the algorithmic bytes
    f_fetch = fetch["copy_calibration"]["value"] / copy_kib
    f_write = write["copy_calibration"]["value"] / copy_kib
    ops = {}
    for name in names:
        if name == "copy_calibration":
            continue
        rb = fetch[name]["value"] / f_fetch * 1024.0
        wb = write[name]["value"] / f_write * 1024.0
        ops[name] = {"kernel": fetch[name]["kernel"], "fetch_kib": round(fetch[name]["value"], 1),
                     "write_kib": round(write[name]["value"], 1), "read_bytes": int(round(rb)),
                     "write_bytes": int(round(wb)), "traffic": int(round(rb + wb)), "alg_bytes": alg[name],
                     "traffic_over_algorithmic": round((rb + wb) / alg[name], 4)}
    return {"sources_digest": bench_line.get("sources_digest"), "workload": bench_line["config"]["workload"],
            "calibration": {"copy_kib_each_way": copy_kib, "fetch_kib": round(fetch["copy_calibration"]["value"], 1),
                            "write_kib": round(write["copy_calibration"]["value"], 1),
                            "fetch_factor": round(f_fetch, 6), "write_factor": round(f_write, 6)},
            "ops": ops}


def markdown_table(summary: dict) -> str:
    lines = ["| launch | kernel | FETCH_SIZE KiB | WRITE_SIZE KiB | read MB | write MB | traffic MB | algorithmic MB "
             "| traffic / algorithmic |", "|---|---|---|---|---|---|---|---|---|"]
    for name, o in summary["ops"].items():
        lines.append("| %s | `%s` | %.1f | %.1f | %.2f | %.2f | %.2f | %.2f | %.4f |" % (
            name, o["kernel"], o["fetch_kib"], o["write_kib"], o["read_bytes"] / 1e6, o["write_bytes"] / 1e6,
            o["traffic"] / 1e6, o["alg_bytes"] / 1e6, o["traffic_over_algorithmic"]))
    return "\n".join(lines)


def load_for(path: str, digest: str):
    """The traffic table at ``path`` if it was measured on the sources with this digest, else None."""
    try:
        with open(path) as f:
            table = json.load(f)
    except (OSError, ValueError):
        return None
    return table if table.get("sources_digest") == digest else None


def _last_json_line(path: str) -> dict:
    with open(path) as f:
        lines = [ln for ln in f.read().splitlines() if ln.startswith("{")]
    return json.loads(lines[-1])


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--fetch", required=True, help="output folder of the rocprofv3 --pmc FETCH_SIZE run")
    ap.add_argument("--write", required=True, help="output folder of the rocprofv3 --pmc WRITE_SIZE run")
    ap.add_argument("--bench-line", required=True, help="file holding the JSON line bench.py printed in either run")
    ap.add_argument("--out", required=True, help="JSON file to write (under profiles/)")
    args = ap.parse_args(argv)
    summary = summarise(args.fetch, args.write, _last_json_line(args.bench_line))
    with open(args.out, "w") as f:
        json.dump(summary, f, indent=1)
        f.write("\n")
    print(markdown_table(summary))
    return 0


if __name__ == "__main__":
    sys.exit(main())

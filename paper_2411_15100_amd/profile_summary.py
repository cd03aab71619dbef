"""Summaries of rocprofv3 runs for `profiles/`.

    python -m paper_2411_15100_amd.profile_summary trace <results.db> <out.txt> "<command>" ["<note>" ...]
        the per-kernel totals of a `rocprofv3 --kernel-trace --stats` run (view top_kernels of the rocpd
        database it writes), as text.

    python -m paper_2411_15100_amd.profile_summary counters <out.txt> <traffic.json> "<note>" <name>=<results.db> ...
        the per-kernel averages of `rocprofv3 --pmc <counter>` runs (one database per counter run), as text;
        and, from the FETCH_SIZE and WRITE_SIZE runs, HBM bytes per launch of the fill / apply kernels into
        traffic.json together with a hash of the kernel sources, which bench.py compares with the sources it
        runs: the figures are dropped (null) once a kernel has changed.  The counters are in KiB per
        dispatch and are scaled by what they read for a plain copy of known size in the same run
        (torch's bf16 <- fp32 copy of the logits buffers: 4 bytes read and 2 written per element).
        "-" as <traffic.json> writes the text only (runs of other workloads than the serving step).
"""

from __future__ import annotations

import hashlib
import json
import os
import sqlite3
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
KERNEL_SOURCES = ["kernels.hip", "kernels.hpp", "walk.hpp"]
COPY_KERNEL = "bfloat16_copy_kernel"         # torch's fp32 -> bf16 copy of one logits buffer


def kernel_source_hash() -> str:
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2411_15100_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def short(name: str) -> str:
    for prefix in ("void ", "xgm::(anonymous namespace)::"):
        name = name.replace(prefix, "")
    return name.split("(")[0][:70]


def trace(db: str, out: str, cmd: str, notes):
    c = sqlite3.connect(db)
    rows = list(c.execute("select name,total_calls,total_duration,average,percentage from top_kernels"))
    with open(out, "w") as f:
        f.write("# rocprofv3 kernel-trace summary (view top_kernels of the rocpd database; durations in microseconds)\n")
        f.write("# command: " + cmd + "\n")
        for n in notes:
            f.write("# " + n + "\n")
        f.write(f"{'calls':>7} {'total_us':>14} {'avg_us':>11} {'pct':>6}  kernel\n")
        for name, calls, total, avg, pct in rows:
            f.write(f"{calls:7d} {total:14.1f} {avg:11.2f} {pct:6.2f}  {short(name)}\n")
    print(open(out).read())


def counter_averages(db: str):
    """{counter: {kernel: (dispatches, mean value)}} of one --pmc run."""
    c = sqlite3.connect(db)
    tables = [r[0] for r in c.execute("select name from sqlite_master where type in ('table','view')")]
    view = "counters_collection" if "counters_collection" in tables else None
    if view is None:
        raise SystemExit(f"{db}: no counters_collection view (tables: {tables})")
    cols = [r[1] for r in c.execute(f"pragma table_info({view})")]
    kcol = "kernel_name" if "kernel_name" in cols else "name"
    out = {}
    for kernel, counter, n, mean in c.execute(
            f"select {kcol}, counter_name, count(*), avg(value) from {view} group by {kcol}, counter_name"):
        out.setdefault(counter, {})[kernel] = (n, mean)
    return out


def counters(out: str, traffic_json: str, note: str, runs):
    text = ["# rocprofv3 --pmc summary: mean counter value per dispatch, by kernel", "# " + note]
    fetch, write = {}, {}
    for label, db in runs:
        text.append(f"# run {label}: {db}")
        for counter, per_kernel in sorted(counter_averages(db).items()):
            text.append(f"{counter}:")
            for kernel, (n, mean) in sorted(per_kernel.items(), key=lambda kv: -kv[1][1])[:14]:
                text.append(f"  {n:7d} dispatches  mean {mean:14.1f}  {short(kernel)}")
            if counter == "FETCH_SIZE":
                fetch = per_kernel
            if counter == "WRITE_SIZE":
                write = per_kernel

    def find(per_kernel, part):
        return [v for k, v in per_kernel.items() if part in k]

    traffic = {"kernel_source_hash": kernel_source_hash(), "bytes_per_launch": {}, "scale": {}}
    copy_f, copy_w = find(fetch, COPY_KERNEL), find(write, COPY_KERNEL)
    if copy_f and copy_w:
        # the copy reads 4 bytes and writes 2 per element; its size is taken from what it writes at factor 1
        elems = copy_w[0][1] * 1024.0 / 2.0
        f_scale = (4.0 * elems) / (copy_f[0][1] * 1024.0)
        traffic["scale"] = {"FETCH_SIZE": f_scale, "WRITE_SIZE": 1.0,
                            "copy_kernel_KiB": {"FETCH_SIZE": copy_f[0][1], "WRITE_SIZE": copy_w[0][1]}}
        text.append(f"# scale: WRITE_SIZE taken at 1.0 (the copy writes {copy_w[0][1]:.0f} KiB); FETCH_SIZE x {f_scale:.3f} "
                    f"(the copy reads twice what it writes, the counter shows {copy_f[0][1]:.0f} KiB)")
        for key, part in (("fill_kernel<false, 2>", "fill_kernel<false, 2>"), ("fill_kernel<false, 0>", "fill_kernel<false, 0>"),
                          ("apply_kernel<2>", "apply_kernel<2>")):
            f_, w_ = find(fetch, part), find(write, part)
            if f_ and w_:
                traffic["bytes_per_launch"][key] = (f_[0][1] * f_scale + w_[0][1]) * 1024.0
                traffic.setdefault("fetched_written", {})[key] = [f_[0][1] * f_scale * 1024.0, w_[0][1] * 1024.0]
                text.append(f"# {key}: fetched {f_[0][1] * f_scale * 1024 / 1e6:.2f} MB + written {w_[0][1] * 1024 / 1e6:.2f} MB per launch")
    with open(out, "w") as f:
        f.write("\n".join(text) + "\n")
    if traffic_json != "-":
        with open(traffic_json, "w") as f:
            json.dump(traffic, f, indent=1)
            f.write("\n")
    print("\n".join(text))


if __name__ == "__main__":
    if len(sys.argv) >= 5 and sys.argv[1] == "trace":
        trace(sys.argv[2], sys.argv[3], sys.argv[4], sys.argv[5:])
    elif len(sys.argv) >= 6 and sys.argv[1] == "counters":
        counters(sys.argv[2], sys.argv[3], sys.argv[4], [a.split("=", 1) for a in sys.argv[5:]])
    else:
        raise SystemExit(__doc__)

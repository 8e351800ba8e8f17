"""Summarises rocprofv3 CSV output (``--output-format csv``) per kernel.

    python -m paper_2601_12247_amd.profsum <output dir> [--top N]

* ``*_kernel_trace.csv``       -> calls, total, mean, min, max duration and share per kernel;
  stage-1 launches are also split by grid size (one workgroup of 1024 threads per logits row).
* ``*_counter_collection.csv`` -> mean counter value per dispatch, per kernel.  FETCH_SIZE and
  WRITE_SIZE are in KiB; the plain device-to-device copy that ``bench.py --pmc-reference``
  issues (256 MiB read, 256 MiB written) shows what the counters read for a known size.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import os
import re


def short(name: str) -> str:
    name = re.sub(r"\(anonymous namespace\)::", "", name)
    m = re.match(r"_ZN3pvf12_GLOBAL__N_1\d+([a-z0-9_]+kernel)I(.*?)EEv", name)
    if m:                                            # mangled template instance: keep the arguments readable
        args = re.sub(r"L[ibj](\d+)E", r"\1,", m.group(2)).replace("DF16b", "bf16,").replace("NS_12GemmEpilogueE", "")
        return f"{m.group(1)}<{args.strip(',')}>"
    if name.startswith(("void at::", "at::")):
        return "torch: " + name[:60]
    return name[:100]


def kernel_trace(path: str, top: int) -> None:
    acc = collections.defaultdict(list)
    s1 = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        d = int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
        k = short(r["Kernel_Name"])
        acc[k].append(d)
        if "stage1_vec" in k:
            s1[int(r.get("Grid_Size", r.get("Grid_Size_X", 0)))].append(d)
    tot = sum(sum(v) for v in acc.values())
    print(f"{'kernel':70s} {'calls':>6s} {'total_ms':>9s} {'avg_us':>9s} {'min_us':>8s} {'max_us':>8s} {'%':>6s}")
    for k, v in sorted(acc.items(), key=lambda kv: -sum(kv[1]))[:top]:
        print(f"{k:70s} {len(v):6d} {sum(v) / 1e6:9.2f} {sum(v) / len(v) / 1e3:9.2f} {min(v) / 1e3:8.2f} "
              f"{max(v) / 1e3:8.2f} {100 * sum(v) / tot:6.2f}")
    g = [v for k, v in acc.items() if k.startswith("gemm_bf16_mfma_kernel")]
    if g:
        n, t = sum(len(v) for v in g), sum(sum(v) for v in g)
        print(f"\nall gemm_bf16_mfma_kernel launches: {n} calls, mean {t / n / 1e3:.2f} us")
    for grid, v in sorted(s1.items()):
        print(f"stage1_vec_kernel grid {grid:8d} ({grid // 1024:5d} rows): calls {len(v):4d} mean {sum(v) / len(v) / 1e3:8.2f} us "
              f"min {min(v) / 1e3:8.2f} us")


def counters(path: str) -> None:
    acc = collections.defaultdict(lambda: [0.0, 0])
    for r in csv.DictReader(open(path)):
        k = short(r["Kernel_Name"])
        if "stage1_vec" in k or "copyBuffer" in k:
            k += f" grid={r.get('Grid_Size', r.get('Grid_Size_X', '?'))}"
        a = acc[(r["Counter_Name"], k)]
        a[0] += float(r["Counter_Value"]); a[1] += 1
    groups = collections.defaultdict(lambda: [0.0, 0])
    print(f"{'counter':12s} {'kernel':80s} {'dispatches':>10s} {'mean/dispatch':>16s}")
    for (c, k), (v, n) in sorted(acc.items()):
        if k.startswith("gemm_bf16_mfma_kernel"):
            g = groups[(c, "gemm_bf16_mfma_kernel (all instances)")]
            g[0] += v; g[1] += n
        print(f"{c:12s} {k:80s} {n:10d} {v / n:16.1f}")
    for (c, k), (v, n) in sorted(groups.items()):
        print(f"{c:12s} {k:80s} {n:10d} {v / n:16.1f}")


def main() -> None:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("dir")
    ap.add_argument("--top", type=int, default=24)
    a = ap.parse_args()
    for f in sorted(glob.glob(os.path.join(a.dir, "**", "*kernel_trace.csv"), recursive=True)):
        print(f"# {os.path.relpath(f, a.dir)}")
        kernel_trace(f, a.top)
    for f in sorted(glob.glob(os.path.join(a.dir, "**", "*counter_collection.csv"), recursive=True)):
        print(f"# {os.path.relpath(f, a.dir)}")
        counters(f)


if __name__ == "__main__":
    main()

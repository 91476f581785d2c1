"""Condenses rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2512_10411_amd.profile_summary stats   <dir with *kernel_stats.csv>
    python -m paper_2512_10411_amd.profile_summary traffic <FETCH_SIZE dir> <WRITE_SIZE dir> <copy MiB>

`traffic` scales the attention kernel's FETCH_SIZE / WRITE_SIZE readings (KiB per
dispatch) by what the same counters read for the plain copy kernel of known size
that `bench.py --copy-probe-mib` runs in the same process.
"""
from __future__ import annotations

import csv
import glob
import os
import sys


def _find(d, pattern):
    files = glob.glob(os.path.join(d, "**", pattern), recursive=True)
    if not files:
        raise SystemExit(f"no {pattern} under {d}")
    return files[0]


def stats(d):
    rows = list(csv.DictReader(open(_find(d, "*kernel_stats.csv"))))
    print("kernel, calls, total ns, average ns, min ns, max ns, percent")
    for r in rows:
        print(", ".join(r[k] for k in ("Name", "Calls", "TotalDurationNs", "AverageNs", "MinNs", "MaxNs", "Percentage")))


def _counter_per_kernel(d, counter):
    acc = {}
    for r in csv.DictReader(open(_find(d, "*counter_collection.csv"))):
        if r["Counter_Name"] != counter:
            continue
        a = acc.setdefault(r["Kernel_Name"], [0.0, 0])
        a[0] += float(r["Counter_Value"])
        a[1] += 1
    return {k: (v[0] / v[1], v[1]) for k, v in acc.items()}


def _largest_dispatch(d, counter, exclude):
    """(kernel name, reading) of the single largest dispatch of a kernel whose name lacks `exclude`."""
    best = None
    for r in csv.DictReader(open(_find(d, "*counter_collection.csv"))):
        if r["Counter_Name"] != counter or exclude in r["Kernel_Name"]:
            continue
        v = float(r["Counter_Value"])
        if best is None or v > best[1]:
            best = (r["Kernel_Name"], v)
    return best


def traffic(fetch_dir, write_dir, copy_mib):
    copy_bytes = float(copy_mib) * (1 << 20)
    out = {}
    for label, d, counter in (("read", fetch_dir, "FETCH_SIZE"), ("write", write_dir, "WRITE_SIZE")):
        per = _counter_per_kernel(d, counter)
        # the probe is the largest dispatch that is not ours (small host-to-device copies use the same kernel)
        probe = _largest_dispatch(d, counter, "swaa")
        attn = {k: v for k, v in per.items() if "swaa" in k}
        if probe is None or probe[1] * 1024 < 0.25 * copy_bytes or not attn:
            raise SystemExit(f"{counter}: copy kernel or attention kernel not found in {d}")
        ck, cval = probe
        factor = copy_bytes / (cval * 1024.0)
        for k, (val, n) in attn.items():
            out.setdefault(k, {})[label] = val * 1024.0 * factor
            print(f"{counter}: {k[:60]}: {val:.0f} KiB/dispatch raw (n={n}); copy kernel {ck[:40]} read as "
                  f"{cval:.0f} KiB for {copy_bytes / 1024:.0f} KiB -> factor {factor:.4f}")
    for k, v in out.items():
        tot = v.get("read", 0.0) + v.get("write", 0.0)
        print(f"HBM bytes per launch, {k[:60]}: read {v.get('read', 0):.4g} + write {v.get('write', 0):.4g} = {tot:.4g}")


if __name__ == "__main__":
    if len(sys.argv) >= 3 and sys.argv[1] == "stats":
        stats(sys.argv[2])
    elif len(sys.argv) >= 5 and sys.argv[1] == "traffic":
        traffic(sys.argv[2], sys.argv[3], sys.argv[4])
    else:
        raise SystemExit(__doc__)

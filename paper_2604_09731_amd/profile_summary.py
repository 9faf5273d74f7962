"""Summaries of rocprofv3 output folders for this library's kernels (text, for profiles/).

  python -m paper_2604_09731_amd.profile_summary stats <dir>
      per-kernel table of a `rocprofv3 --kernel-trace --stats --output-format csv -d <dir>` run
  python -m paper_2604_09731_amd.profile_summary pmc <dir>
      per-kernel mean / min / max of every counter of a `rocprofv3 --pmc ... --output-format csv -d <dir>` run
  python -m paper_2604_09731_amd.profile_summary traffic <fetch_dir> <write_dir> <workload> <kv> [<out file>]
      HBM bytes per launch of the dominant kernel (tva_prefix_kernel) from a FETCH_SIZE run and a WRITE_SIZE run of
      `bench.py --workload <workload> --copy-calibration`: each counter is scaled by what it reads for the plain
      1 GiB device copy of that same run (the runtime's copy kernel reads and writes 1 048 576 KiB).  Prints the
      figures and rewrites the workload's line of the out file (default profiles/hbm_traffic.txt), which bench.py
      reads for `roofline.traffic`.
"""
from __future__ import annotations

import collections
import csv
import glob
import os
import sys

COPY_KIB = float(1 << 20)          # the calibration copy: 1 GiB read, 1 GiB written
DOMINANT = "tva_prefix_kernel"
COPY_KERNEL = "copyBuffer"


def stats(folder):
    for f in sorted(glob.glob(folder + "/**/*kernel_stats.csv", recursive=True)):
        print("| kernel | calls | average ns | min ns | max ns | % of GPU time |\n|---|---|---|---|---|---|")
        for r in csv.DictReader(open(f)):
            print("| %s | %s | %s | %s | %s | %s |" % (r["Name"][:70], r["Calls"], r["AverageNs"], r["MinNs"], r["MaxNs"],
                                                       r["Percentage"]))


def counters(folder):
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for f in glob.glob(folder + "/**/*counter_collection.csv", recursive=True):
        for r in csv.DictReader(open(f)):
            acc[r["Kernel_Name"]][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return acc


def pmc(folder):
    print("| kernel | counter | dispatches | mean | min | max |\n|---|---|---|---|---|---|")
    for k, cs in sorted(counters(folder).items()):
        for c, v in sorted(cs.items()):
            print("| %s | %s | %d | %.1f | %.1f | %.1f |" % (k[:70], c, len(v), sum(v) / len(v), min(v), max(v)))


def _mean_of(acc, kernel_part, counter):
    vals = [v for k, cs in acc.items() if kernel_part in k for v in cs.get(counter, [])]
    if not vals:
        raise SystemExit(f"no {counter} values for a kernel named *{kernel_part}*")
    return sum(vals) / len(vals), len(vals)


def _largest_of(acc, kernel_part, counter):
    """Mean over the dispatches within 1 % of the largest one: the run's other copies (set-up, smaller buffers) go
    through the same copy kernel, the 1 GiB calibration copy is the biggest of them."""
    vals = [v for k, cs in acc.items() if kernel_part in k for v in cs.get(counter, [])]
    if not vals:
        raise SystemExit(f"no {counter} values for a kernel named *{kernel_part}*")
    top = max(vals)
    near = [v for v in vals if v >= 0.99 * top]
    return sum(near) / len(near)


def traffic(fetch_dir, write_dir, workload, kv, out_file):
    fa, wa = counters(fetch_dir), counters(write_dir)
    copy_fetch = _largest_of(fa, COPY_KERNEL, "FETCH_SIZE")
    copy_write = _largest_of(wa, COPY_KERNEL, "WRITE_SIZE")
    fscale, wscale = COPY_KIB / copy_fetch, COPY_KIB / copy_write
    fetch, n = _mean_of(fa, DOMINANT, "FETCH_SIZE")
    write, _ = _mean_of(wa, DOMINANT, "WRITE_SIZE")
    fetched, written = fetch * fscale * 1024.0, write * wscale * 1024.0
    print(f"calibration copy: FETCH_SIZE {copy_fetch:.1f} KiB (x {fscale:.3f}), WRITE_SIZE {copy_write:.1f} KiB (x {wscale:.3f})")
    print(f"{DOMINANT} ({n} dispatches): FETCH_SIZE {fetch:.1f} KiB -> {fetched / 1e6:.2f} MB fetched, "
          f"WRITE_SIZE {write:.1f} KiB -> {written / 1e6:.2f} MB written, {(fetched + written) / 1e6:.2f} MB per launch")
    lines = []
    if os.path.exists(out_file):
        lines = [l for l in open(out_file).read().splitlines()
                 if l.startswith("#") or l.split()[:2] != [workload, kv]]
    if not lines:
        lines = ["# HBM bytes per launch of the dominant kernel by the byte counters (FETCH_SIZE and WRITE_SIZE of two",
                 "# rocprofv3 --pmc runs, each scaled by the plain 1 GiB copy of the same run); written by",
                 "# python -m paper_2604_09731_amd.profile_summary traffic; read by bench.py",
                 "# workload kv kernel bytes_per_launch fetched_bytes written_bytes fetch_scale write_scale"]
    lines.append(f"{workload} {kv} {DOMINANT} {fetched + written:.0f} {fetched:.0f} {written:.0f} {fscale:.3f} {wscale:.3f}")
    with open(out_file, "w") as f:
        f.write("\n".join(lines) + "\n")


def main(argv):
    if len(argv) >= 3 and argv[1] == "stats":
        stats(argv[2])
    elif len(argv) >= 3 and argv[1] == "pmc":
        pmc(argv[2])
    elif len(argv) >= 6 and argv[1] == "traffic":
        here = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
        traffic(argv[2], argv[3], argv[4], argv[5], argv[6] if len(argv) > 6 else os.path.join(here, "profiles", "hbm_traffic.txt"))
    else:
        raise SystemExit(__doc__)


if __name__ == "__main__":
    main(sys.argv)

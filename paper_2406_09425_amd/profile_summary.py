"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

  python -m paper_2406_09425_amd.profile_summary stats <dir> <command...>
      per-kernel table from <dir>/**/*kernel_stats.csv
  python -m paper_2406_09425_amd.profile_summary pmc <fetch_dir> <write_dir> <command...>
      HBM traffic per dispatch from the FETCH_SIZE and WRITE_SIZE runs (KiB per
      dispatch), scaled by what the same counters read for the 256 MiB + 256 MiB
      calibration copy (bn_relu_kernel) in the same runs

The command line that produced the data is echoed into the summary.
"""
from __future__ import annotations

import collections
import csv
import glob
import os
import sys


def _find(d, pat):
    return sorted(glob.glob(os.path.join(d, "**", pat), recursive=True))


def stats(d: str, cmd: str) -> str:
    rows = []
    for f in _find(d, "*kernel_stats.csv"):
        rows += list(csv.DictReader(open(f)))
    out = [f"command: {cmd}", "", f"{'kernel':<92}{'calls':>7}{'avg us':>10}{'total ms':>10}{'%':>7}"]
    for r in rows:
        out.append(f"{r['Name'][:90]:<92}{r['Calls']:>7}{float(r['AverageNs']) / 1e3:>10.2f}"
                   f"{float(r['TotalDurationNs']) / 1e6:>10.3f}{float(r['Percentage']):>7.2f}")
    return "\n".join(out) + "\n"


def _per_kernel(d: str, counter: str):
    """Average counter value per dispatch, keyed by (kernel name, grid size): the
    same kernel launched at different sizes is reported as different rows."""
    tot, cnt = collections.defaultdict(float), collections.Counter()
    for f in _find(d, "*counter_collection.csv"):
        for r in csv.DictReader(open(f)):
            if r["Counter_Name"] == counter:
                key = (r["Kernel_Name"], int(r["Grid_Size"]))
                tot[key] += float(r["Counter_Value"])
                cnt[key] += 1
    return {k: (tot[k] / cnt[k], cnt[k]) for k in tot}


def pmc(fetch_dir: str, write_dir: str, cmd: str) -> str:
    fetch, write = _per_kernel(fetch_dir, "FETCH_SIZE"), _per_kernel(write_dir, "WRITE_SIZE")
    # the calibration copy is the bn_relu launch with the largest grid (256 MiB each way)
    calib = sorted((k for k in fetch if "bn_relu_kernel" in k[0]), key=lambda k: -k[1])
    known_kib = 256.0 * 1024.0
    ff = known_kib / fetch[calib[0]][0] if calib else 1.0
    wf = known_kib / write[calib[0]][0] if calib and calib[0] in write else 1.0
    sizes = collections.Counter(k[0] for k in fetch)
    out = [f"command: {cmd}", "",
           f"calibration copy: FETCH_SIZE reads {fetch[calib[0]][0]:.0f} KiB, WRITE_SIZE reads "
           f"{write[calib[0]][0]:.0f} KiB for 262144 KiB each way -> factors {ff:.4f} (fetch), {wf:.4f} (write)"
           if calib else "no calibration copy found: factors 1.0", "",
           f"{'kernel':<92}{'disp':>6}{'fetch MB':>12}{'write MB':>12}   (per dispatch, scaled)"]
    for k in sorted(fetch, key=lambda k: -fetch[k][0]):
        f_mb = fetch[k][0] * ff * 1024 / 1e6
        w_mb = write.get(k, (0.0, 0))[0] * wf * 1024 / 1e6
        name = k[0][:90] if sizes[k[0]] == 1 else f"{k[0][:70]} [grid {k[1]}]"
        out.append(f"{name:<92}{fetch[k][1]:>6}{f_mb:>12.2f}{w_mb:>12.2f}")
    return "\n".join(out) + "\n"


if __name__ == "__main__":
    if len(sys.argv) >= 4 and sys.argv[1] == "stats":
        sys.stdout.write(stats(sys.argv[2], " ".join(sys.argv[3:])))
    elif len(sys.argv) >= 5 and sys.argv[1] == "pmc":
        sys.stdout.write(pmc(sys.argv[2], sys.argv[3], " ".join(sys.argv[4:])))
    else:
        sys.exit(__doc__)

"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

  python -m paper_2406_09425_amd.profile_summary stats <dir> <command...>
      per-kernel table from <dir>/**/*kernel_stats.csv
  python -m paper_2406_09425_amd.profile_summary pmc <fetch_dir> <write_dir> <command...>
      HBM traffic per dispatch from the FETCH_SIZE and WRITE_SIZE runs (KiB per
      dispatch), scaled by what the same counters read for the 256 MiB + 256 MiB
      calibration copy (bn_relu_kernel) in the same runs

  python -m paper_2406_09425_amd.profile_summary sq <dir> [<dir> ...] -- <command...>
      SQ counters per dispatch of every sgprs kernel (one rocprofv3 --pmc run per
      directory, at most 8 SQ counters each), as fractions of the SIMD cycles of the
      dispatch where that makes sense

  python -m paper_2406_09425_amd.profile_summary concurrency <dir> <command...>
      from a --kernel-trace run (<dir>/**/*kernel_trace.csv): per hardware queue the number of
      kernels and their busy time, and how the traced interval divides by the number of kernels
      (and of distinct queues) in flight at once

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


def concurrency(d: str, cmd: str, skip_first_fraction: float = 0.3) -> str:
    """Who ran beside whom: the kernels of the last (1 - skip_first_fraction) of the trace (the
    steady state after warm-up) as intervals [start, end) per queue."""
    rows = []
    for f in _find(d, "*kernel_trace.csv"):
        for r in csv.DictReader(open(f)):
            if "sgprs" in r["Kernel_Name"]:
                rows.append((int(r["Start_Timestamp"]), int(r["End_Timestamp"]), r["Queue_Id"], r["Kernel_Name"]))
    if not rows:
        return f"command: {cmd}\n\nno sgprs kernels in the trace\n"
    rows.sort()
    t_lo = rows[0][0] + int((rows[-1][1] - rows[0][0]) * skip_first_fraction)
    rows = [r for r in rows if r[0] >= t_lo]
    span = max(r[1] for r in rows) - min(r[0] for r in rows)
    per_q = collections.defaultdict(lambda: [0, 0])
    events = []
    for st, en, q, _ in rows:
        per_q[q][0] += 1
        per_q[q][1] += en - st
        events.append((st, 1, q))
        events.append((en, -1, q))
    events.sort(key=lambda e: (e[0], e[1]))
    in_flight, q_active = 0, collections.Counter()
    by_kernels, by_queues = collections.Counter(), collections.Counter()
    prev = events[0][0]
    for t, dlt, q in events:
        by_kernels[in_flight] += t - prev
        by_queues[sum(1 for v in q_active.values() if v > 0)] += t - prev
        prev = t
        in_flight += dlt
        q_active[q] += dlt
    out = [f"command: {cmd}", "",
           f"{len(rows)} sgprs kernels in the last {100 * (1 - skip_first_fraction):.0f} % of the trace, {span / 1e3:.1f} us, "
           f"sum of kernel durations {sum(r[1] - r[0] for r in rows) / 1e3:.1f} us, "
           f"median kernel {sorted(r[1] - r[0] for r in rows)[len(rows) // 2] / 1e3:.2f} us", "",
           f"{'queue id':<12}{'kernels':>9}{'busy us':>12}{'busy share of the interval':>30}"]
    for q in sorted(per_q, key=lambda q: int(q) if q.isdigit() else 0):
        out.append(f"{q:<12}{per_q[q][0]:>9}{per_q[q][1] / 1e3:>12.1f}{per_q[q][1] / span:>30.3f}")
    out += ["", f"{'kernels in flight':<20}{'share of the interval':>24}"]
    for k in sorted(by_kernels):
        out.append(f"{k:<20}{by_kernels[k] / span:>24.3f}")
    out += ["", f"{'queues with a kernel in flight':<34}{'share of the interval':>24}"]
    for k in sorted(by_queues):
        out.append(f"{k:<34}{by_queues[k] / span:>24.3f}")
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


def sq(dirs, cmd: str) -> str:
    """Shares of a dispatch's SIMD cycles.  SQ_BUSY_CYCLES counts per shader engine (32 on this
    part, 4 per die), the *_CYCLES / ACTIVE_INST / WAIT counters count in units of 4 cycles per
    SIMD, SQ_VALU_MFMA_BUSY_CYCLES in cycles per SIMD."""
    vals = collections.defaultdict(dict)
    disp = collections.Counter()
    for d in dirs:
        names = set()
        for f in _find(d, "*counter_collection.csv"):
            for r in csv.DictReader(open(f)):
                if "sgprs::" not in r["Kernel_Name"]:
                    continue
                k = r["Kernel_Name"]
                vals[k][r["Counter_Name"]] = vals[k].get(r["Counter_Name"], 0.0) + float(r["Counter_Value"])
                names.add(r["Counter_Name"])
                disp[(k, r["Counter_Name"])] += 1
    out = [f"command: {cmd}", "one run per group of at most 8 SQ counters; values are per dispatch", "",
           f"{'kernel':<62}{'cycles':>8}{'waves':>7}{'MFMA busy':>10}{'VALU':>7}{'scalar':>7}{'LDS':>6}{'VMEM':>6}"
           f"{'any inst':>9}{'waiting':>8}{'VALU/wave':>10}{'SALU/wave':>10}{'LDS/wave':>9}{'bank confl.':>12}"]
    for k, v in sorted(vals.items(), key=lambda kv: -kv[1].get("SQ_BUSY_CYCLES", 0) / max(1, disp[(kv[0], "SQ_BUSY_CYCLES")])):
        g = lambda n: v.get(n, 0.0) / max(1, disp[(k, n)])
        cycles = g("SQ_BUSY_CYCLES") / 32.0
        simd = cycles * 1024.0
        if simd <= 0:
            continue
        waves = max(1.0, g("SQ_WAVES"))
        pct = lambda x: f"{100.0 * x / simd:.1f}%"
        lds_active = g("SQ_ACTIVE_INST_LDS") * 4
        out.append(f"{k.replace('void sgprs::', '')[:60]:<62}{cycles:>8.0f}{waves:>7.0f}{pct(g('SQ_VALU_MFMA_BUSY_CYCLES')):>10}"
                   f"{pct(g('SQ_ACTIVE_INST_VALU') * 4):>7}{pct(g('SQ_ACTIVE_INST_SCA') * 4):>7}{pct(lds_active):>6}"
                   f"{pct(g('SQ_ACTIVE_INST_VMEM') * 4):>6}{pct(g('SQ_ACTIVE_INST_ANY') * 4):>9}{pct(g('SQ_WAIT_INST_ANY') * 4):>8}"
                   f"{g('SQ_INSTS_VALU') / waves:>10.0f}{g('SQ_INSTS_SALU') / waves:>10.0f}{g('SQ_INSTS_LDS') / waves:>9.0f}"
                   f"{(100.0 * g('SQ_LDS_BANK_CONFLICT') / max(1.0, g('SQ_LDS_IDX_ACTIVE'))):>11.1f}%")
    out += ["", "MFMA busy: SQ_VALU_MFMA_BUSY_CYCLES / (SQ_BUSY_CYCLES / 32 * 1024 SIMDs).  VALU, scalar, LDS, VMEM, any inst:",
            "SQ_ACTIVE_INST_* * 4 over the same SIMD cycles (issue activity; VALU includes the MFMA issue slots).  waiting:",
            "SQ_WAIT_INST_ANY * 4 over the same (wave-cycles spent waiting, summed over the resident waves, so it can exceed",
            "100 %).  bank confl.: SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE."]
    return "\n".join(out) + "\n"


if __name__ == "__main__":
    if len(sys.argv) >= 4 and sys.argv[1] == "concurrency":
        sys.stdout.write(concurrency(sys.argv[2], " ".join(sys.argv[3:])))
    elif len(sys.argv) >= 4 and sys.argv[1] == "stats":
        sys.stdout.write(stats(sys.argv[2], " ".join(sys.argv[3:])))
    elif len(sys.argv) >= 5 and sys.argv[1] == "pmc":
        sys.stdout.write(pmc(sys.argv[2], sys.argv[3], " ".join(sys.argv[4:])))
    elif len(sys.argv) >= 5 and sys.argv[1] == "sq" and "--" in sys.argv:
        i = sys.argv.index("--")
        sys.stdout.write(sq(sys.argv[2:i], " ".join(sys.argv[i + 1:])))
    else:
        sys.exit(__doc__)

"""Turns a rocprofv3 CSV output directory into the few lines worth keeping.

    python -m paper_2409_19256_amd.rocprof_summary <dir> [--calib-bytes N]

* kernel trace (`rocprofv3 --kernel-trace --stats --output-format csv`): calls, average,
  min and max duration per kernel and grid size, from the per-dispatch trace (launches of
  one kernel over different work lists, e.g. the SKIP_OWN and the COPY_OWN transition of
  one process, have different grids and are listed apart).
* counters (`rocprofv3 --pmc FETCH_SIZE` or `WRITE_SIZE`, one counter per run): average
  counter value per dispatch of every kernel.  With --calib-bytes N the dispatch of the
  library's `calib_copy` kernel (known to read N and write N bytes) gives the factor that
  turns counter units into bytes, and every kernel's HBM bytes per dispatch are printed.
"""
from __future__ import annotations

import collections
import csv
import glob
import os
import sys


def _find(d, pattern):
    hits = sorted(glob.glob(os.path.join(d, "**", pattern), recursive=True))
    return hits[0] if hits else None


def summarise(d: str, calib_bytes: int = 0) -> str:
    out = []
    trace = _find(d, "*kernel_trace.csv")
    if trace:
        dur = collections.defaultdict(list)
        for r in csv.DictReader(open(trace)):
            grid = "x".join(str(r[c]) for c in sorted(r) if c.startswith("Grid_Size")) or "?"
            dur[(r["Kernel_Name"], grid)].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e6)
        out.append(f"# kernel trace: {os.path.basename(trace)}")
        out.append(f"{'kernel':72s} {'grid (threads)':>18s} {'calls':>6s} {'avg ms':>10s} {'min ms':>10s} {'max ms':>10s} {'total ms':>10s}")
        for (k, g), v in sorted(dur.items(), key=lambda kv: -sum(kv[1]))[:14]:
            out.append(f"{k[:72]:72s} {g:>18s} {len(v):6d} {sum(v)/len(v):10.4f} {min(v):10.4f} {max(v):10.4f} {sum(v):10.3f}")
    ctr = _find(d, "*counter_collection.csv")
    if ctr:
        val = collections.defaultdict(list)
        for r in csv.DictReader(open(ctr)):
            val[(r["Kernel_Name"], r["Counter_Name"])].append(float(r["Counter_Value"]))
        out.append(f"# counters: {os.path.basename(ctr)}")
        factor = {}
        if calib_bytes:
            for (k, c), v in val.items():
                if "calib_copy" in k and sum(v) > 0:   # a counter that reads 0 for the copy (a stall counter) has no byte scale
                    factor[c] = calib_bytes / (sum(v) / len(v))
                    out.append(f"calibration: calib_copy moved {calib_bytes} bytes each way and read {c} = {sum(v)/len(v):.1f} "
                               f"-> {factor[c]:.2f} bytes per counter unit")
        out.append(f"{'kernel':72s} {'counter':12s} {'calls':>6s} {'avg per dispatch':>18s} {'HBM bytes per dispatch':>24s}")
        for (k, c), v in sorted(val.items(), key=lambda kv: -sum(kv[1]))[:16]:
            avg = sum(v) / len(v)
            b = f"{avg * factor[c]:24.0f}" if c in factor else f"{'':24s}"
            out.append(f"{k[:72]:72s} {c:12s} {len(v):6d} {avg:18.1f} {b}")
    if not out:
        out.append(f"no rocprofv3 CSV output under {d}")
    return "\n".join(out)


if __name__ == "__main__":
    args = sys.argv[1:]
    calib = 0
    if "--calib-bytes" in args:
        i = args.index("--calib-bytes")
        calib = int(args[i + 1])
        del args[i:i + 2]
    print(summarise(args[0], calib))

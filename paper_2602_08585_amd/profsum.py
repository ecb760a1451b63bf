"""Short text summaries of rocprofv3 output for runs of bench.py (the figures kept under profiles/).

    python -m paper_2602_08585_amd.profsum trace   <dir of a --kernel-trace --stats run>
    python -m paper_2602_08585_amd.profsum traffic <dir of a --pmc FETCH_SIZE run> <dir of a --pmc WRITE_SIZE run> [out.json]

`trace` prints calls / average / min / max duration of every kernel of the library and the mean
gap between consecutive kernels.  `traffic` prints HBM bytes per launch of every kernel: the two
counters are KiB per dispatch, averaged over a kernel's dispatches and scaled by what the same
counter reads for the library's plain copy kernel, whose size is known (bench.py runs it over
64 MiB: 64 MiB read, 64 MiB written); with a third argument the figures are also written as JSON,
the file bench.py reads for `roofline.traffic`.
"""
from __future__ import annotations

import collections
import csv
import glob
import json
import os
import sys

COPY_BYTES = 64 << 20       # bench.py's CEILING_BYTES
SHORT = {"score_stats_kernel": "score_stats", "score_accum_kernel": "score_accum", "sel_hist_kernel": "sel_hist",
         "sel_tail_kernel": "sel_tail", "sel_emit_kernel": "sel_emit", "sel_head_kernel": "sel_head",
         "sel_gather_kernel": "sel_gather"}


def _one(d: str, pattern: str) -> str:
    hits = glob.glob(os.path.join(d, "**", pattern), recursive=True)
    if not hits:
        raise SystemExit("no %s under %s" % (pattern, d))
    return hits[0]


def _short(name: str) -> str:
    return name.split("(")[0].replace("void ", "").replace("lukv::", "").split("<")[0]


def trace(d: str) -> None:
    rows = [r for r in csv.DictReader(open(_one(d, "*_kernel_stats.csv"))) if "lukv::" in r["Name"]]
    print("%-28s %6s %10s %10s %10s" % ("kernel", "calls", "avg_us", "min_us", "max_us"))
    for r in rows:
        print("%-28s %6s %10.2f %10.2f %10.2f" % (_short(r["Name"])[:28], r["Calls"], float(r["AverageNs"]) / 1e3,
                                                  float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3))
    tr = [r for r in csv.DictReader(open(_one(d, "*_kernel_trace.csv"))) if "lukv::" in r["Kernel_Name"]]
    tr.sort(key=lambda r: int(r["Start_Timestamp"]))
    gaps = [(int(b["Start_Timestamp"]) - int(a["End_Timestamp"])) / 1e3 for a, b in zip(tr[:-1], tr[1:])]
    gaps = [g for g in gaps if 0 <= g < 100]
    if gaps:
        print("gap between consecutive kernels under the profiler: mean %.2f us over %d gaps"
              % (sum(gaps) / len(gaps), len(gaps)))


def _counter(d: str, counter: str):
    agg = collections.defaultdict(list)
    for r in csv.DictReader(open(_one(d, "*counter_collection.csv"))):
        if r["Counter_Name"] == counter and "lukv::" in r["Kernel_Name"]:
            agg[_short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return agg


def traffic(fetch_dir: str, write_dir: str, out_json: str | None) -> None:
    F, W = _counter(fetch_dir, "FETCH_SIZE"), _counter(write_dir, "WRITE_SIZE")
    if "copy_kernel" not in F or "copy_kernel" not in W:
        raise SystemExit("the runs hold no dispatch of the copy kernel (bench.py launches it)")
    med = lambda v: sorted(v)[len(v) // 2]
    cf, cw = med(F["copy_kernel"]) * 1024, med(W["copy_kernel"]) * 1024
    sf, sw = COPY_BYTES / cf, COPY_BYTES / cw
    print("copy kernel over %d MiB: FETCH_SIZE reads %.1f MiB -> factor %.4f ; WRITE_SIZE reads %.1f MiB -> factor %.4f"
          % (COPY_BYTES >> 20, cf / 2**20, sf, cw / 2**20, sw))
    out = {}
    for k in sorted(F):
        f = sum(F[k]) / len(F[k]) * 1024 * sf
        wv = W.get(k, [0.0])
        wb = sum(wv) / len(wv) * 1024 * sw
        print("%-22s dispatches %4d  fetch %11.0f B  write %11.0f B" % (k, len(F[k]), f, wb))
        out[SHORT.get(k, k)] = {"fetch_bytes": int(round(f)), "write_bytes": int(round(wb)),
                                "fetch_scale": round(sf, 4), "write_scale": round(sw, 4)}
    if out_json:
        json.dump(out, open(out_json, "w"), indent=1, sort_keys=True)


def main(argv) -> int:
    if len(argv) >= 2 and argv[0] == "trace":
        trace(argv[1])
        return 0
    if len(argv) >= 3 and argv[0] == "traffic":
        traffic(argv[1], argv[2], argv[3] if len(argv) > 3 else None)
        return 0
    sys.stderr.write(__doc__)
    return 2


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))

"""Turn two rocprofv3 --pmc counter files (FETCH_SIZE, WRITE_SIZE) of a bench.py run made with
--copy-calibration into HBM traffic per launch of the library's kernels.

The calibration kernel (y = x * 1 over 2^28 floats) reads 1 GiB and writes 1 GiB; each counter is
scaled by (1 GiB in KiB) / (what the counter reads for that kernel).

usage: python -m paper_2404_08698_amd.pmc_summary FETCH.csv WRITE.csv [out.json]
"""
from __future__ import annotations

import collections
import csv
import json
import sys

GIB_KIB = float(1 << 20)


def _load(path: str, counter: str):
    per = collections.defaultdict(list)
    cal = []
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        name = r["Kernel_Name"]
        val = float(r["Counter_Value"])
        if "MulFunctor<float>" in name and r["Grid_Size"] == str(1 << 26):
            cal.append(val)
        elif "anpd::" in name:
            per[name.replace("void ", "").split("(")[0]].append(val)
    if not cal:
        raise SystemExit("no calibration kernel in %s (run bench.py with --copy-calibration)" % path)
    factor = GIB_KIB / (sum(cal) / len(cal))
    return {k: (sum(v) / len(v) * factor * 1024.0, len(v)) for k, v in per.items()}, factor


def main(argv):
    fetch, f_factor = _load(argv[1], "FETCH_SIZE")
    write, w_factor = _load(argv[2], "WRITE_SIZE")
    out = {"fetch_scale": f_factor, "write_scale": w_factor, "kernels": {}}
    print("scale factors: FETCH_SIZE x %.4f, WRITE_SIZE x %.4f" % (f_factor, w_factor))
    print("%-40s %8s %16s %16s" % ("kernel", "calls", "read MB/launch", "written MB/launch"))
    for k in sorted(fetch, key=lambda k_: -fetch[k_][0]):
        rd, n = fetch[k]
        wr = write.get(k, (0.0, 0))[0]
        out["kernels"][k] = {"calls": n, "read_bytes": rd, "written_bytes": wr}
        print("%-40s %8d %16.3f %16.3f" % (k, n, rd / 1e6, wr / 1e6))
    if len(argv) > 3:
        json.dump(out, open(argv[3], "w"), indent=1)


if __name__ == "__main__":
    main(sys.argv)

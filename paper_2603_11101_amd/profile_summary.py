"""Condense rocprofv3 output into the short text summaries kept under profiles/.

    python -m paper_2603_11101_amd.profile_summary stats  <results.db>
    python -m paper_2603_11101_amd.profile_summary hbm    <fetch_dir> <write_dir> [<out.json>]

`stats` reads the rocpd database of a `--kernel-trace --stats` run and prints calls and average /
minimum / maximum duration per kernel.  `hbm` reads the counter CSVs of two `--pmc` runs of
`bench.py --copy-calibration` (FETCH_SIZE in one, WRITE_SIZE in the other, KiB per dispatch), scales
each counter by what it reads for the 256 MiB device-to-device copy, and prints HBM bytes per launch
of every attention kernel; with <out.json> it also writes {kernel: bytes per launch}, the file
bench.py reports as `roofline.traffic`.
"""
import collections
import csv
import glob
import json
import re
import sqlite3
import sys

COPY_BYTES = 256 << 20
SHORT = {"fwd_bf16_kernel": "fwd_bf16", "bwd_delta_kernel": "bwd_delta", "bwd_dkdv_kernel": "bwd_dkdv",
         "bwd_dq_kernel": "bwd_dq", "fwd_fp8_kernel": "fwd_fp8", "copyBuffer": "copy"}


def short_name(name):
    if re.search(r"fwd_fp8_kernel<\d+, true", name):  # second template argument: block-wise scales
        return "fwd_fp8_blockwise"
    if "quant_blockwise" in name:
        return "quant_blockwise"
    for key, val in SHORT.items():
        if key in name:
            return val
    return None


def stats(db):
    con = sqlite3.connect(db)
    rows = con.execute("select name, count(*), avg(end-start), min(end-start), max(end-start), sum(end-start) "
                       "from kernels group by name order by sum(end-start) desc").fetchall()
    total = sum(r[5] for r in rows)
    print(f"{'kernel':60s} {'calls':>6s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'total_ms':>9s} {'pct':>6s}")
    for name, calls, avg, mn, mx, sm in rows:
        name = re.sub(r"va::\(anonymous namespace\)::|\(va::AttnParams\)|void ", "", name)
        print(f"{name[:60]:60s} {calls:6d} {avg / 1e3:9.2f} {mn / 1e3:9.2f} {mx / 1e3:9.2f} {sm / 1e6:9.3f} "
              f"{100 * sm / total:6.1f}")


def counter_means(directory, counter):
    path = glob.glob(directory + "/**/*counter_collection.csv", recursive=True)[0]
    acc = collections.defaultdict(list)
    for row in csv.DictReader(open(path)):
        name = short_name(row["Kernel_Name"])
        if name and row["Counter_Name"] == counter:
            acc[name].append(float(row["Counter_Value"]))
    # small staging copies run through the same copy kernel: keep the calibration copies only
    if "copy" in acc:
        acc["copy"] = [x for x in acc["copy"] if x >= 0.5 * max(acc["copy"])]
    return {k: (sum(v) / len(v), len(v)) for k, v in acc.items()}


def hbm(fetch_dir, write_dir, out=None):
    fetch = counter_means(fetch_dir, "FETCH_SIZE")
    write = counter_means(write_dir, "WRITE_SIZE")
    f_scale = COPY_BYTES / (fetch["copy"][0] * 1024.0)
    w_scale = COPY_BYTES / (write["copy"][0] * 1024.0)
    print(f"copy of {COPY_BYTES} bytes: FETCH_SIZE {fetch['copy'][0]:.1f} KiB, WRITE_SIZE {write['copy'][0]:.1f} KiB "
          f"-> scale factors {f_scale:.4f} (fetch), {w_scale:.4f} (write)")
    result = {}
    print(f"{'kernel':12s} {'launches':>8s} {'fetch_MB':>10s} {'write_MB':>10s} {'total_MB':>10s}")
    for k in sorted(fetch):
        if k == "copy":
            continue
        fb = fetch[k][0] * 1024.0 * f_scale
        wb = write.get(k, (0.0, 0))[0] * 1024.0 * w_scale
        result[k] = fb + wb
        print(f"{k:12s} {fetch[k][1]:8d} {fb / 1e6:10.2f} {wb / 1e6:10.2f} {(fb + wb) / 1e6:10.2f}")
    if out:
        with open(out, "w") as f:
            json.dump(result, f, indent=1)
            f.write("\n")


if __name__ == "__main__":
    if len(sys.argv) >= 3 and sys.argv[1] == "stats":
        stats(sys.argv[2])
    elif len(sys.argv) >= 4 and sys.argv[1] == "hbm":
        hbm(sys.argv[2], sys.argv[3], sys.argv[4] if len(sys.argv) > 4 else None)
    else:
        print(__doc__)
        sys.exit(2)

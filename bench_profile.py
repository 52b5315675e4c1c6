#!/usr/bin/env python3
"""Condense rocprofv3 output of `bench.py --profile-leg` runs into the short summaries kept under profiles/.

    python bench_profile.py stats <results.db> [--last <steps>]
    python bench_profile.py hbm   <fetch_dir> <write_dir> [<out.json>]
    python bench_profile.py pmc   <pmc_dir> [<pmc_dir> ...] [--json <out.json>]

`stats` reads the rocpd database of a `--kernel-trace --stats` run and prints calls and average /
minimum / maximum duration per kernel.  `hbm` reads the counter CSVs of two `--pmc` runs of
`bench.py --profile-leg --copy-calibration` (FETCH_SIZE in one, WRITE_SIZE in the other, KiB per dispatch),
scales each counter by what it reads for the 256 MiB device-to-device copy, and prints HBM bytes per launch
of every attention kernel; with <out.json> it also writes {kernel: bytes per launch}, the file bench.py
reports as `roofline.traffic`.  `pmc` reads the CSVs of one or more `--pmc` runs with shader counters and
prints, per kernel, the mean of every counter per dispatch and the derived figures: matrix-unit busy
fraction (SQ_VALU_MFMA_BUSY_CYCLES / (4 SIMDs x SQ_BUSY_CU_CYCLES), i.e. of the cycles a CU was busy), MFMA
FLOPs issued (SQ_INSTS_VALU_MFMA_MOPS_* x 512) and the shader clock the counters imply where a trace
duration is known.  JSON outputs carry the digest of the sources they were measured with.
"""
import collections
import csv
import glob
import json
import re
import sqlite3
import sys

from bench import source_digest

COPY_BYTES = 256 << 20
SHORT = {"fwd_bf16_kernel": "fwd_bf16", "bwd_delta_kernel": "bwd_delta", "bwd_dkdv_kernel": "bwd_dkdv",
         "bwd_dkdv_reduce_kernel": "bwd_dkdv_reduce", "bwd_dq_kernel": "bwd_dq", "fwd_fp8_kernel": "fwd_fp8",
         "copyBuffer": "copy"}


def short_name(name):
    if re.search(r"fwd_fp8_kernel<\d+, true", name):  # second template argument: block-wise scales
        return "fwd_fp8_blockwise"
    if "quant_blockwise" in name:
        return "quant_blockwise"
    if "bwd_dkdv_reduce" in name:
        return "bwd_dkdv_reduce"
    for key, val in SHORT.items():
        if key in name:
            return val
    return None


def stats(db, last=0):
    """Per kernel: calls, average / min / max duration and share of the total; with `last` > 0 also the average
    over the last `last` launches of the kernel (the timed steps of the profiled program, which come after its
    clock ramp and warm-up steps: the figure to hold against the program's own milliseconds per step)."""
    con = sqlite3.connect(db)
    rows = con.execute("select name, count(*), avg(end-start), min(end-start), max(end-start), sum(end-start) "
                       "from kernels group by name order by sum(end-start) desc").fetchall()
    total = sum(r[5] for r in rows)
    tail = f" {'last' + str(last) + '_avg_us':>14s}" if last else ""
    print(f"{'kernel':60s} {'calls':>6s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'total_ms':>9s} {'pct':>6s}{tail}")
    for name, calls, avg, mn, mx, sm in rows:
        extra = ""
        if last:
            d = [r[0] for r in con.execute("select end-start from kernels where name = ? order by start desc limit ?",
                                           (name, last))]
            extra = f" {sum(d) / len(d) / 1e3:14.2f}"
        name = re.sub(r"va::\(anonymous namespace\)::|\(va::AttnParams\)|void ", "", name)
        print(f"{name[:60]:60s} {calls:6d} {avg / 1e3:9.2f} {mn / 1e3:9.2f} {mx / 1e3:9.2f} {sm / 1e6:9.3f} "
              f"{100 * sm / total:6.1f}{extra}")


def counter_rows(directory):
    path = glob.glob(directory + "/**/*counter_collection.csv", recursive=True)[0]
    return csv.DictReader(open(path))


def counter_means(directory, counter):
    acc = collections.defaultdict(list)
    for row in counter_rows(directory):
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
    print(f"{'kernel':18s} {'launches':>8s} {'fetch_MB':>10s} {'write_MB':>10s} {'total_MB':>10s}")
    for k in sorted(fetch):
        if k == "copy":
            continue
        fb = fetch[k][0] * 1024.0 * f_scale
        wb = write.get(k, (0.0, 0))[0] * 1024.0 * w_scale
        result[k] = fb + wb
        print(f"{k:18s} {fetch[k][1]:8d} {fb / 1e6:10.2f} {wb / 1e6:10.2f} {(fb + wb) / 1e6:10.2f}")
    if out:
        result["source_digest"] = source_digest()
        with open(out, "w") as f:
            json.dump(result, f, indent=1)
            f.write("\n")


def pmc(dirs, out=None):
    # counter -> kernel -> per-dispatch values; a dispatch reports one row per counter (and per dimension
    # instance for some counters: those are summed per dispatch first)
    per = collections.defaultdict(lambda: collections.defaultdict(lambda: collections.defaultdict(float)))
    for d in dirs:
        for row in counter_rows(d):
            name = short_name(row["Kernel_Name"])
            if name and name != "copy":
                per[row["Counter_Name"]][name][(d, row["Dispatch_Id"])] += float(row["Counter_Value"])
    kernels = sorted({k for c in per for k in per[c]})
    means = {k: {c: sum(per[c][k].values()) / len(per[c][k]) for c in per if k in per[c]} for k in kernels}
    result = {}
    for k in kernels:
        m = means[k]
        print(f"{k}: {max(len(per[c][k]) for c in per if k in per[c])} dispatches")
        for c in sorted(m):
            print(f"    {c:36s} {m[c]:18.1f}")
        derived = {}
        if "SQ_VALU_MFMA_BUSY_CYCLES" in m and "SQ_BUSY_CU_CYCLES" in m and m["SQ_BUSY_CU_CYCLES"] > 0:
            derived["mfma_busy_of_cu_busy"] = m["SQ_VALU_MFMA_BUSY_CYCLES"] / (4.0 * m["SQ_BUSY_CU_CYCLES"])
        if "SQ_VALU_MFMA_BUSY_CYCLES" in m and "GRBM_GUI_ACTIVE" in m and m["GRBM_GUI_ACTIVE"] > 0:
            # the "MfmaUtil" expression of the tool: busy cycles summed over the SIMDs / (kernel cycles x SIMDs)
            derived["mfma_busy_of_kernel_cycles"] = m["SQ_VALU_MFMA_BUSY_CYCLES"] / (m["GRBM_GUI_ACTIVE"] * 1024.0)
        mops = sum(m.get(c, 0.0) for c in ("SQ_INSTS_VALU_MFMA_MOPS_BF16", "SQ_INSTS_VALU_MFMA_MOPS_F8",
                                           "SQ_INSTS_VALU_MFMA_MOPS_F16", "SQ_INSTS_VALU_MFMA_MOPS_F32"))
        if mops > 0:
            derived["mfma_flops_issued"] = mops * 512.0
        if "SQ_ACTIVE_INST_VALU" in m and "SQ_BUSY_CU_CYCLES" in m and m["SQ_BUSY_CU_CYCLES"] > 0:
            derived["valu_active_of_cu_busy"] = m["SQ_ACTIVE_INST_VALU"] / (4.0 * m["SQ_BUSY_CU_CYCLES"])
        for n, v in derived.items():
            print(f"    -> {n:33s} {v:18.4g}")
        result[k] = {"counters": m, **derived}
    if out:
        result["source_digest"] = source_digest()
        with open(out, "w") as f:
            json.dump(result, f, indent=1)
            f.write("\n")


if __name__ == "__main__":
    if len(sys.argv) >= 3 and sys.argv[1] == "stats":
        stats(sys.argv[2], int(sys.argv[4]) if len(sys.argv) >= 5 and sys.argv[3] == "--last" else 0)
    elif len(sys.argv) >= 4 and sys.argv[1] == "hbm":
        hbm(sys.argv[2], sys.argv[3], sys.argv[4] if len(sys.argv) > 4 else None)
    elif len(sys.argv) >= 3 and sys.argv[1] == "pmc":
        rest = sys.argv[2:]
        out = None
        if "--json" in rest:
            i = rest.index("--json")
            out = rest[i + 1]
            rest = rest[:i] + rest[i + 2:]
        pmc(rest, out)
    else:
        print(__doc__)
        sys.exit(2)

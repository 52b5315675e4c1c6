"""Writes tests/golden/workload_bins.json: for each synthetic workload, the
first bin produced by the ORACLE's first-fit on the seeded length pool (sample
count, token count, longest sample, allowed (query, key) pairs per head).

Calls only ``oracle/`` and the seeded length generator; the GPU path is never
involved.  The paper prints no packing example, so these are regression values
for the generator + oracle pair, not values from the paper.

Run from the repository root:  python tests/golden/make_workload_bins.py
"""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import packing as op                       # noqa: E402
from paper_2603_11101_amd import workloads as wl       # noqa: E402


def main():
    out = {}
    for name, w in wl.WORKLOADS.items():
        lens, prefix = wl.sample_lengths(name)
        bin_of, pos, nb = op.first_fit(lens, w.budget)
        idx = op.bin_members(bin_of, pos, 0)
        L = [int(lens[i]) for i in idx]
        mode = op.MASK_THREE_BLOCK if w.three_block else op.MASK_PREFIX_BIDIR_SUFFIX if w.prefix_lm else op.MASK_CAUSAL
        if w.three_block:
            pairs = sum(op.allowed_pairs(int(lens[i]), int(prefix[i][0]), mode, int(prefix[i][1])) for i in idx)
        elif w.prefix_lm:
            pairs = sum(int(prefix[i]) ** 2 + (int(lens[i]) - int(prefix[i])) * int(lens[i]) for i in idx)
        else:
            pairs = sum(l * (l + 1) // 2 for l in L)
        out[name] = {"num_bins": int(nb), "bin0_samples": len(L), "bin0_tokens": sum(L), "bin0_max_len": max(L),
                     "bin0_pairs_per_head": int(pairs), "bin0_first_sample_ids": [int(i) for i in idx[:8]],
                     "mask_mode": mode}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "workload_bins.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1, sort_keys=True)
        f.write("\n")
    print(json.dumps(out, indent=1, sort_keys=True))


if __name__ == "__main__":
    main()

"""Packed variable-length attention against the padded fixed-length layout, on one MI355X.

    python -m paper_2603_11101_amd.padding_sweep [--quick]

The paper's only attention micro-benchmark (section 3.2.1, "varlen vs fixlen") sweeps batch size,
sequence length and padding rate on Qwen2.5-VL shapes and reports the time the variable-length
interface saves and the TFLOP/s of both.  This script repeats the sweep with this library: the same
kernels run once on the packed stream of the true lengths and once on a stream in which every
sample is padded to the maximum length (what a fixed-length batch computes), causal mask, 16 query /
8 KV heads, head_dim 128, forward + backward.  Lengths are seeded: B samples, uniform around
(1 - padding rate) * S, clipped to [16, S], one sample forced to S so that S is the batch maximum.
Prints one row per configuration.
"""
import argparse
import sys

import numpy as np
import torch

from . import binding as va

HQ, HKV, D = 16, 8, 128


def lengths(batch, seq, pad_rate, rng):
    mean = (1.0 - pad_rate) * seq
    half = min(mean - 16, seq - mean, 0.5 * mean)
    lens = rng.integers(int(mean - half), int(mean + half) + 1, size=batch).astype(np.int64)
    lens = np.clip(lens, 16, seq)
    lens[0] = seq
    return lens


def time_stream(lens, steps, dev):
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    T = int(cu[-1])
    ps = va.PackedStream(cu, None, va.VA_MASK_CAUSAL, HQ, HKV, D, device=dev)
    g = torch.Generator(device=dev)
    g.manual_seed(T)
    q = torch.randn((T, HQ, D), device=dev, generator=g).to(torch.bfloat16)
    k = torch.randn((T, HKV, D), device=dev, generator=g).to(torch.bfloat16)
    v = torch.randn((T, HKV, D), device=dev, generator=g).to(torch.bfloat16)
    do = torch.randn((T, HQ, D), device=dev, generator=g).to(torch.bfloat16)
    out, dq = torch.empty_like(q), torch.empty_like(q)
    dk, dv = torch.empty_like(k), torch.empty_like(v)
    lse = torch.empty((HQ, T), dtype=torch.float32, device=dev)
    scale = 1.0 / float(np.sqrt(D))

    def step():
        ps.fwd(q, k, v, scale, out, lse)
        ps.bwd(q, k, v, out, lse, do, scale, dq, dk, dv)

    step()
    step()
    best = float("inf")
    for _ in range(3):  # best of three short runs: one slow run (clock ramp, allocator) must not decide a row
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            step()
        e1.record()
        e1.synchronize()
        best = min(best, e0.elapsed_time(e1) / steps)
    return best


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--quick", action="store_true", help="a 2 x 2 x 3 corner of the sweep")
    args = ap.parse_args()
    if not torch.cuda.is_available():
        print("padding_sweep: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    batches = (8, 32) if args.quick else (8, 16, 32)
    seqs = (1024, 8192) if args.quick else (1024, 2048, 4096, 8192)
    rates = (0.03, 0.5, 0.9) if args.quick else (0.03, 0.25, 0.5, 0.75, 0.9)
    rng = np.random.default_rng(7)
    print(f"{'batch':>5s} {'seq':>6s} {'target':>7s} {'padding':>8s} {'packed_ms':>10s} {'padded_ms':>10s} "
          f"{'saved':>7s} {'packed_TF':>10s} {'padded_TF':>10s}")
    for b in batches:
        for s in seqs:
            padded = np.full(b, s, dtype=np.int64)
            steps = max(2, min(10, int(1e9 / (b * s * s))))
            t_padded = time_stream(padded, steps, dev)
            flops_padded = 14.0 * D * HQ * float((padded * (padded + 1) // 2).sum())
            for r in rates:
                lens = lengths(b, s, r, rng)
                pad = 1.0 - lens.sum() / float(b * s)
                t_packed = time_stream(lens, steps, dev)
                flops = 14.0 * D * HQ * float((lens * (lens + 1) // 2).sum())
                # the padded batch is credited with the useful pairs only
                print(f"{b:5d} {s:6d} {r:7.2f} {pad:8.3f} {t_packed:10.3f} {t_padded:10.3f} "
                      f"{1.0 - t_packed / t_padded:7.1%} {flops / t_packed / 1e9:10.0f} {flops / t_padded / 1e9:10.0f}",
                      flush=True)
    print(f"# padded batch at full credit: last configuration {flops_padded / t_padded / 1e9:.0f} TFLOP/s")


if __name__ == "__main__":
    main()

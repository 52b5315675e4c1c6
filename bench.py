#!/usr/bin/env python3
"""Benchmark of the packed variable-length attention hot path on one MI355X.

One step = forward + backward (dQ and dK/dV kernels, and a delta pass where the dQ kernel does not
compute delta itself) of one packed batch:
the first first-fit bin of the `vlm` workload (causal VLM-backbone layer,
16 query / 8 KV heads, head_dim 128, 16384-token budget), synthetic N(0,1)
bf16 inputs resident in HBM before the timed region.  Buffers rotate over
several independent sets so the inputs of a step are not cache-resident from
the step before.

Prints ONE JSON line: the metric (useful TFLOP/s: 14 * D * Hq * allowed (q, k)
pairs per step), tokens/s, a roofline object for the dominant kernel (measured
live with HIP events on the launch stream) and the CPU oracle's throughput on a
bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0
PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
WORKLOAD = "vlm"
NUM_BUFFER_SETS = 4
COPY_CALIBRATION_BYTES = 256 << 20


def allowed_pairs(lens, prefix):
    lens = np.asarray(lens, dtype=np.int64)
    if prefix is None:
        return int((lens * (lens + 1) // 2).sum())
    prefix = np.asarray(prefix, dtype=np.int64)
    if prefix.ndim == 2:  # three blocks ending at P, P2, L: each row sees its own block and those before it
        P, P2 = prefix[:, 0], prefix[:, 1]
        return int((P * P + (P2 - P) * P2 + (lens - P2) * lens).sum())
    return int((prefix * prefix + (lens - prefix) * lens).sum())


def mask_modes(w, va):
    """(library mask mode, oracle mask mode) of a workload"""
    if w.three_block:
        return va.VA_MASK_THREE_BLOCK, 3
    return (va.VA_MASK_PREFIX_LM, 1) if w.prefix_lm else (va.VA_MASK_CAUSAL, 0)


def build_bin(name, va, wl, which=0):
    """Layout of bin `which` of the first-fit packing of the workload's pool (None if there is no such bin)."""
    w = wl.WORKLOADS[name]
    lens, prefix = wl.sample_lengths(name)
    bin_of, pos, nbins = va.va_pack_first_fit(lens, w.budget)
    if which >= nbins:
        return None
    idx = np.array(sorted(np.nonzero(bin_of == which)[0], key=lambda i: pos[i]), dtype=np.int64)
    cu, pl, mx = va.va_bin_layout(lens[idx], None if prefix is None else prefix[idx])
    return w, lens[idx], (None if prefix is None else prefix[idx]), cu, pl, mx


def build_bin0(name, va, wl):
    return build_bin(name, va, wl, 0)


def cpu_baseline(name, va, wl, budget_s=12.0, max_s=30.0):
    """The oracle as it stands, on the host cores: forward + backward of whole bins of the same workload,
    bin 0 first, until about `budget_s` seconds of CPU work are done (a bin is only started if the rate
    so far says it ends before `max_s`)."""
    from oracle import attn as oa
    nthreads = oa.num_threads()
    flops = tokens = samples = bins = 0
    dt = 0.0
    while True:
        b = build_bin(name, va, wl, bins)
        if b is None:
            break
        w, lens, prefix, cu, pl, mx = b
        D, Hq, Hkv = w.head_dim, w.num_q_heads, w.num_kv_heads
        f = 14.0 * D * Hq * allowed_pairs(lens, prefix)
        if bins > 0 and (dt >= budget_s or dt + f * dt / flops > max_s):
            break
        q, k, v, do = wl.tensor_values(w.seed + 1000 * bins, int(cu[-1]), Hq, Hkv, D)
        scale = 1.0 / float(np.sqrt(D))
        t0 = time.perf_counter()
        oa.attn_fwd(q, k, v, cu, prefix, scale=scale, mask_mode=mask_modes(w, va)[1])
        oa.attn_bwd(q, k, v, do, cu, prefix, scale=scale, mask_mode=mask_modes(w, va)[1])
        dt += time.perf_counter() - t0
        flops += f
        tokens += int(cu[-1])
        samples += len(lens)
        bins += 1
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": nthreads, "kind": "oracle",
            "sample": f"fp64 oracle fwd+bwd on the first {bins} bins of the first-fit packing "
                      f"({samples} samples, {tokens} tokens, {dt:.1f} s)",
            "tokens_per_s": tokens / dt}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=WORKLOAD, choices=["vlm", "pi05", "pi0", "longtail", "vit", "tiny"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a device-to-device copy of 256 MiB three times, the reference that scales the "
                         "HBM byte counters of a counter-collection run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2603_11101_amd import binding as va
    from paper_2603_11101_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    w, lens, prefix, cu, pl, mx = build_bin0(args.workload, va, wl)
    T, Hq, Hkv, D = int(cu[-1]), w.num_q_heads, w.num_kv_heads, w.head_dim
    mask = mask_modes(w, va)[0]
    scale = 1.0 / float(np.sqrt(D))
    pairs = allowed_pairs(lens, prefix)
    flops_fwd = 4.0 * D * Hq * pairs
    flops_bwd = 10.0 * D * Hq * pairs

    torch.zeros(1, device=dev)  # first touch of the device (context, allocator) is not part of the plan
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ps = va.PackedStream(cu, pl, mask, Hq, Hkv, D, max_seqlen=mx, device=dev)  # three work lists, built and uploaded
    torch.cuda.synchronize()
    host_plan_ms = (time.perf_counter() - t0) * 1e3

    def dev_bf16(x):
        return torch.from_numpy(wl.bf16_bits(x).view(np.int16)).view(torch.bfloat16).to(dev)

    q, k, v, do = wl.tensor_values(w.seed, T, Hq, Hkv, D)
    sets = []
    for i in range(NUM_BUFFER_SETS):
        s = {"q": dev_bf16(q), "k": dev_bf16(k), "v": dev_bf16(v), "do": dev_bf16(do)}
        s["out"] = torch.empty_like(s["q"])
        s["lse"] = torch.empty((Hq, T), dtype=torch.float32, device=dev)
        s["dq"], s["dk"], s["dv"] = torch.empty_like(s["q"]), torch.empty_like(s["k"]), torch.empty_like(s["v"])
        sets.append(s)
    ps.workspace()

    def step(s):
        ps.fwd(s["q"], s["k"], s["v"], scale, s["out"], s["lse"])
        ps.bwd(s["q"], s["k"], s["v"], s["out"], s["lse"], s["do"], scale, s["dq"], s["dk"], s["dv"])

    if args.copy_calibration:
        src = torch.ones(COPY_CALIBRATION_BYTES // 4, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for i in range(args.warmup):
        step(sets[i % NUM_BUFFER_SETS])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(sets[i % NUM_BUFFER_SETS])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3

    # per-kernel durations with HIP events on the launch stream, over the same rotation: many launches of one
    # kernel between two events, so that the cost of an event on the stream is spread over all of them
    iters = max(8, min(args.steps, 40))
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]

    def time_block(launch):
        # a warm-up as long as a block, then three blocks with no wait in between: the stream stays busy
        # and the clocks stay up from the first event to the last
        for i in range(iters):
            launch(i)
        evs[0].record()
        for blk in range(3):
            for i in range(iters):
                launch(i)
            evs[blk + 1].record()
        evs[3].synchronize()
        return float(np.median([evs[blk].elapsed_time(evs[blk + 1]) / iters for blk in range(3)]))

    def launch_fwd(i):
        s = sets[i % NUM_BUFFER_SETS]
        ps.fwd(s["q"], s["k"], s["v"], scale, s["out"], s["lse"])

    time_block(launch_fwd)  # the first train of forward-only launches after the mixed loop runs slow: not taken
    fwd_ms = time_block(launch_fwd)
    kms = np.zeros(3)
    per_set = max(2, iters // NUM_BUFFER_SETS)
    for i in range(NUM_BUFFER_SETS):
        s = sets[i]
        kms += np.array(ps.bwd_profile(s["q"], s["k"], s["v"], s["out"], s["lse"], s["do"], scale,
                                       s["dq"], s["dk"], s["dv"], iters=per_set))
    kms /= NUM_BUFFER_SETS
    # algorithmic work per launch: forward 2 products; dK/dV kernel 4 (scores, dP, dV, dK); dQ kernel 1 (dQ;
    # its recomputation of the scores and dP is overhead and is not counted)
    kernels = {
        "fwd_bf16": {"ms": fwd_ms, "flops": flops_fwd},
        "bwd_delta": {"ms": float(kms[0]), "flops": 2.0 * T * Hq * D},  # dropped below where no such kernel runs
        "bwd_dkdv": {"ms": float(kms[1]), "flops": 8.0 * D * Hq * pairs},
        "bwd_dq": {"ms": float(kms[2]), "flops": 2.0 * D * Hq * pairs},
    }
    # algorithmic bytes per launch: every input read once, every output written once
    fused = not va.va_bwd_has_delta_kernel(D)
    kernels["fwd_bf16"]["bytes"] = 2.0 * T * D * (2 * Hq + 2 * Hkv) + 4.0 * T * Hq
    kernels["bwd_dkdv"]["bytes"] = 2.0 * T * D * (2 * Hq + 4 * Hkv) + 8.0 * T * Hq
    kernels["bwd_dq"]["bytes"] = (2.0 * T * D * (4 * Hq + 2 * Hkv) + 12.0 * T * Hq if fused
                                  else 2.0 * T * D * (3 * Hq + 2 * Hkv) + 8.0 * T * Hq)
    kernels["bwd_delta"]["bytes"] = 4.0 * T * D * Hq + 12.0 * T * Hq
    if not va.va_bwd_has_delta_kernel(D):
        del kernels["bwd_delta"]
    dominant = max(("fwd_bf16", "bwd_dkdv", "bwd_dq"), key=lambda n: kernels[n]["ms"])
    achieved = kernels[dominant]["flops"] / (kernels[dominant]["ms"] * 1e-3) / 1e12
    traffic = None
    tpath = os.path.join(ROOT, "profiles", f"hbm_traffic_{args.workload}.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            traffic = json.load(f).get(dominant)

    # FP8 (E4M3) forward on the same batch, outside the timed region: per-head quantisation on the device,
    # then back-to-back launches between events as above
    fp8 = None
    if D == 128:
        codes = {}
        s0 = sets[0]
        for name in ("q", "k", "v"):
            c8 = torch.empty(s0[name].shape, dtype=torch.uint8, device=dev)
            descale = torch.empty((s0[name].shape[1],), dtype=torch.float32, device=dev)
            va.va_quantize_e4m3_per_head_device(s0[name], c8, descale)
            codes[name] = (c8, descale)
        for _ in range(3):
            ps.fwd_fp8(codes["q"][0], codes["k"][0], codes["v"][0], codes["q"][1], codes["k"][1], codes["v"][1],
                       scale, s0["out"], s0["lse"])
        fp8_ms = time_block(lambda i: ps.fwd_fp8(codes["q"][0], codes["k"][0], codes["v"][0], codes["q"][1],
                                                 codes["k"][1], codes["v"][1], scale, s0["out"], s0["lse"]))
        fp8 = {"ms": fp8_ms, "tflops": flops_fwd / (fp8_ms * 1e-3) / 1e12, "peak": 5000.0,
               "frac": flops_fwd / (fp8_ms * 1e-3) / 1e12 / 5000.0}
        # the same with block-wise scales (one per 128 tokens of a sample and head); the three quantiser
        # launches are timed on their own, against the bytes they must move (read twice, codes and scales out)
        cu_dev = torch.from_numpy(np.asarray(ps.cu_seqlens, dtype=np.int32)).to(dev)
        bcodes = {}
        for name in ("q", "k", "v"):
            c8 = torch.empty(s0[name].shape, dtype=torch.uint8, device=dev)
            d_tok = torch.empty(s0[name].shape[:2], dtype=torch.float32, device=dev)
            bcodes[name] = (c8, d_tok)

        def quantise_all(_):
            for name in ("q", "k", "v"):
                va.va_quantize_e4m3_blockwise_device(s0[name], ps.cu_seqlens, cu_dev, bcodes[name][0], bcodes[name][1])

        def fwd_block(_):
            ps.fwd_fp8_blockwise(bcodes["q"][0], bcodes["k"][0], bcodes["v"][0], bcodes["q"][1], bcodes["k"][1],
                                 bcodes["v"][1], scale, s0["out"], s0["lse"])

        for _ in range(3):
            quantise_all(0)
            fwd_block(0)
        q_ms = time_block(quantise_all)
        fb_ms = time_block(fwd_block)
        q_bytes = sum(s0[n].numel() * (2 + 1) + s0[n].shape[0] * s0[n].shape[1] * 4 for n in ("q", "k", "v"))
        fp8["blockwise"] = {"ms": fb_ms, "tflops": flops_fwd / (fb_ms * 1e-3) / 1e12,
                            "frac": flops_fwd / (fb_ms * 1e-3) / 1e12 / 5000.0,
                            "quantise_qkv_ms": q_ms, "quantise_gbps": q_bytes / (q_ms * 1e-3) / 1e9}

    useful_tflops = (flops_fwd + flops_bwd) / (ms_per_step * 1e-3) / 1e12
    result = {
        "metric": "packed varlen attn fwd+bwd useful TFLOP/s",
        "value": useful_tflops,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: bin 0 of the first-fit packing, {len(lens)} samples, {T} tokens, "
                               f"{Hq} q heads / {Hkv} kv heads, head_dim {D}, "
                               f"{'three-block' if w.three_block else 'prefix-LM' if w.prefix_lm else 'causal'}, budget {w.budget}",
                   "tokens": T, "samples": int(len(lens)), "pairs_per_head": pairs,
                   "buffer_sets": NUM_BUFFER_SETS},
        "tokens_per_s": T / (ms_per_step * 1e-3),
        "mfma_util_useful": useful_tflops / PEAK_BF16_TFLOPS,
        "host_plan_ms": host_plan_ms,
        "kernels_ms": {n: kernels[n]["ms"] for n in kernels},
        "kernels_tflops": {n: kernels[n]["flops"] / (kernels[n]["ms"] * 1e-3) / 1e12 for n in kernels},
        "fwd_fp8": fp8,
        "roofline": {"bound": "mfma", "kernel": dominant, "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic,
                     # the same launch against the other roof: short samples put this workload at the ridge
                     "hbm": {"achieved": kernels[dominant]["bytes"] / (kernels[dominant]["ms"] * 1e-3) / 1e9,
                             "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                             "frac": kernels[dominant]["bytes"] / (kernels[dominant]["ms"] * 1e-3) / 1e9 / PEAK_HBM_GBPS,
                             "algorithmic_bytes": kernels[dominant]["bytes"]}},
        "kernels_gbps": {n: kernels[n]["bytes"] / (kernels[n]["ms"] * 1e-3) / 1e9 for n in kernels},
        "paper_context": "paper reports 1.88x end-to-end training throughput from packing + varlen attention "
                         "(section 3.2; NVIDIA GPU model unstated); no absolute attention numbers",
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(args.workload, va, wl)
    print(json.dumps(result))


if __name__ == "__main__":
    main()

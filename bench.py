#!/usr/bin/env python3
"""Benchmark of the packed variable-length attention hot path on one MI355X.

One step = forward + backward (dQ and dK/dV kernels, plus the delta pass where the dQ kernel does not
compute delta itself) of one packed batch, synthetic N(0,1) bf16 inputs resident in HBM before the
timed region.  The headline workload is `longtail` (the largest single-GPU configuration: 65 536-token
budget, heavy-tailed lengths, 16 query / 8 KV heads, head_dim 128, causal), bin 0 of its first-fit packing.
Buffers rotate over several independent sets ("cold": the inputs of a step are not cache-resident from
the step before); the same-buffer ("warm") time and the time of a captured-graph replay are reported next
to it, and so is the mean over the first 8 bins.

Prints ONE JSON line: the metric (useful TFLOP/s: 14 * D * Hq * allowed (q, k) pairs per step), tokens/s,
per-kernel durations (HIP events around trains of launches of one kernel on the launch stream), a roofline
object for the dominant kernel against the roof that binds it, the same fields for the other configurations
(`configs`: vlm, pi05, the FP8 forward on the vlm shapes, and the latency of the tiny configuration), and the
CPU oracle's throughput on a bounded sample of the headline workload.

Other modes:
  --profile-leg        only the steps of --workload (plus FP8 forward launches at head_dim 128 and, with
                       --copy-calibration, three 256 MiB device copies): the program rocprofv3 runs
  --sweep              packed against padded fixed-length batches (the paper's section 3.2.1 sweep)
"""
import argparse
import hashlib
import glob
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0
PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_FP8_TFLOPS = 5000.0
HEADLINE = "longtail"
OTHER_CONFIGS = ("vlm", "pi05")
NUM_BUFFER_SETS = 4
COPY_CALIBRATION_BYTES = 256 << 20
CLOCK_RAMP_MS = 100.0         # untimed work before the warm-up steps, so that a short run sees the clocks a long one sees


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


def source_digest():
    """Digest of the kernel and host sources: profiles/ files carry the one they were measured with."""
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(ROOT, "paper_2603_11101_amd", "csrc", "*"))):
        if path.endswith((".hip", ".cpp", ".h")):
            h.update(os.path.basename(path).encode())
            h.update(open(path, "rb").read())
    return h.hexdigest()[:16]


class Case:
    """One packed batch on the device: work lists, `n_sets` independent buffer sets, algorithmic work."""

    def __init__(self, name, va, wl, torch, which=0, n_sets=NUM_BUFFER_SETS, host_values=True, dev="cuda:0"):
        self.name, self.va, self.torch = name, va, torch
        self.w, self.lens, self.prefix, self.cu, self.pl, self.mx = build_bin(name, va, wl, which)
        w = self.w
        self.T, self.Hq, self.Hkv, self.D = int(self.cu[-1]), w.num_q_heads, w.num_kv_heads, w.head_dim
        T, Hq, Hkv, D = self.T, self.Hq, self.Hkv, self.D
        self.mask = mask_modes(w, va)[0]
        self.scale = 1.0 / float(np.sqrt(D))
        self.pairs = allowed_pairs(self.lens, self.prefix)
        self.flops_fwd = 4.0 * D * Hq * self.pairs
        self.flops_bwd = 10.0 * D * Hq * self.pairs
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        self.ps = va.PackedStream(self.cu, self.pl, self.mask, Hq, Hkv, D, max_seqlen=self.mx, device=dev)
        torch.cuda.synchronize()
        self.host_plan_ms = (time.perf_counter() - t0) * 1e3   # three work lists, built and uploaded
        if host_values:
            self.host = wl.tensor_values(w.seed, T, Hq, Hkv, D)     # q, k, v, do as float32 holding bf16 values
            first = [torch.from_numpy(wl.bf16_bits(x).view(np.int16)).view(torch.bfloat16).to(dev) for x in self.host]
        else:
            g = torch.Generator(device=dev)
            g.manual_seed(1000 * which + w.seed)
            first = [torch.randn(shape, device=dev, generator=g).to(torch.bfloat16)
                     for shape in ((T, Hq, D), (T, Hkv, D), (T, Hkv, D), (T, Hq, D))]
        self.sets = []
        for i in range(n_sets):
            q, k, v, do = first if i == 0 else [x.clone() for x in first]
            s = {"q": q, "k": k, "v": v, "do": do, "out": torch.empty_like(q),
                 "lse": torch.empty((Hq, T), dtype=torch.float32, device=dev),
                 "dq": torch.empty_like(q), "dk": torch.empty_like(k), "dv": torch.empty_like(v)}
            self.sets.append(s)
        self.ps.workspace()
        self.fused = not va.va_bwd_has_delta_kernel(D)

    # -- launches
    def fwd(self, i=0):
        s = self.sets[i % len(self.sets)]
        self.ps.fwd(s["q"], s["k"], s["v"], self.scale, s["out"], s["lse"])

    def bwd(self, i=0, stages=None):
        s = self.sets[i % len(self.sets)]
        if stages is None:
            self.ps.bwd(s["q"], s["k"], s["v"], s["out"], s["lse"], s["do"], self.scale, s["dq"], s["dk"], s["dv"])
        else:
            self.ps.bwd_stages(s["q"], s["k"], s["v"], s["out"], s["lse"], s["do"], self.scale, s["dq"], s["dk"], s["dv"],
                               stages)

    def step(self, i=0):
        self.fwd(i)
        self.bwd(i)

    # -- timing
    def clock_ramp(self, ms=CLOCK_RAMP_MS):
        torch = self.torch
        t0 = time.perf_counter()
        i = 0
        while (time.perf_counter() - t0) * 1e3 < ms:
            for _ in range(4):
                self.step(i)
                i += 1
            torch.cuda.synchronize()

    def time_steps(self, steps, warmup, rotate=True):
        """milliseconds per step over exactly `steps` steps, wall clock between two device synchronisations"""
        torch = self.torch
        for i in range(warmup):
            self.step(i if rotate else 0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            self.step(i if rotate else 0)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    def time_graph(self, steps):
        """one step captured into a graph, replayed `steps` times back to back"""
        torch = self.torch
        g = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(g):
            self.step(0)
        for _ in range(3):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            g.replay()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    def time_train(self, launch, iters):
        """average milliseconds per launch: a warm-up train, then three trains between events with no wait in
        between (the stream stays busy and the clocks stay up from the first event to the last); median"""
        torch = self.torch
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        for i in range(iters):
            launch(i)
        evs[0].record()
        for blk in range(3):
            for i in range(iters):
                launch(i)
            evs[blk + 1].record()
        evs[3].synchronize()
        return float(np.median([evs[b].elapsed_time(evs[b + 1]) / iters for b in range(3)]))

    def time_in_step(self, iters):
        """{kernel: average milliseconds per launch} inside whole steps: `iters` steps of forward + backward in the
        library's own kernel order, buffer sets rotating, an event on the launch stream between every two kernels
        (the backward goes through varlen_attn_bwd_stages one kernel at a time, which launches what
        varlen_attn_bwd launches).  These are the durations a kernel trace of the step shows."""
        torch, va = self.torch, self.va
        order = ([("bwd_dq", va.VA_BWD_STAGE_DQ), ("bwd_dkdv", va.VA_BWD_STAGE_DKDV)] if self.fused else
                 [("bwd_delta", va.VA_BWD_STAGE_DELTA), ("bwd_dkdv", va.VA_BWD_STAGE_DKDV), ("bwd_dq", va.VA_BWD_STAGE_DQ)])
        names = ["fwd_bf16"] + [n for n, _ in order]
        for i in range(4):
            self.step(i)
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(len(names) + 1)] for _ in range(iters)]
        for i in range(iters):
            evs[i][0].record()
            self.fwd(i)
            evs[i][1].record()
            for j, (_, stage) in enumerate(order):
                self.bwd(i, stage)
                evs[i][j + 2].record()
        evs[-1][-1].synchronize()
        return {n: float(np.mean([evs[i][j].elapsed_time(evs[i][j + 1]) for i in range(iters)])) for j, n in enumerate(names)}

    def kernels(self, iters):
        """{kernel: {ms, ms_train, flops, bytes}}: duration inside the step (time_in_step) and in a train of
        back-to-back launches of the one kernel, and the algorithmic work per launch.  Forward 2 products; dK/dV
        kernel 4 (scores, dP, dV, dK); dQ kernel 1 (dQ; its recomputation of the scores and dP is overhead and is
        not counted).  Bytes: every input read once, every output written once."""
        va = self.va
        T, Hq, Hkv, D, pairs = self.T, self.Hq, self.Hkv, self.D, self.pairs
        self.step(0)  # the workspace holds delta and the rescaled LSE of every set the dK/dV train reads
        for i in range(1, len(self.sets)):
            self.step(i)
        self.time_train(self.fwd, iters)  # the first train of one kernel after the mixed loop runs slow: not taken
        k = {"fwd_bf16": {"ms_train": self.time_train(self.fwd, iters), "flops": self.flops_fwd,
                          "bytes": 2.0 * T * D * (2 * Hq + 2 * Hkv) + 4.0 * T * Hq}}
        k["bwd_dq"] = {"ms_train": self.time_train(lambda i: self.bwd(i, va.VA_BWD_STAGE_DQ), iters),
                       "flops": 2.0 * D * Hq * pairs,
                       "bytes": (2.0 * T * D * (4 * Hq + 2 * Hkv) + 12.0 * T * Hq if self.fused
                                 else 2.0 * T * D * (3 * Hq + 2 * Hkv) + 8.0 * T * Hq)}
        # one workspace serves all buffer sets; they hold the same values, so the delta and rescaled LSE the dQ
        # train left there are those of every set
        k["bwd_dkdv"] = {"ms_train": self.time_train(lambda i: self.bwd(i, va.VA_BWD_STAGE_DKDV), iters),
                         "flops": 8.0 * D * Hq * pairs,
                         "bytes": 2.0 * T * D * (2 * Hq + 4 * Hkv) + 8.0 * T * Hq}
        if not self.fused:
            k["bwd_delta"] = {"ms_train": self.time_train(lambda i: self.bwd(i, va.VA_BWD_STAGE_DELTA), iters),
                              "flops": 2.0 * T * Hq * D, "bytes": 4.0 * T * D * Hq + 12.0 * T * Hq}
        in_step = self.time_in_step(iters)
        for n in k:
            k[n]["ms"] = in_step[n]
        return k


def load_profile_json(kind, workload):
    path = os.path.join(ROOT, "profiles", f"{kind}_{workload}.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        return json.load(f)


def roofline_of(kernels, workload, peak_tflops=PEAK_BF16_TFLOPS):
    """The dominant kernel against the roof that binds it: the larger of flops / peak and bytes / 8 TB/s."""
    dominant = max((n for n in kernels if n != "bwd_delta"), key=lambda n: kernels[n]["ms"])
    kd = kernels[dominant]
    sec = kd["ms"] * 1e-3
    t_mfma, t_hbm = kd["flops"] / (peak_tflops * 1e12), kd["bytes"] / (PEAK_HBM_GBPS * 1e9)
    mfma = {"achieved": kd["flops"] / sec / 1e12, "peak": peak_tflops, "unit": "TFLOP/s"}
    hbm = {"achieved": kd["bytes"] / sec / 1e9, "peak": PEAK_HBM_GBPS, "unit": "GB/s"}
    for r in (mfma, hbm):
        r["frac"] = r["achieved"] / r["peak"]
    traffic = load_profile_json("hbm_traffic", workload)
    stale = None if traffic is None else traffic.get("source_digest") != source_digest()
    t = None if traffic is None else traffic.get(dominant)
    main, other, bound = (mfma, hbm, "mfma") if t_mfma >= t_hbm else (hbm, mfma, "hbm")
    return {"bound": bound, "kernel": dominant, **main, "traffic": t,
            "traffic_over_algorithmic": None if t is None else t / kd["bytes"],
            "traffic_source": None if traffic is None else f"profiles/hbm_traffic_{workload}.json"
                              + (" (measured on other sources than this build)" if stale else ""),
            "algorithmic_bytes": kd["bytes"], "algorithmic_flops": kd["flops"],
            "floor_us": {"mfma": t_mfma * 1e6, "hbm": t_hbm * 1e6},
            "other_roof": {"bound": "hbm" if bound == "mfma" else "mfma", **other}}


def measure(case, steps, warmup, iters, full=True):
    """The fields of one configuration."""
    case.clock_ramp()
    ms = case.time_steps(steps, warmup, rotate=True)
    flops = case.flops_fwd + case.flops_bwd
    w = case.w
    r = {"workload": f"{case.name}: bin 0 of the first-fit packing, {len(case.lens)} samples, {case.T} tokens, "
                     f"{case.Hq} q heads / {case.Hkv} kv heads, head_dim {case.D}, "
                     f"{'three-block' if w.three_block else 'prefix-LM' if w.prefix_lm else 'causal'}, budget {w.budget}",
         "tokens": case.T, "samples": int(len(case.lens)), "pairs_per_head": case.pairs,
         "ms_per_step": ms, "value": flops / (ms * 1e-3) / 1e12, "unit": "TFLOP/s",
         "tokens_per_s": case.T / (ms * 1e-3), "mfma_util_useful": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
         "host_plan_ms": case.host_plan_ms}
    if full:
        warm = case.time_steps(steps, min(warmup, 5), rotate=False)
        r["ms_per_step_warm"] = warm
        r["value_warm"] = flops / (warm * 1e-3) / 1e12
        gms = case.time_graph(steps)
        r["ms_per_step_graph"] = gms
        r["value_graph"] = flops / (gms * 1e-3) / 1e12
    k = case.kernels(iters)
    r["kernels_ms"] = {n: k[n]["ms"] for n in k}               # inside the step: what the roofline is priced with
    r["kernels_ms_train"] = {n: k[n]["ms_train"] for n in k}   # back-to-back launches of the one kernel
    r["kernels_tflops"] = {n: k[n]["flops"] / (k[n]["ms"] * 1e-3) / 1e12 for n in k}
    r["kernels_gbps"] = {n: k[n]["bytes"] / (k[n]["ms"] * 1e-3) / 1e9 for n in k}
    r["roofline"] = roofline_of(k, case.name)
    # whole step against the floors of section "measurement": every tensor once, every counted product once
    step_bytes = (2.0 * case.T * case.D * (2 * case.Hq + 2 * case.Hkv) + 4.0 * case.T * case.Hq
                  + 2.0 * case.T * case.D * (4 * case.Hq + 4 * case.Hkv) + 12.0 * case.T * case.Hq)
    floor_us = max(flops / (PEAK_BF16_TFLOPS * 1e12), step_bytes / (PEAK_HBM_GBPS * 1e9)) * 1e6
    r["step_floor_us"] = floor_us
    r["step_frac_of_floor"] = floor_us / (ms * 1e3)
    pmc = load_profile_json("pmc", case.name)
    if pmc is not None:
        r["rocprof_counters"] = {"file": f"profiles/pmc_{case.name}.json",
                                 "stale": pmc.get("source_digest") != source_digest(),
                                 **{n: pmc[n] for n in pmc if n != "source_digest"}}
    return r


def fp8_forward(case, iters):
    """FP8 (E4M3) forward on the batch of `case` (head_dim 128): per-head quantisation on the device, then
    trains of launches between events; the same with block-wise scales, and the quantiser itself."""
    torch, va, ps = case.torch, case.va, case.ps
    s0, scale, dev = case.sets[0], case.scale, case.sets[0]["q"].device
    codes = {}
    for name in ("q", "k", "v"):
        c8 = torch.empty(s0[name].shape, dtype=torch.uint8, device=dev)
        descale = torch.empty((s0[name].shape[1],), dtype=torch.float32, device=dev)
        va.va_quantize_e4m3_per_head_device(s0[name], c8, descale)
        codes[name] = (c8, descale)

    def fwd(_):
        ps.fwd_fp8(codes["q"][0], codes["k"][0], codes["v"][0], codes["q"][1], codes["k"][1], codes["v"][1],
                   scale, s0["out"], s0["lse"])

    for _ in range(3):
        fwd(0)
    ms = case.time_train(fwd, iters)
    T, Hq, Hkv, D = case.T, case.Hq, case.Hkv, case.D
    k = {"fwd_fp8": {"ms": ms, "flops": case.flops_fwd, "bytes": 1.0 * T * D * (Hq + 2 * Hkv) + 2.0 * T * D * Hq + 4.0 * T * Hq}}
    r = {"workload": f"{case.name}_fp8: FP8 (E4M3, per-head scales) forward on the {case.name} batch",
         "ms": ms, "value": case.flops_fwd / (ms * 1e-3) / 1e12, "unit": "TFLOP/s", "dtype": "f8e4m3",
         "roofline": roofline_of(k, case.name, PEAK_FP8_TFLOPS)}
    cu_dev = torch.from_numpy(np.asarray(ps.cu_seqlens, dtype=np.int32)).to(dev)
    bcodes = {name: (torch.empty(s0[name].shape, dtype=torch.uint8, device=dev),
                     torch.empty(s0[name].shape[:2], dtype=torch.float32, device=dev)) for name in ("q", "k", "v")}

    def quantise_all(_):
        for name in ("q", "k", "v"):
            va.va_quantize_e4m3_blockwise_device(s0[name], ps.cu_seqlens, cu_dev, bcodes[name][0], bcodes[name][1])

    def fwd_block(_):
        ps.fwd_fp8_blockwise(bcodes["q"][0], bcodes["k"][0], bcodes["v"][0], bcodes["q"][1], bcodes["k"][1],
                             bcodes["v"][1], scale, s0["out"], s0["lse"])

    for _ in range(3):
        quantise_all(0)
        fwd_block(0)
    q_ms = case.time_train(quantise_all, iters)
    fb_ms = case.time_train(fwd_block, iters)
    q_bytes = sum(s0[n].numel() * (2 + 1) + s0[n].shape[0] * s0[n].shape[1] * 4 for n in ("q", "k", "v"))
    r["blockwise"] = {"ms": fb_ms, "tflops": case.flops_fwd / (fb_ms * 1e-3) / 1e12,
                      "frac": case.flops_fwd / (fb_ms * 1e-3) / 1e12 / PEAK_FP8_TFLOPS,
                      "quantise_qkv_ms": q_ms, "quantise_gbps": q_bytes / (q_ms * 1e-3) / 1e9}
    return r


def gemm_reference(torch, dev, n=8192, seconds=1.0):
    """What the vendor's dense bf16 GEMM (hipBLASLt through torch.matmul, n^3, standard normal operands) reaches on
    this box right now: context for the published 2.5 PFLOP/s that the rooflines are priced with.  Not part of the
    path; nothing of the library is used here."""
    a = torch.randn((n, n), device=dev).to(torch.bfloat16)
    b = torch.randn((n, n), device=dev).to(torch.bfloat16)
    c = torch.empty((n, n), dtype=torch.bfloat16, device=dev)
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < 0.3 * seconds:      # clocks up, library warmed
        for _ in range(8):
            torch.matmul(a, b, out=c)
        torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    iters = 200
    e0.record()
    for _ in range(iters):
        torch.matmul(a, b, out=c)
    e1.record()
    e1.synchronize()
    ms = e0.elapsed_time(e1) / iters
    tf = 2.0 * n ** 3 / (ms * 1e-3) / 1e12
    return {"what": f"torch.matmul (hipBLASLt) bf16 {n}x{n}x{n}, standard normal operands", "ms": ms, "tflops": tf,
            "frac_of_peak": tf / PEAK_BF16_TFLOPS}


def gemm_reference_fp8(torch, dev, n=8192):
    """The same for E4M3 operands (torch._scaled_mm, unit scales, bf16 result): context for the 5 PFLOP/s the FP8
    forward is priced with.  None where this PyTorch build has no such routine."""
    try:
        a = torch.randn((n, n), device=dev).to(torch.float8_e4m3fn)
        b = torch.randn((n, n), device=dev).to(torch.float8_e4m3fn)
        one = torch.ones((), device=dev)
        run = lambda: torch._scaled_mm(a, b.t(), scale_a=one, scale_b=one, out_dtype=torch.bfloat16)
        for _ in range(30):
            run()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(200):
            run()
        e1.record()
        e1.synchronize()
    except Exception as exc:  # noqa: BLE001 - a reference figure only
        return {"what": "torch._scaled_mm not available", "error": repr(exc)[:200]}
    ms = e0.elapsed_time(e1) / 200
    tf = 2.0 * n ** 3 / (ms * 1e-3) / 1e12
    return {"what": f"torch._scaled_mm (hipBLASLt) e4m3 {n}x{n}x{n}, standard normal operands, bf16 result", "ms": ms,
            "tflops": tf, "frac_of_peak": tf / PEAK_FP8_TFLOPS}


def tiny_latency(va, wl, torch, reps=200):
    """Configuration 1 is a latency case: microseconds per forward + backward call pair, eager and as a graph
    replay, and the host microseconds the two calls take to return; the oracle on one thread beside it."""
    case = Case("tiny", va, wl, torch, n_sets=1)
    case.clock_ramp(20.0)
    eager = case.time_steps(reps, 20, rotate=False) * 1e3
    graph = case.time_graph(reps) * 1e3
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        case.step(0)
    host = (time.perf_counter() - t0) / reps * 1e6
    torch.cuda.synchronize()
    from oracle import attn as oa
    q, k, v, do = case.host
    t0 = time.perf_counter()
    for _ in range(5):
        oa.attn_fwd(q, k, v, case.cu, None, scale=case.scale, nthreads=1)
        oa.attn_bwd(q, k, v, do, case.cu, None, scale=case.scale, nthreads=1)
    oracle_us = (time.perf_counter() - t0) / 5 * 1e6
    return {"workload": "tiny: 3 samples of 17, 64, 95 tokens, 2 / 2 heads, head_dim 64, causal",
            "latency_us": eager, "latency_graph_us": graph, "host_call_us": host,
            "oracle_1_thread_us": oracle_us}


def host_call_cost(case, reps=200):
    """(microseconds the forward + backward calls of one step take on the host through the Python binding,
    the same through the bare C ABI with arguments marshalled once): validation of the three work lists and
    the kernel launches; the second figure leaves out what ctypes and numpy add per call."""
    import ctypes
    torch, va = case.torch, case.va
    torch.cuda.synchronize()
    best = float("inf")
    for _ in range(3):
        t0 = time.perf_counter()
        for i in range(reps):
            case.step(i)
        best = min(best, (time.perf_counter() - t0) / reps * 1e6)
        torch.cuda.synchronize()
    ps, s = case.ps, case.sets[0]
    P = va._ptr
    lists = {pid: (P(ps.worklist[pid]), P(ps.worklist_host[pid])) for pid in ps.worklist}
    shape, scale = ctypes.byref(ps.shape), ctypes.c_float(case.scale)
    cu, pl, stream = P(ps.cu_seqlens), P(ps.prefix_lens), va._stream_ptr(None)
    ws = ps.workspace()
    fwd_args = (P(s["q"]), P(s["k"]), P(s["v"]), cu, pl, *lists[va.VA_PASS_FWD], shape, scale, P(s["out"]), P(s["lse"]), stream)
    bwd_args = (P(s["q"]), P(s["k"]), P(s["v"]), P(s["out"]), P(s["lse"]), P(s["do"]), cu, pl, *lists[va.VA_PASS_BWD_DKDV],
                *lists[va.VA_PASS_BWD_DQ], shape, scale, P(s["dq"]), P(s["dk"]), P(s["dv"]), P(ws), ctypes.c_size_t(ws.numel()), stream)
    bare = float("inf")
    for _ in range(3):
        t0 = time.perf_counter()
        for i in range(reps):
            rc = va._lib.varlen_attn_fwd(*fwd_args) | va._lib.varlen_attn_bwd(*bwd_args)
        bare = min(bare, (time.perf_counter() - t0) / reps * 1e6)
        torch.cuda.synchronize()
        assert rc == 0
    return best, bare


def cpu_baseline(case, va, budget_s=14.0):
    """The oracle as it stands, on the host cores: forward + backward of the first m samples of the headline
    batch (a packed stream of its own), m chosen from the rate on the first sample so that the work takes
    about `budget_s` seconds."""
    from oracle import attn as oa
    nthreads = oa.num_threads()
    w, cu, lens, prefix = case.w, case.cu, case.lens, case.prefix
    D, Hq = case.D, case.Hq
    omode = mask_modes(w, va)[1]
    q, k, v, do = case.host

    def run(m):
        rows = int(cu[m])
        sub_cu = np.ascontiguousarray(cu[:m + 1])
        sub_p = None if prefix is None else np.ascontiguousarray(prefix[:m])
        t0 = time.perf_counter()
        oa.attn_fwd(q[:rows], k[:rows], v[:rows], sub_cu, sub_p, scale=case.scale, mask_mode=omode)
        oa.attn_bwd(q[:rows], k[:rows], v[:rows], do[:rows], sub_cu, sub_p, scale=case.scale, mask_mode=omode)
        return time.perf_counter() - t0

    def flops(m):
        return 14.0 * D * Hq * allowed_pairs(lens[:m], None if prefix is None else prefix[:m])

    # rate from a few samples (enough of them to occupy every thread), then as many as fit the budget
    m0 = min(len(lens), max(4, nthreads // max(1, case.Hkv)))
    rate = flops(m0) / run(m0)
    m = m0
    while m < len(lens) and flops(m + 1) / rate <= budget_s:
        m += 1
    dt = run(m)
    return {"value": flops(m) / dt / 1e12, "unit": "TFLOP/s", "cores": nthreads, "kind": "oracle",
            "sample": f"fp64 oracle fwd+bwd on the first {m} of {len(lens)} samples of the {case.name} batch "
                      f"({int(cu[m])} tokens, {dt:.1f} s)",
            "tokens_per_s": int(cu[m]) / dt}


def bins_mean(name, va, wl, torch, steps, warmup, first_ms, nbins=8):
    """Mean over the first `nbins` bins: total useful flops / total time (bin 0 is the headline case, already
    timed; the other bins take device-drawn N(0,1) values and two buffer sets)."""
    flops, tokens, ms_sum, n = 0.0, 0, 0.0, 0
    per_bin = []
    for b in range(nbins):
        if build_bin(name, va, wl, b) is None:
            break
        if b == 0:
            c = None
            w, lens, prefix, cu, pl, mx = build_bin(name, va, wl, 0)
            f = 14.0 * w.head_dim * w.num_q_heads * allowed_pairs(lens, prefix)
            ms, T = first_ms, int(cu[-1])
        else:
            c = Case(name, va, wl, torch, which=b, n_sets=2, host_values=False)
            ms = c.time_steps(max(10, steps // 4), max(3, warmup // 4))
            f, T = c.flops_fwd + c.flops_bwd, c.T
        per_bin.append({"bin": b, "tokens": T, "ms_per_step": ms, "tflops": f / (ms * 1e-3) / 1e12})
        flops, tokens, ms_sum, n = flops + f, tokens + T, ms_sum + ms, n + 1
        del c
        torch.cuda.empty_cache()
    return {"bins": n, "tflops": flops / (ms_sum * 1e-3) / 1e12, "tokens_per_s": tokens / (ms_sum * 1e-3), "per_bin": per_bin}


# ---------------------------------------------------------------- packed against padded (section 3.2.1)

SWEEP_HQ, SWEEP_HKV, SWEEP_D = 16, 8, 128


def sweep_lengths(batch, seq, pad_rate, rng):
    mean = (1.0 - pad_rate) * seq
    half = min(mean - 16, seq - mean, 0.5 * mean)
    lens = rng.integers(int(mean - half), int(mean + half) + 1, size=batch).astype(np.int64)
    lens = np.clip(lens, 16, seq)
    lens[0] = seq
    return lens


def sweep_time(va, torch, lens, steps, dev="cuda:0"):
    HQ, HKV, D = SWEEP_HQ, SWEEP_HKV, SWEEP_D
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


def sweep(va, torch, quick):
    """The paper's varlen-against-fixlen sweep with this library: the same kernels once on the packed stream
    of the true lengths and once on a stream in which every sample is padded to the maximum length (what a
    fixed-length batch computes), causal, 16 / 8 heads, head_dim 128, forward + backward.  Lengths are seeded:
    B samples, uniform around (1 - padding rate) * S, clipped to [16, S], one sample forced to S.  Prints the
    table and, under it, the statements of the paper's section 3.2.1 checked against the rows."""
    HQ, D = SWEEP_HQ, SWEEP_D
    batches = (8, 32) if quick else (8, 16, 32)
    seqs = (1024, 8192) if quick else (1024, 2048, 4096, 8192, 16384, 32768)
    rates = (0.03, 0.5, 0.9) if quick else (0.03, 0.25, 0.5, 0.75, 0.9)
    rng = np.random.default_rng(7)
    print("# Packed variable-length attention against the padded fixed-length layout (forward + backward, causal,\n"
          f"# {HQ} query / {SWEEP_HKV} KV heads, head_dim {D}) on one MI355X: the sweep of the paper's section 3.2.1 (batch, sequence\n"
          "# length, padding rate) with this library's kernels.  Command:\n"
          f"#   python3 bench.py --sweep{' --quick' if quick else ''}\n"
          "# 'target' is the padding rate the lengths were drawn for, 'padding' the rate of the drawn batch (one sample\n"
          "# always has the full length); 'saved' = 1 - packed/padded time; packed_TF and padded_TF count the useful pairs\n"
          "# only; fixlen_TF credits the padded batch with every pair it computes (14 * D * Hq * B * S (S + 1) / 2 over the\n"
          "# padded time): the figure a fixed-length benchmark reports.")
    print(f"{'batch':>5s} {'seq':>6s} {'target':>7s} {'padding':>8s} {'packed_ms':>10s} {'padded_ms':>10s} "
          f"{'saved':>7s} {'packed_TF':>10s} {'padded_TF':>10s} {'fixlen_TF':>10s}")
    rows = []
    for b in batches:
        for s in seqs:
            padded = np.full(b, s, dtype=np.int64)
            steps = max(2, min(10, int(1e9 / (b * s * s))))
            t_padded = sweep_time(va, torch, padded, steps)
            fixlen = 14.0 * D * HQ * b * (s * (s + 1) // 2) / t_padded / 1e9
            for r in rates:
                lens = sweep_lengths(b, s, r, rng)
                pad = 1.0 - lens.sum() / float(b * s)
                t_packed = sweep_time(va, torch, lens, steps)
                flops = 14.0 * D * HQ * float((lens * (lens + 1) // 2).sum())
                # the padded batch is credited with the useful pairs only
                rows.append({"b": b, "s": s, "r": r, "pad": pad, "packed": t_packed, "padded": t_padded,
                             "saved": 1.0 - t_packed / t_padded, "tf": flops / t_packed / 1e9, "fixlen": fixlen})
                print(f"{b:5d} {s:6d} {r:7.2f} {pad:8.3f} {t_packed:10.3f} {t_padded:10.3f} "
                      f"{1.0 - t_packed / t_padded:7.1%} {flops / t_packed / 1e9:10.0f} {flops / t_padded / 1e9:10.0f} "
                      f"{fixlen:10.0f}", flush=True)
    sweep_statements(rows, batches, seqs, rates)


def sweep_statements(rows, batches, seqs, rates):
    """The four statements of the paper's section 3.2.1 (its hardware, its kernels) held against the rows."""
    pick = lambda **kw: [x for x in rows if all(x[k] == v for k, v in kw.items())]
    span = lambda xs, key, f="{:.1%}": f.format(min(x[key] for x in xs)) + " ... " + f.format(max(x[key] for x in xs))
    lo_r, hi_r = min(rates), max(rates)
    print("#\n# The paper's statements (section 3.2.1; other hardware, other kernels), checked against the table:")
    print(f"# 1. 'varlen latency is consistently lower than fixlen': packed_ms < padded_ms in all {len(rows)} rows: "
          f"{all(x['packed'] < x['padded'] for x in rows)}.")
    print(f"#    'savings rise from 2.28 % at 3 % padding to 89.73 % at 90 %': here {span(pick(r=lo_r), 'saved')} at "
          f"{lo_r:.0%} and {span(pick(r=hi_r), 'saved')} at {hi_r:.0%} (drawn padding at that target: "
          f"{span(pick(r=hi_r), 'pad', '{:.0%}')}; one sample is full length);")
    print("#    savings exceed the padding rate because causal cost grows with the square of the length.")
    if 2048 in seqs:
        peak = {b: max(x["tf"] for x in pick(b=b, s=2048)) for b in batches}
        b0, b1 = min(batches), max(batches)
        at = pick(b=b1, s=2048)
        print(f"# 2. 'at 2048 tokens the peak TFLOPS grows 1.2x from batch {b0} to {b1}, and varlen stays below fixlen': peak "
              f"packed_TF {peak[b0]:.0f} -> {peak[b1]:.0f} ({peak[b1] / peak[b0]:.2f}x); at batch {b1} packed_TF by padding "
              f"target {' / '.join(format(x['tf'], '.0f') for x in at)} against fixlen_TF {at[0]['fixlen']:.0f}.")
    top = pick(s=max(seqs))
    ratio = [x["tf"] / x["fixlen"] for x in top]
    print(f"#    'at {max(seqs)} tokens varlen is on par with or above fixlen': packed_TF / fixlen_TF is {min(ratio):.2f} ... "
          f"{max(ratio):.2f} in the {len(top)} rows of that length.")
    if 16 in batches:
        long_rows = [x for x in pick(b=16) if x["s"] > 8192 and x["r"] >= 0.25]
        if long_rows:
            print(f"# 3. 'batch 16, sequences above 8k: savings of 25-90 %': here {span(long_rows, 'saved')} for padding "
                  f"targets of 25 % and more.")
    bmid = 16 if 16 in batches else max(batches)
    best = ", ".join(f"{s}: {max(x['tf'] for x in pick(b=bmid, s=s)):.0f}" for s in seqs)
    print(f"# 4. 'TFLOPS rises quickly from 1k to 8k and is flat beyond': best packed_TF at batch {bmid} by length: {best}.")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=HEADLINE, choices=["vlm", "pi05", "pi0", "longtail", "vit"])
    ap.add_argument("--configs", default=",".join(OTHER_CONFIGS) + ",vlm_fp8,tiny",
                    help="comma-separated configurations reported beside the headline (or 'none')")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-bins", action="store_true", help="skip the mean over the first 8 bins")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a device-to-device copy of 256 MiB three times, the reference that scales the "
                         "HBM byte counters of a counter-collection run")
    ap.add_argument("--profile-leg", action="store_true")
    ap.add_argument("--sweep", action="store_true")
    ap.add_argument("--quick", action="store_true", help="with --sweep: a 2 x 2 x 3 corner")
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
    torch.zeros(1, device=dev)  # first touch of the device (context, allocator) is not part of any plan time
    torch.cuda.synchronize()

    if args.sweep:
        sweep(va, torch, args.quick)
        return

    if args.profile_leg:
        case = Case(args.workload, va, wl, torch, host_values=False)
        if args.copy_calibration:
            src = torch.ones(COPY_CALIBRATION_BYTES // 4, dtype=torch.float32, device=dev)
            dst = torch.empty_like(src)
            for _ in range(3):
                dst.copy_(src)
            torch.cuda.synchronize()
            del src, dst
        case.clock_ramp(30.0)
        ms = case.time_steps(args.steps, args.warmup)
        if case.D == 128:
            fp8_forward(case, max(4, min(args.steps, 20)))
        print(json.dumps({"profile_leg": args.workload, "steps": args.steps, "ms_per_step": ms}))
        return

    iters = max(8, min(args.steps, 40))
    case = Case(args.workload, va, wl, torch)
    head = measure(case, args.steps, args.warmup, iters, full=True)
    head["host_call_us"], head["host_call_us_c_abi"] = host_call_cost(case)
    result = {
        "metric": "packed varlen attn fwd+bwd useful TFLOP/s",
        "value": head["value"],
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": head["workload"], "tokens": head["tokens"], "samples": head["samples"],
                   "pairs_per_head": head["pairs_per_head"], "buffer_sets": NUM_BUFFER_SETS,
                   "clock_ramp_ms": CLOCK_RAMP_MS},
        **{n: head[n] for n in ("tokens_per_s", "mfma_util_useful", "ms_per_step_warm", "value_warm",
                                "ms_per_step_graph", "value_graph", "host_plan_ms", "host_call_us", "host_call_us_c_abi", "kernels_ms", "kernels_ms_train",
                                "kernels_tflops", "kernels_gbps", "step_floor_us", "step_frac_of_floor")},
        "roofline": head["roofline"],
        "source_digest": source_digest(),
        "paper_context": "paper reports 1.88x end-to-end training throughput from packing + varlen attention "
                         "(section 3.2; NVIDIA GPU model unstated); no absolute attention numbers",
    }
    if "rocprof_counters" in head:
        result["rocprof_counters"] = head["rocprof_counters"]
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(case, va)
    first_ms = head["ms_per_step"]
    del case
    torch.cuda.empty_cache()
    if not args.no_bins:
        result["bins8"] = bins_mean(args.workload, va, wl, torch, args.steps, args.warmup, first_ms)
    configs = {}
    wanted = [] if args.configs == "none" else [c for c in args.configs.split(",") if c]
    for name in wanted:
        if name == "tiny":
            configs["tiny"] = tiny_latency(va, wl, torch)
        elif name.endswith("_fp8"):
            c = Case(name[:-4], va, wl, torch, n_sets=1)
            c.clock_ramp()
            configs[name] = fp8_forward(c, iters)
            del c
        elif name != args.workload:
            c = Case(name, va, wl, torch)
            configs[name] = measure(c, max(args.steps, 100), args.warmup, iters, full=True)
            configs[name]["host_call_us"], configs[name]["host_call_us_c_abi"] = host_call_cost(c)
            del c
        torch.cuda.empty_cache()
    if configs:
        result["configs"] = configs
    if not args.no_bins:    # the full default run only
        result["gemm_reference"] = gemm_reference(torch, dev)
        result["gemm_reference_fp8"] = gemm_reference_fp8(torch, dev)
        if result["roofline"]["unit"] == "TFLOP/s":   # the dominant kernel against what a plain GEMM gets here
            result["roofline"]["achieved_over_gemm_reference"] = result["roofline"]["achieved"] / result["gemm_reference"]["tflops"]
    print(json.dumps(result))


if __name__ == "__main__":
    main()

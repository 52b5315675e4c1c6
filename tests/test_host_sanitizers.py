"""The host-only part of the library (first-fit packer, bin layout, work lists with their schedules and
split tiles, both E4M3 quantisers) built with AddressSanitizer and UndefinedBehaviorSanitizer and run on the
cases of the host-library tests and on the benchmark's batches: no report from either sanitiser, and every
output byte equal to what the shipped library returns."""
import os
import shutil
import struct
import subprocess

import numpy as np
import pytest

from paper_2603_11101_amd import binding as va
from paper_2603_11101_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2603_11101_amd", "csrc")


def build_driver(tmp):
    exe = os.path.join(tmp, "host_sanitize")
    # the sanitiser runtimes are linked statically, so that their place in the process's library list does not matter
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-static-libasan", "-static-libubsan", os.path.join(ROOT, "tests", "host_sanitize_main.cpp"),
           os.path.join(CSRC, "host_pack.cpp"), "-o", exe]
    subprocess.check_call(cmd)
    return exe


def bf16_values(n, seed):
    """the driver's pseudo-random bf16 bit patterns"""
    x = np.zeros(n, dtype=np.uint16)
    s = (seed * 2654435761 + 1) & 0xffffffff
    for i in range(n):
        s ^= (s << 13) & 0xffffffff
        s ^= s >> 17
        s ^= (s << 5) & 0xffffffff
        x[i] = ((s >> 31) << 15) | ((110 + (s >> 8) % 30) << 7) | (s & 0x7f)
        if (s >> 16) % 37 == 0:
            x[i] = 0
    return x


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = build_driver(str(tmp_path))
    r = np.random.default_rng(77)
    cases = []
    for _ in range(6):
        budget = int(r.integers(1, 400))
        lens = r.integers(0, budget + 1, size=int(r.integers(0, 120)))
        cases.append(("pack", budget, [int(x) for x in lens]))
    cases.append(("pack", 10, [5, 11]))                          # a sample longer than the budget: an error, outputs untouched
    small = [1, 0, 300, 129, 64, 17, 200, 33]
    for mask in range(5):
        for (Hq, Hkv, D) in ((2, 2, 64), (16, 8, 128), (8, 1, 256), (4, 4, 80)):
            if mask == va.VA_MASK_CAUSAL:
                prefix = []
            elif mask == va.VA_MASK_THREE_BLOCK:
                prefix = [int(x) for x in wl.random_block_ends(D + mask, small).reshape(-1)]
            elif mask == va.VA_MASK_SLIDING_WINDOW:
                prefix = [int(x) for x in r.integers(1, 200, size=len(small))]
            else:
                prefix = [int(r.integers(0, L + 1)) for L in small]
            for pass_id in range(3):
                cases.append(("list", mask, pass_id, D, Hq, Hkv, small, prefix))
    cases.append(("list", va.VA_MASK_PREFIX_LM, va.VA_PASS_FWD, 64, 2, 2, [10, 20], [11, 0]))     # prefix beyond the sample: refused
    for name in ("vlm", "pi05", "longtail", "pi0"):              # the benchmark's batches: schedules, split tiles, launch order
        w = wl.WORKLOADS[name]
        lens, prefix = wl.sample_lengths(name)
        b, p, _ = va.va_pack_first_fit(lens, w.budget)
        idx = np.array(sorted(np.nonzero(b == 0)[0], key=lambda i: p[i]))
        mask = va.VA_MASK_THREE_BLOCK if w.three_block else va.VA_MASK_PREFIX_LM if w.prefix_lm else va.VA_MASK_CAUSAL
        pre = [] if prefix is None else [int(x) for x in np.asarray(prefix[idx]).reshape(-1)]
        for pass_id in range(3):
            cases.append(("list", mask, pass_id, w.head_dim, w.num_q_heads, w.num_kv_heads, [int(x) for x in lens[idx]], pre))
    cases.append(("quant", 70, 3, 48, 5))
    cases.append(("quantb", 3, 48, 6, [5, 128, 0, 129, 300, 1]))

    def words(xs):
        return " ".join(str(int(x)) for x in xs)

    def text(c):
        if c[0] == "pack":
            return f"pack {c[1]} {len(c[2])} {words(c[2])}"
        if c[0] == "list":
            return f"list {words(c[1:6])} {len(c[6])} {words(c[6])} {words(c[7])}"
        if c[0] == "quant":
            return f"quant {words(c[1:])}"
        return f"quantb {words(c[1:4])} {len(c[4])} {words(c[4])}"

    inp, outp = tmp_path / "cases.txt", tmp_path / "out.bin"
    inp.write_text("\n".join(text(c) for c in cases) + "\n")
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe, str(inp), str(outp)], capture_output=True, text=True, env=env)
    assert run.returncode == 0, run.stderr[-3000:]
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr and "LeakSanitizer" not in run.stderr, run.stderr[-3000:]

    blob = outp.read_bytes()
    at = 0

    def take(n):
        nonlocal at
        piece = blob[at:at + n]
        assert len(piece) == n, "the driver wrote less than the cases call for"
        at += n
        return piece

    def take_i32():
        return struct.unpack("<i", take(4))[0]

    for c in cases:
        if c[0] == "pack":
            _, budget, lens = c
            rc, bins = take_i32(), take_i32()
            bin_of, pos = np.frombuffer(take(4 * len(lens)), np.int32), np.frombuffer(take(4 * len(lens)), np.int32)
            try:
                wb, wp, wn = va.va_pack_first_fit(lens, budget)
                assert rc == 0 and bins == wn and np.array_equal(bin_of, wb) and np.array_equal(pos, wp)
            except va.VarlenAttnError as e:
                assert rc == e.code and np.all(bin_of == -1) and np.all(pos == -1)
        elif c[0] == "list":
            _, mask, pass_id, D, Hq, Hkv, lens, prefix = c
            assert take_i32() == 0
            cu = np.frombuffer(take(4 * (len(lens) + 1)), np.int32)
            assert np.array_equal(cu, va.va_bin_layout(lens)[0])
            assert take_i32() == 0
            rc, items = take_i32(), take_i32()
            pre = None if not prefix else np.array(prefix, dtype=np.int32)
            try:
                want = va.va_build_worklist(cu, pre, mask, pass_id, D, Hq, Hkv)
                got = np.frombuffer(take(want.nbytes), np.int32).reshape(-1, 8)
                assert rc == 0 and items == want[0, 6] and np.array_equal(got, want)
            except va.VarlenAttnError as e:
                assert rc == e.code
        elif c[0] == "quant":
            _, T, H, D, seed = c
            assert take_i32() == 0
            x = np.frombuffer(take(2 * T * H * D), np.uint16)
            assert np.array_equal(x, bf16_values(T * H * D, seed))
            codes, descale = va.va_quantize_e4m3_per_head(x.reshape(T, H, D))
            assert np.array_equal(np.frombuffer(take(T * H * D), np.uint8), codes.reshape(-1))
            assert np.array_equal(np.frombuffer(take(4 * H), np.float32).view(np.uint32), descale.view(np.uint32))
        else:
            _, H, D, seed, lens = c
            cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
            T = int(cu[-1])
            assert take_i32() == 0
            x = np.frombuffer(take(2 * T * H * D), np.uint16)
            codes, descale = va.va_quantize_e4m3_blockwise(x.reshape(T, H, D), cu)
            assert np.array_equal(np.frombuffer(take(T * H * D), np.uint8), codes.reshape(-1))
            assert np.array_equal(np.frombuffer(take(4 * T * H), np.float32).view(np.uint32), descale.reshape(-1).view(np.uint32))
    assert at == len(blob)

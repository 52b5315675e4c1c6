"""Two packed streams on two HIP streams at once, launched from two host threads: the library keeps no state
between calls besides the caller's buffers (and the thread-local error string and validation bitmap), so the
results must be the bits of the same calls made one after the other."""
import threading

import numpy as np
import pytest
import torch

from paper_2603_11101_amd import binding as va
from paper_2603_11101_amd import workloads as wl

from gpu_util import DEV, to_dev_bf16

pytestmark = pytest.mark.gpu


def _case(seed, lens, Hq, Hkv, D, mode):
    cu, prefix, q, k, v, do = wl.random_stream(seed, lens, Hq, Hkv, D, prefix_frac=0.5)
    if mode == va.VA_MASK_CAUSAL:
        prefix = None
    ps = va.PackedStream(cu, prefix, mode, Hq, Hkv, D, device=DEV)
    t = {n: to_dev_bf16(x) for n, x in (("q", q), ("k", k), ("v", v), ("do", do))}
    T = int(cu[-1])
    ps.workspace()
    return ps, t, T, Hq, Hkv, D


def _buffers(T, Hq, Hkv, D):
    return {"out": torch.zeros((T, Hq, D), dtype=torch.bfloat16, device=DEV),
            "lse": torch.zeros((Hq, T), dtype=torch.float32, device=DEV),
            "dq": torch.zeros((T, Hq, D), dtype=torch.bfloat16, device=DEV),
            "dk": torch.zeros((T, Hkv, D), dtype=torch.bfloat16, device=DEV),
            "dv": torch.zeros((T, Hkv, D), dtype=torch.bfloat16, device=DEV)}


def _run(ps, t, b, scale, stream, reps):
    for _ in range(reps):
        ps.fwd(t["q"], t["k"], t["v"], scale, b["out"], b["lse"], stream=stream)
        ps.bwd(t["q"], t["k"], t["v"], b["out"], b["lse"], t["do"], scale, b["dq"], b["dk"], b["dv"], stream=stream)


def test_two_streams_from_two_threads_give_the_bits_of_sequential_calls():
    a = _case(81, [300, 77, 1, 512, 130], 8, 2, 128, va.VA_MASK_CAUSAL)
    c = _case(82, [200, 640, 64, 0, 333], 4, 1, 256, va.VA_MASK_PREFIX_LM)
    print("two streams, two threads", flush=True)
    ref = []
    for ps, t, T, Hq, Hkv, D in (a, c):
        b = _buffers(T, Hq, Hkv, D)
        _run(ps, t, b, 1.0 / np.sqrt(D), None, 1)
        torch.cuda.synchronize()
        ref.append({n: x.clone() for n, x in b.items()})
    streams = [torch.cuda.Stream(device=DEV), torch.cuda.Stream(device=DEV)]   # default priority
    bufs = [_buffers(*a[2:]), _buffers(*c[2:])]
    errors = []

    def worker(i, case):
        try:
            ps, t, T, Hq, Hkv, D = case
            _run(ps, t, bufs[i], 1.0 / np.sqrt(D), streams[i], 20)
        except Exception as exc:  # noqa: BLE001 - reported by the main thread
            errors.append(exc)

    torch.cuda.synchronize()
    threads = [threading.Thread(target=worker, args=(i, case)) for i, case in enumerate((a, c))]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    for s in streams:
        s.synchronize()
    assert not errors, errors
    for i in range(2):
        for n in ref[i]:
            assert torch.equal(ref[i][n], bufs[i][n]), (i, n)

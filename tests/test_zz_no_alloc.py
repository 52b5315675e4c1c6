"""varlen_attn_bwd_static (the backward whose scratch is a device array inside the library) against
varlen_attn_bwd with a caller's workspace: same inputs, bit-identical outputs, two calls in a row, the second
on a smaller stream, so that what the first call left in the shared array is there when the second runs."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2603_11101_amd import binding as va
from paper_2603_11101_amd import workloads as wl

from gpu_util import DEV, to_dev_bf16

pytestmark = pytest.mark.gpu


def run_both(cu, prefix, mode, Hq, Hkv, D, seed):
    lens = np.diff(cu)
    _, _, q, k, v, do = wl.random_stream(seed, [int(x) for x in lens], Hq, Hkv, D)
    T = int(cu[-1])
    scale = 1.0 / np.sqrt(D)
    ps = va.PackedStream(cu, prefix, mode, Hq, Hkv, D, device=DEV)
    tq, tk, tv, tdo = (to_dev_bf16(x) for x in (q, k, v, do))
    out = torch.empty_like(tq)
    lse = torch.empty((Hq, T), dtype=torch.float32, device=DEV)
    ps.fwd(tq, tk, tv, scale, out, lse)
    want = [torch.full_like(t, 5.0) for t in (tq, tk, tv)]
    got = [torch.full_like(t, 7.0) for t in (tq, tk, tv)]
    ps.bwd(tq, tk, tv, out, lse, tdo, scale, *want)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    ps.bwd_static(tq, tk, tv, out, lse, tdo, scale, *got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for name, g, w in zip(("dq", "dk", "dv"), got, want):
        assert torch.isfinite(w.float()).all(), name
        assert torch.equal(g, w), f"{name} differs from varlen_attn_bwd"
    return ps


def test_static_workspace_backward_matches_and_survives_a_smaller_second_call():
    # first call: 257 equal works on the 256 slots of head_dim 256, so one key tile is split and the partial-sum
    # slots of the array are used as well as its per-row part; second call: a small stream, other shapes
    print("no-alloc backward, first call (split key tile)", flush=True)
    n, L = 257, 96
    cu = np.arange(n + 1, dtype=np.int32) * L
    prefix = np.full(n, 60, dtype=np.int32)
    ps = run_both(cu, prefix, va.VA_MASK_PREFIX_LM, 8, 1, 256, seed=41)
    assert ps.worklist_host[va.VA_PASS_BWD_DKDV][1, 7] >= 1
    print("no-alloc backward, second call (smaller stream)", flush=True)
    cu2 = np.array([0, 70, 199, 240, 241], dtype=np.int32)
    run_both(cu2, None, va.VA_MASK_CAUSAL, 4, 2, 128, seed=42)


def test_static_workspace_refuses_shapes_beyond_its_size():
    # T * Hq * 8 bytes of per-row scratch alone exceed the array: refused on the host, nothing is launched
    T, Hq, Hkv, D = 1 << 20, 16, 8, 128
    shape = va.make_shape(T, 1, Hq, Hkv, D, T, va.VA_MASK_CAUSAL)
    assert va.varlen_attn_bwd_workspace_bytes(shape) > (32 << 20)
    buf = torch.zeros(4096, dtype=torch.uint8, device=DEV)
    cu = np.array([0, T], dtype=np.int32)
    rc = va._lib.varlen_attn_bwd_static(*([va._ptr(buf)] * 6), va._ptr(cu), ctypes.c_void_p(0), *([va._ptr(buf)] * 4),
                                        ctypes.byref(shape), ctypes.c_float(0.1), *([va._ptr(buf)] * 3), ctypes.c_void_p(0))
    assert rc == va.VA_ESIZE and "built-in buffer" in va.va_last_error()

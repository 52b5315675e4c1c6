"""The device calls allocate nothing and wait for nothing, so a forward + backward can be captured
into a HIP graph and replayed; every replay must reproduce the eager result of the same inputs bit
for bit (the kernels are deterministic)."""
import numpy as np
import pytest
import torch

from paper_2603_11101_amd import binding as va
from paper_2603_11101_amd import workloads as wl

from gpu_util import DEV, to_dev_bf16

pytestmark = pytest.mark.gpu


def test_forward_and_backward_replay_from_a_graph():
    Hq, Hkv, D = 4, 2, 128
    lens = [70, 129, 40, 300, 1]
    scale = 1.0 / np.sqrt(D)
    print("graph capture and replay", flush=True)
    sets = []
    for seed in (21, 22, 23):
        cu, _, q, k, v, do = wl.random_stream(seed, lens, Hq, Hkv, D)
        sets.append([to_dev_bf16(x) for x in (q, k, v, do)])
    T = int(cu[-1])
    ps = va.PackedStream(cu, None, va.VA_MASK_CAUSAL, Hq, Hkv, D, device=DEV)
    ps.workspace()
    q, k, v, do = (torch.empty_like(x) for x in sets[0])
    out, dq = torch.empty_like(q), torch.empty_like(q)
    dk, dv = torch.empty_like(k), torch.empty_like(v)
    lse = torch.empty((Hq, T), dtype=torch.float32, device=DEV)
    outputs = (out, lse, dq, dk, dv)

    def load(i):
        for dst, src in zip((q, k, v, do), sets[i]):
            dst.copy_(src)
        for t in outputs:
            t.fill_(7.0)

    def step():
        ps.fwd(q, k, v, scale, out, lse)
        ps.bwd(q, k, v, out, lse, do, scale, dq, dk, dv)

    eager = []
    for i in range(len(sets)):
        load(i)
        step()
        torch.cuda.synchronize()
        eager.append([t.clone() for t in outputs])

    graph = torch.cuda.CUDAGraph()
    load(0)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        step()
    for i in (2, 0, 1, 2, 2):
        load(i)                      # eager work and a synchronisation between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, got, want in zip(("out", "lse", "dq", "dk", "dv"), outputs, eager[i]):
            assert torch.equal(got, want), f"replay of input set {i}: {name} differs from the eager run"


def test_backward_with_a_split_key_tile_replays_from_a_graph():
    # 257 equal dK/dV works for the 256 workgroup slots of head_dim 256: one key tile is split, so the captured
    # backward holds the pieces' float32 partial sums in the workspace and the merge kernel behind the dK/dV kernel
    Hq, Hkv, D, n, L = 8, 1, 256, 257, 96
    lens = [L] * n
    scale = 1.0 / np.sqrt(D)
    print("graph capture and replay, split key tile", flush=True)
    sets = []
    for seed in (51, 52):
        cu, prefix, q, k, v, do = wl.random_stream(seed, lens, Hq, Hkv, D, prefix_frac=0.6)
        sets.append([to_dev_bf16(x) for x in (q, k, v, do)])
    cu, prefix, *_ = wl.random_stream(51, lens, Hq, Hkv, D, prefix_frac=0.6)
    T = int(cu[-1])
    ps = va.PackedStream(cu, prefix, va.VA_MASK_PREFIX_LM, Hq, Hkv, D, device=DEV)
    assert ps.worklist_host[va.VA_PASS_BWD_DKDV][1, 7] >= 1
    ps.workspace()
    q, k, v, do = (torch.empty_like(x) for x in sets[0])
    out, dq = torch.empty_like(q), torch.empty_like(q)
    dk, dv = torch.empty_like(k), torch.empty_like(v)
    lse = torch.empty((Hq, T), dtype=torch.float32, device=DEV)
    outputs = (out, lse, dq, dk, dv)

    def load(i):
        for dst, src in zip((q, k, v, do), sets[i]):
            dst.copy_(src)
        for t in outputs:
            t.fill_(7.0)
        ps.workspace().fill_(0x7F)

    def step():
        ps.fwd(q, k, v, scale, out, lse)
        ps.bwd(q, k, v, out, lse, do, scale, dq, dk, dv)

    eager = []
    for i in range(len(sets)):
        load(i)
        step()
        torch.cuda.synchronize()
        eager.append([t.clone() for t in outputs])
    graph = torch.cuda.CUDAGraph()
    load(0)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        step()
    for i in (1, 0, 1, 1):
        load(i)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, got, want in zip(("out", "lse", "dq", "dk", "dv"), outputs, eager[i]):
            assert torch.equal(got, want), f"replay of input set {i}: {name} differs from the eager run"


def test_blockwise_fp8_quantise_and_forward_replay_from_a_graph():
    # the block-wise quantiser (one kernel per tensor, block search on the device) and the FP8 forward that
    # reads its per-token-row scales: captured together, replayed on changing inputs, against eager runs
    Hq, Hkv, D = 4, 2, 128
    lens = [70, 129, 40, 300, 1]
    scale = 1.0 / np.sqrt(D)
    print("graph capture and replay, block-wise FP8", flush=True)
    sets = []
    for seed in (31, 32, 33):
        cu, _, q, k, v, _ = wl.random_stream(seed, lens, Hq, Hkv, D)
        sets.append([to_dev_bf16(x) for x in (q, k, v)])
    T = int(cu[-1])
    ps = va.PackedStream(cu, None, va.VA_MASK_CAUSAL, Hq, Hkv, D, device=DEV, passes=(va.VA_PASS_FWD,))
    cu_dev = torch.from_numpy(np.asarray(cu, dtype=np.int32)).to(DEV)
    q, k, v = (torch.empty_like(x) for x in sets[0])
    codes = [torch.empty(x.shape, dtype=torch.uint8, device=DEV) for x in (q, k, v)]
    scales = [torch.empty(x.shape[:2], dtype=torch.float32, device=DEV) for x in (q, k, v)]
    out = torch.empty((T, Hq, D), dtype=torch.bfloat16, device=DEV)
    lse = torch.empty((Hq, T), dtype=torch.float32, device=DEV)
    outputs = (out, lse, *codes, *scales)

    def load(i):
        for dst, src in zip((q, k, v), sets[i]):
            dst.copy_(src)
        for t in (out, lse, *scales):
            t.fill_(7.0)
        for t in codes:
            t.fill_(0x55)

    def step():
        for x, c, s in zip((q, k, v), codes, scales):
            va.va_quantize_e4m3_blockwise_device(x, cu, cu_dev, c, s)
        ps.fwd_fp8_blockwise(codes[0], codes[1], codes[2], scales[0], scales[1], scales[2], scale, out, lse)

    eager = []
    for i in range(len(sets)):
        load(i)
        step()
        torch.cuda.synchronize()
        eager.append([t.clone() for t in outputs])
    assert not torch.equal(eager[0][0], eager[1][0])

    graph = torch.cuda.CUDAGraph()
    load(0)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        step()
    for i in (2, 0, 1, 2, 2):
        load(i)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n, (got, want) in enumerate(zip(outputs, eager[i])):
            assert torch.equal(got, want), f"replay of input set {i}: output {n} differs from the eager run"

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

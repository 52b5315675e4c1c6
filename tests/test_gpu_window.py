"""GPU parity of the sliding-window mask (row i sees the W most recent keys, W per sample) against
the fp64 oracle: forward, backward and the FP8 forward, through the C ABI."""
import numpy as np
import pytest

from oracle import attn as oa
from paper_2603_11101_amd import binding as va
from paper_2603_11101_amd import workloads as wl

from gpu_util import (DeviceRun, TOL_FWD_ABS, TOL_FWD_REL, TOL_GRAD_REL, TOL_LSE_ABS, max_abs, rel_l2)

pytestmark = pytest.mark.gpu

MODE = va.VA_MASK_SLIDING_WINDOW
LENS = [17, 64, 95, 200, 1, 130, 0, 257, 700]
# per sample: wider than the sample; one key tile; a few keys; two and a half tiles; self only; exactly a
# tile; (empty sample); just over a tile; a band far from the first tile
WINDOWS = np.array([40, 64, 7, 150, 1, 64, 3, 65, 100], dtype=np.int32)


def check_fwd(run, ref_out, ref_lse, cu, label):
    print(f"{label}: out rel-L2 {rel_l2(run.out, ref_out):.2e} max-abs {max_abs(run.out, ref_out):.2e} "
          f"lse max-abs {max_abs(run.lse, ref_lse):.2e}", flush=True)
    assert np.isfinite(run.out).all() and np.isfinite(run.lse).all()
    assert rel_l2(run.out, ref_out) <= TOL_FWD_REL
    assert max_abs(run.out, ref_out) <= TOL_FWD_ABS
    assert max_abs(run.lse, ref_lse) <= TOL_LSE_ABS
    for s in range(len(cu) - 1):
        sl = slice(cu[s], cu[s + 1])
        if cu[s + 1] > cu[s]:
            assert rel_l2(run.out[sl], ref_out[sl]) <= TOL_FWD_REL, f"sample {s}"
    assert run.tail_untouched("out")


@pytest.mark.parametrize("Hq,Hkv,D", [(2, 2, 64), (4, 2, 128), (8, 1, 256), (4, 1, 128), (16, 1, 64), (2, 1, 256),
                                      (4, 4, 80), (2, 1, 48), (2, 2, 96), (2, 1, 160), (4, 2, 192)])
def test_window_forward_parity(Hq, Hkv, D):
    seed = Hq * 100 + D + 40
    cu, _, q, k, v, do = wl.random_stream(seed, LENS, Hq, Hkv, D)
    scale = 1.0 / np.sqrt(D)
    print(f"window forward Hq={Hq} Hkv={Hkv} D={D} seed={seed}", flush=True)
    run = DeviceRun(cu, WINDOWS, MODE, q, k, v, do, scale, backward=False)
    ref_out, ref_lse = oa.attn_fwd(q, k, v, cu, WINDOWS, scale=scale, mask_mode=oa.MASK_SLIDING_WINDOW)
    check_fwd(run, ref_out, ref_lse, cu, f"window {Hq}/{Hkv}x{D}")


def test_a_window_as_long_as_the_sample_gives_the_causal_bits():
    Hq, Hkv, D = 4, 2, 128
    lens = [100, 33, 180]
    cu, _, q, k, v, do = wl.random_stream(43, lens, Hq, Hkv, D)
    print("window >= L against causal", flush=True)
    a = DeviceRun(cu, None, va.VA_MASK_CAUSAL, q, k, v, do, 0.11, backward=False)
    b = DeviceRun(cu, np.array([100, 500, 180], dtype=np.int32), MODE, q, k, v, do, 0.11, backward=False)
    assert np.array_equal(a.out, b.out) and np.array_equal(a.lse, b.lse)


def test_window_of_one_returns_the_values():
    Hq, Hkv, D = 4, 2, 64
    lens = [70, 129]
    cu, _, q, k, v, do = wl.random_stream(44, lens, Hq, Hkv, D)
    print("window of one key", flush=True)
    run = DeviceRun(cu, np.array([1, 1], dtype=np.int32), MODE, q, k, v, do, 0.2, backward=False)
    assert np.array_equal(run.out, np.repeat(v, Hq // Hkv, axis=1))      # p = 1 exactly: O is V, bit for bit
    want_lse = 0.2 * np.einsum("thd,thd->ht", q.astype(np.float64), np.repeat(k, Hq // Hkv, axis=1).astype(np.float64))
    assert max_abs(run.lse, want_lse) <= TOL_LSE_ABS


def check_bwd(run, ref, cu, label):
    names = ("dq", "dk", "dv")
    got = (run.dq, run.dk, run.dv)
    print(label + ": " + " ".join(f"{n} rel-L2 {rel_l2(g, r):.2e}" for n, g, r in zip(names, got, ref)), flush=True)
    for n, g, r in zip(names, got, ref):
        assert np.isfinite(g).all(), n
        assert rel_l2(g, r) <= TOL_GRAD_REL, n
        for s in range(len(cu) - 1):
            sl = slice(cu[s], cu[s + 1])
            if cu[s + 1] - cu[s] > 1 and np.abs(r[sl]).max() > 0:   # a window of one key has dq = dk = 0 exactly
                assert rel_l2(g[sl], r[sl]) <= TOL_GRAD_REL, f"{n} sample {s}"
    assert run.tail_untouched("dq", "dk", "dv")


@pytest.mark.parametrize("Hq,Hkv,D", [(2, 2, 64), (4, 2, 128), (8, 1, 256), (4, 1, 128), (16, 1, 64), (2, 1, 256),
                                      (4, 4, 80), (2, 1, 48), (2, 2, 96), (2, 1, 160), (4, 2, 192)])
def test_window_backward_parity(Hq, Hkv, D):
    seed = Hq * 100 + D + 41
    cu, _, q, k, v, do = wl.random_stream(seed, LENS, Hq, Hkv, D)
    scale = 1.0 / np.sqrt(D)
    print(f"window backward Hq={Hq} Hkv={Hkv} D={D} seed={seed}", flush=True)
    run = DeviceRun(cu, WINDOWS, MODE, q, k, v, do, scale)
    ref = oa.attn_bwd(q, k, v, do, cu, WINDOWS, scale=scale, mask_mode=oa.MASK_SLIDING_WINDOW)
    check_bwd(run, ref, cu, f"window {Hq}/{Hkv}x{D}")
    # a window of one key: p = 1, so dS = dP - delta vanishes up to the float32 rounding of the two sums, whose
    # size is |dO . v| (up to about 40 at head_dim 256: half a unit in the last place is 2e-6, a few of them
    # accumulate over the k-steps), times scale * |q| (about 0.2): 5e-6 bounds it at every head dimension
    s4 = slice(cu[4], cu[5])
    assert np.abs(run.dq[s4]).max() <= 5e-6 and np.abs(run.dk[s4]).max() <= 5e-6


@pytest.mark.parametrize("Hq,Hkv,D,n,L", [(4, 4, 128, 129, 96), (4, 4, 256, 65, 96), (2, 2, 64, 129, 256)])
def test_window_backward_with_split_key_tiles(Hq, Hkv, D, n, L):
    # a few equal works more than the workgroup slots, widths drawn per sample: key tiles cut into pieces over
    # query ranges that end where the window of the tile's last key ends
    lens = [L] * n
    widths = np.random.default_rng(9 + D).integers(1, L + 1, size=n).astype(np.int32)
    cu, _, q, k, v, do = wl.random_stream(47 + D, lens, Hq, Hkv, D)
    scale = 1.0 / np.sqrt(D)
    print(f"window backward with split key tiles Hq={Hq} Hkv={Hkv} D={D} samples={n} L={L}", flush=True)
    run = DeviceRun(cu, widths, MODE, q, k, v, do, scale)
    assert run.ps.worklist_host[va.VA_PASS_BWD_DKDV][1, 7] >= 1, "this case is meant to hold a split tile"
    ref = oa.attn_bwd(q, k, v, do, cu, widths, scale=scale, mask_mode=oa.MASK_SLIDING_WINDOW)
    check_bwd(run, ref, cu, f"window split {Hq}/{Hkv}x{D}")


def test_a_window_as_long_as_the_sample_gives_the_causal_gradient_bits():
    Hq, Hkv, D = 4, 2, 128
    lens = [100, 33, 180]
    cu, _, q, k, v, do = wl.random_stream(45, lens, Hq, Hkv, D)
    print("window >= L against causal, backward", flush=True)
    a = DeviceRun(cu, None, va.VA_MASK_CAUSAL, q, k, v, do, 0.11)
    b = DeviceRun(cu, np.array([100, 500, 180], dtype=np.int32), MODE, q, k, v, do, 0.11)
    assert np.array_equal(a.dq, b.dq) and np.array_equal(a.dk, b.dk) and np.array_equal(a.dv, b.dv)


@pytest.mark.parametrize("blockwise", [False, True])
@pytest.mark.parametrize("Hq,Hkv,D", [(4, 2, 128), (8, 1, 128), (4, 2, 64), (8, 1, 256), (2, 2, 256), (8, 2, 64)])
def test_window_fp8_forward_parity(Hq, Hkv, D, blockwise):
    import torch
    from oracle import e4m3 as oe
    from gpu_util import DEV, TOL_FP8_REL, from_dev_bf16
    cu, _, q, k, v, _ = wl.random_stream(46 + Hq, LENS, Hq, Hkv, D)
    T = int(cu[-1])
    scale = 1.0 / np.sqrt(D)
    print(f"window fp8 forward Hq={Hq} Hkv={Hkv} D={D} blockwise={blockwise}", flush=True)
    ps = va.PackedStream(cu, WINDOWS, MODE, Hq, Hkv, D, device=DEV, passes=(va.VA_PASS_FWD,))
    out = torch.full((T + 2, Hq, D), 768.0, dtype=torch.bfloat16, device=DEV)
    lse = torch.empty((Hq, T), dtype=torch.float32, device=DEV)
    if blockwise:
        quant = [va.va_quantize_e4m3_blockwise(wl.bf16_bits(x), cu) for x in (q, k, v)]
        deq = []
        for x, (codes, d_tok) in zip((q, k, v), quant):
            oc, od = oe.quantize_blockwise(x, cu)
            assert np.array_equal(codes, oc)
            deq.append(oe.dequantize_blockwise(oc, od, cu).astype(np.float32))
        args = [torch.from_numpy(c).to(DEV) for c, _ in quant] + [torch.from_numpy(d).to(DEV) for _, d in quant]
        ps.fwd_fp8_blockwise(*args, scale, out, lse)
    else:
        quant = [va.va_quantize_e4m3_per_head(wl.bf16_bits(x)) for x in (q, k, v)]
        deq = [oe.dequantize_per_head(c, d).astype(np.float32) for c, d in quant]
        args = [torch.from_numpy(c).to(DEV) for c, _ in quant] + [torch.from_numpy(d).to(DEV) for _, d in quant]
        ps.fwd_fp8(*args, scale, out, lse)
    torch.cuda.synchronize()
    got = from_dev_bf16(out)
    assert np.all(got[T:] == 768.0)
    got, lse = got[:T], lse.cpu().numpy().astype(np.float64)
    ref_out, ref_lse = oa.attn_fwd(*deq, cu, WINDOWS, scale=scale, mask_mode=oa.MASK_SLIDING_WINDOW)
    print(f"  out rel-L2 {rel_l2(got, ref_out):.2e} lse max-abs {max_abs(lse, ref_lse):.2e}", flush=True)
    assert np.isfinite(got).all() and np.isfinite(lse).all()
    assert rel_l2(got, ref_out) <= TOL_FP8_REL and max_abs(lse, ref_lse) <= TOL_LSE_ABS
    for s in range(len(LENS)):
        if LENS[s]:
            sl = slice(cu[s], cu[s + 1])
            assert rel_l2(got[sl], ref_out[sl]) <= TOL_FP8_REL, f"sample {s}"

"""GPU parity of the bf16 backward (delta, dK/dV, dQ kernels) against the fp64
oracle, element by element, through the C ABI."""
import numpy as np
import pytest

from oracle import attn as oa
from paper_2603_11101_amd import binding as va
from paper_2603_11101_amd import workloads as wl

from gpu_util import DeviceRun, TOL_FWD_REL, TOL_GRAD_REL, TOL_LSE_ABS, max_abs, rel_l2

pytestmark = pytest.mark.gpu

MODES = {va.VA_MASK_CAUSAL: oa.MASK_CAUSAL, va.VA_MASK_PREFIX_LM: oa.MASK_PREFIX_BIDIR_SUFFIX,
         va.VA_MASK_PREFIX_LM_CAUSAL: oa.MASK_PREFIX_CAUSAL_SUFFIX, va.VA_MASK_THREE_BLOCK: oa.MASK_THREE_BLOCK}


def check_bwd(run, ref, cu, label):
    names = ("dq", "dk", "dv")
    got = (run.dq, run.dk, run.dv)
    print(label + ": " + " ".join(f"{n} rel-L2 {rel_l2(g, r):.2e}" for n, g, r in zip(names, got, ref)), flush=True)
    for n, g, r in zip(names, got, ref):
        assert rel_l2(g, r) <= TOL_GRAD_REL, n
        for s in range(len(cu) - 1):
            sl = slice(cu[s], cu[s + 1])
            if cu[s + 1] - cu[s] > 1:      # single-token samples have dq = dk = 0 exactly: no relative error
                assert rel_l2(g[sl], r[sl]) <= TOL_GRAD_REL, f"{n} sample {s}"
    assert run.tail_untouched("dq", "dk", "dv")


def test_tiny_workload_backward():
    w = wl.WORKLOADS["tiny"]
    lens, _ = wl.sample_lengths("tiny")
    cu, _, mx = va.va_bin_layout(lens)
    q, k, v, do = wl.tensor_values(w.seed, int(cu[-1]), w.num_q_heads, w.num_kv_heads, w.head_dim)
    scale = 1.0 / np.sqrt(w.head_dim)
    print("tiny backward", flush=True)
    run = DeviceRun(cu, None, va.VA_MASK_CAUSAL, q, k, v, do, scale)
    check_bwd(run, oa.attn_bwd(q, k, v, do, cu, None, scale=scale), cu, "tiny")


LENS = [17, 64, 95, 200, 1, 130, 0, 257]


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("Hq,Hkv,D", [(2, 2, 64), (4, 2, 128), (8, 1, 256), (4, 1, 128), (6, 2, 64), (16, 1, 64), (2, 1, 256), (4, 4, 80), (4, 1, 80), (2, 1, 48), (2, 2, 96), (2, 1, 160), (4, 2, 192)])
def test_backward_parity(mode, Hq, Hkv, D):
    seed = Hq * 100 + D + mode
    cu, prefix, q, k, v, do = wl.random_stream(seed, LENS, Hq, Hkv, D, prefix_frac=-1.0)
    if mode == va.VA_MASK_CAUSAL:
        prefix = None
    elif mode == va.VA_MASK_THREE_BLOCK:
        prefix = wl.random_block_ends(seed, LENS)
        prefix[3], prefix[7], prefix[5] = (200, 200), (0, 0), (0, 130)   # one block only, three ways
    else:
        prefix[3], prefix[7] = 200, 0
    scale = 1.0 / np.sqrt(D)
    print(f"backward parity mode={mode} Hq={Hq} Hkv={Hkv} D={D} seed={seed}", flush=True)
    run = DeviceRun(cu, prefix, mode, q, k, v, do, scale)
    ref = oa.attn_bwd(q, k, v, do, cu, prefix, scale=scale, mask_mode=MODES[mode])
    check_bwd(run, ref, cu, f"mode {mode} {Hq}/{Hkv}x{D}")
    # single-token sample (index 4): dQ = dK = 0 up to float32 summation noise in (dP - delta), and
    # dV = sum of dO over the group, up to bf16 rounding
    t = cu[4]
    assert np.abs(run.dq[t]).max() < 1e-4 and np.abs(run.dk[t]).max() < 1e-4
    G = Hq // Hkv
    want = do[t].astype(np.float64).reshape(Hkv, G, D).sum(axis=1)
    assert np.allclose(run.dv[t], want, rtol=2.0 ** -8, atol=1e-6)


def test_backward_packing_invariance_no_leak_and_determinism():
    Hq, Hkv, D = 4, 2, 128
    lens = [70, 129, 40]
    cu, _, q, k, v, do = wl.random_stream(4, lens, Hq, Hkv, D)
    scale = 1.0 / np.sqrt(D)
    print("backward packing invariance", flush=True)
    full = DeviceRun(cu, None, va.VA_MASK_CAUSAL, q, k, v, do, scale)
    again = DeviceRun(cu, None, va.VA_MASK_CAUSAL, q, k, v, do, scale)
    for n in ("dq", "dk", "dv"):
        assert np.array_equal(getattr(full, n), getattr(again, n))
    for s, L in enumerate(lens):
        sl = slice(cu[s], cu[s + 1])
        one = DeviceRun(np.array([0, L], dtype=np.int32), None, va.VA_MASK_CAUSAL, q[sl], k[sl], v[sl], do[sl], scale)
        for n in ("dq", "dk", "dv"):
            assert np.array_equal(getattr(one, n), getattr(full, n)[sl]), (n, s)
    q2, k2, v2, do2 = q.copy(), k.copy(), v.copy(), do.copy()
    bad = slice(cu[1], cu[2])
    q2[bad], k2[bad], v2[bad], do2[bad] = np.nan, np.inf, np.nan, np.nan
    poisoned = DeviceRun(cu, None, va.VA_MASK_CAUSAL, q2, k2, v2, do2, scale)
    keep = np.r_[0:cu[1], cu[2]:cu[3]]
    for n in ("dq", "dk", "dv"):
        assert np.array_equal(getattr(poisoned, n)[keep], getattr(full, n)[keep]), n


@pytest.mark.parametrize("Hq,Hkv,D", [(4, 2, 128), (8, 1, 64)])
def test_many_tiny_samples_forward_and_backward(Hq, Hkv, D):
    # thousands of works of one or two tiles each: every persistent workgroup switches works many times,
    # so descriptors fetched ahead, the wait that lets output rows drain and the cross-work prefetch all
    # run back to back; lengths 1..70 also put a ragged block at almost every switch
    rng = np.random.default_rng(5 + D)
    lens = rng.integers(1, 71, size=1600)
    lens[::97] = 0                                   # empty samples in between
    cu, _, q, k, v, do = wl.random_stream(11 + D, [int(x) for x in lens], Hq, Hkv, D)
    scale = 1.0 / np.sqrt(D)
    print(f"many tiny samples Hq={Hq} Hkv={Hkv} D={D} T={int(cu[-1])}", flush=True)
    run = DeviceRun(cu, None, va.VA_MASK_CAUSAL, q, k, v, do, scale)
    ref_out, ref_lse = oa.attn_fwd(q, k, v, cu, None, scale=scale)
    assert rel_l2(run.out, ref_out) <= TOL_FWD_REL and max_abs(run.lse, ref_lse) <= TOL_LSE_ABS
    ref = oa.attn_bwd(q, k, v, do, cu, None, scale=scale)
    for n, g, r in zip(("dq", "dk", "dv"), (run.dq, run.dk, run.dv), ref):
        print(f"  {n} rel-L2 {rel_l2(g, r):.2e}", flush=True)
        assert rel_l2(g, r) <= TOL_GRAD_REL, n
    # per sample as well: with 1600 samples a wrong one would vanish in the global norm
    worst = 0.0
    for s in range(len(lens)):
        sl = slice(cu[s], cu[s + 1])
        if cu[s + 1] > cu[s]:
            worst = max(worst, rel_l2(run.out[sl], ref_out[sl]), rel_l2(run.dq[sl], ref[0][sl]),
                        rel_l2(run.dk[sl], ref[1][sl]), rel_l2(run.dv[sl], ref[2][sl]))
    print(f"  worst per-sample rel-L2 over all samples and tensors {worst:.2e}", flush=True)
    assert worst <= TOL_GRAD_REL
    assert run.tail_untouched("out") and run.tail_untouched("dq") and run.tail_untouched("dk")


@pytest.mark.parametrize("trial", range(8))
def test_random_configurations_forward_and_backward(trial):
    # shapes, head groupings, masks and block ends drawn together, so that combinations the fixed
    # cases above do not pair up are met as well (zero-length samples and one-block samples included)
    r = np.random.default_rng(4000 + trial)
    Hkv = int(r.choice([1, 2, 3]))
    G = int(r.choice([1, 2, 3, 4, 8]))
    D = int(r.choice([48, 64, 80, 96, 128, 160, 192, 256]))
    mode = int(r.choice(list(MODES)))
    lens = [int(x) for x in r.choice([0, 1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 190, 300, 450], size=int(r.integers(2, 7)))]
    if sum(lens) == 0:
        lens.append(77)
    cu, prefix, q, k, v, do = wl.random_stream(5000 + trial, lens, G * Hkv, Hkv, D, prefix_frac=-1.0)
    if mode == va.VA_MASK_CAUSAL:
        prefix = None
    elif mode == va.VA_MASK_THREE_BLOCK:
        prefix = wl.random_block_ends(5000 + trial, lens)
    scale = float(r.choice([1.0 / np.sqrt(D), 0.05, 0.2]))
    print(f"random configuration {trial}: mode={mode} Hq={G * Hkv} Hkv={Hkv} D={D} lens={lens} scale={scale:.3f}", flush=True)
    run = DeviceRun(cu, prefix, mode, q, k, v, do, scale)
    ref_out, ref_lse = oa.attn_fwd(q, k, v, cu, prefix, scale=scale, mask_mode=MODES[mode])
    assert rel_l2(run.out, ref_out) <= TOL_FWD_REL and max_abs(run.lse, ref_lse) <= TOL_LSE_ABS
    check_bwd(run, oa.attn_bwd(q, k, v, do, cu, prefix, scale=scale, mask_mode=MODES[mode]), cu, f"random {trial}")
    assert run.tail_untouched("out")


@pytest.mark.parametrize("D", [48, 64, 80, 96, 128, 160, 192, 256])
@pytest.mark.parametrize("G", [1, 2, 4, 8])
def test_every_head_dimension_with_every_head_stacking(D, G):
    # The forward and dQ kernels are instantiated per (head dimension, query heads stacked in a block of rows:
    # 1, 2, 4 or 8 = the group size here): each of the 32 once, forward and backward, the mask cycling with the case.
    Hkv = 2 if G <= 2 else 1
    mode = list(MODES)[(D // 16 + G) % len(MODES)]
    lens = [70, 0, 129, 33, 200]
    seed = 7000 + 10 * D + G
    cu, prefix, q, k, v, do = wl.random_stream(seed, lens, G * Hkv, Hkv, D, prefix_frac=-1.0)
    if mode == va.VA_MASK_CAUSAL:
        prefix = None
    elif mode == va.VA_MASK_THREE_BLOCK:
        prefix = wl.random_block_ends(seed, lens)
    scale = 1.0 / np.sqrt(D)
    print(f"head_dim {D}, {G} heads per KV head ({Hkv} KV heads), mode={mode}", flush=True)
    run = DeviceRun(cu, prefix, mode, q, k, v, do, scale)
    ref_out, ref_lse = oa.attn_fwd(q, k, v, cu, prefix, scale=scale, mask_mode=MODES[mode])
    assert rel_l2(run.out, ref_out) <= TOL_FWD_REL and max_abs(run.lse, ref_lse) <= TOL_LSE_ABS
    check_bwd(run, oa.attn_bwd(q, k, v, do, cu, prefix, scale=scale, mask_mode=MODES[mode]), cu, f"D={D} G={G}")
    assert run.tail_untouched("out")


@pytest.mark.parametrize("mode,Hq,Hkv,D", [(va.VA_MASK_CAUSAL, 4, 2, 128), (va.VA_MASK_PREFIX_LM, 2, 1, 64),
                                           (va.VA_MASK_CAUSAL, 2, 2, 256)])
def test_peaked_softmax_with_a_rising_row_maximum(mode, Hq, Hkv, D):
    # Scores with a standard deviation of about 8 whose size grows along the sample: the running maximum
    # of a row moves up by many units from one key tile to the next, so the reference point of the
    # exponentials has to follow every time, and nearly all of a row's weight sits on a few keys.
    lens = [330, 70, 200]
    cu, prefix, q, k, v, do = wl.random_stream(91 + D, lens, Hq, Hkv, D, prefix_frac=0.4)
    if mode == va.VA_MASK_CAUSAL:
        prefix = None
    ramp = np.concatenate([1.0 + 3.0 * np.arange(L) / L for L in lens]).astype(np.float32)
    k = wl.round_to_bf16(k * ramp[:, None, None])
    scale = 8.0 / np.sqrt(D) / 2.5
    print(f"peaked softmax mode={mode} Hq={Hq} Hkv={Hkv} D={D}", flush=True)
    run = DeviceRun(cu, prefix, mode, q, k, v, do, scale)
    ref_out, ref_lse = oa.attn_fwd(q, k, v, cu, prefix, scale=scale, mask_mode=MODES[mode])
    print(f"  largest |LSE| {np.abs(ref_lse).max():.1f}; out rel-L2 {rel_l2(run.out, ref_out):.2e} "
          f"lse max-abs {max_abs(run.lse, ref_lse):.2e}", flush=True)
    assert np.isfinite(run.out).all() and np.isfinite(run.lse).all()
    assert rel_l2(run.out, ref_out) <= TOL_FWD_REL
    # float32 LSE of magnitude ~50 carries 4e-6 of rounding per operation; the bound stays the stated one
    assert max_abs(run.lse, ref_lse) <= TOL_LSE_ABS
    check_bwd(run, oa.attn_bwd(q, k, v, do, cu, prefix, scale=scale, mask_mode=MODES[mode]), cu, "peaked")


@pytest.mark.parametrize("mode,Hq,Hkv,n,L,D", [
    (va.VA_MASK_CAUSAL, 4, 4, 65, 64, 256), (va.VA_MASK_PREFIX_LM, 8, 1, 257, 96, 256),
    (va.VA_MASK_CAUSAL, 4, 4, 129, 64, 128), (va.VA_MASK_PREFIX_LM, 8, 4, 129, 96, 128), (va.VA_MASK_CAUSAL, 4, 4, 65, 256, 64),
    (va.VA_MASK_CAUSAL, 4, 4, 129, 96, 80), (va.VA_MASK_PREFIX_LM_CAUSAL, 2, 2, 129, 256, 48), (va.VA_MASK_CAUSAL, 4, 4, 65, 96, 160),
    (va.VA_MASK_PREFIX_LM, 2, 2, 129, 64, 192), (va.VA_MASK_CAUSAL, 2, 2, 257, 128, 96),
    (va.VA_MASK_THREE_BLOCK, 4, 4, 65, 96, 256), (va.VA_MASK_THREE_BLOCK, 4, 2, 257, 96, 128)])
def test_split_key_tiles_against_the_oracle(mode, Hq, Hkv, n, L, D):
    # A few equal works more than the workgroup slots of the head dimension (256 at 256, else 512): the host cuts
    # the query tiles of the last key tiles into pieces, their workgroups write float32 partial sums into the
    # workspace and the merge kernel (one instantiation per head dimension) adds them.  Every sample against the
    # oracle, and twice for determinism.
    lens = [L] * n
    cu, prefix, q, k, v, do = wl.random_stream(300 + n, lens, Hq, Hkv, D, prefix_frac=0.6)
    if mode == va.VA_MASK_CAUSAL:
        prefix = None
    elif mode == va.VA_MASK_THREE_BLOCK:
        prefix = wl.random_block_ends(300 + n, lens)
    scale = 1.0 / np.sqrt(D)
    print(f"split key tiles mode={mode} Hq={Hq} Hkv={Hkv} samples={n} L={L} D={D}", flush=True)
    run = DeviceRun(cu, prefix, mode, q, k, v, do, scale)
    dkdv_list = run.ps.worklist_host[va.VA_PASS_BWD_DKDV]
    assert dkdv_list[1, 7] >= 1, "this case is meant to hold a split tile"
    print(f"  {int(dkdv_list[1, 7])} split tile(s), {int((va.worklist_items(dkdv_list)[:, 1] >> 8 > 0).sum())} pieces", flush=True)
    ref = oa.attn_bwd(q, k, v, do, cu, prefix, scale=scale, mask_mode=MODES[mode])
    check_bwd(run, ref, cu, "split")
    again = DeviceRun(cu, prefix, mode, q, k, v, do, scale)
    for name in ("dq", "dk", "dv"):
        assert np.array_equal(getattr(run, name), getattr(again, name)), name


@pytest.mark.parametrize("Hq,Hkv,D", [(4, 2, 128), (8, 1, 256)])
def test_backward_by_stages_equals_the_whole_backward(Hq, Hkv, D):
    # varlen_attn_bwd_stages: dQ alone (frozen keys and values), then dK/dV alone reading what the first call
    # left in the workspace, give the bits of varlen_attn_bwd; outputs of stages not selected stay untouched
    import torch
    from gpu_util import DEV, to_dev_bf16
    lens = [70, 129, 40, 300, 1]
    cu, _, q, k, v, do = wl.random_stream(80 + D, lens, Hq, Hkv, D)
    scale = 1.0 / np.sqrt(D)
    T = int(cu[-1])
    print(f"backward by stages Hq={Hq} Hkv={Hkv} D={D}", flush=True)
    ps = va.PackedStream(cu, None, va.VA_MASK_CAUSAL, Hq, Hkv, D, device=DEV)
    tq, tk, tv, tdo = (to_dev_bf16(x) for x in (q, k, v, do))
    out, lse = torch.empty_like(tq), torch.empty((Hq, T), dtype=torch.float32, device=DEV)
    ps.fwd(tq, tk, tv, scale, out, lse)
    want = [torch.empty_like(t) for t in (tq, tk, tv)]
    ps.bwd(tq, tk, tv, out, lse, tdo, scale, *want)
    torch.cuda.synchronize()
    ps.workspace().fill_(0xFF)                      # nothing of the whole backward's scratch may be relied upon
    got = [torch.full_like(t, 3.0) for t in (tq, tk, tv)]
    first = va.VA_BWD_STAGE_DQ | (va.VA_BWD_STAGE_DELTA if va.va_bwd_has_delta_kernel(D) else 0)
    ps.bwd_stages(tq, tk, tv, out, lse, tdo, scale, *got, first)
    torch.cuda.synchronize()
    assert torch.equal(got[0], want[0]) and torch.all(got[1] == 3.0) and torch.all(got[2] == 3.0)
    got[0].fill_(3.0)
    ps.bwd_stages(tq, tk, tv, out, lse, tdo, scale, *got, va.VA_BWD_STAGE_DKDV)
    torch.cuda.synchronize()
    assert torch.all(got[0] == 3.0) and torch.equal(got[1], want[1]) and torch.equal(got[2], want[2])
    with pytest.raises(va.VarlenAttnError) as e:
        ps.bwd_stages(tq, tk, tv, out, lse, tdo, scale, *got, 0)
    assert e.value.code == va.VA_EINVAL
    with pytest.raises(va.VarlenAttnError) as e:
        ps.bwd_stages(tq, tk, tv, out, lse, tdo, scale, *got, 8)
    assert e.value.code == va.VA_EINVAL

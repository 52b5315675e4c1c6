"""GPU parity of the bf16 forward against the fp64 oracle, element by element,
through the C ABI.  Sizes are small enough for the oracle to finish in seconds
and still span several query/key tiles with ragged tails."""
import numpy as np
import pytest

from oracle import attn as oa
from paper_2603_11101_amd import binding as va
from paper_2603_11101_amd import workloads as wl

from gpu_util import DeviceRun, TOL_FWD_ABS, TOL_FWD_REL, TOL_LSE_ABS, max_abs, rel_l2

pytestmark = pytest.mark.gpu

MODES = {va.VA_MASK_CAUSAL: oa.MASK_CAUSAL, va.VA_MASK_PREFIX_LM: oa.MASK_PREFIX_BIDIR_SUFFIX,
         va.VA_MASK_PREFIX_LM_CAUSAL: oa.MASK_PREFIX_CAUSAL_SUFFIX, va.VA_MASK_THREE_BLOCK: oa.MASK_THREE_BLOCK}


def check_fwd(run, ref_out, ref_lse, cu, label):
    print(f"{label}: out rel-L2 {rel_l2(run.out, ref_out):.2e} max-abs {max_abs(run.out, ref_out):.2e} "
          f"lse max-abs {max_abs(run.lse, ref_lse):.2e}", flush=True)
    assert rel_l2(run.out, ref_out) <= TOL_FWD_REL
    assert max_abs(run.out, ref_out) <= TOL_FWD_ABS
    assert max_abs(run.lse, ref_lse) <= TOL_LSE_ABS
    for s in range(len(cu) - 1):          # per sample, so a bad short sample cannot hide behind long ones
        sl = slice(cu[s], cu[s + 1])
        if cu[s + 1] > cu[s]:
            assert rel_l2(run.out[sl], ref_out[sl]) <= TOL_FWD_REL, f"sample {s}"
    assert run.tail_untouched("out")


def test_tiny_workload_forward():
    w = wl.WORKLOADS["tiny"]
    lens, _ = wl.sample_lengths("tiny")
    cu, _, mx = va.va_bin_layout(lens)
    q, k, v, do = wl.tensor_values(w.seed, int(cu[-1]), w.num_q_heads, w.num_kv_heads, w.head_dim)
    scale = 1.0 / np.sqrt(w.head_dim)
    print("tiny forward", flush=True)
    run = DeviceRun(cu, None, va.VA_MASK_CAUSAL, q, k, v, do, scale, backward=False)
    ref_out, ref_lse = oa.attn_fwd(q, k, v, cu, None, scale=scale)
    check_fwd(run, ref_out, ref_lse, cu, "tiny")


LENS = [17, 64, 95, 200, 1, 130, 0, 257]


@pytest.mark.parametrize("mode", list(MODES))
@pytest.mark.parametrize("Hq,Hkv,D", [(2, 2, 64), (4, 2, 128), (8, 1, 256), (4, 1, 128), (6, 2, 64), (16, 1, 64), (2, 1, 256), (4, 4, 80), (4, 1, 80), (2, 1, 48), (2, 2, 96), (2, 1, 160), (4, 2, 192)])
def test_forward_parity(mode, Hq, Hkv, D):
    seed = Hq * 100 + D + mode
    cu, prefix, q, k, v, do = wl.random_stream(seed, LENS, Hq, Hkv, D, prefix_frac=-1.0)
    if mode == va.VA_MASK_CAUSAL:
        prefix = None
    elif mode == va.VA_MASK_THREE_BLOCK:
        prefix = wl.random_block_ends(seed, LENS)
        prefix[3], prefix[7], prefix[5] = (200, 200), (0, 0), (0, 130)   # one block only, three ways
    else:
        prefix[3], prefix[7] = 200, 0       # whole sample prefix / empty prefix
    scale = 1.0 / np.sqrt(D)
    print(f"forward parity mode={mode} Hq={Hq} Hkv={Hkv} D={D} seed={seed}", flush=True)
    run = DeviceRun(cu, prefix, mode, q, k, v, do, scale, backward=False)
    ref_out, ref_lse = oa.attn_fwd(q, k, v, cu, prefix, scale=scale, mask_mode=MODES[mode])
    check_fwd(run, ref_out, ref_lse, cu, f"mode {mode} {Hq}/{Hkv}x{D}")


def test_forward_does_not_depend_on_max_seqlen_slack_and_is_deterministic():
    Hq, Hkv, D = 4, 2, 128
    cu, prefix, q, k, v, do = wl.random_stream(3, [100, 33, 180], Hq, Hkv, D)
    scale = 0.11
    print("max_seqlen slack / determinism", flush=True)
    a = DeviceRun(cu, None, va.VA_MASK_CAUSAL, q, k, v, do, scale, max_seqlen=180, backward=False)
    b = DeviceRun(cu, None, va.VA_MASK_CAUSAL, q, k, v, do, scale, max_seqlen=360, backward=False)
    assert np.array_equal(a.out, b.out) and np.array_equal(a.lse, b.lse)


def test_forward_packing_invariance_and_no_leak_on_gpu():
    # each sample alone gives the same bits as inside the packed stream, and NaN/Inf in one
    # sample (and in the rows beyond T) never reaches another
    Hq, Hkv, D = 4, 2, 128
    lens = [70, 129, 40]
    cu, _, q, k, v, do = wl.random_stream(4, lens, Hq, Hkv, D)
    scale = 1.0 / np.sqrt(D)
    print("packing invariance", flush=True)
    full = DeviceRun(cu, None, va.VA_MASK_CAUSAL, q, k, v, do, scale, backward=False)
    for s, L in enumerate(lens):
        sl = slice(cu[s], cu[s + 1])
        one = DeviceRun(np.array([0, L], dtype=np.int32), None, va.VA_MASK_CAUSAL, q[sl], k[sl], v[sl], do[sl], scale,
                     backward=False)
        assert np.array_equal(one.out, full.out[sl]) and np.array_equal(one.lse, full.lse[:, sl])
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    bad = slice(cu[1], cu[2])
    q2[bad], k2[bad], v2[bad] = np.nan, np.inf, np.nan
    poisoned = DeviceRun(cu, None, va.VA_MASK_CAUSAL, q2, k2, v2, do, scale, backward=False)
    keep = np.r_[0:cu[1], cu[2]:cu[3]]
    assert np.array_equal(poisoned.out[keep], full.out[keep]) and np.array_equal(poisoned.lse[:, keep], full.lse[:, keep])


@pytest.mark.parametrize("mode,Hq,Hkv,D", [(va.VA_MASK_CAUSAL, 4, 2, 128), (va.VA_MASK_PREFIX_LM, 8, 1, 256),
                                           (va.VA_MASK_PREFIX_LM_CAUSAL, 2, 2, 64), (va.VA_MASK_SLIDING_WINDOW, 4, 1, 128)])
def test_zero_queries_give_the_mean_of_the_visible_values(mode, Hq, Hkv, D):
    # Q = 0: every score is 0, the softmax is uniform over the keys a row sees, so O is the plain mean of their V
    # rows and LSE = ln(their number) -- closed forms written here from the mask definition, no oracle involved.
    # The gradient of K is then exactly zero (dS is multiplied by Q = 0).
    lens = [1, 70, 129, 300]
    cu, prefix, q, k, v, do = wl.random_stream(31 + D, lens, Hq, Hkv, D, prefix_frac=0.4)
    q[:] = 0.0
    if mode == va.VA_MASK_CAUSAL:
        prefix = None
    elif mode == va.VA_MASK_SLIDING_WINDOW:
        prefix = np.array([1, 16, 200, 65], dtype=np.int32)
    print(f"zero queries mode={mode} Hq={Hq} Hkv={Hkv} D={D}", flush=True)
    run = DeviceRun(cu, prefix, mode, q, k, v, do, 0.3)
    G = Hq // Hkv
    for s, L in enumerate(lens):
        c = int(cu[s])
        for i in range(L):
            if mode == va.VA_MASK_CAUSAL:
                lo, hi = 0, i + 1
            elif mode == va.VA_MASK_PREFIX_LM:
                lo, hi = 0, (int(prefix[s]) if i < prefix[s] else L)
            elif mode == va.VA_MASK_PREFIX_LM_CAUSAL:
                lo, hi = 0, (int(prefix[s]) if i < prefix[s] else i + 1)
            else:
                lo, hi = max(0, i + 1 - int(prefix[s])), i + 1
            want = v[c + lo:c + hi].astype(np.float64).mean(axis=0)          # [Hkv, D]
            got = run.out[c + i].reshape(Hkv, G, D)
            # bf16 P (1/n rounded) and bf16 output rounding: 2^-8 relative to the largest value averaged
            tol = 2.0 ** -7 * np.abs(v[c + lo:c + hi]).max() + 1e-6
            assert np.abs(got - want[:, None, :]).max() <= tol, (s, i)
            assert np.abs(run.lse[:, c + i] - np.log(hi - lo)).max() <= 1e-5, (s, i)
    assert np.all(run.dk == 0.0)
    assert run.tail_untouched("out", "dq", "dk", "dv")

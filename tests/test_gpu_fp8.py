"""GPU parity of the FP8 (E4M3) forward against the fp64 oracle run on the
dequantised inputs.  Quantised codes and descales must equal the oracle
quantiser's bit for bit; the attention output must be within rel-L2 5e-2
(the requantisation of the probabilities is not modelled by the oracle)."""
import numpy as np
import pytest
import torch

from oracle import attn as oa
from oracle import e4m3 as oe
from paper_2603_11101_amd import binding as va
from paper_2603_11101_amd import workloads as wl

from gpu_util import DEV, TOL_FP8_REL, TOL_LSE_ABS, from_dev_bf16, max_abs, rel_l2

pytestmark = pytest.mark.gpu


def run_fp8(cu, prefix, mode, q, k, v, scale):
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    q8, qd = va.va_quantize_e4m3_per_head(wl.bf16_bits(q))
    k8, kd = va.va_quantize_e4m3_per_head(wl.bf16_bits(k))
    v8, vd = va.va_quantize_e4m3_per_head(wl.bf16_bits(v))
    for x, codes, ds in ((q, q8, qd), (k, k8, kd), (v, v8, vd)):
        oc, od = oe.quantize_per_head(x)
        assert np.array_equal(codes, oc) and np.array_equal(ds, od)      # bit-exact quantiser
    ps = va.PackedStream(cu, prefix, mode, Hq, Hkv, D, device=DEV, passes=(va.VA_PASS_FWD,))
    out = torch.full((T + 2, Hq, D), 768.0, dtype=torch.bfloat16, device=DEV)
    lse = torch.empty((Hq, T), dtype=torch.float32, device=DEV)
    pad = np.full((2,) + q8.shape[1:], 0x7F, dtype=np.uint8)            # NaN codes beyond T
    padk = np.full((2,) + k8.shape[1:], 0x7F, dtype=np.uint8)
    tq = torch.from_numpy(np.concatenate([q8, pad])).to(DEV)
    tk = torch.from_numpy(np.concatenate([k8, padk])).to(DEV)
    tv = torch.from_numpy(np.concatenate([v8, padk])).to(DEV)
    ps.fwd_fp8(tq, tk, tv, torch.from_numpy(qd).to(DEV), torch.from_numpy(kd).to(DEV), torch.from_numpy(vd).to(DEV),
               scale, out, lse)
    torch.cuda.synchronize()
    got = from_dev_bf16(out)
    assert np.all(got[T:] == 768.0)
    deq = [oe.dequantize_per_head(c, d).astype(np.float32) for c, d in ((q8, qd), (k8, kd), (v8, vd))]
    return got[:T], lse.cpu().numpy().astype(np.float64), deq


@pytest.mark.parametrize("D", [128, 64, 256])
@pytest.mark.parametrize("mode,Hq,Hkv", [(va.VA_MASK_CAUSAL, 4, 2), (va.VA_MASK_PREFIX_LM, 8, 1), (va.VA_MASK_CAUSAL, 2, 2),
                                         (va.VA_MASK_PREFIX_LM_CAUSAL, 4, 1), (va.VA_MASK_THREE_BLOCK, 4, 2)])
def test_fp8_forward_parity(mode, Hq, Hkv, D):
    lens = [17, 64, 95, 200, 1, 130, 0, 257]
    cu, prefix, q, k, v, _ = wl.random_stream(50 + Hq + mode + D, lens, Hq, Hkv, D, prefix_frac=-1.0)
    if mode == va.VA_MASK_CAUSAL:
        prefix = None
    elif mode == va.VA_MASK_THREE_BLOCK:
        prefix = wl.random_block_ends(50 + Hq, lens)
    scale = 1.0 / np.sqrt(D)
    print(f"fp8 forward mode={mode} Hq={Hq} Hkv={Hkv} D={D}", flush=True)
    out, lse, (qd, kd, vd) = run_fp8(cu, prefix, mode, q, k, v, scale)
    omode = {va.VA_MASK_CAUSAL: oa.MASK_CAUSAL, va.VA_MASK_PREFIX_LM: oa.MASK_PREFIX_BIDIR_SUFFIX,
             va.VA_MASK_PREFIX_LM_CAUSAL: oa.MASK_PREFIX_CAUSAL_SUFFIX, va.VA_MASK_THREE_BLOCK: oa.MASK_THREE_BLOCK}[mode]
    ref_out, ref_lse = oa.attn_fwd(qd, kd, vd, cu, prefix, scale=scale, mask_mode=omode)
    print(f"  out rel-L2 {rel_l2(out, ref_out):.2e} max-abs {max_abs(out, ref_out):.2e} lse max-abs {max_abs(lse, ref_lse):.2e}",
          flush=True)
    assert rel_l2(out, ref_out) <= TOL_FP8_REL
    assert max_abs(lse, ref_lse) <= TOL_LSE_ABS
    for s in range(len(lens)):
        if lens[s]:
            sl = slice(cu[s], cu[s + 1])
            assert rel_l2(out[sl], ref_out[sl]) <= TOL_FP8_REL, f"sample {s}"


def test_fp8_uniform_keys_is_exact_for_power_of_two_counts():
    # every key equal: p = 1 / (i + 1); for rows where i + 1 is a power of two, p * 2^8 is exactly
    # representable in E4M3, so O is the exact mean of the (quantised) values up to bf16 rounding
    for D in (128, 64, 256):
        Hq, Hkv, L = 2, 1, 64
        cu, _, q, k, v, _ = wl.random_stream(60 + D, [L], Hq, Hkv, D)
        k[:] = k[0]
        print(f"fp8 uniform keys D={D}", flush=True)
        out, lse, (qd, kd, vd) = run_fp8(cu, None, va.VA_MASK_CAUSAL, q, k, v, 0.05)
        for i in (0, 1, 3, 7, 15, 31, 63):
            want = vd[:i + 1, 0].astype(np.float64).mean(axis=0)
            # bf16 rounding of the result, plus the matrix unit's own summation (about 17 significant bits,
            # relative to the largest term: it shows where the values of a column nearly cancel)
            atol = 2.0 ** -16 * np.abs(vd[:i + 1, 0]).max()
            for h in range(Hq):
                assert np.allclose(out[i, h], want, rtol=2.0 ** -7, atol=atol), (D, i, h)


@pytest.mark.gpu
def test_device_quantisers_equal_the_host_routines_on_non_finite_inputs():
    # a NaN of either sign in one head, infinities in another: the device routines return the bytes and
    # scales of the host routines (whose behaviour the host-library tests tie to the oracle's quantiser)
    T, H, D = 300, 3, 64
    r = np.random.default_rng(8)
    bits = wl.bf16_bits(wl.round_to_bf16(r.standard_normal((T, H, D)).astype(np.float32) * 3.0)).copy()
    bits[T // 3, 0, 5], bits[T - 1, 0, D - 1] = 0x7fc0, 0xffc1
    bits[1, 1, 0], bits[T // 2, 1, 7] = 0x7f80, 0xff80
    cu = np.array([0, 130, 131, 300], dtype=np.int32)
    print("device quantisers, non-finite inputs", flush=True)
    xt = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(DEV)
    codes = torch.full((T, H, D), 0xAA, dtype=torch.uint8, device=DEV)
    descale = torch.full((H,), -1.0, dtype=torch.float32, device=DEV)
    va.va_quantize_e4m3_per_head_device(xt, codes, descale)
    bcodes = torch.full((T, H, D), 0xAA, dtype=torch.uint8, device=DEV)
    bdescale = torch.full((T, H), -1.0, dtype=torch.float32, device=DEV)
    va.va_quantize_e4m3_blockwise_device(xt, cu, torch.from_numpy(cu).to(DEV), bcodes, bdescale)
    torch.cuda.synchronize()
    hc, hd = va.va_quantize_e4m3_per_head(bits)
    assert np.array_equal(codes.cpu().numpy(), hc) and np.array_equal(descale.cpu().numpy().view(np.uint32), hd.view(np.uint32))
    assert hc[T // 3, 0, 5] == 0x7F and hc[T - 1, 0, D - 1] == 0x7F and np.isfinite(hd[0]) and np.isinf(hd[1])
    hbc, hbd = va.va_quantize_e4m3_blockwise(bits, cu)
    assert np.array_equal(bcodes.cpu().numpy(), hbc)
    assert np.array_equal(bdescale.cpu().numpy().view(np.uint32), hbd.view(np.uint32))


@pytest.mark.gpu
@pytest.mark.parametrize("T,H,D", [(1, 1, 64), (77, 3, 64), (513, 8, 128), (300, 5, 256), (0, 4, 128)])
def test_device_quantiser_is_bit_identical_to_the_oracle(T, H, D):
    # per-head amax, descale and every code byte: the oracle's nearest-value search decides, the device
    # uses the conversion instruction after clamping; values hit subnormals, ties and the saturation edge
    print(f"device quantiser T={T} H={H} D={D}", flush=True)
    rng = np.random.default_rng(100 + T + H)
    x = rng.standard_normal((T, H, D)).astype(np.float32)
    if T > 0:
        x[0, 0, :8] = [0.0, -0.0, 1e-6, -3e-5, 448.0, -448.0, 1.0, -1.0]
        x[:, -1, :] *= 1e-3           # a head with a tiny range
        if H > 1:
            x[:, 1, :] = 0.0          # an all-zero head: descale 1
        x.flat[:: 7] *= 37.0          # spread over many binades
    x = wl.round_to_bf16(x)
    bits = wl.bf16_bits(x)
    xt = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(DEV)
    codes = torch.full((T, H, D), 0xAA, dtype=torch.uint8, device=DEV)
    descale = torch.full((H,), -1.0, dtype=torch.float32, device=DEV)
    va.va_quantize_e4m3_per_head_device(xt, codes, descale)
    torch.cuda.synchronize()
    if T == 0:  # nothing to look at: every head is "all zero"
        assert np.array_equal(descale.cpu().numpy(), np.ones(H, dtype=np.float32))
        return
    ref_codes, ref_descale = oe.quantize_per_head(x)
    assert np.array_equal(descale.cpu().numpy().view(np.uint32), ref_descale.astype(np.float32).view(np.uint32))
    assert np.array_equal(codes.cpu().numpy(), ref_codes)
    host_codes, host_descale = va.va_quantize_e4m3_per_head(bits)
    assert np.array_equal(host_codes, ref_codes) and np.array_equal(host_descale, ref_descale.astype(np.float32))


def test_fp8_peaked_softmax_with_a_rising_row_maximum():
    # as the bf16 case of the same name: the row maximum climbs from tile to tile and most of a row's
    # weight sits on a few keys, so the reference point of the stored probabilities has to follow
    Hq, Hkv, D = 4, 2, 128
    lens = [330, 70, 200]
    cu, _, q, k, v, _ = wl.random_stream(93, lens, Hq, Hkv, D)
    ramp = np.concatenate([1.0 + 3.0 * np.arange(L) / L for L in lens]).astype(np.float32)
    k = wl.round_to_bf16(k * ramp[:, None, None])
    # half the size of the bf16 case: the matrix unit sums FP8 products with about 17 significant bits, so
    # the scores (and the LSE) carry a relative error of about 1.4e-5, which the absolute LSE bound of
    # 1e-3 absorbs up to |LSE| of about 70 (measured 7e-4 at |LSE| = 50, 4e-5 at ordinary sizes)
    scale = 4.0 / np.sqrt(D) / 2.5
    print("fp8 peaked softmax", flush=True)
    out, lse, (qd, kd, vd) = run_fp8(cu, None, va.VA_MASK_CAUSAL, q, k, v, scale)
    ref_out, ref_lse = oa.attn_fwd(qd, kd, vd, cu, None, scale=scale, mask_mode=oa.MASK_CAUSAL)
    print(f"  largest |LSE| {np.abs(ref_lse).max():.1f}; out rel-L2 {rel_l2(out, ref_out):.2e} lse max-abs {max_abs(lse, ref_lse):.2e}",
          flush=True)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    assert rel_l2(out, ref_out) <= TOL_FP8_REL and max_abs(lse, ref_lse) <= TOL_LSE_ABS

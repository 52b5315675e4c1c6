"""GPU parity of the block-wise scaled FP8 path: the device quantiser (one
scale per 128 tokens of a sample and head) against the oracle's, bit for bit,
and the FP8 forward fed with per-token-row scales against the fp64 oracle run
on the block-wise dequantised inputs (rel-L2 5e-2, LSE 1e-3 as for the
per-head kernel)."""
import numpy as np
import pytest
import torch

from oracle import attn as oa
from oracle import e4m3 as oe
from paper_2603_11101_amd import binding as va
from paper_2603_11101_amd import workloads as wl

from gpu_util import DEV, TOL_FP8_REL, TOL_LSE_ABS, from_dev_bf16, max_abs, rel_l2

pytestmark = pytest.mark.gpu


def expand(descale, cu, H):
    """The oracle's [num_blocks, H] block scales, one row per token (the library's layout)."""
    starts = oe.block_starts(cu)
    out = np.zeros((int(cu[-1]), H), dtype=np.float32)
    for s in range(len(cu) - 1):
        for t in range(int(cu[s]), int(cu[s + 1])):
            out[t] = descale[int(starts[s]) + (t - int(cu[s])) // oe.BLOCK_TOKENS]
    return out


def drifting(seed, x, period, lo=-6, hi=6):
    """x with its magnitude changed by a random power of two every `period` tokens, rounded to bf16."""
    r = np.random.default_rng(seed)
    T = x.shape[0]
    f = np.exp2(r.integers(lo, hi + 1, size=(T // period + 1, x.shape[1]))).astype(np.float32)
    return wl.round_to_bf16(x * f[np.arange(T) // period][:, :, None])


def to_dev_bf16(x):
    return torch.from_numpy(wl.bf16_bits(x).view(np.int16)).view(torch.bfloat16).to(DEV)


def quantise_on_device(x, cu):
    T, H, D = x.shape
    codes = torch.full((T + 1, H, D), 0xAA, dtype=torch.uint8, device=DEV)
    descale = torch.full((T + 1, H), -1.0, dtype=torch.float32, device=DEV)
    cu_dev = torch.from_numpy(np.asarray(cu, dtype=np.int32)).to(DEV)
    va.va_quantize_e4m3_blockwise_device(to_dev_bf16(x), cu, cu_dev, codes[:T], descale[:T])
    torch.cuda.synchronize()
    assert torch.all(codes[T] == 0xAA) and torch.all(descale[T] == -1.0)     # nothing past the last token
    return codes[:T], descale[:T]


@pytest.mark.parametrize("lens,H,D", [([1], 1, 64), ([128], 2, 128), ([129, 0, 5], 3, 64), ([300, 17, 256, 1, 700], 5, 128),
                                      ([0, 0], 4, 128), (list(range(1, 151)), 2, 48), ([1000], 9, 256), ([130, 40], 2, 512),
                                      ([700, 3], 3, 40)])
def test_device_blockwise_quantiser_is_bit_identical_to_the_oracle(lens, H, D):
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(cu[-1])
    print(f"device block-wise quantiser samples={len(lens)} T={T} H={H} D={D}", flush=True)
    rng = np.random.default_rng(200 + T + H)
    x = rng.standard_normal((T, H, D)).astype(np.float32)
    if T > 0:
        x = drifting(300 + T, x, 37, -14, 6)
        x[0, 0, :8] = [0.0, -0.0, 1e-6, -3e-5, 448.0, -448.0, 1.0, -1.0]
        if T > 140:
            x[128:140, -1, :] = 0.0   # zero rows inside a block
        if T >= 300 and len(lens) > 1:
            x[cu[1] - 44:cu[1], 0, :] = 0.0      # the short last block of sample 0, all zero: descale 1
        x = wl.round_to_bf16(x)
    codes, descale = quantise_on_device(x, cu)
    if T == 0:
        return
    ref_codes, ref_descale = oe.quantize_blockwise(x, cu)
    want = expand(ref_descale, cu, H)
    assert np.array_equal(descale.cpu().numpy().view(np.uint32), want.view(np.uint32))
    assert np.array_equal(codes.cpu().numpy(), ref_codes)
    host_codes, host_descale = va.va_quantize_e4m3_blockwise(wl.bf16_bits(x), cu)
    assert np.array_equal(host_codes, ref_codes) and np.array_equal(host_descale, want)


def run_blockwise(cu, prefix, mode, q, k, v, scale):
    """Quantise on the device, run the block-wise FP8 forward, return (out, lse, dequantised inputs)."""
    T, Hq, D = q.shape
    Hkv = k.shape[1]
    dev = [quantise_on_device(x, cu) for x in (q, k, v)]
    deq = []
    for x, (codes, descale) in zip((q, k, v), dev):
        oc, od = oe.quantize_blockwise(x, cu)
        assert np.array_equal(codes.cpu().numpy(), oc)
        assert np.array_equal(descale.cpu().numpy(), expand(od, cu, x.shape[1]))
        deq.append(oe.dequantize_blockwise(oc, od, cu).astype(np.float32))
    ps = va.PackedStream(cu, prefix, mode, Hq, Hkv, D, device=DEV, passes=(va.VA_PASS_FWD,))
    out = torch.full((T + 2, Hq, D), 768.0, dtype=torch.bfloat16, device=DEV)
    lse = torch.empty((Hq, T), dtype=torch.float32, device=DEV)
    (q8, qd), (k8, kd), (v8, vd) = dev
    ps.fwd_fp8_blockwise(q8.contiguous(), k8.contiguous(), v8.contiguous(), qd.contiguous(), kd.contiguous(),
                         vd.contiguous(), scale, out, lse)
    torch.cuda.synchronize()
    got = from_dev_bf16(out)
    assert np.all(got[T:] == 768.0)
    return got[:T], lse.cpu().numpy().astype(np.float64), deq


OMODE = {va.VA_MASK_CAUSAL: oa.MASK_CAUSAL, va.VA_MASK_PREFIX_LM: oa.MASK_PREFIX_BIDIR_SUFFIX,
         va.VA_MASK_PREFIX_LM_CAUSAL: oa.MASK_PREFIX_CAUSAL_SUFFIX, va.VA_MASK_THREE_BLOCK: oa.MASK_THREE_BLOCK}


@pytest.mark.parametrize("mode,Hq,Hkv,D", [(va.VA_MASK_CAUSAL, 4, 2, 128), (va.VA_MASK_PREFIX_LM, 8, 1, 128), (va.VA_MASK_CAUSAL, 2, 2, 128),
                                           (va.VA_MASK_PREFIX_LM_CAUSAL, 4, 1, 128), (va.VA_MASK_THREE_BLOCK, 16, 2, 128),
                                           (va.VA_MASK_CAUSAL, 4, 2, 64), (va.VA_MASK_PREFIX_LM, 8, 1, 256), (va.VA_MASK_CAUSAL, 2, 2, 256),
                                           (va.VA_MASK_THREE_BLOCK, 4, 1, 64), (va.VA_MASK_CAUSAL, 2, 2, 64), (va.VA_MASK_PREFIX_LM, 8, 1, 64),
                                           (va.VA_MASK_CAUSAL, 4, 2, 256), (va.VA_MASK_PREFIX_LM_CAUSAL, 4, 1, 256)])
def test_fp8_blockwise_forward_parity(mode, Hq, Hkv, D):
    # magnitudes of Q, K and V drift by powers of two along the stream (period 90 tokens, so blocks
    # differ and some blocks straddle a change), which is what block scales are for
    lens = [17, 64, 95, 200, 1, 130, 0, 257, 600]
    cu, prefix, q, k, v, _ = wl.random_stream(70 + Hq + mode + D, lens, Hq, Hkv, D, prefix_frac=-1.0)
    q, k, v = drifting(1, q, 90, -4, 1), drifting(2, k, 90, -4, 1), drifting(3, v, 90, -5, 5)
    if mode == va.VA_MASK_CAUSAL:
        prefix = None
    elif mode == va.VA_MASK_THREE_BLOCK:
        prefix = wl.random_block_ends(70 + Hq, lens)
    # sizes that keep |LSE| small: the FP8 products carry a relative error of about 1.4e-5 into the scores,
    # which the absolute LSE bound absorbs only up to |LSE| of a few tens
    scale = 1.0 / np.sqrt(D)
    print(f"fp8 block-wise forward mode={mode} Hq={Hq} Hkv={Hkv} D={D}", flush=True)
    out, lse, (qd, kd, vd) = run_blockwise(cu, prefix, mode, q, k, v, scale)
    ref_out, ref_lse = oa.attn_fwd(qd, kd, vd, cu, prefix, scale=scale, mask_mode=OMODE[mode])
    print(f"  largest |LSE| {np.abs(ref_lse).max():.1f}; out rel-L2 {rel_l2(out, ref_out):.2e} max-abs {max_abs(out, ref_out):.2e} "
          f"lse max-abs {max_abs(lse, ref_lse):.2e}", flush=True)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    assert rel_l2(out, ref_out) <= TOL_FP8_REL
    assert max_abs(lse, ref_lse) <= TOL_LSE_ABS
    for s in range(len(lens)):
        if lens[s]:
            sl = slice(cu[s], cu[s + 1])
            assert rel_l2(out[sl], ref_out[sl]) <= TOL_FP8_REL, f"sample {s}"


def test_fp8_blockwise_equals_per_head_when_every_block_has_the_same_scale():
    # one entry of magnitude 448 * 2^-5 in every (block, head) pins every descale to 2^-5 exactly: both
    # kernels then see the same codes and scales, and log2 / reciprocal of a power of two are exact, so the
    # two outputs may differ only through the order of the float operations on the scales
    Hq, Hkv, D = 4, 2, 128
    lens = [200, 64, 331]
    cu, _, q, k, v, _ = wl.random_stream(81, lens, Hq, Hkv, D)
    peak = np.float32(448.0 * 2.0 ** -5)
    for x in (q, k, v):
        np.clip(x, -peak, peak, out=x)
        for s in range(len(lens)):
            x[cu[s]:cu[s + 1]:64, :, 0] = peak        # at least one per block, heads alike
    scale = 1.0 / np.sqrt(D)
    print("fp8 block-wise against per-head, equal scales", flush=True)
    out_b, lse_b, _ = run_blockwise(cu, None, va.VA_MASK_CAUSAL, q, k, v, scale)
    T = int(cu[-1])
    codes = [va.va_quantize_e4m3_per_head(wl.bf16_bits(x)) for x in (q, k, v)]
    assert all(np.all(d == np.float32(2.0 ** -5)) for _, d in codes)
    ps = va.PackedStream(cu, None, va.VA_MASK_CAUSAL, Hq, Hkv, D, device=DEV, passes=(va.VA_PASS_FWD,))
    out = torch.zeros((T, Hq, D), dtype=torch.bfloat16, device=DEV)
    lse = torch.empty((Hq, T), dtype=torch.float32, device=DEV)
    args = [torch.from_numpy(c).to(DEV) for c, _ in codes] + [torch.from_numpy(d).to(DEV) for _, d in codes]
    ps.fwd_fp8(*args, scale, out, lse)
    torch.cuda.synchronize()
    out_h = from_dev_bf16(out)
    print(f"  out max-abs {max_abs(out_b, out_h):.2e} lse max-abs {max_abs(lse_b, lse.cpu().numpy()):.2e}", flush=True)
    assert rel_l2(out_b, out_h) <= 2e-3 and max_abs(lse_b, lse.cpu().numpy().astype(np.float64)) <= 1e-5


def test_fp8_blockwise_is_closer_to_the_unquantised_result_than_per_head_on_drifting_magnitudes():
    # the reason for block scales: where the magnitude of V grows along a sample by more than E4M3's range
    # (here by 2^4 per 128 tokens, from 2^-16), one scale per head leaves the early stretches in the
    # subnormals or at zero, and under a causal mask the early rows, which see only those keys, lose their
    # output; compare both FP8 paths, row by row, with the oracle on the original bf16 inputs
    Hq, Hkv, D = 4, 2, 128
    lens = [600, 300]
    cu, _, q, k, v, _ = wl.random_stream(83, lens, Hq, Hkv, D)
    for s in range(len(lens)):
        growth = np.exp2(np.minimum(0, -16 + 4 * (np.arange(lens[s]) // 128))).astype(np.float32)
        v[cu[s]:cu[s + 1]] *= growth[:, None, None]
    v = wl.round_to_bf16(v)
    scale = 1.0 / np.sqrt(D)
    print("fp8 block-wise against per-head, accuracy", flush=True)
    out_b, _, _ = run_blockwise(cu, None, va.VA_MASK_CAUSAL, q, k, v, scale)
    T = int(cu[-1])
    codes = [va.va_quantize_e4m3_per_head(wl.bf16_bits(x)) for x in (q, k, v)]
    ps = va.PackedStream(cu, None, va.VA_MASK_CAUSAL, Hq, Hkv, D, device=DEV, passes=(va.VA_PASS_FWD,))
    out = torch.zeros((T, Hq, D), dtype=torch.bfloat16, device=DEV)
    lse = torch.empty((Hq, T), dtype=torch.float32, device=DEV)
    args = [torch.from_numpy(c).to(DEV) for c, _ in codes] + [torch.from_numpy(d).to(DEV) for _, d in codes]
    ps.fwd_fp8(*args, scale, out, lse)
    torch.cuda.synchronize()
    out_h = from_dev_bf16(out)
    ref, _ = oa.attn_fwd(q, k, v, cu, None, scale=scale, mask_mode=oa.MASK_CAUSAL)

    def row_err(got):
        num = np.sqrt(((got - ref) ** 2).sum(axis=2))
        return num / np.sqrt((ref ** 2).sum(axis=2))

    eb, eh = row_err(out_b), row_err(out_h)
    print(f"  row-wise relative error against the unquantised result: block-wise median {np.median(eb):.3e} "
          f"worst {eb.max():.3e}; per-head median {np.median(eh):.3e} worst {eh.max():.3e}", flush=True)
    assert eb.max() <= 0.15 and eh.max() >= 3 * eb.max() and np.median(eb) <= np.median(eh)

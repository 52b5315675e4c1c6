"""Pins for the E4M3 oracle: the format's definition (exhaustive over all 256
codes), round-to-nearest-even at every midpoint, saturation, and PyTorch's CPU
float8_e4m3fn cast as an independent library routine."""
import numpy as np
import torch

from oracle import e4m3


def test_known_values_of_the_format():
    # 1-4-3, bias 7: 0x38 = 1.0, 0x40 = 2.0, 0x7E = 448 (largest), 0x08 = 2^-6 (smallest normal),
    # 0x01 = 2^-9 (smallest subnormal), 0x7F = NaN, sign bit 0x80
    assert e4m3.decode_scalar(0x38) == 1.0
    assert e4m3.decode_scalar(0x40) == 2.0
    assert e4m3.decode_scalar(0x7E) == 448.0
    assert e4m3.decode_scalar(0x08) == 2.0 ** -6
    assert e4m3.decode_scalar(0x01) == 2.0 ** -9
    assert e4m3.decode_scalar(0x07) == 7 * 2.0 ** -9
    assert np.isnan(e4m3.decode_scalar(0x7F)) and np.isnan(e4m3.decode_scalar(0xFF))
    assert e4m3.decode_scalar(0xB8) == -1.0
    assert e4m3.decode_scalar(0x80) == 0.0 and np.signbit(e4m3.decode_scalar(0x80))


def test_all_codes_round_trip():
    for c in range(256):
        v = e4m3.decode_scalar(c)
        if np.isnan(v):
            assert e4m3.encode_scalar(v) == 0x7F
            continue
        assert e4m3.encode_scalar(v) == c
        assert int(e4m3.encode(np.array([v]))[0]) == c


def test_midpoints_round_to_even_and_neighbours_round_to_nearest():
    for c in range(0x7E):
        lo, hi = e4m3.decode_scalar(c), e4m3.decode_scalar(c + 1)
        mid = (lo + hi) / 2
        even = c if c % 2 == 0 else c + 1
        assert e4m3.encode_scalar(mid) == even
        assert e4m3.encode_scalar(-mid) == even | 0x80
        just_below = np.nextafter(np.float32(mid), np.float32(0))
        just_above = np.nextafter(np.float32(mid), np.float32(1e9))
        got = e4m3.encode(np.array([mid, just_below, just_above], dtype=np.float32))
        assert list(got) == [even, c, c + 1]


def test_saturation_and_nan():
    x = np.array([448.0, 449.0, 463.99, 464.0, 480.0, 1e30, np.inf, -1e30, -np.inf, np.nan], dtype=np.float32)
    got = e4m3.encode(x)
    assert list(got) == [0x7E, 0x7E, 0x7E, 0x7E, 0x7E, 0x7E, 0x7E, 0xFE, 0xFE, 0x7F]
    assert [e4m3.encode_scalar(float(v)) for v in x] == list(got)


def test_vector_encode_equals_scalar_search():
    r = np.random.default_rng(0)
    x = np.concatenate([r.standard_normal(3000) * s for s in (1e-3, 0.02, 1.0, 40.0, 300.0)]).astype(np.float32)
    assert list(e4m3.encode(x)) == [e4m3.encode_scalar(float(v)) for v in x]


def test_against_torch_cpu_float8_cast():
    codes = torch.arange(256, dtype=torch.uint8)
    tv = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    ov = e4m3.decode(codes.numpy())
    assert np.array_equal(np.isnan(tv), np.isnan(ov))
    assert np.array_equal(tv[~np.isnan(tv)], ov[~np.isnan(ov)])
    r = np.random.default_rng(1)
    x = np.concatenate([r.standard_normal(20000) * s for s in (1e-3, 0.05, 1.0, 30.0, 150.0)]).astype(np.float32)
    x = x[np.abs(x) < 464.0]   # beyond that torch produces NaN where the oracle saturates
    t = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(t, e4m3.encode(x))


def test_per_head_quantiser():
    r = np.random.default_rng(2)
    x = (r.standard_normal((50, 3, 16)) * np.array([0.1, 1.0, 7.0])[None, :, None]).astype(np.float32)
    x[:, 1, :] = 0.0
    codes, descale = e4m3.quantize_per_head(x)
    amax = np.abs(x).max(axis=(0, 2))
    assert descale[1] == 1.0 and np.all(codes[:, 1, :] == 0)
    for h in (0, 2):
        assert descale[h] == np.float32(amax[h]) / np.float32(448.0)
        assert e4m3.decode(codes[:, h, :]).max() <= 448.0
        deq = e4m3.dequantize_per_head(codes, descale)[:, h, :]
        # e4m3 keeps 3 mantissa bits: relative error <= 2^-4 for normal numbers
        big = np.abs(x[:, h, :]) > descale[h] * 2.0 ** -6
        assert np.all(np.abs(deq - x[:, h, :])[big] <= np.abs(x[:, h, :])[big] * 2.0 ** -4 * 1.0001)
    # the element with the largest magnitude maps to +-448 exactly
    assert np.abs(e4m3.decode(codes[:, 2, :])).max() == 448.0


def test_blockwise_quantiser():
    # blocks are 128 tokens of one sample by one head: every block is, taken alone, the per-head rule
    r = np.random.default_rng(3)
    cu = np.array([0, 5, 5, 140, 140 + 256, 140 + 256 + 129], dtype=np.int32)        # a short, an empty, ragged and whole blocks
    T, H, D = int(cu[-1]), 2, 16
    x = (r.standard_normal((T, H, D)) * np.exp(r.standard_normal((T, 1, 1)))).astype(np.float32)
    x[140:268, 1, :] = 0.0                                                            # one all-zero block
    codes, descale = e4m3.quantize_blockwise(x, cu)
    starts = e4m3.block_starts(cu)
    assert starts.tolist() == [0, 1, 1, 3, 5, 7] and descale.shape == (7, H)
    b = 0
    for s in range(len(cu) - 1):
        for r0 in range(int(cu[s]), int(cu[s + 1]), 128):
            rows = slice(r0, min(int(cu[s + 1]), r0 + 128))
            want_codes, want_descale = e4m3.quantize_per_head(x[rows])
            assert np.array_equal(codes[rows], want_codes) and np.array_equal(descale[b], want_descale)
            b += 1
    assert b == 7 and descale[3, 1] == 1.0 and np.all(codes[140:268, 1, :] == 0)
    # the largest element of every non-zero block maps to +-448; the round trip keeps 2^-4 relative
    deq = e4m3.dequantize_blockwise(codes, descale, cu)
    assert np.abs(e4m3.decode(codes[0:5, 0, :])).max() == 448.0
    big = np.abs(x) > 0
    rel = np.abs(deq - x)[big] / np.abs(x)[big]
    assert np.percentile(rel, 50) <= 2.0 ** -4 and deq.shape == x.shape
    # one block per sample and one sample: the per-head rule itself
    one = np.array([0, 100], dtype=np.int32)
    c1, d1 = e4m3.quantize_blockwise(x[:100], one)
    c2, d2 = e4m3.quantize_per_head(x[:100])
    assert np.array_equal(c1, c2) and np.array_equal(d1[0], d2)

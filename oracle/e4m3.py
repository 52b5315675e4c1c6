"""Oracle for the OCP FP8 E4M3 ("e4m3fn") number format and the per-head input
quantiser of the fp8 forward.

TEST INFRASTRUCTURE ONLY.  Written from the format's definition: 1 sign bit,
4 exponent bits with bias 7, 3 mantissa bits; no infinities; the only NaN is
S.1111.111; exponent field 0 holds subnormals m * 2**-9; the largest finite
value is S.1111.110 = 448.  Encoding is "the nearest representable value, ties
to the code with an even mantissa, magnitudes beyond the largest finite value
saturate to it".

The paper (section 2.2.3, scaling granularity) defines per-tensor, per-channel
and block-wise scales; the attention fp8 forward uses one scale per head (the
per-channel rule applied along the head axis): descale[h] = amax_h / 448 in
float32 and code = encode(float32(x / descale[h])), both operations in float32.
"""
import numpy as np

E4M3_MAX = 448.0
NAN_CODE = 0x7F


def decode_scalar(code: int) -> float:
    code = int(code) & 0xFF
    sign = -1.0 if code & 0x80 else 1.0
    e = (code >> 3) & 0xF
    m = code & 0x7
    if e == 0xF and m == 0x7:
        return float("nan")
    if e == 0:
        return sign * m * 2.0 ** -9
    return sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)


# magnitudes of the 127 finite non-negative codes 0x00..0x7E, increasing
_MAG = np.array([decode_scalar(c) for c in range(0x7F)], dtype=np.float64)


def decode(codes) -> np.ndarray:
    """uint8 codes -> float64 values (exact)."""
    table = np.array([decode_scalar(c) for c in range(256)], dtype=np.float64)
    return table[np.asarray(codes, dtype=np.uint8)]


def encode_scalar(x: float) -> int:
    """Nearest-even encode of one value by exhaustive search over all codes."""
    if np.isnan(x):
        return NAN_CODE
    sign = 0x80 if np.signbit(x) else 0
    a = abs(float(x))
    if a >= E4M3_MAX:
        return sign | 0x7E
    best = None
    for c in range(0x7F):
        d = abs(_MAG[c] - a)
        if best is None or d < best[0] or (d == best[0] and (c & 1) == 0 and (best[1] & 1) == 1):
            best = (d, c)
    return sign | best[1]


def encode(x) -> np.ndarray:
    """Vectorised nearest-even encode of float32/float64 values -> uint8."""
    x = np.asarray(x)
    a = np.abs(x.astype(np.float64))
    hi = np.searchsorted(_MAG, a, side="left")          # first code with value >= a
    hi = np.clip(hi, 0, 0x7E)
    lo = np.clip(hi - 1, 0, 0x7E)
    d_hi = np.abs(_MAG[hi] - a)
    d_lo = np.abs(a - _MAG[lo])
    pick_lo = (d_lo < d_hi) | ((d_lo == d_hi) & ((lo & 1) == 0))
    code = np.where(pick_lo, lo, hi)
    code = np.where(a >= E4M3_MAX, 0x7E, code)
    code = code.astype(np.uint8) | np.where(np.signbit(x), 0x80, 0).astype(np.uint8)
    code = np.where(np.isnan(x), NAN_CODE, code).astype(np.uint8)
    return code


def quantize_per_head(x):
    """x [T, H, D] float32 -> (codes uint8 [T, H, D], descale float32 [H])."""
    x = np.asarray(x, dtype=np.float32)
    amax = np.max(np.abs(x), axis=(0, 2)).astype(np.float32)
    descale = (amax / np.float32(448.0)).astype(np.float32)
    descale = np.where(descale > 0, descale, np.float32(1.0)).astype(np.float32)
    scaled = (x / descale[None, :, None]).astype(np.float32)
    return encode(scaled), descale


def dequantize_per_head(codes, descale):
    """codes [T, H, D], descale [H] -> float64 values code_value * descale."""
    return decode(codes) * np.asarray(descale, dtype=np.float64)[None, :, None]


# ---------------------------------------------------------------- block-wise scaling
#
# The paper's third granularity (section 2.2.3: one scale per 128 x 128 block of the tensor).  Read for
# the attention operands [T, H, D] of a packed stream as: 128 consecutive tokens of ONE sample by the
# 128 values of one head, so a block never mixes two samples; sample s of length L_s has ceil(L_s / 128)
# token blocks (the last one shorter) and the blocks of the stream are numbered sample after sample.

BLOCK_TOKENS = 128


def block_starts(cu_seqlens, block=BLOCK_TOKENS):
    """First block number of every sample, and the total number of blocks (last entry)."""
    out = [0]
    for s in range(len(cu_seqlens) - 1):
        L = int(cu_seqlens[s + 1]) - int(cu_seqlens[s])
        out.append(out[-1] + (L + block - 1) // block)
    return np.array(out, dtype=np.int32)


def quantize_blockwise(x, cu_seqlens, block=BLOCK_TOKENS):
    """x [T, H, D] float32 -> (codes uint8 [T, H, D], descale float32 [num_blocks, H]): descale =
    amax of the block / 448 (1 where the block is all zero), code = encode(float32(x / descale))."""
    x = np.asarray(x, dtype=np.float32)
    T, H, D = x.shape
    starts = block_starts(cu_seqlens, block)
    descale = np.ones((int(starts[-1]), H), dtype=np.float32)
    codes = np.zeros((T, H, D), dtype=np.uint8)
    for s in range(len(cu_seqlens) - 1):
        c, e = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        for b, r0 in enumerate(range(c, e, block)):
            rows = slice(r0, min(e, r0 + block))
            amax = np.max(np.abs(x[rows]), axis=(0, 2)).astype(np.float32)
            d = (amax / np.float32(448.0)).astype(np.float32)
            d = np.where(d > 0, d, np.float32(1.0)).astype(np.float32)
            descale[int(starts[s]) + b] = d
            codes[rows] = encode((x[rows] / d[None, :, None]).astype(np.float32))
    return codes, descale


def dequantize_blockwise(codes, descale, cu_seqlens, block=BLOCK_TOKENS):
    """codes [T, H, D], descale [num_blocks, H] -> float64 values code_value * descale of the block."""
    vals = decode(codes)
    starts = block_starts(cu_seqlens, block)
    out = np.zeros_like(vals)
    for s in range(len(cu_seqlens) - 1):
        c, e = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        for b, r0 in enumerate(range(c, e, block)):
            rows = slice(r0, min(e, r0 + block))
            out[rows] = vals[rows] * np.asarray(descale[int(starts[s]) + b], dtype=np.float64)[None, :, None]
    return out

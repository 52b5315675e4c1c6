"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws numbers: sample lengths and tensor values.  It holds
none of the method's arithmetic (no packing, no tiling, no attention, no
quantisation) so that both the HIP path and the CPU oracle can be fed from it
without sharing any logic.  It imports neither of them.

The paper trains VLA backbones on multi-camera robot samples: a few hundred
image tokens per camera, a short instruction and a handful of state/action
tokens (section 2.2.1 for the Qwen2.5-VL decoder, section 2.2.2 for pi-0.5).
Its datasets are not available here, so the workloads below draw lengths
with that structure from fixed seeds (`vit` stands for the vision side, which
the paper runs through the same variable-length interface, section 2.2.1 (1)):

  tiny      3 samples of 17, 64, 95 tokens; 2 q heads / 2 kv heads, D = 64; causal
  vlm       pool of 512 samples: 256 * U{1,2,3} image tokens + U{10..60} text
            + 17 state/action tokens; 16 / 8 heads, D = 128; causal; budget 16384
  pi05      pool of 512: prefix = 768 image + U{20..200} text tokens
            (bidirectional), suffix = 50 action tokens; 8 / 1 heads, D = 256;
            prefix-LM; budget 32768
  longtail  pool of 2048: lognormal lengths (median 600, sigma 0.8) clipped to
            [16, 4096]; 16 / 8 heads, D = 128; causal; budget 65536
  vlm_fp8   the `vlm` lengths and values, for the FP8 forward
  pi0       pool of 512: three blocks, each seeing itself and those before it:
            768 image + U{20..200} text tokens, one state token, 50 action
            tokens; 8 / 1 heads, D = 256; budget 32768; the second value
            returned by sample_lengths is then [pool, 2]: the ends of the first
            two blocks
  vit       pool of 512 images of side U{16,24,32,38} patches, side^2 tokens
            each; 16 / 16 heads, D = 80 (the encoder's 1280 / 16); every token sees its whole image
            (prefix = length); budget 16384

Tensor values are float32 standard normal draws rounded once to bfloat16
(round-to-nearest-even), from a stream separate from the one that draws the
lengths, in the order Q, K, V, dO.
"""
from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    seed: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    prefix_lm: bool
    budget: int
    pool: int
    three_block: bool = False


WORKLOADS = {
    "tiny": Workload("tiny", 1, 2, 2, 64, False, 176, 3),
    "vlm": Workload("vlm", 2, 16, 8, 128, False, 16384, 512),
    "pi05": Workload("pi05", 3, 8, 1, 256, True, 32768, 512),
    "longtail": Workload("longtail", 4, 16, 8, 128, False, 65536, 2048),
    "vlm_fp8": Workload("vlm_fp8", 2, 16, 8, 128, False, 16384, 512),
    "vit": Workload("vit", 5, 16, 16, 80, True, 16384, 512),
    "pi0": Workload("pi0", 6, 8, 1, 256, True, 32768, 512, three_block=True),
}


def sample_lengths(name: str):
    """Pool of sample lengths (int32) and prefix lengths (int32 or None)."""
    w = WORKLOADS[name]
    r = np.random.default_rng(w.seed)
    if name == "tiny":
        return np.array([17, 64, 95], dtype=np.int32), None
    if name in ("vlm", "vlm_fp8"):
        cams = r.integers(1, 4, size=w.pool)
        text = r.integers(10, 61, size=w.pool)
        return (256 * cams + text + 17).astype(np.int32), None
    if name == "pi05":
        text = r.integers(20, 201, size=w.pool)
        prefix = 768 + text
        return (prefix + 50).astype(np.int32), prefix.astype(np.int32)
    if name == "vit":
        side = r.choice(np.array([16, 24, 32, 38]), size=w.pool)
        L = (side * side).astype(np.int32)
        return L, L.copy()
    if name == "pi0":
        text = r.integers(20, 201, size=w.pool)
        prefix = 768 + text
        ends = np.stack([prefix, prefix + 1], axis=1).astype(np.int32)
        return (prefix + 51).astype(np.int32), ends
    if name == "longtail":
        z = r.standard_normal(w.pool)
        L = np.clip(np.rint(np.exp(np.log(600.0) + 0.8 * z)), 16, 4096)
        return L.astype(np.int32), None
    raise KeyError(name)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 -> float32 holding the nearest bfloat16 value (ties to even)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000))
    return rounded.view(np.float32)


def bf16_bits(x_rounded: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that already are bfloat16 numbers."""
    u = np.ascontiguousarray(x_rounded, dtype=np.float32).view(np.uint32)
    return (u >> np.uint32(16)).astype(np.uint16)


def bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float32."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def tensor_values(seed: int, T: int, Hq: int, Hkv: int, D: int, with_dout: bool = True):
    """Q [T,Hq,D], K, V [T,Hkv,D], dO [T,Hq,D]: float32 arrays of bf16 values."""
    r = np.random.default_rng(1000 + seed)
    q = round_to_bf16(r.standard_normal((T, Hq, D), dtype=np.float32))
    k = round_to_bf16(r.standard_normal((T, Hkv, D), dtype=np.float32))
    v = round_to_bf16(r.standard_normal((T, Hkv, D), dtype=np.float32))
    do = round_to_bf16(r.standard_normal((T, Hq, D), dtype=np.float32)) if with_dout else None
    return q, k, v, do


def random_stream(seed: int, lens, Hq: int, Hkv: int, D: int, prefix_frac=None):
    """A free-form packed stream for tests: cu_seqlens, prefix_lens (or None)
    and tensor values, for arbitrary sample lengths."""
    lens = np.asarray(lens, dtype=np.int32)
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    r = np.random.default_rng(77000 + seed)
    prefix = None
    if prefix_frac is not None:
        prefix = np.array([int(r.integers(0, L + 1)) if prefix_frac < 0 else int(round(prefix_frac * L))
                           for L in lens], dtype=np.int32)
    q, k, v, do = tensor_values(seed, int(cu[-1]), Hq, Hkv, D)
    return cu, prefix, q, k, v, do


def random_block_ends(seed: int, lens) -> np.ndarray:
    """[num_seqs, 2] int32 ends (P, P2) of the first two of three blocks, 0 <= P <= P2 <= L, for tests
    of the three-block mask; empty blocks occur."""
    r = np.random.default_rng(88000 + seed)
    out = np.zeros((len(lens), 2), dtype=np.int32)
    for s, L in enumerate(lens):
        L = int(L)
        P = int(r.integers(0, L + 1))
        out[s] = (P, int(r.integers(P, L + 1)))
    return out


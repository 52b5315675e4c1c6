"""Helpers of the GPU parity tests: run the HIP path through the C ABI on a
packed stream and hand back numpy arrays; error metrics."""
import numpy as np
import torch

from paper_2603_11101_amd import binding as va
from paper_2603_11101_amd import workloads as wl

DEV = "cuda:0"

# tolerances stated for the path: bf16 forward rel-L2 1e-2 and max-abs 2e-2, LSE abs 1e-3,
# gradients rel-L2 2e-2, fp8 forward rel-L2 5e-2
TOL_FWD_REL, TOL_FWD_ABS, TOL_LSE_ABS, TOL_GRAD_REL, TOL_FP8_REL = 1e-2, 2e-2, 1e-3, 2e-2, 5e-2


def to_dev_bf16(x_f32, pad_rows=0, pad_value=float("nan")):
    """float32 array of bf16 values -> bf16 device tensor, optionally followed by
    `pad_rows` extra rows of a poison value (rows >= T must never be read)."""
    t = torch.from_numpy(wl.bf16_bits(x_f32).view(np.int16)).view(torch.bfloat16)
    if pad_rows:
        pad = torch.full((pad_rows,) + tuple(t.shape[1:]), pad_value, dtype=torch.bfloat16)
        t = torch.cat([t, pad])
    return t.to(DEV)


def from_dev_bf16(t):
    return wl.bits_to_f32(t.cpu().view(torch.int16).numpy().view(np.uint16)).astype(np.float64)


def rel_l2(x, ref):
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.sqrt((ref * ref).sum())
    return float(np.sqrt(((x - ref) ** 2).sum()) / den) if den > 0 else float(np.abs(x).max())


def max_abs(x, ref):
    return float(np.abs(np.asarray(x, dtype=np.float64) - ref).max()) if np.size(ref) else 0.0


class DeviceRun:
    """Forward (and backward) of one stream on the GPU; outputs as float64 numpy."""

    SENTINEL = 768.0   # exactly representable in bfloat16

    def __init__(self, cu, prefix, mask_mode, q, k, v, do, scale, max_seqlen=None, pad_rows=3, backward=True):
        T, Hq, D = q.shape
        Hkv = k.shape[1]
        self.T, self.pad = T, pad_rows
        self.ps = va.PackedStream(cu, prefix, mask_mode, Hq, Hkv, D, max_seqlen=max_seqlen, device=DEV)
        dq_, dk_, dv_, ddo = (to_dev_bf16(x, pad_rows) for x in (q, k, v, do))
        out = torch.full((T + pad_rows, Hq, D), self.SENTINEL, dtype=torch.bfloat16, device=DEV)
        lse = torch.full((Hq, T), self.SENTINEL, dtype=torch.float32, device=DEV)
        self.ps.fwd(dq_, dk_, dv_, scale, out, lse)
        torch.cuda.synchronize()
        self.out_full = from_dev_bf16(out)
        self.out = self.out_full[:T]
        self.lse = lse.cpu().numpy().astype(np.float64)
        if backward:
            gq = torch.full((T + pad_rows, Hq, D), self.SENTINEL, dtype=torch.bfloat16, device=DEV)
            gk = torch.full((T + pad_rows, Hkv, D), self.SENTINEL, dtype=torch.bfloat16, device=DEV)
            gv = torch.full((T + pad_rows, Hkv, D), self.SENTINEL, dtype=torch.bfloat16, device=DEV)
            self.ps.bwd(dq_, dk_, dv_, out, lse, ddo, scale, gq, gk, gv)
            torch.cuda.synchronize()
            self.dq_full, self.dk_full, self.dv_full = from_dev_bf16(gq), from_dev_bf16(gk), from_dev_bf16(gv)
            self.dq, self.dk, self.dv = self.dq_full[:T], self.dk_full[:T], self.dv_full[:T]

    def tail_untouched(self, *names):
        return all(np.all(getattr(self, n + "_full")[self.T:] == self.SENTINEL) for n in names)

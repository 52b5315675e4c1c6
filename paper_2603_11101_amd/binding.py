"""ctypes binding of ``libvarlen_attn.so`` with the same names as the C ABI
(``include/varlen_attn.h``).  Argument marshalling only: every step of the
path runs in the library.  PyTorch is used for device memory and streams.

The library must have been built (``python -m paper_2603_11101_amd.build``);
there is no fallback of any kind: a missing library raises.
"""
import ctypes
import os

import numpy as np
# torch first: the library then binds to the HIP runtime torch has already loaded, so both
# share one runtime (and one view of the device) inside the process
import torch  # noqa: F401

VA_OK = 0
VA_EINVAL, VA_EUNSUPPORTED, VA_EALIGN, VA_ESIZE, VA_EHIP = -1, -2, -3, -4, -5
VA_MASK_CAUSAL, VA_MASK_PREFIX_LM, VA_MASK_PREFIX_LM_CAUSAL, VA_MASK_THREE_BLOCK, VA_MASK_SLIDING_WINDOW = 0, 1, 2, 3, 4
VA_PASS_FWD, VA_PASS_BWD_DKDV, VA_PASS_BWD_DQ = 0, 1, 2
VA_BWD_STAGE_DELTA, VA_BWD_STAGE_DKDV, VA_BWD_STAGE_DQ, VA_BWD_STAGE_ALL = 1, 2, 4, 7

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvarlen_attn.so")


class VarlenAttnError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"[{code}] {message}")
        self.code = code


class va_shape(ctypes.Structure):
    _fields_ = [("total_tokens", ctypes.c_int32), ("num_seqs", ctypes.c_int32),
                ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("max_seqlen", ctypes.c_int32),
                ("mask_mode", ctypes.c_int32)]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_11101_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    lib.va_last_error.restype = ctypes.c_char_p
    lib.varlen_attn_bwd_workspace_bytes.restype = ctypes.c_size_t
    lib.varlen_attn_bwd_workspace_bytes.argtypes = [ctypes.POINTER(va_shape)]
    return lib


_lib = _load()

EXPORTS = ["va_last_error", "va_pack_first_fit", "va_bin_layout", "va_tile_shape", "va_worklist_size",
           "va_build_worklist", "va_check_worklist", "va_quantize_e4m3_per_head", "va_quantize_e4m3_per_head_device",
           "varlen_attn_bwd_workspace_bytes", "va_bwd_has_delta_kernel",
           "varlen_attn_fwd", "varlen_attn_bwd", "varlen_attn_bwd_stages", "varlen_attn_bwd_static", "varlen_attn_fwd_fp8",
           "va_quantize_e4m3_blockwise", "va_quantize_e4m3_blockwise_device", "varlen_attn_fwd_fp8_blockwise"]


def _check(rc):
    if rc != VA_OK:
        raise VarlenAttnError(rc, _lib.va_last_error().decode())


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _prefix(prefix_lens, mask_mode, num_seqs):
    """The prefix_lens argument as the C side reads it: one entry per sample, or the pairs (P, P2)
    of VA_MASK_THREE_BLOCK, given as [num_seqs, 2] or flat.  The library cannot see the array's
    length, so it is checked here."""
    if prefix_lens is None:
        return None
    pl = _i32(prefix_lens).reshape(-1)
    want = 2 * num_seqs if mask_mode == VA_MASK_THREE_BLOCK else num_seqs
    if mask_mode != VA_MASK_CAUSAL and pl.size != want:
        raise ValueError(f"prefix_lens holds {pl.size} entries, mask mode {mask_mode} needs {want}")
    return pl


def _ptr(a):
    """Pointer of a numpy array, a torch tensor, or None."""
    if a is None:
        return ctypes.c_void_p(0)
    if isinstance(a, np.ndarray):
        return a.ctypes.data_as(ctypes.c_void_p)
    return ctypes.c_void_p(a.data_ptr())


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def va_last_error() -> str:
    return _lib.va_last_error().decode()


def va_pack_first_fit(lens, budget):
    lens = _i32(lens)
    n = len(lens)
    bin_of = np.zeros(n, dtype=np.int32)
    pos = np.zeros(n, dtype=np.int32)
    nb = ctypes.c_int32(0)
    _check(_lib.va_pack_first_fit(_ptr(lens), ctypes.c_int32(n), ctypes.c_int32(budget),
                                  _ptr(bin_of), _ptr(pos), ctypes.byref(nb)))
    return bin_of, pos, nb.value


def va_bin_layout(lens, prefix=None):
    """cu_seqlens, prefix_lens, max_seqlen of one bin.  A [n, 2] ``prefix`` (the block ends of
    VA_MASK_THREE_BLOCK) goes through the library one column at a time and comes back as [n, 2]."""
    lens = _i32(lens)
    n = len(lens)
    if prefix is not None and np.ndim(prefix) == 2:
        cols = [va_bin_layout(lens, np.asarray(prefix)[:, j]) for j in range(2)]
        return cols[0][0], np.stack([cols[0][1], cols[1][1]], axis=1), cols[0][2]
    pre = None if prefix is None else _i32(prefix)
    cu = np.zeros(n + 1, dtype=np.int32)
    pl = None if prefix is None else np.zeros(n, dtype=np.int32)
    mx = ctypes.c_int32(0)
    _check(_lib.va_bin_layout(_ptr(lens), _ptr(pre), ctypes.c_int32(n), _ptr(cu), _ptr(pl), ctypes.byref(mx)))
    return cu, pl, mx.value


def va_tile_shape(pass_id, head_dim, num_q_heads, num_kv_heads):
    rows, cols = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(_lib.va_tile_shape(ctypes.c_int32(pass_id), ctypes.c_int32(head_dim), ctypes.c_int32(num_q_heads),
                              ctypes.c_int32(num_kv_heads), ctypes.byref(rows), ctypes.byref(cols)))
    return rows.value, cols.value


def va_worklist_size(cu_seqlens, pass_id, head_dim, num_q_heads, num_kv_heads):
    cu = _i32(cu_seqlens)
    nbytes = ctypes.c_size_t(0)
    _check(_lib.va_worklist_size(_ptr(cu), ctypes.c_int32(len(cu) - 1), ctypes.c_int32(pass_id),
                                  ctypes.c_int32(head_dim), ctypes.c_int32(num_q_heads),
                                  ctypes.c_int32(num_kv_heads), ctypes.byref(nbytes)))
    return nbytes.value


def va_build_worklist(cu_seqlens, prefix_lens, mask_mode, pass_id, head_dim, num_q_heads, num_kv_heads):
    """Returns the whole work list as an int32 array of 8-word records (see ``worklist_items`` and
    ``worklist_schedule`` for its parts)."""
    cu = _i32(cu_seqlens)
    pl = _prefix(prefix_lens, mask_mode, len(cu) - 1)
    nbytes = va_worklist_size(cu, pass_id, head_dim, num_q_heads, num_kv_heads)
    buf = np.zeros((nbytes // 32, 8), dtype=np.int32)
    n_items = ctypes.c_int32(0)
    _check(_lib.va_build_worklist(_ptr(cu), _ptr(pl), ctypes.c_int32(len(cu) - 1), ctypes.c_int32(mask_mode),
                                  ctypes.c_int32(pass_id), ctypes.c_int32(head_dim), ctypes.c_int32(num_q_heads),
                                  ctypes.c_int32(num_kv_heads), _ptr(buf), ctypes.c_size_t(nbytes),
                                  ctypes.byref(n_items)))
    assert n_items.value == buf[0, 6]
    return buf


def va_check_worklist(worklist_host, pass_id, cu_seqlens, prefix_lens, shape):
    """Raises VarlenAttnError unless the device calls would accept this host copy of a work list."""
    cu = _i32(cu_seqlens)
    pl = _prefix(prefix_lens, shape.mask_mode, len(cu) - 1)
    wl = np.ascontiguousarray(worklist_host, dtype=np.int32)
    _check(_lib.va_check_worklist(_ptr(wl), ctypes.c_int32(pass_id), _ptr(cu), _ptr(pl), ctypes.byref(shape)))


def worklist_items(wl):
    """Item records [num_items, 8] of a work list."""
    return wl[2:2 + wl[0, 6]]


def worklist_merges(wl):
    """Merge records [num_merges, 8] of a dK/dV work list: one per key tile whose query tiles were cut into
    pieces, {kv_row0, kv_rows, first partial slot, pieces, qt_first, qt_count, 0, 0}."""
    n = int(wl[1, 7])
    first = int(wl[1, 6]) - n
    return wl[first:first + n]


def worklist_schedule(wl):
    """(table [num_workgroups, 2] of (first work, count), work ids [num_works]) of a work list.  A table
    entry is 16 words: the item of the workgroup's first work, that work's id, the id of the second one,
    then first schedule position and count."""
    flat = wl.reshape(-1)
    P, W = int(wl[1, 0]), int(wl[1, 1])
    table = flat[8 * wl[1, 4]:8 * wl[1, 4] + 16 * P].reshape(P, 16)[:, 10:12]
    ids = flat[8 * wl[1, 5]:8 * wl[1, 5] + W]
    return table, ids


def va_quantize_e4m3_per_head(x_bf16_bits):
    """x: uint16 array [T, H, D] of bfloat16 bit patterns -> (uint8 codes, float32 descale[H])."""
    x = np.ascontiguousarray(x_bf16_bits, dtype=np.uint16)
    T, H, D = x.shape
    codes = np.zeros((T, H, D), dtype=np.uint8)
    descale = np.zeros(H, dtype=np.float32)
    _check(_lib.va_quantize_e4m3_per_head(_ptr(x), ctypes.c_int32(T), ctypes.c_int32(H), ctypes.c_int32(D),
                                          _ptr(codes), _ptr(descale)))
    return codes, descale


def va_quantize_e4m3_per_head_device(x, codes, descale, stream=None):
    """x: bfloat16 device tensor [T, H, D]; codes: uint8 device tensor [T, H, D]; descale: float32 device
    tensor [H].  Enqueues the quantisation on the stream."""
    T, H, D = x.shape
    _check(_lib.va_quantize_e4m3_per_head_device(_ptr(x), ctypes.c_int32(T), ctypes.c_int32(H), ctypes.c_int32(D),
                                                 _ptr(codes), _ptr(descale), _stream_ptr(stream)))


def va_quantize_e4m3_blockwise(x_bf16_bits, cu_seqlens):
    """x: uint16 array [T, H, D] of bfloat16 bit patterns, T = cu_seqlens[-1] -> (uint8 codes [T, H, D],
    float32 descale_tok [T, H]: one scale per 128 tokens of a sample and head, repeated on its rows)."""
    x = np.ascontiguousarray(x_bf16_bits, dtype=np.uint16)
    cu = _i32(cu_seqlens)
    T, H, D = x.shape
    if T != int(cu[-1]):
        raise ValueError(f"x holds {T} rows, cu_seqlens ends at {int(cu[-1])}")
    codes = np.zeros((T, H, D), dtype=np.uint8)
    descale_tok = np.zeros((T, H), dtype=np.float32)
    _check(_lib.va_quantize_e4m3_blockwise(_ptr(x), _ptr(cu), ctypes.c_int32(len(cu) - 1), ctypes.c_int32(H),
                                           ctypes.c_int32(D), _ptr(codes), _ptr(descale_tok)))
    return codes, descale_tok


def va_quantize_e4m3_blockwise_device(x, cu_seqlens, cu_seqlens_device, codes, descale_tok, stream=None):
    """x: bfloat16 device tensor [T, H, D]; cu_seqlens: host int32 array; cu_seqlens_device: the same
    values in an int32 device tensor; codes: uint8 device tensor [T, H, D]; descale_tok: float32 device
    tensor [T, H].  Enqueues the quantisation on the stream."""
    cu = _i32(cu_seqlens)
    T, H, D = x.shape
    if T != int(cu[-1]) or cu_seqlens_device.numel() != len(cu) or tuple(codes.shape) != (T, H, D) \
            or tuple(descale_tok.shape) != (T, H):
        raise ValueError("shapes of x, cu_seqlens, codes and descale_tok disagree")
    _check(_lib.va_quantize_e4m3_blockwise_device(_ptr(x), _ptr(cu), _ptr(cu_seqlens_device), ctypes.c_int32(len(cu) - 1),
                                                  ctypes.c_int32(H), ctypes.c_int32(D), _ptr(codes), _ptr(descale_tok),
                                                  _stream_ptr(stream)))


def make_shape(total_tokens, num_seqs, num_q_heads, num_kv_heads, head_dim, max_seqlen, mask_mode):
    return va_shape(int(total_tokens), int(num_seqs), int(num_q_heads), int(num_kv_heads), int(head_dim),
                    int(max_seqlen), int(mask_mode))


def varlen_attn_bwd_workspace_bytes(shape):
    return int(_lib.varlen_attn_bwd_workspace_bytes(ctypes.byref(shape)))


def va_bwd_has_delta_kernel(head_dim):
    return bool(_lib.va_bwd_has_delta_kernel(ctypes.c_int32(head_dim)))


def varlen_attn_fwd(q, k, v, cu_seqlens, prefix_lens, worklist, worklist_host, shape, scale, out, lse, stream=None):
    cu = _i32(cu_seqlens)
    pl = _prefix(prefix_lens, shape.mask_mode, len(cu) - 1)
    _check(_lib.varlen_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(cu), _ptr(pl), _ptr(worklist), _ptr(worklist_host),
                                ctypes.byref(shape), ctypes.c_float(scale), _ptr(out), _ptr(lse), _stream_ptr(stream)))


def varlen_attn_bwd(q, k, v, out, lse, dout, cu_seqlens, prefix_lens, worklist_dkdv, worklist_dkdv_host,
                    worklist_dq, worklist_dq_host, shape, scale, dq, dk, dv, workspace, workspace_bytes, stream=None):
    cu = _i32(cu_seqlens)
    pl = _prefix(prefix_lens, shape.mask_mode, len(cu) - 1)
    _check(_lib.varlen_attn_bwd(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(dout), _ptr(cu), _ptr(pl),
                                _ptr(worklist_dkdv), _ptr(worklist_dkdv_host), _ptr(worklist_dq), _ptr(worklist_dq_host),
                                ctypes.byref(shape), ctypes.c_float(scale), _ptr(dq), _ptr(dk), _ptr(dv),
                                _ptr(workspace), ctypes.c_size_t(workspace_bytes), _stream_ptr(stream)))


def varlen_attn_bwd_static(q, k, v, out, lse, dout, cu_seqlens, prefix_lens, worklist_dkdv, worklist_dkdv_host,
                           worklist_dq, worklist_dq_host, shape, scale, dq, dk, dv, stream=None):
    cu = _i32(cu_seqlens)
    pl = _prefix(prefix_lens, shape.mask_mode, len(cu) - 1)
    _check(_lib.varlen_attn_bwd_static(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(dout), _ptr(cu), _ptr(pl),
                                       _ptr(worklist_dkdv), _ptr(worklist_dkdv_host), _ptr(worklist_dq),
                                       _ptr(worklist_dq_host), ctypes.byref(shape), ctypes.c_float(scale),
                                       _ptr(dq), _ptr(dk), _ptr(dv), _stream_ptr(stream)))


def varlen_attn_bwd_stages(q, k, v, out, lse, dout, cu_seqlens, prefix_lens, worklist_dkdv, worklist_dkdv_host,
                           worklist_dq, worklist_dq_host, shape, scale, dq, dk, dv, workspace, workspace_bytes,
                           stages, stream=None):
    cu = _i32(cu_seqlens)
    pl = _prefix(prefix_lens, shape.mask_mode, len(cu) - 1)
    _check(_lib.varlen_attn_bwd_stages(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), _ptr(dout), _ptr(cu), _ptr(pl),
                                       _ptr(worklist_dkdv), _ptr(worklist_dkdv_host), _ptr(worklist_dq),
                                       _ptr(worklist_dq_host), ctypes.byref(shape), ctypes.c_float(scale),
                                       _ptr(dq), _ptr(dk), _ptr(dv), _ptr(workspace), ctypes.c_size_t(workspace_bytes),
                                       _stream_ptr(stream), ctypes.c_uint32(stages)))


def varlen_attn_fwd_fp8(q8, k8, v8, q_descale, k_descale, v_descale, cu_seqlens, prefix_lens, worklist, worklist_host,
                        shape, scale, out, lse, stream=None):
    cu = _i32(cu_seqlens)
    pl = _prefix(prefix_lens, shape.mask_mode, len(cu) - 1)
    _check(_lib.varlen_attn_fwd_fp8(_ptr(q8), _ptr(k8), _ptr(v8), _ptr(q_descale), _ptr(k_descale), _ptr(v_descale),
                                    _ptr(cu), _ptr(pl), _ptr(worklist), _ptr(worklist_host), ctypes.byref(shape),
                                    ctypes.c_float(scale), _ptr(out), _ptr(lse), _stream_ptr(stream)))


def varlen_attn_fwd_fp8_blockwise(q8, k8, v8, q_descale_tok, k_descale_tok, v_descale_tok, cu_seqlens, prefix_lens,
                                  worklist, worklist_host, shape, scale, out, lse, stream=None):
    cu = _i32(cu_seqlens)
    pl = _prefix(prefix_lens, shape.mask_mode, len(cu) - 1)
    T = int(shape.total_tokens)
    for name, d, h in (("q", q_descale_tok, shape.num_q_heads), ("k", k_descale_tok, shape.num_kv_heads),
                       ("v", v_descale_tok, shape.num_kv_heads)):
        if d is not None and tuple(d.shape) != (T, h):  # the library cannot see the arrays' lengths
            raise ValueError(f"{name}_descale_tok has shape {tuple(d.shape)}, expected {(T, h)}")
    _check(_lib.varlen_attn_fwd_fp8_blockwise(_ptr(q8), _ptr(k8), _ptr(v8), _ptr(q_descale_tok), _ptr(k_descale_tok),
                                              _ptr(v_descale_tok), _ptr(cu), _ptr(pl), _ptr(worklist),
                                              _ptr(worklist_host), ctypes.byref(shape), ctypes.c_float(scale),
                                              _ptr(out), _ptr(lse), _stream_ptr(stream)))


class PackedStream:
    """Everything the device calls need for one packed stream, kept together:
    the host index arrays, the three work lists (host copies and device copies)
    and the shape record.  Plumbing only."""

    def __init__(self, cu_seqlens, prefix_lens, mask_mode, num_q_heads, num_kv_heads, head_dim,
                 max_seqlen=None, device="cuda:0", passes=(VA_PASS_FWD, VA_PASS_BWD_DKDV, VA_PASS_BWD_DQ)):
        self.cu_seqlens = _i32(cu_seqlens)
        self.prefix_lens = _prefix(prefix_lens, int(mask_mode), len(self.cu_seqlens) - 1)
        self.mask_mode = int(mask_mode)
        n = len(self.cu_seqlens) - 1
        lens = np.diff(self.cu_seqlens)
        if max_seqlen is None:
            max_seqlen = int(lens.max()) if n else 0
        self.shape = make_shape(self.cu_seqlens[-1], n, num_q_heads, num_kv_heads, head_dim, max_seqlen, mask_mode)
        self.worklist_host = {}
        self.worklist = {}
        for pid in passes:
            wl = va_build_worklist(self.cu_seqlens, self.prefix_lens, mask_mode, pid, head_dim, num_q_heads, num_kv_heads)
            self.worklist_host[pid] = wl
            self.worklist[pid] = torch.from_numpy(wl).to(device)
        self.device = device
        self._workspace = None

    def workspace(self):
        if self._workspace is None:
            nbytes = max(256, varlen_attn_bwd_workspace_bytes(self.shape))
            self._workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        return self._workspace

    def fwd(self, q, k, v, scale, out, lse, stream=None):
        varlen_attn_fwd(q, k, v, self.cu_seqlens, self.prefix_lens, self.worklist[VA_PASS_FWD],
                        self.worklist_host[VA_PASS_FWD], self.shape, scale, out, lse, stream)

    def bwd(self, q, k, v, out, lse, dout, scale, dq, dk, dv, stream=None):
        ws = self.workspace()
        varlen_attn_bwd(q, k, v, out, lse, dout, self.cu_seqlens, self.prefix_lens,
                        self.worklist[VA_PASS_BWD_DKDV], self.worklist_host[VA_PASS_BWD_DKDV],
                        self.worklist[VA_PASS_BWD_DQ], self.worklist_host[VA_PASS_BWD_DQ],
                        self.shape, scale, dq, dk, dv, ws, ws.numel(), stream)

    def bwd_static(self, q, k, v, out, lse, dout, scale, dq, dk, dv, stream=None):
        varlen_attn_bwd_static(q, k, v, out, lse, dout, self.cu_seqlens, self.prefix_lens,
                               self.worklist[VA_PASS_BWD_DKDV], self.worklist_host[VA_PASS_BWD_DKDV],
                               self.worklist[VA_PASS_BWD_DQ], self.worklist_host[VA_PASS_BWD_DQ],
                               self.shape, scale, dq, dk, dv, stream)

    def bwd_stages(self, q, k, v, out, lse, dout, scale, dq, dk, dv, stages, stream=None):
        ws = self.workspace()
        varlen_attn_bwd_stages(q, k, v, out, lse, dout, self.cu_seqlens, self.prefix_lens,
                               self.worklist[VA_PASS_BWD_DKDV], self.worklist_host[VA_PASS_BWD_DKDV],
                               self.worklist[VA_PASS_BWD_DQ], self.worklist_host[VA_PASS_BWD_DQ],
                               self.shape, scale, dq, dk, dv, ws, ws.numel(), stages, stream)

    def fwd_fp8_blockwise(self, q8, k8, v8, q_descale_tok, k_descale_tok, v_descale_tok, scale, out, lse, stream=None):
        varlen_attn_fwd_fp8_blockwise(q8, k8, v8, q_descale_tok, k_descale_tok, v_descale_tok, self.cu_seqlens,
                                      self.prefix_lens, self.worklist[VA_PASS_FWD], self.worklist_host[VA_PASS_FWD],
                                      self.shape, scale, out, lse, stream)

    def fwd_fp8(self, q8, k8, v8, q_descale, k_descale, v_descale, scale, out, lse, stream=None):
        varlen_attn_fwd_fp8(q8, k8, v8, q_descale, k_descale, v_descale, self.cu_seqlens, self.prefix_lens,
                            self.worklist[VA_PASS_FWD], self.worklist_host[VA_PASS_FWD], self.shape, scale,
                            out, lse, stream)

"""Thin ctypes binding over the C ABI in include/qlora.h.

Argument marshalling only: every step of the path runs in the HIP library.  torch is
used for device memory and for the current stream handle.  There is no CPU or eager
fallback: if the shared library is missing the import of a function raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, byref, c_float, c_int32, c_int64, c_size_t, c_void_p

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libqlora_hip.so")

EXPORTS = [
    "qlora_status_string", "qlora_last_hip_error", "qlora_nf4_sizes", "qlora_nf4_quantize",
    "qlora_nf4_dequant", "qlora_linear_fwd_sizes", "qlora_linear_bwd_sizes", "qlora_linear_fwd",
    "qlora_linear_bwd", "qlora_linear_bwd_acc", "qlora_linear_fwd_multi_sizes", "qlora_linear_fwd_multi", "qlora_workspace_init",
    "qlora_profile_gemm", "qlora_profile_gemm_read",
    "qlora_linear_dropout_sizes", "qlora_linear_fwd_dropout", "qlora_linear_bwd_dropout",
    "qlora_codebook_4bit", "qlora_quantize_4bit", "qlora_quant_sizes", "qlora_quantize_int8",
    "qlora_linear_fwd_list_sizes", "qlora_linear_bwd_list_sizes", "qlora_linear_fwd_list", "qlora_linear_bwd_list",
    "qlora_workspace_check", "qlora_fewtok_poll_limit", "qlora_bwd_fused_dequant", "qlora_mfma_probe", "qlora_hbm_probe", "qlora_nf4_quantize_static",
    "qlora_grad_sqnorm", "qlora_adam_step", "qlora_linear_fwd_stacked_sizes", "qlora_linear_fwd_stacked",
    "qlora_linear_bwd_stacked_sizes", "qlora_linear_bwd_stacked",
    "qlora_kbit_sizes", "qlora_kbit_pack", "qlora_kbit_unpack",
]


class qlora_adam_config(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_double), ("beta1", ctypes.c_double), ("beta2", ctypes.c_double),
                ("eps", ctypes.c_double), ("weight_decay", ctypes.c_double), ("grad_scale", ctypes.c_double),
                ("max_grad_norm", ctypes.c_double), ("step", c_int64), ("zero_grad", c_int32), ("reserved", c_int32)]


class QloraError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{message} (status {status})")
        self.status = status


class qlora_nf4_view(Structure):
    _fields_ = [("packed", c_void_p), ("c2_code", c_void_p), ("c1", c_void_p), ("c2_mean", c_void_p),
                ("rows", c_int64), ("cols", c_int64), ("blocksize", c_int32), ("dq_blocksize", c_int32),
                ("dtype", c_int32), ("reserved", c_int32)]


_lib = None


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2305_14314_amd.build` "
                          "(there is no fallback path)")
    L = ctypes.CDLL(LIB_PATH)
    vp, sp = c_void_p, POINTER(c_size_t)
    L.qlora_status_string.restype = ctypes.c_char_p
    L.qlora_status_string.argtypes = [c_int32]
    L.qlora_last_hip_error.restype = ctypes.c_int
    L.qlora_nf4_sizes.argtypes = [c_int64, c_int64, c_int32, c_int32, sp, sp, sp, sp]
    L.qlora_nf4_quantize.argtypes = [vp, c_int64, c_int64, c_int32, c_int32, vp, vp, vp, vp, vp, c_size_t, vp]
    L.qlora_nf4_quantize_static.argtypes = [vp, c_int64, c_int64, c_int32, c_int32, vp, vp, vp, vp, vp]
    L.qlora_quantize_4bit.argtypes = [vp, c_int64, c_int64, c_int32, c_int32, c_int32, vp, vp, vp, vp, vp, c_size_t, vp]
    L.qlora_codebook_4bit.argtypes = [c_int32, vp]
    L.qlora_quant_sizes.argtypes = [c_int64, c_int64, c_int32, c_int32, c_int32, sp, sp, sp, sp]
    L.qlora_quantize_int8.argtypes = [vp, c_int64, c_int64, c_int32, c_int32, vp, vp, vp, vp, vp, c_size_t, vp]
    L.qlora_nf4_dequant.argtypes = [POINTER(qlora_nf4_view), vp, vp]
    L.qlora_linear_fwd_sizes.argtypes = [c_int64, c_int64, c_int64, c_int32, sp]
    L.qlora_linear_bwd_sizes.argtypes = [c_int64, c_int64, c_int64, c_int32, sp]
    L.qlora_linear_fwd.argtypes = [vp, POINTER(qlora_nf4_view), vp, vp, c_float, c_int64, c_int32, vp, vp,
                                   vp, c_size_t, vp]
    L.qlora_linear_bwd.argtypes = [vp, vp, POINTER(qlora_nf4_view), vp, vp, c_float, c_int64, c_int32, vp,
                                   vp, vp, vp, vp, c_size_t, vp]
    L.qlora_linear_bwd_acc.argtypes = list(L.qlora_linear_bwd.argtypes)
    L.qlora_linear_fwd_multi_sizes.argtypes = [c_int64, c_int32, c_int64, POINTER(c_int64), POINTER(c_int32), sp]
    L.qlora_linear_fwd_multi.argtypes = [vp, c_int32, POINTER(qlora_nf4_view), POINTER(vp), POINTER(vp), POINTER(c_float),
                                         c_int64, POINTER(c_int32), POINTER(vp), vp, c_size_t, vp]
    L.qlora_linear_fwd_stacked_sizes.argtypes = list(L.qlora_linear_fwd_multi_sizes.argtypes)
    L.qlora_linear_fwd_stacked.argtypes = [vp, c_int32, POINTER(qlora_nf4_view), POINTER(vp), POINTER(vp), POINTER(c_float),
                                           c_int64, POINTER(c_int32), vp, POINTER(vp), vp, c_size_t, vp]
    L.qlora_linear_bwd_stacked_sizes.argtypes = list(L.qlora_linear_fwd_multi_sizes.argtypes)
    L.qlora_linear_bwd_stacked.argtypes = [vp, vp, c_int32, POINTER(qlora_nf4_view), POINTER(vp), POINTER(vp), POINTER(c_float),
                                           c_int64, POINTER(c_int32), POINTER(vp), vp, POINTER(vp), POINTER(vp), vp,
                                           c_size_t, vp]
    L.qlora_linear_dropout_sizes.argtypes = [c_int64, c_int64, c_int64, c_int32, sp, sp]
    L.qlora_linear_fwd_dropout.argtypes = [vp, POINTER(qlora_nf4_view), vp, vp, c_float, c_int64, c_int32, vp, c_float,
                                           vp, vp, vp, c_size_t, vp]
    L.qlora_linear_bwd_dropout.argtypes = [vp, vp, POINTER(qlora_nf4_view), vp, vp, c_float, c_int64, c_int32, vp, c_float,
                                           vp, vp, vp, vp, vp, vp, vp, c_size_t, vp]
    L.qlora_linear_fwd_list_sizes.argtypes = [c_int64, c_int32, POINTER(c_int64), POINTER(c_int64), POINTER(c_int32), sp]
    L.qlora_linear_bwd_list_sizes.argtypes = list(L.qlora_linear_fwd_list_sizes.argtypes)
    L.qlora_linear_fwd_list.argtypes = [c_int32, POINTER(vp), POINTER(qlora_nf4_view), POINTER(vp), POINTER(vp),
                                        POINTER(c_float), c_int64, POINTER(c_int32), POINTER(vp), vp, c_size_t, vp]
    L.qlora_linear_bwd_list.argtypes = list(L.qlora_linear_fwd_list.argtypes)
    L.qlora_workspace_check.argtypes = [vp, c_size_t, vp]
    L.qlora_fewtok_poll_limit.argtypes = [c_int32]
    L.qlora_bwd_fused_dequant.argtypes = [c_int32]
    L.qlora_mfma_probe.argtypes = [c_int32, c_int32, vp, c_size_t, vp]
    L.qlora_hbm_probe.argtypes = [c_int32, vp, vp, c_int64, vp, c_int32, vp]
    L.qlora_grad_sqnorm.argtypes = [vp, c_int64, vp, vp]
    L.qlora_kbit_sizes.argtypes = [c_int64, c_int64, c_int32, sp]
    L.qlora_kbit_pack.argtypes = [vp, c_int64, c_int64, c_int32, vp, vp]
    L.qlora_kbit_unpack.argtypes = [vp, c_int64, c_int64, c_int32, vp, vp]
    L.qlora_adam_step.argtypes = [vp, vp, vp, vp, vp, c_int64, POINTER(qlora_adam_config), vp, vp]
    L.qlora_fewtok_poll_limit.restype = None
    L.qlora_profile_gemm.argtypes = [ctypes.c_int]
    L.qlora_profile_gemm.restype = None
    L.qlora_profile_gemm_read.argtypes = [POINTER(ctypes.c_double), POINTER(c_int64), POINTER(ctypes.c_double)]
    for name in EXPORTS:
        if name not in ("qlora_status_string", "qlora_last_hip_error", "qlora_profile_gemm", "qlora_fewtok_poll_limit"):
            getattr(L, name).restype = c_int32
    _lib = L
    return L


def _check(st: int):
    if st != 0:
        raise QloraError(st, lib().qlora_status_string(st).decode())


def _ptr(t):
    return None if t is None else c_void_p(t.data_ptr())


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return c_void_p(s.cuda_stream)


class NF4Weight:
    """Device buffers of one quantised h x o weight plus the view struct the C ABI takes."""

    def __init__(self, rows, cols, packed, code, c1, mean, blocksize=64, dq_blocksize=256, dtype=0):
        self.rows, self.cols = int(rows), int(cols)
        self.blocksize, self.dq_blocksize = int(blocksize), int(dq_blocksize)
        self.packed, self.code, self.c1, self.mean = packed, code, c1, mean
        self.dtype = int(dtype)                               # NF4 = 0, or FP4_E2M1 / FP4_E3M0 / INT4 / INT8

    def view(self) -> qlora_nf4_view:
        ptr = lambda t: None if t is None or t.numel() == 0 else t.data_ptr()
        per_byte = 1 if self.dtype == 4 else 2                # weights per byte of `packed`: INT8 one, the 4-bit types two
        if self.packed.numel() * per_byte != self.rows * self.cols:
            raise ValueError("NF4Weight: size of `packed` does not match rows, cols and dtype")
        return qlora_nf4_view(ptr(self.packed), ptr(self.code), ptr(self.c1), ptr(self.mean), self.rows, self.cols,
                              self.blocksize, self.dq_blocksize, self.dtype, 0)

    @property
    def nbytes(self) -> int:
        if self.dq_blocksize == 0:                            # no Double Quantization: c1 holds the fp32 constants c2
            return self.packed.numel() + 4 * self.c1.numel()
        return self.packed.numel() + self.code.numel() + 4 * self.c1.numel() + 4

    def code_flat(self):
        """The 8-bit codes in flattened block order (block row * cols/64 + blk), as a new device tensor.

        The library stores them column-group-major (include/qlora.h): position(row, blk) =
        4 * rows * (blk // 4) + row * w + blk % 4, with w = 4 or, for the last group, cols/64 - 4 * (blk // 4)."""
        bpr = self.cols // self.blocksize
        dev = self.code.device
        row = torch.arange(self.rows, device=dev, dtype=torch.int64).repeat_interleave(bpr)
        blk = torch.arange(bpr, device=dev, dtype=torch.int64).repeat(self.rows)
        grp = blk // 4
        width = torch.clamp(bpr - 4 * grp, max=4)
        return self.code[4 * self.rows * grp + row * width + blk % 4]


def qlora_nf4_sizes(rows, cols, blocksize=64, dq_blocksize=256):
    """(packed_bytes, code_bytes, c1_bytes, scratch_bytes)"""
    out = [c_size_t(0) for _ in range(4)]
    _check(lib().qlora_nf4_sizes(rows, cols, blocksize, dq_blocksize, *[byref(x) for x in out]))
    return tuple(int(x.value) for x in out)


def qlora_quant_sizes(rows, cols, blocksize=64, dq_blocksize=256, dtype=0):
    """(packed_bytes, code_bytes, c1_bytes, scratch_bytes) for any data type (INT8: one byte per weight)."""
    out = [c_size_t(0) for _ in range(4)]
    _check(lib().qlora_quant_sizes(rows, cols, blocksize, dq_blocksize, int(dtype), *[byref(x) for x in out]))
    return tuple(int(x.value) for x in out)


def nf4_alloc(rows, cols, device, blocksize=64, dq_blocksize=256, dtype=0) -> NF4Weight:
    """Uninitialised device buffers for a quantised rows x cols weight."""
    pb, cb, c1b, _ = qlora_quant_sizes(rows, cols, blocksize, dq_blocksize, dtype)
    w = NF4Weight(rows, cols, torch.empty(pb, dtype=torch.uint8, device=device),
                  torch.empty(cb, dtype=torch.uint8, device=device),
                  torch.empty(c1b // 4, dtype=torch.float32, device=device),
                  torch.empty(1, dtype=torch.float32, device=device), blocksize, dq_blocksize)
    w.dtype = int(dtype)
    return w


NF4, FP4_E2M1, FP4_E3M0, INT4, INT8, NF3, NF2 = 0, 1, 2, 3, 4, 5, 6


def qlora_quantize_int8(W, blocksize=64, dq_blocksize=256, scratch=None, stream=None, out=None) -> NF4Weight:
    """Blockwise 8-bit integers (Eq. 1).  The result's `packed` holds the signed bytes (as uint8 storage)."""
    assert W.is_cuda and W.dtype == torch.float32 and W.dim() == 2 and W.is_contiguous()
    rows, cols = W.shape
    sb = qlora_quant_sizes(rows, cols, blocksize, dq_blocksize, INT8)[3]
    if out is None:
        out = nf4_alloc(rows, cols, W.device, blocksize, dq_blocksize, INT8)
    assert (out.rows, out.cols, out.blocksize, out.dq_blocksize, out.dtype) == (rows, cols, blocksize, dq_blocksize, INT8)
    assert out.packed.numel() == rows * cols
    if scratch is None:
        scratch = torch.empty(sb, dtype=torch.uint8, device=W.device)
    _check(lib().qlora_quantize_int8(_ptr(W), rows, cols, blocksize, dq_blocksize, _ptr(out.packed), _ptr(out.code),
                                     _ptr(out.c1), _ptr(out.mean), _ptr(scratch), scratch.numel(), _stream(stream)))
    return out


def qlora_codebook_4bit(dtype):
    """The 16 fp32 values of a 4-bit data type (NF4, FP4_E2M1, FP4_E3M0, INT4), ascending, as a list."""
    out = (c_float * 16)()
    _check(lib().qlora_codebook_4bit(int(dtype), out))
    return list(out)


def qlora_quantize_4bit(W, dtype, blocksize=64, dq_blocksize=256, scratch=None, stream=None, out=None) -> NF4Weight:
    """qlora_nf4_quantize with one of the other 4-bit data types of the paper's comparison."""
    return qlora_nf4_quantize(W, blocksize, dq_blocksize, scratch, stream, out, dtype=dtype)


def qlora_nf4_quantize(W, blocksize=64, dq_blocksize=256, scratch=None, stream=None, out=None, dtype=0) -> NF4Weight:
    """W: fp32 device tensor (h, o).  Returns the quantised weight (in `out` if given, else new buffers)."""
    assert W.is_cuda and W.dtype == torch.float32 and W.dim() == 2 and W.is_contiguous()
    rows, cols = W.shape
    sb = qlora_nf4_sizes(rows, cols, blocksize, dq_blocksize)[3]
    dev = W.device
    if out is None:
        out = nf4_alloc(rows, cols, dev, blocksize, dq_blocksize)
    assert (out.rows, out.cols, out.blocksize, out.dq_blocksize) == (rows, cols, blocksize, dq_blocksize)
    assert int(dtype) in (NF4, FP4_E2M1, FP4_E3M0, INT4, NF3, NF2) and out.packed.numel() == rows * cols // 2
    packed, code, c1, mean = out.packed, out.code, out.c1, out.mean
    if scratch is None:
        scratch = torch.empty(sb, dtype=torch.uint8, device=dev)
    if dtype == 0:
        _check(lib().qlora_nf4_quantize(_ptr(W), rows, cols, blocksize, dq_blocksize, _ptr(packed), _ptr(code),
                                        _ptr(c1), _ptr(mean), _ptr(scratch), scratch.numel(), _stream(stream)))
    else:
        _check(lib().qlora_quantize_4bit(_ptr(W), rows, cols, blocksize, dq_blocksize, int(dtype), _ptr(packed),
                                         _ptr(code), _ptr(c1), _ptr(mean), _ptr(scratch), scratch.numel(),
                                         _stream(stream)))
    out.dtype = int(dtype)
    return out


STATIC_QUANT_MAX_WEIGHTS = 1 << 28


def qlora_nf4_quantize_static(W, out: NF4Weight, stream=None) -> NF4Weight:
    """qlora_nf4_quantize into the caller's buffers `out`, with the scratch in the library's own device array:
    nothing is allocated here or below."""
    assert W.is_cuda and W.dtype == torch.float32 and W.dim() == 2 and W.is_contiguous()
    rows, cols = W.shape
    assert (out.rows, out.cols, out.dtype) == (rows, cols, NF4)
    _check(lib().qlora_nf4_quantize_static(_ptr(W), rows, cols, out.blocksize, out.dq_blocksize, _ptr(out.packed),
                                           _ptr(out.code), _ptr(out.c1), _ptr(out.mean), _stream(stream)))
    return out


def qlora_nf4_dequant(Wq: NF4Weight, out=None, stream=None):
    """Returns the bf16 weight (h, o)."""
    if out is None:
        out = torch.empty((Wq.rows, Wq.cols), dtype=torch.bfloat16, device=Wq.packed.device)
    v = Wq.view()
    _check(lib().qlora_nf4_dequant(byref(v), _ptr(out), _stream(stream)))
    return out


def qlora_linear_fwd_sizes(M, h, o, r) -> int:
    out = c_size_t(0)
    _check(lib().qlora_linear_fwd_sizes(M, h, o, r, byref(out)))
    return int(out.value)


def qlora_linear_bwd_sizes(M, h, o, r) -> int:
    out = c_size_t(0)
    _check(lib().qlora_linear_bwd_sizes(M, h, o, r, byref(out)))
    return int(out.value)


WORKSPACE_HEADER_BYTES = 16384


def _fwd_bytes(Wq, M, h, o, r):
    """Workspace of a forward call: a weight without Double Quantization always takes the large-GEMM path."""
    few = Wq.dq_blocksize and Wq.dtype != INT8
    return qlora_linear_fwd_sizes(M, h, o, r) if few else qlora_linear_dropout_sizes(M, h, o, r)[0]


def _bwd_bytes(Wq, M, h, o, r):
    few = Wq.dq_blocksize and Wq.dtype != INT8
    return qlora_linear_bwd_sizes(M, h, o, r) if few else qlora_linear_dropout_sizes(M, h, o, r)[1]


def qlora_workspace_init(workspace, stream=None):
    """Zeroes the counter header of a workspace buffer: once per buffer, before its first use."""
    _check(lib().qlora_workspace_init(_ptr(workspace), workspace.numel(), _stream(stream)))
    return workspace


def workspace_alloc(nbytes, device="cuda", stream=None):
    """A uint8 workspace of at least `nbytes` whose counter header is zeroed."""
    ws = torch.empty(max(int(nbytes), WORKSPACE_HEADER_BYTES), dtype=torch.uint8, device=device)
    return qlora_workspace_init(ws, stream)


def qlora_linear_fwd(X, Wq: NF4Weight, L1, L2, s, Y=None, T_save=None, workspace=None, stream=None):
    """Y = X dequant(Wq) + s (X L1) L2.  X (M, h), L1 (h, r), L2 (r, o) bf16 device tensors;
    T_save, if given, is an (M, 2r) bf16 tensor that receives X L1 as a [hi | lo] pair."""
    M, h = X.shape
    o = Wq.cols
    r = 0 if L1 is None else L1.shape[1]
    if Y is None:
        Y = torch.empty((M, o), dtype=torch.bfloat16, device=X.device)
    if workspace is None:
        workspace = workspace_alloc(_fwd_bytes(Wq, M, h, o, r), X.device, stream)
    v = Wq.view()
    _check(lib().qlora_linear_fwd(_ptr(X), byref(v), _ptr(L1), _ptr(L2), float(s), M, r, _ptr(Y), _ptr(T_save),
                                  _ptr(workspace), workspace.numel(), _stream(stream)))
    return Y


MULTI_MAX = 4


def qlora_linear_fwd_multi_sizes(M, h, os_, rs) -> int:
    n = len(os_)
    out = c_size_t(0)
    _check(lib().qlora_linear_fwd_multi_sizes(M, n, h, (c_int64 * n)(*os_), (c_int32 * n)(*rs), byref(out)))
    return int(out.value)


def qlora_linear_fwd_multi(X, Wqs, L1s, L2s, ss, Ys=None, workspace=None, stream=None):
    """Y[l] = X dequant(Wqs[l]) + ss[l] (X L1s[l]) L2s[l] for up to MULTI_MAX layers that read the same X (M, h);
    at M <= 16 all of them in one launch.  L1s[l] / L2s[l] may be None (no adapter on that layer)."""
    n = len(Wqs)
    M, h = X.shape
    rs = [0 if L1s[l] is None else L1s[l].shape[1] for l in range(n)]
    if Ys is None:
        Ys = [torch.empty((M, w.cols), dtype=torch.bfloat16, device=X.device) for w in Wqs]
    if workspace is None:
        workspace = workspace_alloc(qlora_linear_fwd_multi_sizes(M, h, [w.cols for w in Wqs], rs), X.device, stream)
    views = (qlora_nf4_view * n)(*[w.view() for w in Wqs])
    ptrs = lambda ts: (c_void_p * n)(*[None if t is None else t.data_ptr() for t in ts])
    _check(lib().qlora_linear_fwd_multi(_ptr(X), n, views, ptrs(L1s), ptrs(L2s), (c_float * n)(*[float(s) for s in ss]),
                                        M, (c_int32 * n)(*rs), ptrs(Ys), _ptr(workspace), workspace.numel(),
                                        _stream(stream)))
    return Ys


def qlora_linear_fwd_stacked_sizes(M, h, os_, rs) -> int:
    n = len(os_)
    out = c_size_t()
    _check(lib().qlora_linear_fwd_stacked_sizes(M, n, h, (c_int64 * n)(*os_), (c_int32 * n)(*rs), ctypes.byref(out)))
    return int(out.value)


def qlora_linear_fwd_stacked(X, Wqs, L1s, L2s, ss, Y=None, T_saves=None, workspace=None, stream=None):
    """The layers of qlora_linear_fwd_multi with one matrix product: returns Y (M, sum o), layer l in the column range
    that starts at o[0] + ... + o[l-1].  T_saves: None or a list of (M, 2 r) bf16 tensors / None per layer."""
    n = len(Wqs)
    M, h = X.shape
    rs = [0 if L1s[l] is None else L1s[l].shape[1] for l in range(n)]
    N = sum(w.cols for w in Wqs)
    if Y is None:
        Y = torch.empty((M, N), dtype=torch.bfloat16, device=X.device)
    assert Y.shape == (M, N) and Y.is_contiguous()
    if workspace is None:
        workspace = workspace_alloc(qlora_linear_fwd_stacked_sizes(M, h, [w.cols for w in Wqs], rs), X.device, stream)
    views = (qlora_nf4_view * n)(*[w.view() for w in Wqs])
    ptrs = lambda ts: (c_void_p * n)(*[None if t is None else t.data_ptr() for t in ts])
    _check(lib().qlora_linear_fwd_stacked(_ptr(X), n, views, ptrs(L1s), ptrs(L2s), (c_float * n)(*[float(s) for s in ss]),
                                          M, (c_int32 * n)(*rs), _ptr(Y), None if T_saves is None else ptrs(T_saves),
                                          _ptr(workspace), workspace.numel(), _stream(stream)))
    return Y


def qlora_linear_bwd_stacked_sizes(M, h, os_, rs) -> int:
    n = len(os_)
    out = c_size_t()
    _check(lib().qlora_linear_bwd_stacked_sizes(M, n, h, (c_int64 * n)(*os_), (c_int32 * n)(*rs), ctypes.byref(out)))
    return int(out.value)


def qlora_linear_bwd_stacked(dY, X, Wqs, L1s, L2s, ss, T_saveds=None, dX=None, need_dL=True, workspace=None, stream=None,
                             dL1s=None, dL2s=None):
    """dY: (M, sum o) in the stacked layout.  Returns (dX (M, h) = the sum of the layers' input gradients, dL1s, dL2s);
    the adapter gradients are lists with None for layers without an adapter (or all None with need_dL=False)."""
    n = len(Wqs)
    M = dY.shape[0]
    h = Wqs[0].rows
    rs = [0 if L1s[l] is None else L1s[l].shape[1] for l in range(n)]
    assert dY.shape == (M, sum(w.cols for w in Wqs)) and dY.is_contiguous()
    dev = dY.device
    if dX is None:
        dX = torch.empty((M, h), dtype=torch.bfloat16, device=dev)
    if dL1s is None:
        dL1s = [torch.empty((h, rs[l]), dtype=torch.bfloat16, device=dev) if need_dL and rs[l] else None for l in range(n)]
    if dL2s is None:
        dL2s = [torch.empty((rs[l], Wqs[l].cols), dtype=torch.bfloat16, device=dev) if need_dL and rs[l] else None
                for l in range(n)]
    if workspace is None:
        workspace = workspace_alloc(qlora_linear_bwd_stacked_sizes(M, h, [w.cols for w in Wqs], rs), dev, stream)
    views = (qlora_nf4_view * n)(*[w.view() for w in Wqs])
    ptrs = lambda ts: (c_void_p * n)(*[None if t is None else t.data_ptr() for t in ts])
    _check(lib().qlora_linear_bwd_stacked(_ptr(dY), _ptr(X), n, views, ptrs(L1s), ptrs(L2s),
                                          (c_float * n)(*[float(s) for s in ss]), M, (c_int32 * n)(*rs),
                                          None if T_saveds is None else ptrs(T_saveds), _ptr(dX), ptrs(dL1s), ptrs(dL2s),
                                          _ptr(workspace), workspace.numel(), _stream(stream)))
    return dX, dL1s, dL2s


LIST_MAX = 8


def qlora_linear_list_sizes(M, hs, os_, rs, backward=False) -> int:
    n = len(hs)
    out = c_size_t(0)
    fn = lib().qlora_linear_bwd_list_sizes if backward else lib().qlora_linear_fwd_list_sizes
    _check(fn(M, n, (c_int64 * n)(*hs), (c_int64 * n)(*os_), (c_int32 * n)(*rs), byref(out)))
    return int(out.value)


def _list_call(fn, ins, Wqs, L1s, L2s, ss, outs, out_dim, workspace, stream, backward):
    n = len(Wqs)
    M = ins[0].shape[0]
    rs = [0 if L1s[l] is None else L1s[l].shape[1] for l in range(n)]
    if outs is None:
        outs = [torch.empty((M, out_dim(w)), dtype=torch.bfloat16, device=ins[0].device) for w in Wqs]
    if workspace is None:
        workspace = workspace_alloc(qlora_linear_list_sizes(M, [w.rows for w in Wqs], [w.cols for w in Wqs], rs, backward),
                                    ins[0].device, stream)
    views = (qlora_nf4_view * n)(*[w.view() for w in Wqs])
    ptrs = lambda ts: (c_void_p * n)(*[None if t is None else t.data_ptr() for t in ts])
    _check(fn(n, ptrs(ins), views, ptrs(L1s), ptrs(L2s), (c_float * n)(*[float(s) for s in ss]), M, (c_int32 * n)(*rs),
              ptrs(outs), _ptr(workspace), workspace.numel(), _stream(stream)))
    return outs


def qlora_linear_fwd_list(Xs, Wqs, L1s, L2s, ss, Ys=None, workspace=None, stream=None):
    """Y[l] = X[l] dequant(Wqs[l]) + ss[l] (X[l] L1s[l]) L2s[l] for up to LIST_MAX independent layers, each with its own
    input of M tokens; at M <= 16 all of them in one persistent launch."""
    return _list_call(lib().qlora_linear_fwd_list, Xs, Wqs, L1s, L2s, ss, Ys, lambda w: w.cols, workspace, stream, False)


def qlora_linear_bwd_list(dYs, Wqs, L1s, L2s, ss, dXs=None, workspace=None, stream=None):
    """dX[l] = dY[l] dequant(Wqs[l])^T + ss[l] (dY[l] L2s[l]^T) L1s[l]^T for up to LIST_MAX independent layers."""
    return _list_call(lib().qlora_linear_bwd_list, dYs, Wqs, L1s, L2s, ss, dXs, lambda w: w.rows, workspace, stream, True)


def qlora_workspace_check(workspace, stream=None) -> bool:
    """Synchronises the stream; True if no kernel has found the workspace's counter header dirty since it was initialised."""
    st = lib().qlora_workspace_check(_ptr(workspace), workspace.numel(), _stream(stream))
    if st == -7:
        return False
    _check(st)
    return True


def qlora_fewtok_poll_limit(polls: int):
    lib().qlora_fewtok_poll_limit(int(polls))


def qlora_hbm_probe(mode: int, src, dst, sink, wgs_per_cu: int = 8, stream=None) -> int:
    """Enqueues a plain stream (0: read src, 1: write dst, 2: copy src to dst); returns the bytes one buffer holds."""
    buf = src if src is not None else dst
    nbytes = buf.numel() * buf.element_size()
    _check(lib().qlora_hbm_probe(int(mode), _ptr(src), _ptr(dst), nbytes, _ptr(sink), int(wgs_per_cu), _stream(stream)))
    return nbytes


def qlora_mfma_probe(lds_traffic: int, iters: int, out=None, stream=None) -> float:
    """Enqueues the register-only MFMA loop (lds_traffic 0: none, 1: fragment reads, 2: and tile writes); returns the
    flops of the call (time it with events around the call)."""
    if out is None:
        out = torch.empty(256 * 256, dtype=torch.float32, device="cuda")
    _check(lib().qlora_mfma_probe(int(lds_traffic), int(iters), _ptr(out), out.numel() * 4, _stream(stream)))
    return 256.0 * 4 * int(iters) * 16 * 16384


def qlora_bwd_fused_dequant(mode: int) -> int:
    """0: dequantise, then multiply; 1: decode the weight's tiles inside the backward product; < 0: query.  Returns the previous mode."""
    return int(lib().qlora_bwd_fused_dequant(int(mode)))


def qlora_linear_bwd(dY, X, Wq: NF4Weight, L1, L2, s, T_saved=None, dX=None, dL1=None, dL2=None,
                     need_dX=True, need_dL=True, workspace=None, stream=None):
    """dX, dL1, dL2 of the layer; adapter gradients only, never dW."""
    M, o = dY.shape
    h = Wq.rows
    r = 0 if L1 is None else L1.shape[1]
    dev = dY.device
    if dX is None and need_dX:
        dX = torch.empty((M, h), dtype=torch.bfloat16, device=dev)
    if r > 0 and need_dL:
        if dL1 is None:
            dL1 = torch.empty((h, r), dtype=torch.bfloat16, device=dev)
        if dL2 is None:
            dL2 = torch.empty((r, o), dtype=torch.bfloat16, device=dev)
    if workspace is None:
        workspace = workspace_alloc(_bwd_bytes(Wq, M, h, o, r), dev, stream)
    v = Wq.view()
    _check(lib().qlora_linear_bwd(_ptr(dY), _ptr(X), byref(v), _ptr(L1), _ptr(L2), float(s), M, r, _ptr(T_saved),
                                  _ptr(dX), _ptr(dL1), _ptr(dL2), _ptr(workspace), workspace.numel(),
                                  _stream(stream)))
    return dX, dL1, dL2


def qlora_linear_bwd_acc(dY, X, Wq: NF4Weight, L1, L2, s, dL1_acc, dL2_acc, T_saved=None, dX=None, need_dX=True,
                         workspace=None, stream=None):
    """The backward pass with the adapter gradients added to the fp32 accumulators dL1_acc (h, r), dL2_acc (r, o)."""
    M, o = dY.shape
    h = Wq.rows
    r = 0 if L1 is None else L1.shape[1]
    dev = dY.device
    if dX is None and need_dX:
        dX = torch.empty((M, h), dtype=torch.bfloat16, device=dev)
    for a in (dL1_acc, dL2_acc):
        assert a is None or (a.dtype == torch.float32 and a.is_contiguous())
    if workspace is None:
        workspace = workspace_alloc(_bwd_bytes(Wq, M, h, o, r), dev, stream)
    v = Wq.view()
    _check(lib().qlora_linear_bwd_acc(_ptr(dY), _ptr(X), byref(v), _ptr(L1), _ptr(L2), float(s), M, r, _ptr(T_saved),
                                      _ptr(dX), _ptr(dL1_acc), _ptr(dL2_acc), _ptr(workspace), workspace.numel(),
                                      _stream(stream)))
    return dX


def qlora_linear_dropout_sizes(M, h, o, r):
    """(forward workspace bytes, backward workspace bytes) of the LoRA-dropout calls."""
    f, b = c_size_t(0), c_size_t(0)
    _check(lib().qlora_linear_dropout_sizes(M, h, o, r, byref(f), byref(b)))
    return int(f.value), int(b.value)


def pack_keep_mask(keep):
    """Boolean (M, h) device tensor, True = kept -> the bit mask the C ABI takes (bit e % 8 of byte e // 8)."""
    k = keep.reshape(-1, 8).to(torch.uint8)
    w = torch.tensor([1, 2, 4, 8, 16, 32, 64, 128], dtype=torch.uint8, device=keep.device)
    return (k * w).sum(dim=1, dtype=torch.int32).to(torch.uint8).contiguous()


def qlora_linear_fwd_dropout(X, Wq: NF4Weight, L1, L2, s, keep_mask, p, Y=None, T_save=None, workspace=None, stream=None):
    """Y = X dequant(Wq) + s ((D o X) L1) L2 with D = keep / (1 - p): LoRA dropout on the adapter's input.
    keep_mask: uint8 device tensor of M * h / 8 bytes (pack_keep_mask)."""
    M, h = X.shape
    o = Wq.cols
    r = 0 if L1 is None else L1.shape[1]
    if Y is None:
        Y = torch.empty((M, o), dtype=torch.bfloat16, device=X.device)
    if workspace is None:
        workspace = workspace_alloc(qlora_linear_dropout_sizes(M, h, o, r)[0], X.device, stream)
    v = Wq.view()
    _check(lib().qlora_linear_fwd_dropout(_ptr(X), byref(v), _ptr(L1), _ptr(L2), float(s), M, r, _ptr(keep_mask),
                                          float(p), _ptr(Y), _ptr(T_save), _ptr(workspace), workspace.numel(),
                                          _stream(stream)))
    return Y


def qlora_linear_bwd_dropout(dY, X, Wq: NF4Weight, L1, L2, s, keep_mask, p, T_saved=None, dX=None, dL1=None, dL2=None,
                             dL1_acc=None, dL2_acc=None, need_dX=True, need_dL=True, workspace=None, stream=None):
    """dX, dL1, dL2 under LoRA dropout (same mask as the forward call); with dL1_acc / dL2_acc the adapter gradients
    are added to those fp32 accumulators instead."""
    M, o = dY.shape
    h = Wq.rows
    r = 0 if L1 is None else L1.shape[1]
    dev = dY.device
    if dX is None and need_dX:
        dX = torch.empty((M, h), dtype=torch.bfloat16, device=dev)
    if r > 0 and need_dL and dL1_acc is None and dL2_acc is None:
        if dL1 is None:
            dL1 = torch.empty((h, r), dtype=torch.bfloat16, device=dev)
        if dL2 is None:
            dL2 = torch.empty((r, o), dtype=torch.bfloat16, device=dev)
    if workspace is None:
        workspace = workspace_alloc(qlora_linear_dropout_sizes(M, h, o, r)[1], dev, stream)
    v = Wq.view()
    _check(lib().qlora_linear_bwd_dropout(_ptr(dY), _ptr(X), byref(v), _ptr(L1), _ptr(L2), float(s), M, r,
                                          _ptr(keep_mask), float(p), _ptr(T_saved), _ptr(dX), _ptr(dL1), _ptr(dL2),
                                          _ptr(dL1_acc), _ptr(dL2_acc), _ptr(workspace), workspace.numel(),
                                          _stream(stream)))
    return dX, dL1, dL2


def qlora_kbit_sizes(rows, cols, k) -> int:
    out = c_size_t()
    _check(lib().qlora_kbit_sizes(rows, cols, k, ctypes.byref(out)))
    return int(out.value)


def qlora_kbit_pack(Wq: NF4Weight, out=None, stream=None):
    """The dense k-bit stream (uint8 tensor) of an NF3 / NF2 weight's codes; the constants stay as they are."""
    k = {NF3: 3, NF2: 2}[Wq.dtype]
    if out is None:
        out = torch.empty(qlora_kbit_sizes(Wq.rows, Wq.cols, k), dtype=torch.uint8, device=Wq.packed.device)
    _check(lib().qlora_kbit_pack(_ptr(Wq.packed), Wq.rows, Wq.cols, k, _ptr(out), _stream(stream)))
    return out


def qlora_kbit_unpack(stream_bytes, Wq: NF4Weight, stream=None) -> NF4Weight:
    """Restores the 4-bit container `Wq.packed` of an NF3 / NF2 weight from its k-bit stream."""
    k = {NF3: 3, NF2: 2}[Wq.dtype]
    assert stream_bytes.is_cuda and stream_bytes.dtype == torch.uint8
    assert stream_bytes.numel() == qlora_kbit_sizes(Wq.rows, Wq.cols, k)
    _check(lib().qlora_kbit_unpack(_ptr(stream_bytes), Wq.rows, Wq.cols, k, _ptr(Wq.packed), _stream(stream)))
    return Wq


def qlora_grad_sqnorm(grad, accum, stream=None):
    """accum (device float64 tensor with one element) += sum of squares of grad (fp32 device tensor)."""
    assert grad.is_cuda and grad.dtype == torch.float32 and grad.is_contiguous()
    assert accum.is_cuda and accum.dtype == torch.float64 and accum.numel() == 1
    _check(lib().qlora_grad_sqnorm(_ptr(grad), grad.numel(), _ptr(accum), _stream(stream)))
    return accum


def qlora_adam_step(param, m, v, grad, step, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, grad_scale=1.0,
                    max_grad_norm=0.0, sqnorm=None, param_bf16=None, zero_grad=False, stream=None):
    """One Adam step in place on the fp32 device tensors param, m, v (grad is cleared when zero_grad is set);
    param_bf16 receives the bf16 copy of the new parameters."""
    n = param.numel()
    for t in (param, m, v, grad):
        assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == n
    if param_bf16 is not None:
        assert param_bf16.is_cuda and param_bf16.dtype == torch.bfloat16 and param_bf16.is_contiguous()
        assert param_bf16.numel() == n
    if sqnorm is not None:
        assert sqnorm.is_cuda and sqnorm.dtype == torch.float64 and sqnorm.numel() == 1
    cfg = qlora_adam_config(lr, beta1, beta2, eps, weight_decay, grad_scale, max_grad_norm, int(step),
                            1 if zero_grad else 0, 0)
    _check(lib().qlora_adam_step(_ptr(param), _ptr(m), _ptr(v), _ptr(grad), _ptr(param_bf16), n, ctypes.byref(cfg),
                                 _ptr(sqnorm), _stream(stream)))


def qlora_profile_gemm(enable: bool):
    """Bracket every main-GEMM launch with HIP events on its stream (benchmark aid)."""
    lib().qlora_profile_gemm(1 if enable else 0)


def qlora_profile_gemm_read():
    """(total kernel ms, launches, total algorithmic FLOPs) since the last read."""
    ms, n, fl = ctypes.c_double(0), c_int64(0), ctypes.c_double(0)
    _check(lib().qlora_profile_gemm_read(byref(ms), byref(n), byref(fl)))
    return ms.value, int(n.value), fl.value

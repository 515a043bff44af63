"""CPU oracle for the QLoRA frozen-linear hot path (numpy front end to the C++ library).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this module;
it is used by ``tests/``, by the smoke check and by the benchmark's ``cpu_baseline``
leg.  It shares no code with the HIP library.  See ``qlora_oracle.h`` for what each
function computes and which passage of the paper it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from ctypes import POINTER, c_double, c_float, c_int32, c_int64, c_uint8, c_uint16, c_void_p

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qlora_oracle.cpp")
_LIB = os.path.join(_HERE, "libqlora_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (plain IEEE arithmetic: no fast-math, no FMA contraction)."""
    stale = (not os.path.exists(_LIB)) or any(
        os.path.getmtime(os.path.join(_HERE, f)) > os.path.getmtime(_LIB)
        for f in ("qlora_oracle.cpp", "qlora_oracle.h"))
    if force or stale:
        cmd = ["g++", "-O2", "-std=c++17", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-Wall", "-Wextra", "-shared", "-fPIC", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    L = ctypes.CDLL(_LIB)
    vp = c_void_p
    L.oracle_num_threads.restype = ctypes.c_int
    L.oracle_nf4_table.argtypes = [vp]
    L.oracle_nf4_derive.argtypes = [c_double, vp]
    L.oracle_nfk_derive.argtypes = [c_int32, vp]
    L.oracle_normal_quantile.argtypes = [c_double]
    L.oracle_normal_quantile.restype = c_double
    L.oracle_nf4_index.argtypes = [c_float]
    L.oracle_nf4_index.restype = ctypes.c_int
    L.oracle_bf16_rne.argtypes = [c_float]
    L.oracle_bf16_rne.restype = c_uint16
    L.oracle_e4m3_encode.argtypes = [c_float]
    L.oracle_e4m3_encode.restype = c_uint8
    L.oracle_e4m3_value.argtypes = [c_uint8]
    L.oracle_e4m3_value.restype = c_float
    L.oracle_e4m3_unit.argtypes = [c_uint8]
    L.oracle_e4m3_unit.restype = c_float
    L.oracle_nf4_quantize.argtypes = [vp, c_int64, c_int64, c_int32, c_int32, vp, vp, vp, vp, vp]
    L.oracle_nf4_dequant.argtypes = [vp, vp, vp, c_float, c_int64, c_int64, c_int32, c_int32, vp, vp]
    L.oracle_codebook4.argtypes = [ctypes.c_int, vp]
    L.oracle_index4.argtypes = [vp, c_float]
    L.oracle_index4.restype = ctypes.c_int
    L.oracle_quantize4.argtypes = [vp] + list(L.oracle_nf4_quantize.argtypes)
    L.oracle_dequant4.argtypes = [vp] + list(L.oracle_nf4_dequant.argtypes)
    L.oracle_dequant4_nodq.argtypes = [vp, vp, vp, c_int64, c_int64, c_int32, vp]
    L.oracle_quantize_int8.argtypes = [vp, c_int64, c_int64, c_int32, c_int32, vp, vp, vp, vp, vp]
    L.oracle_dequant_int8.argtypes = [vp, vp, c_int64, c_int64, c_int32, vp]
    L.oracle_dq_constants.argtypes = [vp, vp, c_float, c_int64, c_int32, vp]
    lin = [vp, vp, vp, vp, c_double, c_int64, c_int64, c_int64, c_int64, vp, c_int64, vp]
    for name in ("oracle_linear_fwd_cols", "oracle_linear_bwd_dx_cols"):
        getattr(L, name).argtypes = lin
    for name in ("oracle_linear_fwd", "oracle_linear_bwd_dx"):
        getattr(L, name).argtypes = lin[:-1] + [vp, vp]      # ..., D, out
    L.oracle_linear_bwd_dl.argtypes = [vp, vp, vp, vp, c_double, c_int64, c_int64, c_int64, c_int64, vp, vp, vp]
    _lib = L
    return L


def _p(a):
    return None if a is None else a.ctypes.data_as(c_void_p)


def _arr(a, dtype, shape=None):
    a = np.ascontiguousarray(a, dtype=dtype)
    if shape is not None:
        assert a.shape == tuple(shape), (a.shape, shape)
    return a


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"{what}: oracle rejected the arguments (code {rc})")


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def nf4_table() -> np.ndarray:
    out = np.empty(16, np.float32)
    _load().oracle_nf4_table(_p(out))
    return out


def nf4_derive(p_max: float) -> np.ndarray:
    out = np.empty(16, np.float64)
    _load().oracle_nf4_derive(float(p_max), _p(out))
    return out


def normal_quantile(p: float) -> float:
    return float(_load().oracle_normal_quantile(float(p)))


def nf4_index(xhat) -> int:
    return int(_load().oracle_nf4_index(np.float32(xhat)))


def bf16_rne(v) -> int:
    return int(_load().oracle_bf16_rne(np.float32(v)))


def e4m3_encode(z) -> int:
    return int(_load().oracle_e4m3_encode(np.float32(z)))


def e4m3_value(code: int) -> float:
    return float(_load().oracle_e4m3_value(int(code)))


def e4m3_unit(code: int) -> np.float32:
    return np.float32(_load().oracle_e4m3_unit(int(code)))


KINDS = {"nf4": 0, "fp4_e2m1": 1, "fp4_e3m0": 2, "int4": 3, "nf3": 5, "nf2": 6}


def nfk_derive(k: int) -> np.ndarray:
    """k-bit NormalFloat values (k = 2, 3, 4) from normal quantiles, fp64: 2^k values ascending, padded with +1 to 16."""
    out = np.empty(16, np.float64)
    _check(_load().oracle_nfk_derive(int(k), _p(out)), "nfk_derive")
    return out


def codebook4(kind) -> np.ndarray:
    """The 16 values (fp32, ascending, in [-1, 1]) of a 4-bit data type: 'nf4', 'fp4_e2m1', 'fp4_e3m0', 'int4'."""
    out = np.empty(16, np.float32)
    _check(_load().oracle_codebook4(KINDS[kind] if isinstance(kind, str) else int(kind), _p(out)), "codebook4")
    return out


def index4(table, xhat) -> int:
    return int(_load().oracle_index4(_p(_arr(table, np.float32, (16,))), np.float32(xhat)))


def nf4_quantize(W, blocksize: int = 64, dq_blocksize: int = 256, table=None):
    """Returns dict(packed u8[P/2], code u8[n], c1 f32[n1], mean f32, c2 f32[n]).
    table: the 16 values of another 4-bit data type (codebook4), None = NF4.
    dq_blocksize = 0: no Double Quantization -- the result carries the fp32 constants c2 only (code, c1, mean None)."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    assert W.ndim == 2
    rows, cols = W.shape
    P = rows * cols
    if dq_blocksize == 0:
        q = nf4_quantize(W, blocksize, 256, table)           # the first step does not depend on the second
        q.update(code=None, c1=None, mean=None, dq_blocksize=0)
        return q
    if blocksize <= 0 or dq_blocksize <= 0 or P % blocksize or P % 2:
        raise ValueError("oracle nf4_quantize: bad shape / blocksize")
    n = P // blocksize
    n1 = -(-n // dq_blocksize)
    packed = np.empty(P // 2, np.uint8)
    code = np.empty(n, np.uint8)
    c1 = np.empty(n1, np.float32)
    mean = np.empty(1, np.float32)
    c2 = np.empty(n, np.float32)
    if table is None:
        _check(_load().oracle_nf4_quantize(_p(W), rows, cols, blocksize, dq_blocksize,
                                           _p(packed), _p(code), _p(c1), _p(mean), _p(c2)), "nf4_quantize")
    else:
        table = _arr(table, np.float32, (16,))
        _check(_load().oracle_quantize4(_p(table), _p(W), rows, cols, blocksize, dq_blocksize,
                                        _p(packed), _p(code), _p(c1), _p(mean), _p(c2)), "quantize4")
    return dict(packed=packed, code=code, c1=c1, mean=np.float32(mean[0]), c2=c2,
                rows=rows, cols=cols, blocksize=blocksize, dq_blocksize=dq_blocksize, table=table)


def nf4_dequant(q, return_c2hat: bool = False):
    """q: the dict from nf4_quantize.  Returns bf16 bit patterns u16[rows, cols]."""
    rows, cols = q["rows"], q["cols"]
    n = rows * cols // q["blocksize"]
    out = np.empty((rows, cols), np.uint16)
    if q["dq_blocksize"] == 0:
        table = nf4_table() if q.get("table") is None else _arr(q["table"], np.float32, (16,))
        _check(_load().oracle_dequant4_nodq(_p(table), _p(_arr(q["packed"], np.uint8)), _p(_arr(q["c2"], np.float32)),
                                            rows, cols, q["blocksize"], _p(out)), "dequant4_nodq")
        return (out, _arr(q["c2"], np.float32).copy()) if return_c2hat else out
    c2hat = np.empty(n, np.float32) if return_c2hat else None
    args = (_p(_arr(q["packed"], np.uint8)), _p(_arr(q["code"], np.uint8)), _p(_arr(q["c1"], np.float32)),
            np.float32(q["mean"]), rows, cols, q["blocksize"], q["dq_blocksize"], _p(out), _p(c2hat))
    if q.get("table") is None:
        _check(_load().oracle_nf4_dequant(*args), "nf4_dequant")
    else:
        _check(_load().oracle_dequant4(_p(_arr(q["table"], np.float32, (16,))), *args), "dequant4")
    return (out, c2hat) if return_c2hat else out


def int8_quantize(W, blocksize: int = 64, dq_blocksize: int = 256):
    """Eq. 1: blockwise 8-bit integers.  Returns dict(q8 i8[P], code, c1, mean (None without Double Quantization),
    c2 f32[n], ...)."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    rows, cols = W.shape
    P = rows * cols
    if blocksize <= 0 or dq_blocksize < 0 or P % blocksize:
        raise ValueError("oracle int8_quantize: bad shape / blocksize")
    n = P // blocksize
    q8 = np.empty(P, np.int8)
    c2 = np.empty(n, np.float32)
    dq = dq_blocksize != 0
    code = np.empty(n, np.uint8) if dq else None
    c1 = np.empty(-(-n // dq_blocksize), np.float32) if dq else None
    mean = np.empty(1, np.float32) if dq else None
    _check(_load().oracle_quantize_int8(_p(W), rows, cols, blocksize, dq_blocksize, _p(q8), _p(code), _p(c1),
                                        _p(mean), _p(c2)), "int8_quantize")
    return dict(q8=q8, code=code, c1=c1, mean=None if mean is None else np.float32(mean[0]), c2=c2, rows=rows,
                cols=cols, blocksize=blocksize, dq_blocksize=dq_blocksize)


def int8_dequant(q):
    """Eq. 2 on the result of int8_quantize.  Returns bf16 bit patterns u16[rows, cols]."""
    rows, cols = q["rows"], q["cols"]
    n = rows * cols // q["blocksize"]
    if q["dq_blocksize"] == 0:
        c2hat = _arr(q["c2"], np.float32)
    else:
        c2hat = np.empty(n, np.float32)
        _check(_load().oracle_dq_constants(_p(_arr(q["code"], np.uint8)), _p(_arr(q["c1"], np.float32)),
                                           np.float32(q["mean"]), n, q["dq_blocksize"], _p(c2hat)), "dq_constants")
    out = np.empty((rows, cols), np.uint16)
    _check(_load().oracle_dequant_int8(_p(_arr(q["q8"], np.int8)), _p(c2hat), rows, cols, q["blocksize"], _p(out)),
           "int8_dequant")
    return out


def _lin_args(A, What, L1, L2, M, h, o):
    r = 0 if L1 is None else int(np.asarray(L1).shape[1])
    What = _arr(What, np.uint16, (h, o))
    L1 = None if r == 0 else _arr(L1, np.uint16, (h, r))
    L2 = None if r == 0 else _arr(L2, np.uint16, (r, o))
    return What, L1, L2, r


def dropout_multipliers(keep, p):
    """LoRA dropout as a matrix of multipliers: 0 where an element of the adapter's input is dropped, 1/(1-p) where
    it is kept (keep: boolean M x h)."""
    return np.ascontiguousarray(np.asarray(keep, bool).astype(np.float64) / (1.0 - float(p)))


def linear_fwd(X, What, L1, L2, s, rows=None, cols=None, D=None):
    """Y = X What + s ((D o X) L1) L2 in fp64 (D: M x h multipliers of LoRA dropout, None = no dropout).
    X/What/L1/L2 are bf16 bit patterns (uint16).
    rows: token rows to compute (all columns), or cols: output columns (all rows; not with D)."""
    X = _arr(X, np.uint16)
    M, h = X.shape
    D = None if D is None else _arr(D, np.float64, (M, h))
    assert D is None or cols is None
    o = np.asarray(What).shape[1]
    What, L1, L2, r = _lin_args(X, What, L1, L2, M, h, o)
    L = _load()
    if cols is not None:
        sel = _arr(cols, np.int64)
        Y = np.empty((M, sel.size), np.float64)
        _check(L.oracle_linear_fwd_cols(_p(X), _p(What), _p(L1), _p(L2), float(s), M, h, o, r,
                                        _p(sel), sel.size, _p(Y)), "linear_fwd_cols")
        return Y
    sel = None if rows is None else _arr(rows, np.int64)
    ns = M if sel is None else sel.size
    Y = np.empty((ns, o), np.float64)
    _check(L.oracle_linear_fwd(_p(X), _p(What), _p(L1), _p(L2), float(s), M, h, o, r,
                               _p(sel), ns, _p(D), _p(Y)), "linear_fwd")
    return Y


def linear_bwd_dx(dY, What, L1, L2, s, rows=None, cols=None, D=None):
    """dX = dY What^T + s D o ((dY L2^T) L1^T) in fp64 (D as in linear_fwd)."""
    dY = _arr(dY, np.uint16)
    M, o = dY.shape
    h = np.asarray(What).shape[0]
    D = None if D is None else _arr(D, np.float64, (M, h))
    assert D is None or cols is None
    What, L1, L2, r = _lin_args(dY, What, L1, L2, M, h, o)
    L = _load()
    if cols is not None:
        sel = _arr(cols, np.int64)
        dX = np.empty((M, sel.size), np.float64)
        _check(L.oracle_linear_bwd_dx_cols(_p(dY), _p(What), _p(L1), _p(L2), float(s), M, h, o, r,
                                           _p(sel), sel.size, _p(dX)), "linear_bwd_dx_cols")
        return dX
    sel = None if rows is None else _arr(rows, np.int64)
    ns = M if sel is None else sel.size
    dX = np.empty((ns, h), np.float64)
    _check(L.oracle_linear_bwd_dx(_p(dY), _p(What), _p(L1), _p(L2), float(s), M, h, o, r,
                                  _p(sel), ns, _p(D), _p(dX)), "linear_bwd_dx")
    return dX


def linear_bwd_dl(dY, X, L1, L2, s, D=None):
    """dL1 = s Xd^T (dY L2^T), dL2 = s (Xd L1)^T dY in fp64, Xd = D o X (D as in linear_fwd)."""
    dY = _arr(dY, np.uint16)
    X = _arr(X, np.uint16)
    M, o = dY.shape
    h = X.shape[1]
    r = np.asarray(L1).shape[1]
    L1 = _arr(L1, np.uint16, (h, r))
    L2 = _arr(L2, np.uint16, (r, o))
    dL1 = np.empty((h, r), np.float64)
    dL2 = np.empty((r, o), np.float64)
    D = None if D is None else _arr(D, np.float64, (M, h))
    _check(_load().oracle_linear_bwd_dl(_p(dY), _p(X), _p(L1), _p(L2), float(s), M, h, o, r,
                                        _p(D), _p(dL1), _p(dL2)), "linear_bwd_dl")
    return dL1, dL2

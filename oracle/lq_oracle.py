"""ctypes access to the CPU oracle  --  TEST INFRASTRUCTURE, not the product.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this module.  It
compiles oracle/lq_oracle.c with gcc on first use (or via build()) and exposes thin numpy wrappers
with no arithmetic of their own.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lq_oracle.c")
_LIB = os.path.join(_HERE, "liblq_oracle.so")

V_DTYPES = {"fp32": 0, "bf16": 1, "fp16": 2}


class Config(C.Structure):
    _fields_ = [("bits", C.c_int32), ("block", C.c_int32), ("scale_block", C.c_int32),
                ("scale_bits", C.c_int32), ("v_dtype", C.c_int32)]


def config(bits, block, scale_block, scale_bits=8, v_dtype="fp32") -> Config:
    return Config(bits, block, scale_block, scale_bits, V_DTYPES[v_dtype] if isinstance(v_dtype, str) else v_dtype)


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC",
               _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.oq_norm_ppf.restype = C.c_double
        L.oq_norm_ppf.argtypes = [C.c_double]
        L.oq_cast_v.restype = C.c_float
        L.oq_cast_v.argtypes = [C.c_float, C.c_int]
        L.oq_storage_bits.restype = C.c_double
        L.oq_storage_bits.argtypes = [C.c_int64, Config]
        L.oq_packed_bytes.restype = C.c_int64
        L.oq_packed_bytes.argtypes = [C.c_int64, C.c_int]
        _lib = L
    return _lib


def _p(a, t):
    return None if a is None else a.ctypes.data_as(C.POINTER(t))


def norm_ppf(p: float) -> float:
    return lib().oq_norm_ppf(p)


def codebook(bits: int) -> np.ndarray:
    out = np.zeros(1 << bits, np.float32)
    rc = lib().oq_codebook(C.c_int(bits), _p(out, C.c_float))
    if rc != 0:
        raise ValueError("bad bits")
    return out


def cast_v(v: float, v_dtype) -> float:
    return lib().oq_cast_v(C.c_float(v), V_DTYPES[v_dtype] if isinstance(v_dtype, str) else v_dtype)


def storage_bits(n: int, cfg: Config) -> float:
    return lib().oq_storage_bits(n, cfg)


def quantize(x: np.ndarray, cfg: Config):
    """-> codes (uint8, unpacked), scale_idx (uint8), v (fp32), s_exact (fp32)."""
    x = np.ascontiguousarray(x, np.float32).ravel()
    n = x.size
    nb = n // cfg.block
    ng = (nb + cfg.scale_block - 1) // cfg.scale_block
    codes = np.zeros(n, np.uint8)
    sidx = np.zeros(nb, np.uint8)
    v = np.zeros(ng, np.float32)
    s = np.zeros(nb, np.float32)
    rc = lib().oq_quantize(_p(x, C.c_float), C.c_int64(n), cfg, _p(codes, C.c_uint8), _p(sidx, C.c_uint8),
                           _p(v, C.c_float), _p(s, C.c_float))
    if rc != 0:
        raise ValueError("oq_quantize failed")
    return codes, sidx, v, s


def dequantize(codes, sidx, v, cfg: Config) -> np.ndarray:
    codes = np.ascontiguousarray(codes, np.uint8)
    sidx = np.ascontiguousarray(sidx, np.uint8)
    v = np.ascontiguousarray(v, np.float32)
    out = np.zeros(codes.size, np.float32)
    rc = lib().oq_dequantize(_p(codes, C.c_uint8), _p(sidx, C.c_uint8), _p(v, C.c_float), C.c_int64(codes.size),
                             cfg, _p(out, C.c_float))
    if rc != 0:
        raise ValueError("oq_dequantize failed")
    return out


def matmul(x, codes, sidx, v, cfg: Config, k: int, l1=None, l2=None, want_abs: bool = False):
    """Y = X (Q + L1 L2) in double; codes unpacked (one per byte).  want_abs: also |X| (|Q| + |L1||L2|)."""
    x = np.ascontiguousarray(x, np.float32)
    codes = np.ascontiguousarray(codes, np.uint8)
    sidx = np.ascontiguousarray(sidx, np.uint8)
    v = np.ascontiguousarray(v, np.float32)
    m, d = x.shape
    assert codes.size == d * k
    r = 0 if l1 is None else l1.shape[1]
    l1 = np.zeros((d, 1), np.float32) if l1 is None else np.ascontiguousarray(l1, np.float32)
    l2 = np.zeros((1, k), np.float32) if l2 is None else np.ascontiguousarray(l2, np.float32)
    y = np.zeros((m, k), np.float64)
    ya = np.zeros((m, k), np.float64) if want_abs else None
    rc = lib().oq_matmul(_p(x, C.c_float), C.c_int(m), C.c_int(d), C.c_int(k), _p(codes, C.c_uint8),
                         _p(sidx, C.c_uint8), _p(v, C.c_float), cfg, _p(l1, C.c_float), _p(l2, C.c_float),
                         C.c_int(r), _p(y, C.c_double), _p(ya, C.c_double) if want_abs else None)
    if rc != 0:
        raise ValueError("oq_matmul failed")
    return (y, ya) if want_abs else y


def pack(codes: np.ndarray, bits: int) -> np.ndarray:
    codes = np.ascontiguousarray(codes, np.uint8)
    out = np.zeros(lib().oq_packed_bytes(codes.size, bits), np.uint8)
    lib().oq_pack(_p(codes, C.c_uint8), C.c_int64(codes.size), C.c_int(bits), _p(out, C.c_uint8))
    return out


def unpack(packed: np.ndarray, n: int, bits: int) -> np.ndarray:
    packed = np.ascontiguousarray(packed, np.uint8)
    assert packed.size >= lib().oq_packed_bytes(n, bits)
    out = np.zeros(n, np.uint8)
    lib().oq_unpack(_p(packed, C.c_uint8), C.c_int64(n), C.c_int(bits), _p(out, C.c_uint8))
    return out


def svd(a: np.ndarray):
    """Exact SVD by one-sided Jacobi: -> U (d x m), S (m), Vt (m x k), float64."""
    a = np.ascontiguousarray(a, np.float64)
    d, k = a.shape
    m = min(d, k)
    u = np.zeros((d, m)); s = np.zeros(m); vt = np.zeros((m, k))
    rc = lib().oq_svd(_p(a, C.c_double), C.c_int(d), C.c_int(k), _p(u, C.c_double), _p(s, C.c_double),
                      _p(vt, C.c_double))
    if rc != 0:
        raise ValueError("oq_svd failed")
    return u, s, vt


def factorize(a: np.ndarray, r: int, row_w=None, col_w=None):
    """-> L1 (d x r) fp32, L2 (r x k) fp32, sigma (r) float64."""
    a = np.ascontiguousarray(a, np.float32)
    d, k = a.shape
    rw = None if row_w is None else np.ascontiguousarray(row_w, np.float32)
    cw = None if col_w is None else np.ascontiguousarray(col_w, np.float32)
    l1 = np.zeros((d, r), np.float32); l2 = np.zeros((r, k), np.float32); sg = np.zeros(r)
    rc = lib().oq_factorize(_p(a, C.c_float), C.c_int(d), C.c_int(k), _p(rw, C.c_float), _p(cw, C.c_float),
                            C.c_int(r), _p(l1, C.c_float), _p(l2, C.c_float), _p(sg, C.c_double))
    if rc != 0:
        raise ValueError("oq_factorize failed")
    return l1, l2, sg


def lq(w: np.ndarray, r: int, cfg: Config, iters: int, early_stop: bool = False, row_w=None, col_w=None,
       init_quantized: bool = False):
    """Algorithm 2.  -> dict(L1, L2, codes, scale_idx, v, Q, err, trace, iters_done, sigma)."""
    w = np.ascontiguousarray(w, np.float32)
    d, k = w.shape
    n = d * k
    nb = n // cfg.block
    ng = (nb + cfg.scale_block - 1) // cfg.scale_block
    rw = None if row_w is None else np.ascontiguousarray(row_w, np.float32)
    cw = None if col_w is None else np.ascontiguousarray(col_w, np.float32)
    out = dict(L1=np.zeros((d, r), np.float32), L2=np.zeros((r, k), np.float32), codes=np.zeros(n, np.uint8),
               scale_idx=np.zeros(nb, np.uint8), v=np.zeros(ng, np.float32), Q=np.zeros((d, k), np.float32),
               trace=np.full(iters, np.nan), sigma=np.zeros(r))
    err = C.c_double(0.0); done = C.c_int32(0)
    rc = lib().oq_lq_init(_p(w, C.c_float), C.c_int(d), C.c_int(k), C.c_int(r), cfg, C.c_int(iters),
                     C.c_int(int(early_stop)), _p(rw, C.c_float), _p(cw, C.c_float),
                     _p(out["L1"], C.c_float), _p(out["L2"], C.c_float), _p(out["codes"], C.c_uint8),
                     _p(out["scale_idx"], C.c_uint8), _p(out["v"], C.c_float), _p(out["Q"], C.c_float),
                     C.byref(err), _p(out["trace"], C.c_double), C.byref(done), _p(out["sigma"], C.c_double),
                     C.c_int(1 if init_quantized else 0))
    if rc != 0:
        raise ValueError("oq_lq failed")
    out["err"] = err.value
    out["iters_done"] = done.value
    return out


def lq_step(w: np.ndarray, q_prev: np.ndarray, r: int, cfg: Config, row_w=None, col_w=None):
    """One pass through Algorithm 2's loop body from a given Q(t-1).
    -> dict(L1, L2, codes, scale_idx, v, Q, err, sigma)."""
    w = np.ascontiguousarray(w, np.float32)
    q_prev = np.ascontiguousarray(q_prev, np.float32)
    d, k = w.shape
    assert q_prev.shape == (d, k)
    n = d * k
    nb = n // cfg.block
    ng = (nb + cfg.scale_block - 1) // cfg.scale_block
    rw = None if row_w is None else np.ascontiguousarray(row_w, np.float32)
    cw = None if col_w is None else np.ascontiguousarray(col_w, np.float32)
    out = dict(L1=np.zeros((d, r), np.float32), L2=np.zeros((r, k), np.float32), codes=np.zeros(n, np.uint8),
               scale_idx=np.zeros(nb, np.uint8), v=np.zeros(ng, np.float32), Q=np.zeros((d, k), np.float32),
               sigma=np.zeros(r))
    err = C.c_double(0.0)
    rc = lib().oq_lq_step(_p(w, C.c_float), C.c_int(d), C.c_int(k), C.c_int(r), cfg, _p(rw, C.c_float),
                          _p(cw, C.c_float), _p(q_prev, C.c_float), _p(out["L1"], C.c_float), _p(out["L2"], C.c_float),
                          _p(out["codes"], C.c_uint8), _p(out["scale_idx"], C.c_uint8), _p(out["v"], C.c_float),
                          _p(out["Q"], C.c_float), C.byref(err), _p(out["sigma"], C.c_double))
    if rc != 0:
        raise ValueError("oq_lq_step failed")
    out["err"] = err.value
    return out


def error_table(w: np.ndarray, r: int, cfgs, iters: int, early_stop: bool = False, row_w=None, col_w=None):
    """Algorithm 3 inner loops.  -> err_sq (n_cfgs), storage_bits (n_cfgs)."""
    w = np.ascontiguousarray(w, np.float32)
    d, k = w.shape
    arr = (Config * len(cfgs))(*cfgs)
    rw = None if row_w is None else np.ascontiguousarray(row_w, np.float32)
    cw = None if col_w is None else np.ascontiguousarray(col_w, np.float32)
    e = np.zeros(len(cfgs)); s = np.zeros(len(cfgs))
    rc = lib().oq_error_table(_p(w, C.c_float), C.c_int(d), C.c_int(k), C.c_int(r), arr, C.c_int(len(cfgs)),
                              C.c_int(iters), C.c_int(1 if early_stop else 0), _p(rw, C.c_float),
                              _p(cw, C.c_float), _p(e, C.c_double), _p(s, C.c_double))
    if rc != 0:
        raise ValueError("oq_error_table failed")
    return e, s


def fisher_row_col(f: np.ndarray):
    f = np.ascontiguousarray(f, np.float64)
    d, k = f.shape
    rw = np.zeros(d, np.float32); cw = np.zeros(k, np.float32)
    lib().oq_fisher_row_col(_p(f, C.c_double), C.c_int(d), C.c_int(k), _p(rw, C.c_float), _p(cw, C.c_float))
    return rw, cw


def assign_bruteforce(err, storage, budget_bits):
    """The integer program of Section 3.2 by definition: every assignment of one configuration per matrix is tried,
    the feasible one with the smallest summed error wins (pure Python; tiny instances only).
    -> (choice list, total error) or (None, inf) when nothing fits."""
    import itertools
    err = np.asarray(err, np.float64)
    storage = np.asarray(storage, np.float64)
    n, c = err.shape
    best, best_err = None, float("inf")
    for pick in itertools.product(range(c), repeat=n):
        used = sum(storage[i, pick[i]] for i in range(n))
        if used > budget_bits:
            continue
        total = sum(err[i, pick[i]] for i in range(n))
        if total < best_err:
            best, best_err = list(pick), total
    return best, best_err

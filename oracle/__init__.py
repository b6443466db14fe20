"""CPU oracle for HCCS -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

`build()` compiles hccs_oracle.c with gcc into this folder; `load()` opens it
with ctypes and declares the argument types.  The numpy helpers below only
marshal arrays into the C functions: there is no arithmetic of the method in
this file.  Nothing outside tests, the smoke check and the benchmark's CPU
baseline may import this package.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hccs_oracle.c")
_LIB = os.path.join(_HERE, "libhccs_oracle.so")
_lib = None

MODE_U8, MODE_I16, MODE_CLB_U8, MODE_CLB_I16 = 0, 1, 2, 3


def build(force=False):
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, i32, p = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        lib.hccs_oracle_check_params.argtypes = [i64, i64, i64, i64, i32]
        for name in ("row_u8", "row_i16", "row_clb_u8", "row_clb_i16"):
            getattr(lib, "hccs_oracle_" + name).argtypes = [p, i64, i64, i64, i64, p, p, p]
        lib.hccs_oracle_softmax.argtypes = [p, p, i64, i64, i64, i64, p, i32, i32, i32]
        lib.hccs_oracle_attention_i8.argtypes = [p, p, p, p, i64, i64, i64, i64, i64, p, p, i32, i32]
        lib.hccs_oracle_requant_logits.argtypes = [p, p, p, i64, i64, i64, i64, i64, p]
        lib.hccs_oracle_reciprocal_u8.argtypes = [p, p, i64]
        lib.hccs_oracle_calibrate.argtypes = [p, i64, i64, i64, i64, p, p, i64, p, p, i32]
        _lib = lib
    return _lib


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def check_params(B, S, D, n, band):
    return load().hccs_oracle_check_params(int(B), int(S), int(D), int(n), int(band))


def row(x, B, S, D, mode=MODE_U8):
    """One row through the C oracle.  Returns (p, Z, rho, status)."""
    x = np.ascontiguousarray(x, dtype=np.int8)
    out = np.zeros(x.shape[0], dtype=np.uint16 if mode & 1 else np.uint8)
    Z, rho = ctypes.c_int64(0), ctypes.c_int64(0)
    fn = [load().hccs_oracle_row_u8, load().hccs_oracle_row_i16,
          load().hccs_oracle_row_clb_u8, load().hccs_oracle_row_clb_i16][mode]
    rc = fn(_ptr(x), x.shape[0], int(B), int(S), int(D), _ptr(out), ctypes.byref(Z), ctypes.byref(rho))
    return out, Z.value, rho.value, rc


def softmax(logits, table, band, mode=MODE_U8, threads=1):
    """logits int8 [B,H,Lq,Lk], table int32 [H,3].  Returns (out, status)."""
    logits = np.ascontiguousarray(logits, dtype=np.int8)
    table = np.ascontiguousarray(table, dtype=np.int32)
    Bt, H, Lq, Lk = logits.shape
    assert table.shape == (H, 3)
    out = np.zeros(logits.shape, dtype=np.uint16 if mode & 1 else np.uint8)
    rc = load().hccs_oracle_softmax(_ptr(logits), _ptr(out), Bt, H, Lq, Lk, _ptr(table),
                                    int(band), int(mode), int(threads))
    return out, rc


def attention(q, k, v, table, requant, band, threads=1):
    """q int8 [B,H,Lq,d]; k,v int8 [B,H,Lk,d]; table int32 [H,3]; requant int32 [H,2].
    Returns (o int32 [B,H,Lq,d], status)."""
    q = np.ascontiguousarray(q, dtype=np.int8)
    k = np.ascontiguousarray(k, dtype=np.int8)
    v = np.ascontiguousarray(v, dtype=np.int8)
    table = np.ascontiguousarray(table, dtype=np.int32)
    requant = np.ascontiguousarray(requant, dtype=np.int32)
    Bt, H, Lq, d = q.shape
    Lk = k.shape[2]
    assert k.shape == (Bt, H, Lk, d) and v.shape == k.shape
    assert table.shape == (H, 3) and requant.shape == (H, 2)
    o = np.zeros(q.shape, dtype=np.int32)
    rc = load().hccs_oracle_attention_i8(_ptr(q), _ptr(k), _ptr(v), _ptr(o), Bt, H, Lq, Lk, d,
                                         _ptr(table), _ptr(requant), int(band), int(threads))
    return o, rc


def requant_logits(q, k, requant):
    q = np.ascontiguousarray(q, dtype=np.int8)
    k = np.ascontiguousarray(k, dtype=np.int8)
    requant = np.ascontiguousarray(requant, dtype=np.int32)
    Bt, H, Lq, d = q.shape
    Lk = k.shape[2]
    x = np.zeros((Bt, H, Lq, Lk), dtype=np.int8)
    rc = load().hccs_oracle_requant_logits(_ptr(q), _ptr(k), _ptr(x), Bt, H, Lq, Lk, d, _ptr(requant))
    return x, rc


def reciprocal_u8(Z):
    Z = np.ascontiguousarray(Z, dtype=np.int64)
    rho = np.zeros_like(Z)
    rc = load().hccs_oracle_reciprocal_u8(_ptr(Z), _ptr(rho), Z.shape[0])
    return rho, rc


def calibrate(logits, alpha, candidates, threads=1):
    """Brute-force calibration objective.  logits int8 [B,H,Lq,Lk], alpha float64 [H],
    candidates int32 [nc,3].  Returns (objective float64 [H,nc], best int32 [H], status)."""
    logits = np.ascontiguousarray(logits, dtype=np.int8)
    alpha = np.ascontiguousarray(alpha, dtype=np.float64)
    candidates = np.ascontiguousarray(candidates, dtype=np.int32)
    Bt, H, Lq, Lk = logits.shape
    nc = candidates.shape[0]
    assert alpha.shape == (H,) and candidates.shape == (nc, 3)
    obj = np.zeros((H, nc), dtype=np.float64)
    best = np.zeros(H, dtype=np.int32)
    rc = load().hccs_oracle_calibrate(_ptr(logits), Bt, H, Lq, Lk, _ptr(alpha), _ptr(candidates), nc,
                                      _ptr(obj), _ptr(best), int(threads))
    return obj, best, rc

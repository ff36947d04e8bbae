"""ctypes front-end of the CPU oracle (oracle/tq_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg.  The product package never imports this module, and this module never
imports the product package.  Arrays are numpy; fp16 travels as uint16 bit patterns or
numpy float16 (same bits).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "tq_oracle.cpp"
_LIB = _HERE / "libtq_oracle.so"


def build(force: bool = False) -> Path:
    """Compile the oracle with g++ (no fast-math, no FMA contraction)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".so.tmp{os.getpid()}")
        cmd = ["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-pthread", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", str(_SRC), "-o", str(tmp)]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(str(_LIB))
        P, I, I64, D = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_double
        L.orc_half_to_float.argtypes = [ctypes.c_uint16]
        L.orc_half_to_float.restype = ctypes.c_float
        L.orc_float_to_half.argtypes = [ctypes.c_float]
        L.orc_float_to_half.restype = ctypes.c_uint16
        L.orc_quantize.argtypes = [P, I64, I, I, P, P, P, I]
        L.orc_dequantize_f64.argtypes = [P, P, P, I64, I, I, P]
        L.orc_dequantize_f16.argtypes = [P, P, P, I64, I, I, P]
        L.orc_attend_dense_f64.argtypes = [P, P, P, I, I, I, I64, I, D, D, P, I]
        L.orc_attend_packed_f64.argtypes = [P, P, P, P, P, P, P, I, I, I, I64, I64, I, I, D, P, I]
        L.orc_attend_alg1_eq6_f64.argtypes = [P, P, P, I, I, I, I64, I, D, P, I, P]
        L.orc_kv_bytes_int4.argtypes = [I64, I64, I64, I64, I64]
        L.orc_kv_bytes_fp16.argtypes = [I64, I64, I64, I64]
        L.orc_kv_bytes_int4.restype = L.orc_kv_bytes_fp16.restype = I64
        _lib = L
    return _lib


def default_threads() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _as_u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        return a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError(f"expected float16/uint16, got {a.dtype}")
    return a


def half_to_float(bits: int) -> float:
    return float(lib().orc_half_to_float(int(bits)))


def float_to_half(x: float) -> int:
    return int(lib().orc_float_to_half(float(x)))


def quantize(x, nthreads: int | None = None, group: int = 32):
    """x: float16 [..., d] -> (codes uint8 [..., d/2], scale float16 [..., d/group], zero float16 [..., d/group])."""
    xu = _as_u16(x)
    d = xu.shape[-1]
    n = xu.size // d
    codes = np.empty(xu.shape[:-1] + (d // 2,), np.uint8)
    scale = np.empty(xu.shape[:-1] + (d // group,), np.uint16)
    zero = np.empty_like(scale)
    rc = lib().orc_quantize(_ptr(xu), n, d, int(group), _ptr(codes), _ptr(scale), _ptr(zero),
                            nthreads or default_threads())
    if rc:
        raise ValueError(f"orc_quantize failed ({rc})")
    return codes, scale.view(np.float16), zero.view(np.float16)


def group_of(codes, scale) -> int:
    """The group size a cache's arrays imply: elements per vector over scales per vector."""
    return int(codes.shape[-1] * 2 // scale.shape[-1])


def dequantize(codes, scale, zero) -> np.ndarray:
    """fp64 value of every stored element, [..., d] (the group size follows from the shapes)."""
    codes = np.ascontiguousarray(codes, np.uint8)
    s, z = _as_u16(scale), _as_u16(zero)
    d = codes.shape[-1] * 2
    out = np.empty(codes.shape[:-1] + (d,), np.float64)
    rc = lib().orc_dequantize_f64(_ptr(codes), _ptr(s), _ptr(z), codes.size // (d // 2), d, group_of(codes, s), _ptr(out))
    if rc:
        raise ValueError(f"orc_dequantize_f64 failed ({rc})")
    return out


def dequantize_f16(codes, scale, zero) -> np.ndarray:
    codes = np.ascontiguousarray(codes, np.uint8)
    s, z = _as_u16(scale), _as_u16(zero)
    d = codes.shape[-1] * 2
    out = np.empty(codes.shape[:-1] + (d,), np.uint16)
    rc = lib().orc_dequantize_f16(_ptr(codes), _ptr(s), _ptr(z), codes.size // (d // 2), d, group_of(codes, s), _ptr(out))
    if rc:
        raise ValueError(f"orc_dequantize_f16 failed ({rc})")
    return out.view(np.float16)


def attend_dense(q, K, V, alpha: float, score_bias: float = 0.0, nthreads: int | None = None) -> np.ndarray:
    """q float16 [B,Hq,d]; K,V float64 [B,Hkv,S,d] -> float64 [B,Hq,d]."""
    qu = _as_u16(q)
    K = np.ascontiguousarray(K, np.float64)
    V = np.ascontiguousarray(V, np.float64)
    B, Hq, d = qu.shape
    _, Hkv, S, _ = K.shape
    out = np.empty((B, Hq, d), np.float64)
    rc = lib().orc_attend_dense_f64(_ptr(qu), _ptr(K), _ptr(V), B, Hq, Hkv, S, d, float(alpha),
                                    float(score_bias), _ptr(out), nthreads or default_threads())
    if rc:
        raise ValueError(f"orc_attend_dense_f64 failed ({rc})")
    return out


def attend_packed(q, k_codes, k_scale, k_zero, v_codes, v_scale, v_zero, seq_len: int, alpha: float,
                  nthreads: int | None = None) -> np.ndarray:
    """Canonical packed cache arrays [B,Hkv,capacity,*] -> float64 out [B,Hq,d] (group size from the shapes)."""
    qu = _as_u16(q)
    kc = np.ascontiguousarray(k_codes, np.uint8)
    vc = np.ascontiguousarray(v_codes, np.uint8)
    ks, kz, vs, vz = (_as_u16(a) for a in (k_scale, k_zero, v_scale, v_zero))
    B, Hq, d = qu.shape
    _, Hkv, cap, _ = kc.shape
    out = np.empty((B, Hq, d), np.float64)
    if group_of(kc, ks) != group_of(vc, vs):
        raise ValueError("K and V are quantised with different group sizes")
    rc = lib().orc_attend_packed_f64(_ptr(qu), _ptr(kc), _ptr(ks), _ptr(kz), _ptr(vc), _ptr(vs), _ptr(vz),
                                     B, Hq, Hkv, cap, int(seq_len), d, group_of(kc, ks), float(alpha), _ptr(out),
                                     nthreads or default_threads())
    if rc:
        raise ValueError(f"orc_attend_packed_f64 failed ({rc})")
    return out


def attend_alg1_eq6(q, K, V, alpha: float, bounds) -> np.ndarray:
    qu = _as_u16(q)
    K = np.ascontiguousarray(K, np.float64)
    V = np.ascontiguousarray(V, np.float64)
    B, Hq, d = qu.shape
    _, Hkv, S, _ = K.shape
    b = np.ascontiguousarray(bounds, np.int64)
    out = np.empty((B, Hq, d), np.float64)
    rc = lib().orc_attend_alg1_eq6_f64(_ptr(qu), _ptr(K), _ptr(V), B, Hq, Hkv, S, d, float(alpha),
                                       _ptr(b), len(b) - 1, _ptr(out))
    if rc:
        raise ValueError(f"orc_attend_alg1_eq6_f64 failed ({rc})")
    return out


def kv_bytes_int4(n_layers, n_kv_heads, seq_len, d, group: int = 32) -> int:
    return int(lib().orc_kv_bytes_int4(n_layers, n_kv_heads, seq_len, d, group))


def kv_bytes_fp16(n_layers, n_kv_heads, seq_len, d) -> int:
    return int(lib().orc_kv_bytes_fp16(n_layers, n_kv_heads, seq_len, d))

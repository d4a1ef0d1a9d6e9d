"""numpy front-end of the CPU oracle (oracle/convrot_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module.
The C file is compiled with gcc on first use (``oracle/build.py`` does the same
explicitly).  All arrays are C-contiguous numpy arrays; bf16 tensors are uint16
bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "convrot_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over rows).  Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-fno-fast-math", "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            i64, i32, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
            lib.oracle_num_threads.restype = i32
            lib.oracle_hadamard.argtypes = [i32, vp, vp]
            lib.oracle_rotate.argtypes = [vp, i64, i64, i32, vp, vp]
            lib.oracle_quantize.argtypes = [vp, i64, i64, i32, vp, vp]
            lib.oracle_pack4.argtypes = [vp, i64, i64, vp]
            lib.oracle_unpack4.argtypes = [vp, i64, i64, vp]
            lib.oracle_int_gemm.argtypes = [vp, vp, i64, i64, i64, vp]
            lib.oracle_dequant.argtypes = [vp, vp, vp, vp, i64, i64, vp]
            lib.oracle_rotquant.argtypes = [vp, i64, i64, i32, i32, vp, vp]
            lib.oracle_convlinear.argtypes = [vp, vp, vp, i64, i64, i64, i32, i32, vp]
            lib.oracle_double_to_bf16.argtypes = [ctypes.c_double]
            lib.oracle_double_to_bf16.restype = ctypes.c_uint16
            _lib = lib
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"oracle.{what} failed with status {rc}")


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def hadamard(g: int, h4: Optional[np.ndarray] = None) -> np.ndarray:
    """H_g (int8, [g, g]) by Kronecker powers of the order-4 base (printed matrix if h4 is None)."""
    H = np.empty((g, g), dtype=np.int8)
    base = None if h4 is None else _c(h4, np.int8).reshape(4, 4)
    _check(_load().oracle_hadamard(int(g), _p(base), _p(H)), "hadamard")
    return H


def rotate(x_bf16: np.ndarray, g: int, H: Optional[np.ndarray] = None) -> np.ndarray:
    """Group-wise rotation of every row: double [rows, K]."""
    x = _c(x_bf16, np.uint16)
    rows, K = x.shape
    H = hadamard(g) if H is None else _c(H, np.int8)
    out = np.empty((rows, K), dtype=np.float64)
    _check(_load().oracle_rotate(_p(x), rows, K, int(g), _p(H), _p(out)), "rotate")
    return out


def quantize(v: np.ndarray, qmax: int = 7) -> Tuple[np.ndarray, np.ndarray]:
    """Per-row symmetric quantiser: (codes int8 [rows, K], scale float32 [rows])."""
    v = _c(v, np.float64)
    rows, K = v.shape
    codes = np.empty((rows, K), dtype=np.int8)
    scale = np.empty((rows,), dtype=np.float32)
    _check(_load().oracle_quantize(_p(v), rows, K, int(qmax), _p(scale), _p(codes)), "quantize")
    return codes, scale


def pack4(codes: np.ndarray) -> np.ndarray:
    c = _c(codes, np.int8)
    rows, K = c.shape
    out = np.empty((rows, K // 2), dtype=np.uint8)
    _check(_load().oracle_pack4(_p(c), rows, K, _p(out)), "pack4")
    return out


def unpack4(packed: np.ndarray) -> np.ndarray:
    p = _c(packed, np.uint8)
    rows, half = p.shape
    out = np.empty((rows, half * 2), dtype=np.int8)
    _check(_load().oracle_unpack4(_p(p), rows, half * 2, _p(out)), "unpack4")
    return out


def int_gemm(qx: np.ndarray, qw: np.ndarray) -> np.ndarray:
    """acc[m, n] = sum_k qx[m, k] * qw[n, k], int32."""
    qx = _c(qx, np.int8)
    qw = _c(qw, np.int8)
    M, K = qx.shape
    N, K2 = qw.shape
    if K != K2:
        raise ValueError("K mismatch")
    acc = np.empty((M, N), dtype=np.int32)
    _check(_load().oracle_int_gemm(_p(qx), _p(qw), M, N, K, _p(acc)), "int_gemm")
    return acc


def dequant(acc: np.ndarray, sx: np.ndarray, sw: np.ndarray, bias: Optional[np.ndarray] = None) -> np.ndarray:
    """Y = bf16(acc * sx[:, None] * sw[None, :] + bias[None, :]) as uint16 bits (bias: bf16 bits [N] or None)."""
    acc = _c(acc, np.int32)
    sx = _c(sx, np.float32)
    sw = _c(sw, np.float32)
    M, N = acc.shape
    b = None if bias is None else _c(bias, np.uint16)
    if b is not None and b.shape != (N,):
        raise ValueError("bias shape")
    y = np.empty((M, N), dtype=np.uint16)
    _check(_load().oracle_dequant(_p(acc), _p(sx), _p(sw), _p(b), M, N, _p(y)), "dequant")
    return y


def rotquant(x_bf16: np.ndarray, g: int, qmax: int = 7) -> Tuple[np.ndarray, np.ndarray]:
    """Rotation + per-row quantisation of one operand: (codes int8 [rows, K], scale f32 [rows])."""
    x = _c(x_bf16, np.uint16)
    rows, K = x.shape
    codes = np.empty((rows, K), dtype=np.int8)
    scale = np.empty((rows,), dtype=np.float32)
    _check(_load().oracle_rotquant(_p(x), rows, K, int(g), int(qmax), _p(codes), _p(scale)), "rotquant")
    return codes, scale


def convlinear(x_bf16: np.ndarray, w_bf16: np.ndarray, g: int, bias: Optional[np.ndarray] = None,
               qmax: int = 7) -> np.ndarray:
    """Whole forward: bf16 X [M,K], bf16 W [N,K] (+ bf16 bias [N]) -> bf16 Y [M,N] (uint16 bits).

    qmax = 7 is ConvLinear4bit (W4A4), qmax = 127 the W8A8 variant."""
    x = _c(x_bf16, np.uint16)
    w = _c(w_bf16, np.uint16)
    M, K = x.shape
    N, K2 = w.shape
    if K != K2:
        raise ValueError("K mismatch")
    b = None if bias is None else _c(bias, np.uint16)
    y = np.empty((M, N), dtype=np.uint16)
    _check(_load().oracle_convlinear(_p(x), _p(w), _p(b), M, N, K, int(g), int(qmax), _p(y)), "convlinear")
    return y


def convlinear4bit(x_bf16: np.ndarray, w_bf16: np.ndarray, g: int, bias: Optional[np.ndarray] = None) -> np.ndarray:
    """ConvLinear4bit forward (W4A4)."""
    return convlinear(x_bf16, w_bf16, g, bias=bias, qmax=7)


def double_to_bf16(v: float) -> int:
    return int(_load().oracle_double_to_bf16(float(v)))

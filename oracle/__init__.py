"""CPU oracle for the ModuLoRA linear layer -- TEST INFRASTRUCTURE ONLY.

A thin ctypes wrapper over ``modulora_oracle.c`` (plain C, float64
accumulation, written from the paper: Section 2.2 eq. (2) for dequantization,
Section 3.1 eq. (3) and Figure 1 for the forward and backward passes).  Only
the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import
this package; the GPU library never does, and nothing here imports the GPU
library.

All arrays are numpy.  16-bit float tensors travel as ``uint16`` bit patterns:
``X``/``dY`` are bfloat16 bits, ``scales`` are IEEE binary16 bits.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "modulora_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (a second or two).  Returns the .so path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
             "-o", tmp, _SRC],
            check=True,
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _p(a, dtype):
    assert a.dtype == dtype and a.flags["C_CONTIGUOUS"], (a.dtype, dtype)
    return a.ctypes.data_as(ctypes.c_void_p)


def _i64(v):
    return ctypes.c_int64(int(v))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def unpack(qweight: np.ndarray, K: int, N: int, bits: int) -> np.ndarray:
    """codes[n][k] (uint8 [N][K]) from the packed bitstream words."""
    assert qweight.shape == (K * bits // 32, N)
    out = np.empty((N, K), dtype=np.uint8)
    rc = _load().oracle_unpack(_p(qweight, np.uint32), _i64(K), _i64(N),
                               ctypes.c_int(bits), _p(out, np.uint8))
    assert rc == 0, rc
    return out


def _check_layer(qweight, scales, zeros, K, N, bits, group):
    assert qweight.shape == (K * bits // 32, N), qweight.shape
    assert scales.shape == (K // group, N) and zeros.shape == (K // group, N)


def dequant_f32(qweight, scales, zeros, K, N, bits, group) -> np.ndarray:
    """Exact float32 (q - zero) * scale, [N][K]."""
    _check_layer(qweight, scales, zeros, K, N, bits, group)
    out = np.empty((N, K), dtype=np.float32)
    rc = _load().oracle_dequant_f32(
        _p(qweight, np.uint32), _p(scales, np.uint16), _p(zeros, np.uint8),
        _i64(K), _i64(N), ctypes.c_int(bits), _i64(group), _p(out, np.float32))
    assert rc == 0, rc
    return out


def dequant_bf16(qweight, scales, zeros, K, N, bits, group) -> np.ndarray:
    """Materialized weight as bfloat16 bit patterns (uint16 [N][K])."""
    _check_layer(qweight, scales, zeros, K, N, bits, group)
    out = np.empty((N, K), dtype=np.uint16)
    rc = _load().oracle_dequant_bf16(
        _p(qweight, np.uint32), _p(scales, np.uint16), _p(zeros, np.uint8),
        _i64(K), _i64(N), ctypes.c_int(bits), _i64(group), _p(out, np.uint16))
    assert rc == 0, rc
    return out


def _ab(A, B, K, N):
    r = A.shape[1] if A is not None else 0
    if r == 0:
        A = np.zeros((K, 0), dtype=np.float32)
        B = np.zeros((0, N), dtype=np.float32)
    assert A.shape == (K, r) and B.shape == (r, N)
    # ctypes needs a valid pointer even for empty arrays
    Ap = _p(A, np.float32) if r else ctypes.c_void_p(0)
    Bp = _p(B, np.float32) if r else ctypes.c_void_p(0)
    return r, Ap, Bp


def fwd(qweight, scales, zeros, K, N, bits, group, X, A, B, lora_scale):
    """Returns (Y float64 [M][N], U = X A float64 [M][r])."""
    _check_layer(qweight, scales, zeros, K, N, bits, group)
    M = X.shape[0]
    assert X.shape == (M, K)
    r, Ap, Bp = _ab(A, B, K, N)
    Y = np.empty((M, N), dtype=np.float64)
    U = np.empty((M, r), dtype=np.float64)
    rc = _load().oracle_fwd(
        _p(qweight, np.uint32), _p(scales, np.uint16), _p(zeros, np.uint8),
        _i64(K), _i64(N), ctypes.c_int(bits), _i64(group), _p(X, np.uint16),
        _i64(M), Ap, Bp, _i64(r), ctypes.c_double(lora_scale),
        _p(Y, np.float64), _p(U, np.float64) if r else ctypes.c_void_p(0))
    assert rc == 0, rc
    return Y, U


def bwd_input(qweight, scales, zeros, K, N, bits, group, dY, A, B, lora_scale):
    """Returns (dX float64 [M][K], T = dY B^T float64 [M][r])."""
    _check_layer(qweight, scales, zeros, K, N, bits, group)
    M = dY.shape[0]
    assert dY.shape == (M, N)
    r, Ap, Bp = _ab(A, B, K, N)
    dX = np.empty((M, K), dtype=np.float64)
    T = np.empty((M, r), dtype=np.float64)
    rc = _load().oracle_bwd_input(
        _p(qweight, np.uint32), _p(scales, np.uint16), _p(zeros, np.uint8),
        _i64(K), _i64(N), ctypes.c_int(bits), _i64(group), _p(dY, np.uint16),
        _i64(M), Ap, Bp, _i64(r), ctypes.c_double(lora_scale),
        _p(dX, np.float64), _p(T, np.float64) if r else ctypes.c_void_p(0))
    assert rc == 0, rc
    return dX, T


def bwd_lora(K, N, X, dY, A, B, lora_scale):
    """Returns (dA float64 [K][r], dB float64 [r][N])."""
    M = X.shape[0]
    assert X.shape == (M, K) and dY.shape == (M, N)
    r, Ap, Bp = _ab(A, B, K, N)
    dA = np.empty((K, r), dtype=np.float64)
    dB = np.empty((r, N), dtype=np.float64)
    if r == 0:
        return dA, dB
    rc = _load().oracle_bwd_lora(
        _i64(K), _i64(N), _i64(M), _i64(r), ctypes.c_double(lora_scale),
        _p(X, np.uint16), _p(dY, np.uint16), Ap, Bp,
        _p(dA, np.float64), _p(dB, np.float64))
    assert rc == 0, rc
    return dA, dB

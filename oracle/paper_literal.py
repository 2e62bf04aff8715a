"""The layer in the paper's own storage convention, numpy -- TEST INFRASTRUCTURE ONLY.

Section 2.2 eq. (2) states the frozen weight as  What = s (.) Wq + z  with a *floating*
zero point z next to the scale s, and Section 3.2 keeps z, s and the materialized What in a
16-bit float; Figure 1 / eq. (3) add a bias to the adapted layer.  This module is that
variant written out plainly (the integer-zero-point, bfloat16 variant is the C oracle):

    What[n][k] = binary16( binary32( q[n][k] * scale[g][n] + z[g][n] ) )      g = k div group
    Y          = X What^T + bias + lora_scale (X A) B
    dX         = dY What + lora_scale (dY B^T) A^T
    dA         = lora_scale X^T (dY B^T)        dB = lora_scale (X A)^T dY

q are the b-bit codes of the same LSB-first bitstream; scale and z are binary16 per group
of `group` consecutive inputs of an output column ([K/group][N]; group = K is the paper's
one-pair-per-row case); X, dY are binary16; A, B float32; all sums in float64.

Rounding of What (the paper is silent): the affine value is formed with one rounding to
binary32 -- what a fused multiply-add returns -- and then rounded to nearest even to
binary16.  For finite, normal-or-zero binary16 scale and z the exact value q*scale + z
fits a float64 (at most 15 + 34 significant bits apart), so `float64 -> float32` below is
that single rounding.  The bias is not an input of the backward pass (Figure 1: the
gradients of the frozen parts are None).

Only the tests (and the benchmark's CPU baseline) may import this module.
"""
from __future__ import annotations

import numpy as np

import oracle


def f16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def dequant_f16(qweight, scales, zeros, K: int, N: int, bits: int, group: int) -> np.ndarray:
    """What as binary16 bit patterns, uint16 [N][K]."""
    q = oracle.unpack(qweight, K, N, bits).astype(np.float64)            # [N][K]
    s = f16_bits_to_f64(scales).reshape(K // group, N)
    z = f16_bits_to_f64(zeros).reshape(K // group, N)
    g = np.arange(K) // group
    exact = q * s[g, :].T + z[g, :].T                                    # exact in float64 (see above)
    w32 = exact.astype(np.float32)                                       # the one rounding of an fma
    return np.ascontiguousarray(w32.astype(np.float16)).view(np.uint16)  # round to nearest even


def _dense(qweight, scales, zeros, K, N, bits, group) -> np.ndarray:
    return f16_bits_to_f64(dequant_f16(qweight, scales, zeros, K, N, bits, group))


def fwd(qweight, scales, zeros, K, N, bits, group, X, A, B, lora_scale, bias=None):
    """X uint16 (binary16 bits) [M][K].  Returns (Y [M][N], XA [M][r]) in float64."""
    W = _dense(qweight, scales, zeros, K, N, bits, group)
    Xd = f16_bits_to_f64(X)
    Y = Xd @ W.T
    XA = np.zeros((Xd.shape[0], 0))
    if A is not None and A.shape[1] > 0:
        XA = Xd @ A.astype(np.float64)
        Y = Y + float(lora_scale) * (XA @ B.astype(np.float64))
    if bias is not None:
        Y = Y + f16_bits_to_f64(bias)[None, :]
    return Y, XA


def bwd_input(qweight, scales, zeros, K, N, bits, group, dY, A, B, lora_scale):
    """dY uint16 (binary16 bits) [M][N].  Returns (dX [M][K], dYBt [M][r]) in float64."""
    W = _dense(qweight, scales, zeros, K, N, bits, group)
    G = f16_bits_to_f64(dY)
    dX = G @ W
    T = np.zeros((G.shape[0], 0))
    if A is not None and A.shape[1] > 0:
        T = G @ B.astype(np.float64).T
        dX = dX + float(lora_scale) * (T @ A.astype(np.float64).T)
    return dX, T


def bwd_lora(X, dY, A, B, lora_scale):
    """Returns (dA [K][r], dB [r][N]) in float64."""
    Xd, G = f16_bits_to_f64(X), f16_bits_to_f64(dY)
    T = G @ B.astype(np.float64).T
    U = Xd @ A.astype(np.float64)
    return float(lora_scale) * (Xd.T @ T), float(lora_scale) * (U.T @ G)

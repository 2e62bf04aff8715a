"""Round-to-nearest (RTN) group quantizer, numpy -- TEST INFRASTRUCTURE ONLY.

The quantizer side (the black-box Q of Section 2.2) in its simplest form, the
round-to-nearest baseline of the paper's quantizer ablation: every group of `g`
consecutive inputs of an output column gets its own affine grid of 2^b levels that spans
the group's range (widened to contain zero), and every weight goes to the nearest level.
The result is in the storage format of the layer (eq. (2) in its integer-zero-point
form): codes q in 0..2^b-1, a binary16 scale and a uint8 zero point per group with

    w  ~=  (q - zero) * scale,      |w - (q - zero) * scale| <= scale * (1/2 + 2^-20).

Where floating point decides an integer, the precision is part of the definition (the
GPU kernel takes the same decisions in the same precision): everything is IEEE float32,

    lo    = min(group, 0),  hi = max(group, 0)
    scale = the smallest binary16 value >= (hi - lo) / (2^b - 1), at least 2^-14 (a normal one)
    zero  = clamp(rne(-lo / scale), 0, 2^b - 1)
    q     = clamp(rne(w / scale) + zero, 0, 2^b - 1)

with rne = round half to even.  Rounding the scale *up* keeps (hi - lo) / scale <= 2^b - 1,
which is what makes the error bound hold also for the weights that the clamp touches.

Only the tests may import this module; the GPU library never does.
"""
from __future__ import annotations

import numpy as np


def f16_round_up(x: np.ndarray) -> np.ndarray:
    """Smallest binary16 >= x (x float32, 0 <= x <= 65504), as uint16 bit patterns."""
    x = np.asarray(x, dtype=np.float32)
    h = x.astype(np.float16)                       # round to nearest even
    bits = h.view(np.uint16).copy()
    low = h.astype(np.float32) < x                 # rounded down: take the next one up
    bits[low] += 1                                 # positive finite values: bit pattern order = value order
    return bits


def quantize(W: np.ndarray, bits: int, group: int):
    """W float32 [N][K] (d_out rows).  Returns (codes uint8 [N][K], scales uint16 [K/group][N]
    binary16 bit patterns, zeros uint8 [K/group][N])."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    N, K = W.shape
    assert K % group == 0
    G = K // group
    maxq = np.float32((1 << bits) - 1)
    Wg = W.reshape(N, G, group)
    lo = np.minimum(Wg.min(axis=2), np.float32(0))
    hi = np.maximum(Wg.max(axis=2), np.float32(0))
    raw = (hi - lo) / maxq                                     # float32 [N][G]
    sbits = f16_round_up(np.maximum(raw, np.float32(2.0 ** -14)))
    s = sbits.view(np.float16).astype(np.float32)
    zero = np.clip(np.rint(-lo / s), 0, maxq)                  # float32 arithmetic, half to even
    q = np.clip(np.rint(Wg / s[:, :, None]) + zero[:, :, None], 0, maxq)
    codes = q.astype(np.uint8).reshape(N, K)
    return codes, np.ascontiguousarray(sbits.T), np.ascontiguousarray(zero.astype(np.uint8).T)


def pack(codes: np.ndarray, bits: int) -> np.ndarray:
    """codes uint8 [N][K] -> words uint32 [K*bits/32][N]: per output column one bitstream
    along K, code k in stream bits [k*bits, (k+1)*bits), stream bit j = bit (j mod 32) of word j // 32."""
    N, K = codes.shape
    assert (K * bits) % 32 == 0
    words = np.zeros((K * bits // 32, N), dtype=np.uint64)
    for k in range(K):
        pos = k * bits
        w, sh = pos // 32, pos % 32
        v = codes[:, k].astype(np.uint64) << np.uint64(sh)
        words[w] |= v & np.uint64(0xFFFFFFFF)
        if sh + bits > 32:
            words[w + 1] |= v >> np.uint64(32)
    return words.astype(np.uint32)


def quantize_packed(W: np.ndarray, bits: int, group: int):
    """(qweight uint32 [K*bits/32][N], scales uint16 [G][N], zeros uint8 [G][N])."""
    codes, scales, zeros = quantize(W, bits, group)
    return pack(codes, bits), scales, zeros

"""Seeded synthetic inputs for the quantized-LoRA layer workloads.

This module only *draws and stores* inputs: random codes, zero points, scales,
activations and adapters with the shapes and value ranges of the LLaMA-shaped
layer configurations the library is measured on.  It holds none of the layer's
arithmetic (no unpacking, no dequantization, no matrix products) and is the one
module that both the GPU tests and the CPU oracle's tests may share.

Storage conventions (the ones the C header states):
  qweight uint32 [K*bits/32][N]  -- per column n one LSB-first bitstream along k
  scales  uint16 [K/g][N]        -- IEEE binary16 bit patterns
  zeros   uint8  [K/g][N]
  X, dY   uint16                 -- bfloat16 bit patterns, [M][K] and [M][N]
  A [K][r], B [r][N] float32
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class LayerConfig:
    name: str
    K: int            # d_in
    N: int            # d_out
    bits: int
    group: int
    M: int            # tokens
    r: int            # LoRA rank
    scale_lo: float = 0.005
    scale_hi: float = 0.02
    lora_scale: float = 2.0
    seed: int = 0

    def with_M(self, M: int) -> "LayerConfig":
        return replace(self, M=M, name="%s_M%d" % (self.name.split("_M")[0], M))

    @property
    def packed_weight_bytes(self) -> int:
        """codes + scales (2 B) + zeros (1 B): what one pass over the frozen weight reads."""
        G = self.K // self.group
        return self.K * self.N * self.bits // 8 + G * self.N * 3

    @property
    def flops_fwd_bwd(self) -> int:
        """2 GEMMs with the frozen weight + 6 rank-r products."""
        return 4 * self.M * self.K * self.N + 6 * self.M * self.r * (self.K + self.N)


# The layer shapes of the benchmark configurations.
CONFIGS = {
    # toy layer, the oracle finishes it instantly
    "c1_toy": LayerConfig("c1_toy", 256, 256, 4, 64, 16, 8),
    # LLaMA-7B attention projection
    "c2_7b_attn": LayerConfig("c2_7b_attn", 4096, 4096, 3, 128, 512, 8),
    # LLaMA-7B MLP
    "c3_7b_gate_up": LayerConfig("c3_7b_gate_up", 4096, 11008, 4, 128, 2048, 16),
    "c3_7b_down": LayerConfig("c3_7b_down", 11008, 4096, 4, 128, 2048, 16),
    # LLaMA-30B, 2-bit
    "c4_30b_attn": LayerConfig("c4_30b_attn", 6656, 6656, 2, 64, 1024, 8, 0.01, 0.04),
    "c4_30b_up": LayerConfig("c4_30b_up", 6656, 17920, 2, 64, 1024, 8, 0.01, 0.04),
    "c4_30b_down": LayerConfig("c4_30b_down", 17920, 6656, 2, 64, 1024, 8, 0.01, 0.04),
    # LLaMA-65B decoder layer, swept over M in {1, 16, 256, 4096}
    "c5_65b_attn": LayerConfig("c5_65b_attn", 8192, 8192, 3, 128, 16, 8),
    "c5_65b_up": LayerConfig("c5_65b_up", 8192, 22016, 3, 128, 16, 8),
    "c5_65b_down": LayerConfig("c5_65b_down", 22016, 8192, 3, 128, 16, 8),
}
C5_M_SWEEP = (1, 16, 256, 4096)

# one independent random stream per tensor, keyed by these ids
_STREAM = {"codes": 1, "zeros": 2, "scales": 3, "X": 4, "dY": 5, "A": 6, "B": 7, "zeros_f16": 8, "bias": 9}


def _rng(seed: int, what: str) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, _STREAM[what]])))


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Store float32 values as bfloat16 (round to nearest even) bit patterns."""
    import torch

    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bf16_bits_to_f64(a: np.ndarray) -> np.ndarray:
    """Widen stored bfloat16 bit patterns to float64 (exact)."""
    return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def f16_bits_to_f64(a: np.ndarray) -> np.ndarray:
    """Widen stored binary16 bit patterns to float64 (exact)."""
    return a.view(np.float16).astype(np.float64)


def pack_codes(codes: np.ndarray, bits: int) -> np.ndarray:
    """Write codes[n][k] into the packed words, one stream bit at a time.

    Column n's stream bit j = k*bits + t holds bit t of codes[n][k]; stream bit
    j lives in bit (j mod 32) of word [j // 32][n].
    """
    N, K = codes.shape
    assert (K * bits) % 32 == 0
    assert int(codes.max(initial=0)) < (1 << bits)
    words = np.zeros((K * bits // 32, N), dtype=np.uint32)
    for k in range(K):
        col = codes[:, k].astype(np.uint32)
        for t in range(bits):
            j = k * bits + t
            words[j // 32] |= ((col >> np.uint32(t)) & np.uint32(1)) << np.uint32(j % 32)
    return words


def make_layer(cfg: LayerConfig, *, zero_B: bool = False, zero_A: bool = False) -> dict:
    """Draw every input of one layer workload.  Deterministic in cfg.seed."""
    K, N, M, r, b, g = cfg.K, cfg.N, cfg.M, cfg.r, cfg.bits, cfg.group
    assert K % g == 0 and (g * b) % 32 == 0
    G = K // g
    codes = _rng(cfg.seed, "codes").integers(0, 1 << b, size=(N, K), dtype=np.uint8)
    zeros = _rng(cfg.seed, "zeros").integers(0, 1 << b, size=(G, N), dtype=np.uint8)
    scales32 = _rng(cfg.seed, "scales").uniform(cfg.scale_lo, cfg.scale_hi, size=(G, N)).astype(np.float32)
    scales = scales32.astype(np.float16).view(np.uint16)
    X = f32_to_bf16_bits(_rng(cfg.seed, "X").standard_normal((M, K), dtype=np.float32))
    dY = f32_to_bf16_bits(_rng(cfg.seed, "dY").standard_normal((M, N), dtype=np.float32))
    A = (0.02 * _rng(cfg.seed, "A").standard_normal((K, r), dtype=np.float32)).astype(np.float32)
    B = (0.02 * _rng(cfg.seed, "B").standard_normal((r, N), dtype=np.float32)).astype(np.float32)
    if zero_A:
        A = np.zeros_like(A)
    if zero_B:
        B = np.zeros_like(B)
    return dict(
        cfg=cfg, K=K, N=N, M=M, r=r, bits=b, group=g, lora_scale=float(cfg.lora_scale),
        codes=codes, qweight=pack_codes(codes, b), zeros=zeros, scales=scales,
        X=X, dY=dY, A=np.ascontiguousarray(A), B=np.ascontiguousarray(B),
    )


def make_layer_f16(cfg: LayerConfig, *, with_bias: bool = True) -> dict:
    """Inputs of the layer in the paper's own storage convention: the same codes, scales, A and B
    as make_layer(), a binary16 additive zero point per group, U[-(2^b - 1) * scale_hi, 0] (the
    range the integer zero points times the scales cover), binary16 activations N(0, 1) and a
    binary16 bias N(0, 0.1)."""
    L = make_layer(cfg)
    G = cfg.K // cfg.group
    span = ((1 << cfg.bits) - 1) * cfg.scale_hi
    z32 = _rng(cfg.seed, "zeros_f16").uniform(-span, 0.0, size=(G, cfg.N)).astype(np.float32)
    L["zeros_f16"] = z32.astype(np.float16).view(np.uint16)
    L["X"] = _rng(cfg.seed, "X").standard_normal((cfg.M, cfg.K), dtype=np.float32).astype(np.float16).view(np.uint16)
    L["dY"] = _rng(cfg.seed, "dY").standard_normal((cfg.M, cfg.N), dtype=np.float32).astype(np.float16).view(np.uint16)
    L["bias"] = None
    if with_bias:
        b32 = (0.1 * _rng(cfg.seed, "bias").standard_normal(cfg.N, dtype=np.float32)).astype(np.float32)
        L["bias"] = b32.astype(np.float16).view(np.uint16)
    del L["zeros"]
    return L


def make_layer_torch(cfg: LayerConfig, device: str = "cuda", seed: int = 0) -> dict:
    """The same distributions as make_layer, drawn with torch's generator on `device` (fast at
    the full benchmark sizes, where the bit-by-bit packer would take minutes).  Uniformly random
    32-bit words are exactly uniformly random codes.  Returns torch tensors: qweight int32,
    scales float16, zeros uint8, X / dY bfloat16, A / B float32."""
    import torch

    K, N, M, r, bits, g = cfg.K, cfg.N, cfg.M, cfg.r, cfg.bits, cfg.group
    G = K // g
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    q = torch.randint(-2 ** 31, 2 ** 31, (K * bits // 32, N), dtype=torch.int64, device=device,
                      generator=gen).to(torch.int32)
    sc = (torch.rand((G, N), device=device, generator=gen) * (cfg.scale_hi - cfg.scale_lo)
          + cfg.scale_lo).to(torch.float16)
    z = torch.randint(0, 1 << bits, (G, N), dtype=torch.uint8, device=device, generator=gen)
    out = {"qweight": q, "scales": sc, "zeros": z, "K": K, "N": N, "M": M, "r": r, "bits": bits, "group": g,
           "lora_scale": cfg.lora_scale}
    out["X"] = torch.randn((M, K), device=device, generator=gen).to(torch.bfloat16)
    out["dY"] = torch.randn((M, N), device=device, generator=gen).to(torch.bfloat16)
    out["A"] = torch.randn((K, max(r, 1)), device=device, generator=gen)[:, :r].contiguous() * 0.02
    out["B"] = torch.randn((max(r, 1), N), device=device, generator=gen)[:r].contiguous() * 0.02
    return out

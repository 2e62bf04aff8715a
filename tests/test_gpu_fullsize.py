"""Parity at the full benchmark sizes, in the launch configuration bench.py times (the library
picks its kernels from the shape alone).  The oracle's cost is linear in the token count, so
Y and dX are checked on a sample of token rows (each row of Y / dX depends only on the same
row of X / dY); dA and dB are checked in full (they need only rank-r products on the CPU);
and the adjoint identity <dY, Y> = <dX, X>, which holds for the layer as a whole at any size,
ties the unsampled rows together."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_16119_amd import binding as b
from paper_2309_16119_amd import synth

from gpu_util import assert_bar, assert_tight, f64

pytestmark = pytest.mark.gpu

CASES = [
    ("c2_7b_attn", None),
    ("c3_7b_gate_up", None),
    ("c3_7b_down", None),
    ("c4_30b_attn", None),
    ("c5_65b_attn", 16),
    ("c5_65b_attn", 1),
    ("c5_65b_attn", 256),
    ("c5_65b_attn", 4096),
    ("c5_65b_up", 16),
    ("c5_65b_down", 16),
    ("c4_30b_up", None),
    ("c4_30b_down", None),
    ("c5_65b_up", 1),
    ("c5_65b_up", 256),
    ("c5_65b_up", 4096),
    ("c5_65b_down", 256),
    ("c5_65b_down", 4096),
]


def host16(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


@pytest.mark.parametrize("name,M", CASES)
def test_full_size_layer_against_oracle(name, M):
    cfg = synth.CONFIGS[name] if M is None else synth.CONFIGS[name].with_M(M)
    L = synth.make_layer_torch(cfg, "cuda", seed=11)
    K, N, M, r, s = cfg.K, cfg.N, cfg.M, cfg.r, cfg.lora_scale
    w = b.QWeight(L["qweight"], L["scales"], L["zeros"], K, N, cfg.bits, cfg.group)
    Y, XA = b.modulora_fwd(w, L["X"], L["A"], L["B"], s)
    dX, T = b.modulora_bwd_input(w, L["dY"], L["A"], L["B"], s)
    dA, dB = b.modulora_bwd_lora(L["X"], L["dY"], L["A"], L["B"], s, XA=XA, dYBt=T)
    torch.cuda.synchronize()

    # host copies for the oracle
    qw = L["qweight"].cpu().numpy().view(np.uint32)
    sc = host16(L["scales"])
    zz = L["zeros"].cpu().numpy()
    Xh, dYh = host16(L["X"]), host16(L["dY"])
    Ah, Bh = L["A"].cpu().numpy(), L["B"].cpu().numpy()
    wargs = (qw, sc, zz, K, N, cfg.bits, cfg.group)

    rng = np.random.default_rng(5)
    n_rows = min(M, 12)
    rows = np.unique(np.concatenate(([0, M - 1], rng.integers(0, M, n_rows)))) if M > 12 else np.arange(M)
    Yr, Ur = oracle.fwd(*wargs, np.ascontiguousarray(Xh[rows]), Ah, Bh, s)
    dXr, Tr = oracle.bwd_input(*wargs, np.ascontiguousarray(dYh[rows]), Ah, Bh, s)

    extra_Y = extra_dX = 0.0
    if M <= 16:   # code-domain arithmetic of the streaming kernels (see test_gpu_parity.py)
        Wabs = np.abs(oracle.dequant_f32(*wargs).astype(np.float64))
        extra_Y = 2.0 ** -8 * (np.abs(synth.bf16_bits_to_f64(Xh[rows])) @ Wabs.T)
        extra_dX = 2.0 ** -7 * (np.abs(synth.bf16_bits_to_f64(dYh[rows])) @ Wabs)
    Yg, dXg = f64(Y)[rows], f64(dX)[rows]
    assert_bar("Y", Yg, Yr)
    assert_tight("Y", Yg, Yr, True, K, extra_Y)
    assert_bar("dX", dXg, dXr)
    assert_tight("dX", dXg, dXr, True, N, extra_dX)
    assert_tight("XA", f64(XA)[rows], Ur, False, K)
    assert_tight("dYBt", f64(T)[rows], Tr, False, N)

    dAr, dBr = oracle.bwd_lora(K, N, Xh, dYh, Ah, Bh, s)
    assert_bar("dA", f64(dA), dAr)
    assert_bar("dB", f64(dB), dBr)
    assert_tight("dA", f64(dA), dAr, False, M * N)
    assert_tight("dB", f64(dB), dBr, False, M * K)

    # adjoint identity over ALL rows: <dY, Y> = <dX, X> for the whole (linear, bias-free) layer.
    # Both sides carry one bfloat16 rounding per output element; random signs, so the sums
    # agree far better than 2^-9 relative to the sum of magnitudes.
    lhs = float((L["dY"].double() * Y.double()).sum())
    rhs = float((dX.double() * L["X"].double()).sum())
    mag = float((L["dY"].double().abs() * Y.double().abs()).sum())
    assert abs(lhs - rhs) <= 2.0 ** -9 * mag, (lhs, rhs, mag)

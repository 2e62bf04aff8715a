"""Randomly drawn layer shapes through both storage conventions, against the two oracles.

The fixed shape lists of the other GPU tests are chosen by hand for the launch configurations
they reach; this sweep draws (bits, d_in, d_out, tokens, rank, group size) at random -- a
handful of tokens, a few hundred, a thousand and more with a deep contraction in either
direction, narrow and wide outputs, one scale per row -- so that combinations nobody thought of
(an output narrower than a tile, a contraction shorter than one step, ...) are exercised too.
Seeded: the same shapes every run."""
import numpy as np
import pytest
import torch

import oracle
from oracle import paper_literal as pl
from paper_2309_16119_amd import binding as b
from paper_2309_16119_amd import synth

from gpu_util import f64, oracle_args, to_device

pytestmark = pytest.mark.gpu


def draw_shapes(seed, count):
    rng = np.random.default_rng(seed)
    shapes = []
    for _ in range(count):
        bits = int(rng.choice([2, 3, 4]))
        group = int(rng.choice([32, 64, 128, 256]))
        K = group * int(rng.integers(1, 24))
        if rng.random() < 0.3:
            group = K
        kind = rng.random()
        if kind < 0.35:
            M = int(rng.integers(1, 17))
        elif kind < 0.7:
            M = int(rng.integers(17, 400))
        else:
            M = int(rng.integers(1024, 1400))
        N = 8 * int(rng.integers(1, 300)) if rng.random() < 0.5 else 128 * int(rng.integers(1, 20))
        if M >= 1024 and rng.random() < 0.6:       # a deep contraction in one of the two directions
            if rng.random() < 0.5:
                K, N = group * max(1, 6400 // group), 8 * int(rng.integers(8, 80))
            else:
                N, K = 128 * int(rng.integers(48, 60)), group * int(rng.integers(1, 6))
        r = int(rng.choice([0, 1, 3, 8, 16, 24, 33, 64]))
        shapes.append((bits, K, N, M, r, group))
    return shapes


def close(name, got, ref, rel, n_sum, extra, ctx):
    """One rounding of the output (rel) plus fp32 accumulation over n_sum terms, plus `extra`."""
    scale = np.abs(ref).max()
    tol = rel * np.abs(ref) + (4e-7 * np.sqrt(n_sum) + 2e-5) * scale + extra
    bad = np.abs(got - ref) > tol
    assert not bad.any(), (name, ctx, int(bad.sum()), float(np.abs(got - ref).max()), float(scale))


def f16_dev(bits_u16):
    return torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16)).cuda().view(torch.float16)


@pytest.mark.parametrize("idx,shape", list(enumerate(draw_shapes(2309, 40))))
def test_random_shape_both_conventions(idx, shape):
    bits, K, N, M, r, group = shape
    cfg = synth.LayerConfig("rnd", K, N, bits, group, M, r, seed=7000 + idx)
    s = 2.0
    # ---- bfloat16 activations, integer zero points
    L = synth.make_layer(cfg)
    D = to_device(L)
    A, B = (L["A"], L["B"]) if r else (None, None)
    Y, XA = b.modulora_fwd(D["w"], D["Xd"], D["Ad"], D["Bd"], s)
    dX, T = b.modulora_bwd_input(D["w"], D["dYd"], D["Ad"], D["Bd"], s)
    Yr, Ur = oracle.fwd(*oracle_args(L), L["X"], A, B, s)
    dXr, Tr = oracle.bwd_input(*oracle_args(L), L["dY"], A, B, s)
    eY = edX = 0.0
    if M <= 32:     # the streaming kernels' code-domain arithmetic (see test_gpu_parity.py)
        Wabs = np.abs(oracle.dequant_f32(*oracle_args(L)).astype(np.float64))
        eY = 2.0 ** -8 * (np.abs(synth.bf16_bits_to_f64(L["X"])) @ Wabs.T)
        edX = 2.0 ** -7 * (np.abs(synth.bf16_bits_to_f64(L["dY"])) @ Wabs)
    close("Y", f64(Y), Yr, 2.0 ** -8, K, eY, shape)
    close("dX", f64(dX), dXr, 2.0 ** -8, N, edX, shape)
    if r:
        close("XA", f64(XA), Ur, 2.0 ** -20, K, 0.0, shape)
        close("dYBt", f64(T), Tr, 2.0 ** -20, N, 0.0, shape)
        dAr, dBr = oracle.bwd_lora(K, N, L["X"], L["dY"], L["A"], L["B"], s)
        for kw in (dict(XA=XA, dYBt=T), dict()):
            dA, dB = b.modulora_bwd_lora(D["Xd"], D["dYd"], D["Ad"], D["Bd"], s, **kw)
            close("dA", f64(dA), dAr, 2.0 ** -20, M * N, 0.0, shape)
            close("dB", f64(dB), dBr, 2.0 ** -20, M * K, 0.0, shape)
    # ---- the paper's storage convention: binary16, added zero point, bias on every other case
    L = synth.make_layer_f16(cfg, with_bias=bool(idx & 1))
    w = b.QWeightF16.from_numpy(L["qweight"], L["scales"], L["zeros_f16"], L["bias"], K, N, bits, group)
    Xd, dYd = f16_dev(L["X"]), f16_dev(L["dY"])
    Ad = torch.from_numpy(L["A"]).cuda() if r else None
    Bd = torch.from_numpy(L["B"]).cuda() if r else None
    oa = (L["qweight"], L["scales"], L["zeros_f16"], K, N, bits, group)
    Y, XA = b.modulora_f16_fwd(w, Xd, Ad, Bd, s)
    dX, T = b.modulora_f16_bwd_input(w, dYd, Ad, Bd, s)
    Yr, Ur = pl.fwd(*oa, L["X"], A, B, s, L["bias"])
    dXr, Tr = pl.bwd_input(*oa, L["dY"], A, B, s)
    eY = edX = 0.0
    if M <= 32:     # see test_gpu_f16.py
        Wabs = np.abs(synth.f16_bits_to_f64(pl.dequant_f16(*oa)))
        eY = 2.0 ** -11 * (np.abs(synth.f16_bits_to_f64(L["X"])) @ Wabs.T)
        edX = 2.0 ** -10 * (np.abs(synth.f16_bits_to_f64(L["dY"])) @ Wabs) + 2.0 ** -25 * 15 * N
    close("Y (binary16)", f64(Y), Yr, 2.0 ** -10, K + r, eY, shape)
    close("dX (binary16)", f64(dX), dXr, 2.0 ** -10, N + r, edX, shape)
    if r:
        close("XA (binary16)", f64(XA), Ur, 2.0 ** -20, K, 0.0, shape)
        close("dYBt (binary16)", f64(T), Tr, 2.0 ** -20, N, 0.0, shape)
        dA, dB = b.modulora_f16_bwd_lora(Xd, dYd, Ad, Bd, s, XA=XA, dYBt=T)
        dAr, dBr = pl.bwd_lora(L["X"], L["dY"], A, B, s)
        close("dA (binary16)", f64(dA), dAr, 2.0 ** -20, M + N, 0.0, shape)
        close("dB (binary16)", f64(dB), dBr, 2.0 ** -20, M + K, 0.0, shape)

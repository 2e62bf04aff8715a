"""Parity at the full benchmark sizes, in the launch configuration bench.py times (the library
picks its kernels from the shape alone).  The oracle's cost is linear in the token count, so
Y and dX are checked against it on a sample of token rows (each row of Y / dX depends only on
the same row of X / dY) that has at least one row in every block of 128 rows -- no row tile of
any kernel is left without an oracle-checked element -- plus the rows either side of tile
boundaries; dA and dB are checked in full (they need only rank-r products on the CPU).  Every
remaining element of Y and dX is compared, on the device, with a plain float32 torch product
over the materialized weight; that weight and that product are themselves tied to the oracle
(bit-exact dequantization, and the torch product against the oracle on the sampled rows), so a
mis-addressed or dropped tile anywhere fails.  The adjoint identity <dY, Y> = <dX, X>, which
holds for the layer as a whole at any size, is asserted with a tolerance sized from the
rounding statistics."""
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
    ("c5_65b_down", 1),
    ("c4_30b_up", None),
    ("c4_30b_down", None),
    ("c5_65b_up", 1),
    ("c5_65b_up", 256),
    ("c5_65b_up", 4096),
    ("c5_65b_down", 256),
    ("c5_65b_down", 4096),
    # the decoder layer of the benchmark at 128 tokens: the 128-row instantiation of the large tile kernel
    ("c5_65b_attn", 32),      # two passes of the streaming kernels
    ("c5_65b_up", 24),
    ("c5_65b_attn", 128),
    ("c5_65b_up", 128),
    ("c5_65b_down", 128),
]


def host16(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def sample_rows(M):
    """Token rows the oracle computes: all of them up to 48; else one random row from every block
    of 128 rows, the first and last row of every block of 128 (either side of every row-tile
    boundary of the 256- and 128-row kernels), and rows 0 and M - 1."""
    if M <= 48:
        return np.arange(M)
    rng = np.random.default_rng(5)
    starts = np.arange(0, M, 128)
    inner = starts + rng.integers(0, 128, starts.size)
    edges = np.concatenate((np.arange(0, M, 128), np.arange(127, M, 128)))
    rows = np.concatenate((inner, edges, [0, M - 1]))
    return np.unique(rows[rows < M])


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

    rows = sample_rows(M)
    Yr, Ur = oracle.fwd(*wargs, np.ascontiguousarray(Xh[rows]), Ah, Bh, s)
    dXr, Tr = oracle.bwd_input(*wargs, np.ascontiguousarray(dYh[rows]), Ah, Bh, s)

    extra_Y = extra_dX = 0.0
    if M <= 32:   # code-domain arithmetic of the streaming kernels (see test_gpu_parity.py)
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

    # every element of Y and dX against a float32 torch product over the materialized weight
    What = b.modulora_dequant(w)
    assert np.array_equal(host16(What), oracle.dequant_bf16(*wargs))               # tied to the oracle, bit for bit
    Wf = What.float()
    del What
    rows_t = torch.from_numpy(rows).cuda()
    torch.backends.cuda.matmul.allow_tf32 = False
    for oname, act, out, P, F_up, ref_rows, Ksum, code_tol in (
            ("Y", L["X"], Y, XA, L["B"], Yr, K, 2.0 ** -8 if M <= 32 else 0.0),
            ("dX", L["dY"], dX, T, L["A"].t(), dXr, N, 2.0 ** -7 if M <= 32 else 0.0)):
        Wm = Wf.t() if oname == "Y" else Wf
        ref = act.float() @ Wm + s * (P @ F_up)
        scale = float(ref.abs().max())
        tol = 2.0 ** -8 * ref.abs() + (4e-7 * np.sqrt(Ksum) + 2e-5) * scale
        if code_tol:
            tol = tol + code_tol * (act.float().abs() @ Wm.abs())
        bad = (out.float() - ref).abs() > tol
        assert not bool(bad.any()), "%s: %d elements off the float32 torch product" % (oname, int(bad.sum()))
        # ... which agrees with the oracle where the oracle was computed
        assert_tight(oname + " (torch product)", ref[rows_t].double().cpu().numpy(), ref_rows, False, Ksum)
        del ref, tol, bad
    del Wf

    # adjoint identity over ALL rows: <dY, Y> = <dX, X> for the whole (linear, bias-free) layer.
    # Each side carries one bfloat16 rounding per output element (uniform within half an ulp:
    # standard deviation 2^-9 / sqrt(3) relative, independent signs), so the two sums differ by
    # about 2^-9 / sqrt(3) * sqrt(sum (dY Y)^2 + sum (dX X)^2); eight standard deviations are
    # allowed.  At M <= 32 the code-domain kernels add per-weight terms of the same size (the
    # skipped rounding of the weight, the rounded scaled activation): three times as much.
    lhs_terms = L["dY"].double() * Y.double()
    rhs_terms = dX.double() * L["X"].double()
    lhs, rhs = float(lhs_terms.sum()), float(rhs_terms.sum())
    sigma = 2.0 ** -9 / np.sqrt(3.0) * float(torch.sqrt((lhs_terms ** 2).sum() + (rhs_terms ** 2).sum()))
    assert abs(lhs - rhs) <= (24.0 if M <= 32 else 8.0) * sigma, (lhs, rhs, sigma)


def test_operands_beyond_four_gib():
    """More tokens than 32-bit byte offsets can address: X, dY, Y and dX are 4.5 GB each, so
    the rows past index 2^20 lie beyond 4 GiB from the start of their matrices.  Only a few
    thousand rows, spread over the whole range and dense at its very end, are non-zero; the
    oracle sees just those rows (every sum over tokens skips zero rows, every output row
    depends on its own input row alone).  An address that wrapped at 4 GiB would read a zero
    row in place of a populated one, or write into a row that must stay zero."""
    K = N = 2048
    bits, group, r, s = 3, 128, 8, 2.0
    M = (1 << 20) + (1 << 16) + 3
    n_live = 4096
    small = synth.LayerConfig("beyond_4gib", K, N, bits, group, n_live, r)
    L = synth.make_layer_torch(small, "cuda", seed=23)
    rng = np.random.default_rng(9)
    live = np.unique(np.concatenate((rng.integers(0, M, n_live - 200), np.arange(M - 150, M), [0, 1 << 20, (1 << 20) + 1])))
    n_live = live.size
    live_t = torch.from_numpy(live).cuda()
    X = torch.zeros((M, K), dtype=torch.bfloat16, device="cuda")
    dY = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    X[live_t] = L["X"][:n_live]
    dY[live_t] = L["dY"][:n_live]
    assert X.numel() * 2 > (1 << 32) and int(live[-1]) * K * 2 > (1 << 32)

    w = b.QWeight(L["qweight"], L["scales"], L["zeros"], K, N, bits, group)
    Y, XA = b.modulora_fwd(w, X, L["A"], L["B"], s)
    dX, T = b.modulora_bwd_input(w, dY, L["A"], L["B"], s)
    dA, dB = b.modulora_bwd_lora(X, dY, L["A"], L["B"], s, XA=XA, dYBt=T)
    torch.cuda.synchronize()

    # rows that must be zero are zero, and no populated row came out empty
    is_live = torch.zeros(M, dtype=torch.bool, device="cuda")
    is_live[live_t] = True
    for name, out in (("Y", Y), ("dX", dX), ("XA", XA), ("dYBt", T)):
        nonzero_rows = out.ne(0).any(dim=1)
        assert torch.equal(nonzero_rows, is_live), name

    qw = L["qweight"].cpu().numpy().view(np.uint32)
    sc = host16(L["scales"])
    zz = L["zeros"].cpu().numpy()
    Ah, Bh = L["A"].cpu().numpy(), L["B"].cpu().numpy()
    wargs = (qw, sc, zz, K, N, bits, group)
    Xl, dYl = host16(L["X"][:n_live]), host16(L["dY"][:n_live])
    # Y and dX on the populated rows from the far end and a sample of the others
    pick = np.unique(np.concatenate((np.arange(n_live - 24, n_live), rng.integers(0, n_live, 24))))
    pick_t = live_t[torch.from_numpy(pick).cuda()]
    Yr, Ur = oracle.fwd(*wargs, np.ascontiguousarray(Xl[pick]), Ah, Bh, s)
    dXr, Tr = oracle.bwd_input(*wargs, np.ascontiguousarray(dYl[pick]), Ah, Bh, s)
    assert_bar("Y", f64(Y[pick_t]), Yr)
    assert_tight("Y", f64(Y[pick_t]), Yr, True, K)
    assert_bar("dX", f64(dX[pick_t]), dXr)
    assert_tight("dX", f64(dX[pick_t]), dXr, True, N)
    assert_tight("XA", f64(XA[pick_t]), Ur, False, K)
    assert_tight("dYBt", f64(T[pick_t]), Tr, False, N)
    # the adapter gradients: sums over all tokens = sums over the populated rows
    dAr, dBr = oracle.bwd_lora(K, N, Xl, dYl, Ah, Bh, s)
    assert_bar("dA", f64(dA), dAr)
    assert_bar("dB", f64(dB), dBr)
    assert_tight("dA", f64(dA), dAr, False, n_live * N)
    assert_tight("dB", f64(dB), dBr, False, n_live * K)

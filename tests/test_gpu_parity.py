"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle,
element by element on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_16119_amd import binding as b
from paper_2309_16119_amd import synth

from gpu_util import (assert_bar, assert_tight, bf16_dev, bits16, f64, oracle_args, to_device)

pytestmark = pytest.mark.gpu


def layer(bits, K, N, M, r, group, seed=1, **kw):
    hi = 0.04 if bits == 2 else 0.02
    cfg = synth.LayerConfig("t", K, N, bits, group, M, r, hi / 4, hi, 2.0, seed)
    return synth.make_layer(cfg, **kw)


# ------------------------------------------------------------------ dequant: bit exact
@pytest.mark.parametrize("bits,K,N,group", [
    (4, 256, 256, 64), (3, 416, 296, 32), (2, 448, 8, 64), (4, 32, 1032, 32),
    (3, 1024, 520, 1024), (2, 2048, 264, 128),
])
def test_dequant_bit_exact(bits, K, N, group):
    L = layer(bits, K, N, 1, 0, group)
    D = to_device(L)
    got = bits16(b.modulora_dequant(D["w"]))
    ref = oracle.dequant_bf16(*oracle_args(L))
    assert np.array_equal(got, ref)


def test_dequant_bit_exact_full_size_llama7b_attention():
    L = synth.make_layer(synth.CONFIGS["c2_7b_attn"].with_M(1))
    D = to_device(L)
    got = bits16(b.modulora_dequant(D["w"]))
    assert np.array_equal(got, oracle.dequant_bf16(*oracle_args(L)))


# --------------------------------------- the fused kernels' own dequantization, observed
@pytest.mark.parametrize("bits", [2, 3, 4])
def test_fused_kernels_reproduce_the_weight_bit_exactly(bits):
    """One-hot activations pick out single weights: Y = What^T rows and dX = What rows,
    exactly, because one nonzero fp32 term and a bfloat16 -> bfloat16 rounding lose nothing.
    This makes the dequantization inside the fused kernels observable."""
    K, N, group = 320, 264, 64
    L = layer(bits, K, N, 1, 0, group, seed=5)
    D = to_device(L)
    What = oracle.dequant_bf16(*oracle_args(L))                          # [N][K] bits
    eyeK = torch.eye(K, dtype=torch.bfloat16, device="cuda")
    Y, _ = b.modulora_fwd(D["w"], eyeK, None, None, 1.0)                 # [K][N] = What^T
    assert np.array_equal(bits16(Y), What.T)
    eyeN = torch.eye(N, dtype=torch.bfloat16, device="cuda")
    dX, _ = b.modulora_bwd_input(D["w"], eyeN, None, None, 1.0)          # [N][K] = What
    assert np.array_equal(bits16(dX), What)
    # a few rows only (small-M launch configuration)
    Ys, _ = b.modulora_fwd(D["w"], eyeK[37:46].contiguous(), None, None, 1.0)
    assert np.array_equal(bits16(Ys), What.T[37:46])
    dXs, _ = b.modulora_bwd_input(D["w"], eyeN[100:101].contiguous(), None, None, 1.0)
    assert np.array_equal(bits16(dXs), What[100:101])


# ------------------------------------------------------------------ forward / backward
SHAPES = [
    # bits, K, N, M, r, group
    (4, 256, 256, 16, 8, 64),        # BASELINE config 1
    (3, 1120, 808, 1, 8, 160),
    (3, 1120, 808, 7, 3, 32),
    (2, 1088, 520, 33, 16, 64),
    (4, 544, 1304, 130, 40, 32),
    (3, 736, 776, 300, 64, 736),     # one scale per row (g = K), maximum rank
    (2, 512, 2056, 515, 5, 128),
    (4, 2048, 512, 64, 0, 128),      # r = 0: the plain low-precision linear map
    # M <= 16 with group sizes the streaming kernels accept (ragged last column block too)
    (3, 1024, 808, 16, 8, 128),
    (3, 2560, 264, 3, 5, 256),
    (2, 768, 296, 5, 4, 64),
    (2, 1024, 1032, 16, 16, 128),
    (4, 512, 1304, 1, 16, 32),
    (4, 1152, 520, 13, 40, 128),
    (3, 1536, 512, 9, 0, 1536),      # one scale per row, no adapter
    # ... and shapes the streaming backward kernel accepts too (N and group multiples of 128)
    (3, 1024, 768, 16, 8, 128),
    (3, 2560, 384, 3, 5, 256),
    (2, 1024, 1152, 5, 16, 256),
    (4, 1152, 640, 13, 40, 128),
    (4, 512, 2304, 1, 16, 512),
    (2, 768, 128, 16, 0, 768),
    # ... with two quantization groups per 128-column backward tile (group 64)
    (2, 768, 384, 5, 4, 64),
    (3, 1024, 2176, 11, 8, 64),
    (4, 512, 640, 16, 16, 64),
    # ... with N split over several workgroups whose waves get unequal numbers of steps
    (3, 1024, 2176, 11, 8, 128),
    (4, 512, 2176, 16, 4, 128),
    (2, 1024, 2176, 2, 8, 256),
    # few 256 x 256 tiles and a deep contraction: the tiles are cut into slices of the
    # contraction whose partial tiles a second kernel adds (ragged M, N and last 64-deep step)
    (3, 8224, 328, 200, 8, 32),      # forward: 2 tiles x 8 slices
    (4, 320, 8232, 300, 16, 64),     # backward: 4 tiles x 8 slices
    (2, 8192, 512, 256, 0, 128),     # no adapter: the partial tiles are the only scratch
    # a hundred-odd tokens (or that many past a multiple of 256): the same kernel with 128-row
    # tiles -- one exactly full tile, ragged ones, an adapter wider than one 64-deep step
    (3, 4096, 1024, 128, 8, 128),
    (2, 4160, 1064, 97, 20, 32),
    (4, 1056, 4136, 330, 40, 32),
    # few rows and a deep contraction: the rank-r projection is split over workgroups too
    (3, 4096, 264, 40, 40, 128),
    (4, 256, 6144, 100, 64, 32),
    # 17 .. 32 tokens over a weight of more than 4 MB of codes: two passes of the streaming kernels
    (3, 4096, 4096, 17, 8, 128),
    (4, 2560, 4096, 32, 16, 64),
    (2, 8192, 2176, 24, 5, 128),
    # about a hundred 128 x 64 tiles: the producer / consumer kernel, with a ragged row tile, a
    # ragged column tile, a ragged last 128-deep step in both directions and 16-deep adapter steps
    (3, 2112, 2136, 300, 8, 64),
    (4, 2144, 2080, 300, 16, 32),
    (2, 2048, 2176, 384, 40, 2048),
    # either side of the token count at which the streaming kernels hand over to the tile kernels
    (3, 1024, 768, 17, 8, 128),
    (4, 512, 520, 32, 8, 64),
]


def test_mid_size_shapes_run_the_producer_consumer_kernel():
    """The shapes above that are meant for the 128 x 64 producer / consumer kernel do reach it."""
    L = layer(3, 2112, 2136, 300, 8, 64, seed=2)
    D = to_device(L)
    b.modulora_profile_begin()
    b.modulora_fwd(D["w"], D["Xd"], D["Ad"], D["Bd"], L["lora_scale"])
    b.modulora_bwd_input(D["w"], D["dYd"], D["Ad"], D["Bd"], L["lora_scale"])
    torch.cuda.synchronize()
    names = set(b.modulora_profile_end())
    assert {"gemm_fwd_128x64s", "gemm_bwd_128x64s"} <= names, names


@pytest.mark.parametrize("bits,K,N,M,r,group", SHAPES)
def test_forward_backward_against_oracle(bits, K, N, M, r, group):
    L = layer(bits, K, N, M, r, group, seed=2)
    D = to_device(L)
    s = L["lora_scale"]
    A, B = (L["A"], L["B"]) if r else (None, None)

    # For a handful of tokens (M <= 32) the library may multiply by the codes directly, i.e. without the oracle's
    # intermediate rounding of What to bfloat16 (half an ulp, at most 2^-8 relative per
    # weight): allow exactly that much, as the rigorous bound 2^-8 * |act| |What|^T.  The
    # backward kernel instead rounds dY * scale to bfloat16 (another 2^-8 per term), hence
    # 2^-7 there.
    extra_Y = extra_dX = 0.0
    if M <= 32:
        Wabs = np.abs(oracle.dequant_f32(*oracle_args(L)).astype(np.float64))      # [N][K]
        extra_Y = 2.0 ** -8 * (np.abs(synth.bf16_bits_to_f64(L["X"])) @ Wabs.T)
        extra_dX = 2.0 ** -7 * (np.abs(synth.bf16_bits_to_f64(L["dY"])) @ Wabs)

    Y, XA = b.modulora_fwd(D["w"], D["Xd"], D["Ad"], D["Bd"], s)
    Yr, Ur = oracle.fwd(*oracle_args(L), L["X"], A, B, s)
    assert_bar("Y", f64(Y), Yr)
    assert_tight("Y", f64(Y), Yr, True, K, extra_Y)

    dX, T = b.modulora_bwd_input(D["w"], D["dYd"], D["Ad"], D["Bd"], s)
    dXr, Tr = oracle.bwd_input(*oracle_args(L), L["dY"], A, B, s)
    assert_bar("dX", f64(dX), dXr)
    assert_tight("dX", f64(dX), dXr, True, N, extra_dX)

    if r == 0:
        assert XA is None and T is None
        return
    assert_tight("XA", f64(XA), Ur, False, K)
    assert_tight("dYBt", f64(T), Tr, False, N)

    dAr, dBr = oracle.bwd_lora(K, N, L["X"], L["dY"], L["A"], L["B"], s)
    # with the hand-offs, and recomputing them inside
    for kw in (dict(XA=XA, dYBt=T), dict()):
        dA, dB = b.modulora_bwd_lora(D["Xd"], D["dYd"], D["Ad"], D["Bd"], s, **kw)
        assert_bar("dA", f64(dA), dAr)
        assert_bar("dB", f64(dB), dBr)
        assert_tight("dA", f64(dA), dAr, False, M * N)
        assert_tight("dB", f64(dB), dBr, False, M * K)


def test_small_token_counts_run_the_streaming_kernels():
    """BASELINE config 1 (group 64) and a group-128 layer reach the streaming kernels in both directions;
    so do 17 .. 32 tokens over a weight of at least 4 MB of codes (two passes: twice the launches), while
    a smaller weight at those token counts and 33 tokens do not."""
    for bits, K, N, M, group, passes in ((4, 256, 256, 16, 64, 1), (3, 1024, 768, 16, 128, 1), (3, 4096, 4096, 17, 128, 2),
                                         (2, 8192, 2176, 32, 128, 2), (3, 1024, 768, 17, 128, 0), (3, 4096, 4096, 33, 128, 0)):
        L = layer(bits, K, N, M, 8, group, seed=2)
        D = to_device(L)
        b.modulora_profile_begin()
        b.modulora_fwd(D["w"], D["Xd"], D["Ad"], D["Bd"], 2.0)
        b.modulora_bwd_input(D["w"], D["dYd"], D["Ad"], D["Bd"], 2.0)
        torch.cuda.synchronize()
        prof = b.modulora_profile_end()
        stream = {k: v[0] for k, v in prof.items() if k.startswith("stream_")}
        want = {k: passes for k in ("stream_fwd", "stream_fwd_finish", "stream_bwd", "stream_bwd_finish")} if passes else {}
        assert stream == want, (bits, K, N, M, group, prof)


@pytest.mark.parametrize("group", [128, 64])
@pytest.mark.parametrize("bits", [2, 3, 4])
def test_streaming_kernels_pick_out_single_weights(bits, group):
    """One-hot rows through the M <= 16 streaming kernels: a single nonzero term, so the
    code-domain arithmetic must land on the same bfloat16 as the materialized weight."""
    K, N = 512, 384
    L = layer(bits, K, N, 1, 0, group, seed=6)
    D = to_device(L)
    What = oracle.dequant_bf16(*oracle_args(L))
    eyeK = torch.eye(K, dtype=torch.bfloat16, device="cuda")
    for lo in (0, 100, 497):
        rows = eyeK[lo:lo + 15].contiguous()
        Y, _ = b.modulora_fwd(D["w"], rows, None, None, 1.0)
        assert np.array_equal(bits16(Y), What.T[lo:lo + 15])
    eyeN = torch.eye(N, dtype=torch.bfloat16, device="cuda")
    # backward: the scale is rounded to bfloat16 before the product, so a picked-out weight
    # may land on a bfloat16 neighbour of the materialized one (one ulp, at most 2^-7 relative)
    Wf = synth.bf16_bits_to_f64(What)
    for lo in (0, 368):
        rows = eyeN[lo:lo + 16].contiguous()
        dX, _ = b.modulora_bwd_input(D["w"], rows, None, None, 1.0)
        assert np.all(np.abs(f64(dX) - Wf[lo:lo + 16]) <= 2.0 ** -7 * np.abs(Wf[lo:lo + 16]))


def test_second_streaming_pass_picks_out_the_right_rows():
    """One-hot rows 0 .. 31 through the two-pass form (17 .. 32 tokens): row m of the output is
    column / row hot[m] of the weight, so a second pass that read or wrote at the wrong row offset
    would put the wrong weights there."""
    K, N = 4096, 4096
    L = layer(3, K, N, 1, 0, 128, seed=8)
    D = to_device(L)
    What = oracle.dequant_bf16(*oracle_args(L))
    hot = (np.arange(29) * 139 + 5) % K
    rows = torch.zeros((29, K), dtype=torch.bfloat16, device="cuda")
    rows[torch.arange(29), torch.from_numpy(hot).cuda()] = 1.0
    b.modulora_profile_begin()
    Y, _ = b.modulora_fwd(D["w"], rows, None, None, 1.0)
    torch.cuda.synchronize()
    assert b.modulora_profile_end()["stream_fwd"][0] == 2
    assert np.array_equal(bits16(Y), What.T[hot])
    hot = (np.arange(32) * 131 + 7) % N
    rows = torch.zeros((32, N), dtype=torch.bfloat16, device="cuda")
    rows[torch.arange(32), torch.from_numpy(hot).cuda()] = 1.0
    dX, _ = b.modulora_bwd_input(D["w"], rows, None, None, 1.0)
    Wf = synth.bf16_bits_to_f64(What)
    assert np.all(np.abs(f64(dX) - Wf[hot]) <= 2.0 ** -7 * np.abs(Wf[hot]))


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_adapter_term_dominant(bits):
    """Large adapters (the LoRA term is most of the output): a dropped, mis-scaled or
    transposed adapter path cannot hide under the base term."""
    K, N, M, r, group = 608, 392, 45, 8, 32
    L = layer(bits, K, N, M, r, group, seed=9)
    rng = np.random.default_rng(1)
    L["A"] = rng.standard_normal((K, r)).astype(np.float32)
    L["B"] = rng.standard_normal((r, N)).astype(np.float32)
    D = to_device(L)
    s = 0.75
    Y, XA = b.modulora_fwd(D["w"], D["Xd"], D["Ad"], D["Bd"], s)
    Yr, _ = oracle.fwd(*oracle_args(L), L["X"], L["A"], L["B"], s)
    Y0, _ = oracle.fwd(*oracle_args(L), L["X"], None, None, s)
    assert np.abs(Yr - Y0).max() > 10 * np.abs(Y0).max()
    assert_tight("Y", f64(Y), Yr, True, K)
    dX, T = b.modulora_bwd_input(D["w"], D["dYd"], D["Ad"], D["Bd"], s)
    dXr, _ = oracle.bwd_input(*oracle_args(L), L["dY"], L["A"], L["B"], s)
    assert_tight("dX", f64(dX), dXr, True, N)


def test_zero_B_gives_exactly_zero_dA_and_no_adapter_part():
    L = layer(4, 512, 264, 40, 8, 64, zero_B=True)
    D = to_device(L)
    Y, XA = b.modulora_fwd(D["w"], D["Xd"], D["Ad"], D["Bd"], 2.0)
    Y0, _ = b.modulora_fwd(D["w"], D["Xd"], None, None, 2.0)
    assert torch.equal(Y, Y0)
    dX, T = b.modulora_bwd_input(D["w"], D["dYd"], D["Ad"], D["Bd"], 2.0)
    assert torch.count_nonzero(T).item() == 0
    dA, dB = b.modulora_bwd_lora(D["Xd"], D["dYd"], D["Ad"], D["Bd"], 2.0, XA=XA, dYBt=T)
    assert torch.count_nonzero(dA).item() == 0
    assert torch.count_nonzero(dB).item() > 0


def test_gradient_accumulation_flag():
    L = layer(3, 256, 264, 70, 8, 32)
    D = to_device(L)
    dA1, dB1 = b.modulora_bwd_lora(D["Xd"], D["dYd"], D["Ad"], D["Bd"], 2.0)
    dA = torch.full_like(dA1, 3.0)
    dB = torch.full_like(dB1, -1.0)
    b.modulora_bwd_lora(D["Xd"], D["dYd"], D["Ad"], D["Bd"], 2.0, dA=dA, dB=dB, accumulate=True)
    assert torch.allclose(dA, dA1 + 3.0, rtol=1e-5, atol=1e-5)
    assert torch.allclose(dB, dB1 - 1.0, rtol=1e-5, atol=1e-5)
    # overwrite ignores what was there (NaN poison)
    dA.fill_(float("nan"))
    dB.fill_(float("nan"))
    b.modulora_bwd_lora(D["Xd"], D["dYd"], D["Ad"], D["Bd"], 2.0, dA=dA, dB=dB, accumulate=False)
    assert torch.allclose(dA, dA1, rtol=1e-5, atol=1e-6) and torch.allclose(dB, dB1, rtol=1e-5, atol=1e-6)


def test_outputs_fully_written_and_deterministic():
    """NaN-poisoned outputs and workspace: every element is overwritten; forward and
    backward-input use no atomics, so two runs agree bit for bit."""
    L = layer(3, 800, 520, 77, 8, 32)
    D = to_device(L)
    ws = b._workspace(D["Xd"].device, b.modulora_workspace_bytes(D["w"], 77, 8))
    ws.view(torch.int16).fill_(0x7FC0)     # bf16 NaN pattern, NaN as fp32 pairs too
    Y = torch.full((77, 520), float("nan"), dtype=torch.bfloat16, device="cuda")
    b.modulora_fwd(D["w"], D["Xd"], D["Ad"], D["Bd"], 2.0, Y=Y)
    assert not torch.isnan(Y).any()
    Y2, _ = b.modulora_fwd(D["w"], D["Xd"], D["Ad"], D["Bd"], 2.0)
    assert torch.equal(Y, Y2)
    dX = torch.full((77, 800), float("nan"), dtype=torch.bfloat16, device="cuda")
    b.modulora_bwd_input(D["w"], D["dYd"], D["Ad"], D["Bd"], 2.0, dX=dX)
    assert not torch.isnan(dX).any()
    dX2, _ = b.modulora_bwd_input(D["w"], D["dYd"], D["Ad"], D["Bd"], 2.0)
    assert torch.equal(dX, dX2)


def test_integer_special_case_on_gpu():
    """scale = 1, zero = 0, sparse X in {-1,0,1}: exact small integers out of the MFMA path."""
    rng = np.random.default_rng(3)
    for bits in (2, 3, 4):
        K, N, M = 256, 264, 50
        codes = rng.integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
        words = synth.pack_codes(codes, bits)
        scales = np.full((1, N), 0x3C00, dtype=np.uint16)
        zeros = np.zeros((1, N), dtype=np.uint8)
        Xi = np.zeros((M, K), dtype=np.int64)
        for m in range(M):
            idx = rng.choice(K, size=8, replace=False)
            Xi[m, idx] = rng.choice([-1, 1], size=8)
        w = b.QWeight.from_numpy(words, scales, zeros, K, N, bits, K)
        Y, _ = b.modulora_fwd(w, bf16_dev(synth.f32_to_bf16_bits(Xi.astype(np.float32))), None, None, 1.0)
        assert np.array_equal(f64(Y), (Xi @ codes.astype(np.int64).T).astype(np.float64))

"""Every tile variant the automatic choice can reach, against the oracle.

The library picks a tile kernel from the shape alone (a table of measured step costs).  Besides
the 256 x 256 and the 128 x 64 producer / consumer kernels that the benchmark shapes land on, ordinary shapes reach four more variants of the generic tile kernel: 64 x 128
with two k-groups (a few dozen tokens, very wide outputs), 64 x 128, 128 x 128 and 256 x 128;
and token counts whose last block of 256 rows would be at most half full take the 256 x 256
kernel's instantiation with 128-row tiles.
Each is driven here in both directions and at all three bit widths by a shape that the table
routes to it -- the kernel that ran is read back through the profiling hook and asserted -- with
a ragged row tile, a ragged column tile, a ragged last contraction step and an adapter."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_16119_amd import binding as b
from paper_2309_16119_amd import synth

from gpu_util import assert_bar, assert_tight, f64, oracle_args, to_device

pytestmark = pytest.mark.gpu

# variant -> (M, forward shape (K, N, group), backward shape (K, N, group))
# forward contracts over K and the tile grid covers N; backward contracts over N and covers K
VARIANTS = {
    "64x128k": (50, (288, 16664, 96), (16672, 264, 32)),
    "64x128": (131, (288, 16664, 32), (16672, 264, 16672)),
    "128x128": (200, (288, 16664, 288), (16672, 264, 32)),
    # the 256 x 256 kernel's second instantiation; eight slices of the contraction per tile + fix-up launch
    "128x256": (100, (4128, 1064, 96), (1056, 4104, 32)),
    "256x128": (1301, (288, 10760, 32), (10784, 264, 10784)),
}


def _layer(bits, K, N, M, r, group, seed):
    hi = 0.04 if bits == 2 else 0.02
    return synth.make_layer(synth.LayerConfig("t", K, N, bits, group, M, r, hi / 4, hi, 2.0, seed))


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("variant", sorted(VARIANTS))
def test_forward_through_variant(variant, bits):
    M, (K, N, group), _ = VARIANTS[variant]
    r = 8
    L = _layer(bits, K, N, M, r, group, seed=31)
    D = to_device(L)
    s = L["lora_scale"]
    b.modulora_profile_begin()
    Y, XA = b.modulora_fwd(D["w"], D["Xd"], D["Ad"], D["Bd"], s)
    torch.cuda.synchronize()
    names = set(b.modulora_profile_end())
    assert "gemm_fwd_" + variant in names, names
    Yr, Ur = oracle.fwd(*oracle_args(L), L["X"], L["A"], L["B"], s)
    assert_bar("Y", f64(Y), Yr)
    assert_tight("Y", f64(Y), Yr, True, K)
    assert_tight("XA", f64(XA), Ur, False, K)


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("variant", sorted(VARIANTS))
def test_backward_through_variant(variant, bits):
    M, _, (K, N, group) = VARIANTS[variant]
    r = 5
    L = _layer(bits, K, N, M, r, group, seed=37)
    D = to_device(L)
    s = L["lora_scale"]
    b.modulora_profile_begin()
    dX, T = b.modulora_bwd_input(D["w"], D["dYd"], D["Ad"], D["Bd"], s)
    torch.cuda.synchronize()
    names = set(b.modulora_profile_end())
    assert "gemm_bwd_" + variant in names, names
    dXr, Tr = oracle.bwd_input(*oracle_args(L), L["dY"], L["A"], L["B"], s)
    assert_bar("dX", f64(dX), dXr)
    assert_tight("dX", f64(dX), dXr, True, N)
    assert_tight("dYBt", f64(T), Tr, False, N)


@pytest.mark.parametrize("variant", sorted(VARIANTS))
def test_variant_reproduces_the_weight_bit_exactly(variant):
    """One-hot activations through each variant: every output is a single weight, which must
    come out with the bit pattern of the materialized one (3-bit: both word straddles)."""
    M, (K, N, group), (Kb, Nb, groupb) = VARIANTS[variant]
    L = _layer(3, K, N, 1, 0, group, seed=41)
    D = to_device(L)
    What = oracle.dequant_bf16(*oracle_args(L))                  # [N][K] bit patterns
    rows = torch.zeros((M, K), dtype=torch.bfloat16, device="cuda")
    hot = torch.arange(M, device="cuda") % K
    rows[torch.arange(M, device="cuda"), hot] = 1.0
    b.modulora_profile_begin()
    Y, _ = b.modulora_fwd(D["w"], rows, None, None, 1.0)
    torch.cuda.synchronize()
    assert "gemm_fwd_" + variant in set(b.modulora_profile_end())
    got = Y.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(got, What.T[hot.cpu().numpy()])

    L = _layer(3, Kb, Nb, 1, 0, groupb, seed=43)
    D = to_device(L)
    What = oracle.dequant_bf16(*oracle_args(L))
    rows = torch.zeros((M, Nb), dtype=torch.bfloat16, device="cuda")
    hot = (torch.arange(M, device="cuda") * 7) % Nb
    rows[torch.arange(M, device="cuda"), hot] = 1.0
    b.modulora_profile_begin()
    dX, _ = b.modulora_bwd_input(D["w"], rows, None, None, 1.0)
    torch.cuda.synchronize()
    assert "gemm_bwd_" + variant in set(b.modulora_profile_end())
    got = dX.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(got, What[hot.cpu().numpy()])

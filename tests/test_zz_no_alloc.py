"""modulora_fwd_static -- the forward pass on the library's own static scratch, for callers that
cannot allocate -- against modulora_fwd on the same inputs: same kernels, so the outputs must be
equal bit for bit (and are therefore inside the stated bar against the oracle, which is checked
too).  Every case makes two calls in a row on the shared scratch, the second with a smaller
input, with the scratch's previous contents left in place."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_16119_amd import binding as b
from paper_2309_16119_amd import synth

from gpu_util import assert_bar, f64, oracle_args, to_device

pytestmark = pytest.mark.gpu


def _layer(bits, K, N, M, r, group, seed):
    hi = 0.04 if bits == 2 else 0.02
    return synth.make_layer(synth.LayerConfig("t", K, N, bits, group, M, r, hi / 4, hi, 2.0, seed))


def _both(L):
    D = to_device(L)
    M, N, r, s = L["M"], L["N"], L["r"], L["lora_scale"]
    Y_ref, XA_ref = b.modulora_fwd(D["w"], D["Xd"], D["Ad"], D["Bd"], s)
    Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    XA = torch.full((M, r), float("nan"), dtype=torch.float32, device="cuda") if r else None
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    b.modulora_fwd_static(D["w"], D["Xd"], D["Ad"], D["Bd"], s, Y, XA)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before or _both.first, "device memory changed during the call"
    _both.first = False
    assert torch.equal(Y.view(torch.int16), Y_ref.view(torch.int16))
    if r:
        assert torch.equal(XA, XA_ref)
    Yr, _ = oracle.fwd(*oracle_args(L), L["X"], L["A"] if r else None, L["B"] if r else None, s)
    assert_bar("Y", f64(Y), Yr)


_both.first = True      # the first call on the GPU loads the array's address (and may map the code object)


@pytest.mark.parametrize("first,second", [
    # M <= 16 streaming kernels: slices of K meet in the scratch
    ((3, 2048, 2176, 16, 8, 128), (3, 1024, 768, 5, 8, 128)),
    ((4, 1152, 520, 13, 40, 128), (2, 768, 296, 5, 0, 64)),
    # two passes of the streaming kernels (24 tokens over 6 MB of codes), then one pass
    ((3, 4096, 4096, 24, 8, 128), (3, 4096, 4096, 9, 8, 128)),
    # 128 x 64 producer / consumer kernel, then a few dozen tokens: adapter operands in the scratch
    ((3, 2112, 2136, 300, 8, 64), (4, 512, 520, 32, 8, 64)),
    # 256 x 256 kernel with a split contraction whose partial tiles (4 MB) fit the scratch, then a
    # layer without adapter whose only scratch is partial tiles
    ((3, 8224, 328, 200, 8, 32), (2, 8192, 512, 256, 0, 128)),
])
def test_static_scratch_forward_equals_workspace_forward(first, second):
    for shape in (first, second):
        bits, K, N, M, r, group = shape
        _both(_layer(bits, K, N, M, r, group, seed=51))


def test_partial_tiles_that_do_not_fit_are_done_without():
    """A shape whose split contraction would need 64 MB of partial tiles: the static entry point
    runs those tiles whole instead (a different summation order inside fp32 accumulation, so the
    comparison with the workspace path is at the oracle's bar, not bit for bit)."""
    L = _layer(3, 8192, 8192, 300, 8, 128, seed=52)        # 64 tiles x 4 slices x 256 KB
    D = to_device(L)
    s = L["lora_scale"]
    Y = torch.full((300, 8192), float("nan"), dtype=torch.bfloat16, device="cuda")
    b.modulora_fwd_static(D["w"], D["Xd"], D["Ad"], D["Bd"], s, Y, None)
    rows = np.array([0, 17, 128, 255, 256, 299])
    Yr, _ = oracle.fwd(*oracle_args(L), np.ascontiguousarray(L["X"][rows]), L["A"], L["B"], s)
    assert_bar("Y", f64(Y)[rows], Yr)
    Y_ref, _ = b.modulora_fwd(D["w"], D["Xd"], D["Ad"], D["Bd"], s)
    assert not torch.isnan(Y.float()).any()
    assert float((Y.float() - Y_ref.float()).abs().max()) <= 2.0 ** -7 * float(Y_ref.float().abs().max())

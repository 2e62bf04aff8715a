"""GPU parity of the round-to-nearest quantizer + packer (C ABI) against the numpy oracle:
bit-exact words, scales and zero points; and the round trip through the library's own
dequantizer within the error bound."""
import numpy as np
import pytest
import torch

import oracle
from oracle import rtn
from paper_2309_16119_amd import binding as b

pytestmark = pytest.mark.gpu


def weight(N, K, seed):
    """Weights like a trained linear layer's: normal, with a heavy-tailed per-row scale and a few
    outliers; plus degenerate rows (all zero, all positive, all negative, constant)."""
    rng = np.random.default_rng(seed)
    W = (rng.normal(size=(N, K)) * rng.lognormal(sigma=1.0, size=(N, 1)) * 0.02).astype(np.float32)
    out = rng.integers(0, N * K, size=max(1, N * K // 500))
    W.reshape(-1)[out] *= 8
    W[0] = 0.0
    W[1] = np.abs(W[1])
    W[2] = -np.abs(W[2])
    W[3] = 0.37
    W[4, : K // 2] = 0.0
    return W


@pytest.mark.parametrize("bits,K,N,group", [
    (4, 256, 256, 64), (3, 416, 296, 32), (2, 448, 8, 64), (4, 32, 1032, 32), (3, 1024, 520, 1024),
    (2, 2048, 264, 128), (3, 2240, 72, 160), (4, 3072, 136, 1536), (2, 4096, 64, 4096), (3, 4096, 4096, 128),
])
def test_quantize_bit_exact(bits, K, N, group):
    W = weight(N, K, seed=bits * 1000 + group)
    qw = b.modulora_quantize_rtn(torch.from_numpy(W).cuda(), bits, group)
    q_ref, s_ref, z_ref = rtn.quantize_packed(W, bits, group)
    assert np.array_equal(qw.scales.cpu().numpy().view(np.uint16), s_ref)
    assert np.array_equal(qw.zeros.cpu().numpy(), z_ref)
    assert np.array_equal(qw.qweight.cpu().numpy().view(np.uint32), q_ref)


def test_quantize_then_dequantize_full_size_within_the_bound():
    """LLaMA-65B up projection (8192 -> 22016), 3-bit, group 128: quantize on the GPU, materialize
    with the library's dequantizer, check |w - what| <= scale (1/2 + 2^-20) + the bfloat16 rounding
    of what (2^-9 relative) everywhere, on the GPU; sampled columns bit-exact against the oracle."""
    K, N, bits, group = 8192, 22016, 3, 128
    g = torch.Generator(device="cuda").manual_seed(11)
    W = torch.randn((N, K), device="cuda", generator=g) * 0.02
    qw = b.modulora_quantize_rtn(W, bits, group)
    What = b.modulora_dequant(qw).float()                                   # [N][K]
    s = qw.scales.float().t().repeat_interleave(group, dim=1)              # [N][K]
    bound = s * (0.5 + 2.0 ** -20) + What.abs() * 2.0 ** -8
    assert bool(torch.all((W - What).abs() <= bound))
    cols = [0, 1, 4097, 22015]
    Wc = W[cols].cpu().numpy()
    q_ref, s_ref, z_ref = rtn.quantize_packed(Wc, bits, group)
    assert np.array_equal(qw.qweight[:, cols].cpu().numpy().view(np.uint32), q_ref)
    assert np.array_equal(qw.scales[:, cols].cpu().numpy().view(np.uint16), s_ref)
    assert np.array_equal(qw.zeros[:, cols].cpu().numpy(), z_ref)


def test_quantized_layer_runs_through_the_forward_pass():
    """The quantizer's output is a valid layer: forward of the library against the oracle's
    forward on the same (GPU-independent) oracle-quantized weight."""
    from paper_2309_16119_amd import synth
    from gpu_util import assert_bar, f64
    K, N, M, bits, group = 512, 384, 40, 4, 128
    W = weight(N, K, seed=3)
    q_ref, s_ref, z_ref = rtn.quantize_packed(W, bits, group)
    qw = b.modulora_quantize_rtn(torch.from_numpy(W).cuda(), bits, group)
    rng = np.random.default_rng(4)
    X = synth.f32_to_bf16_bits(rng.normal(size=(M, K)).astype(np.float32))
    Xd = torch.from_numpy(X.view(np.int16)).cuda().view(torch.bfloat16)
    Y, _ = b.modulora_fwd(qw, Xd, None, None, 0.0)
    Yr, _ = oracle.fwd(q_ref, s_ref, z_ref, K, N, bits, group, X, None, None, 0.0)
    assert_bar("Y", f64(Y), Yr)

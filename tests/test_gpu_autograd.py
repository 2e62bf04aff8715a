"""The torch module over the C-ABI: autograd must deliver exactly what the three library
calls return, and those are checked against the oracle here once more through the module."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_16119_amd import synth
from paper_2309_16119_amd.nn import ModuLoRALinear

from gpu_util import assert_bar, assert_tight, f64, oracle_args, to_device

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("bits,K,N,batch,seq,r,group", [(4, 512, 768, 2, 40, 8, 128), (3, 1024, 384, 1, 9, 16, 128),
                                                       (2, 512, 520, 3, 50, 0, 64)])
def test_module_forward_backward_match_the_oracle(bits, K, N, batch, seq, r, group):
    M = batch * seq
    cfg = synth.LayerConfig(name="t", K=K, N=N, bits=bits, group=group, M=M, r=r, seed=3)
    L = synth.make_layer(cfg)
    D = to_device(L)
    layer = ModuLoRALinear(D["w"], r=r, alpha=2.0 * r if r else 0.0)
    if r:
        with torch.no_grad():
            layer.A.copy_(D["Ad"])
            layer.B.copy_(D["Bd"])
    x = D["Xd"].view(batch, seq, K).clone().requires_grad_(True)
    y = layer(x)
    assert y.shape == (batch, seq, N) and y.dtype == torch.bfloat16
    y.backward(D["dYd"].view(batch, seq, N))

    s = 2.0
    A, B = (L["A"], L["B"]) if r else (None, None)
    Yr, _ = oracle.fwd(*oracle_args(L), L["X"], A, B, s)
    dXr, _ = oracle.bwd_input(*oracle_args(L), L["dY"], A, B, s)
    extra_Y = extra_dX = 0.0
    if M <= 32:
        Wabs = np.abs(oracle.dequant_f32(*oracle_args(L)).astype(np.float64))
        extra_Y = 2.0 ** -8 * (np.abs(synth.bf16_bits_to_f64(L["X"])) @ Wabs.T)
        extra_dX = 2.0 ** -7 * (np.abs(synth.bf16_bits_to_f64(L["dY"])) @ Wabs)
    assert_bar("Y", f64(y).reshape(M, N), Yr)
    assert_tight("Y", f64(y).reshape(M, N), Yr, True, K, extra_Y)
    assert_bar("dX", f64(x.grad).reshape(M, K), dXr)
    assert_tight("dX", f64(x.grad).reshape(M, K), dXr, True, N, extra_dX)
    if r:
        dAr, dBr = oracle.bwd_lora(K, N, L["X"], L["dY"], L["A"], L["B"], s)
        assert_tight("dA", f64(layer.A.grad), dAr, False, M * N)
        assert_tight("dB", f64(layer.B.grad), dBr, False, M * K)
    else:
        assert layer.A is None and layer.B is None


def test_module_over_the_paper_literal_weight():
    """The same module over a QWeightF16: float16 activations, bias inside the frozen weight."""
    from oracle import paper_literal as pl
    from paper_2309_16119_amd import binding as b

    K, N, batch, seq, r = 512, 520, 2, 33, 8
    M = batch * seq
    cfg = synth.LayerConfig(name="t", K=K, N=N, bits=3, group=128, M=M, r=r, seed=6)
    L = synth.make_layer_f16(cfg)
    w = b.QWeightF16.from_numpy(L["qweight"], L["scales"], L["zeros_f16"], L["bias"], K, N, 3, 128)
    layer = ModuLoRALinear(w, r=r, alpha=2.0 * r)
    with torch.no_grad():
        layer.A.copy_(torch.from_numpy(L["A"]).cuda())
        layer.B.copy_(torch.from_numpy(L["B"]).cuda())
    h = lambda a: torch.from_numpy(a.view(np.int16)).cuda().view(torch.float16)
    x = h(L["X"]).view(batch, seq, K).clone().requires_grad_(True)
    y = layer(x)
    assert y.shape == (batch, seq, N) and y.dtype == torch.float16
    y.backward(h(L["dY"]).view(batch, seq, N))
    args = (L["qweight"], L["scales"], L["zeros_f16"], K, N, 3, 128)
    Yr, _ = pl.fwd(*args, L["X"], L["A"], L["B"], 2.0, L["bias"])
    dXr, _ = pl.bwd_input(*args, L["dY"], L["A"], L["B"], 2.0)
    dAr, dBr = pl.bwd_lora(L["X"], L["dY"], L["A"], L["B"], 2.0)
    assert_bar("Y", f64(y).reshape(M, N), Yr)
    assert_bar("dX", f64(x.grad).reshape(M, K), dXr)
    assert_bar("dA", f64(layer.A.grad), dAr)
    assert_bar("dB", f64(layer.B.grad), dBr)
    assert np.abs(f64(y).reshape(M, N) - Yr).max() <= 2.0 ** -10 * np.abs(Yr).max() + 1e-4


def test_module_starts_as_the_plain_quantized_layer_and_trains():
    cfg = synth.LayerConfig(name="t", K=256, N=256, bits=4, group=64, M=32, r=8, seed=4)
    L = synth.make_layer(cfg)
    D = to_device(L)
    layer = ModuLoRALinear(D["w"], r=8, alpha=16.0)
    x = D["Xd"]
    y0 = layer(x)
    Yr, _ = oracle.fwd(*oracle_args(L), L["X"], None, None, 0.0)
    assert_bar("Y (B = 0)", f64(y0), Yr)          # B = 0: the adapter contributes nothing yet
    # a few SGD steps on the adapter towards a shifted target must reduce the loss
    target = (y0.float() + 0.1).detach()
    opt = torch.optim.SGD(layer.parameters(), lr=1e-2)
    losses = []
    for _ in range(5):
        opt.zero_grad()
        out = layer(x).float()
        loss = ((out - target) ** 2).mean()
        loss.backward()
        opt.step()
        losses.append(float(loss.detach()))
    assert losses[-1] < losses[0]
    assert layer.B.grad is not None and layer.A.grad is not None


def test_fused_adamw_over_two_modules_matches_the_oracle():
    """Two layers of different shape in one flat buffer.  (a) autograd accumulates into the flat
    gradient in place; (b) with seeded gradients written into it, three optimizer steps leave
    every factor equal to the float64 AdamW oracle applied to that factor alone."""
    from oracle import optim as oracle_optim
    from paper_2309_16119_amd.nn import FusedAdapterAdamW

    cfg1 = synth.LayerConfig(name="t1", K=256, N=384, bits=4, group=64, M=48, r=8, seed=5)
    cfg2 = synth.LayerConfig(name="t2", K=384, N=264, bits=3, group=128, M=48, r=5, seed=6)   # 5 * 264: not a multiple of 4
    D1, D2 = to_device(synth.make_layer(cfg1)), to_device(synth.make_layer(cfg2))
    l1, l2 = ModuLoRALinear(D1["w"], r=8, alpha=16.0), ModuLoRALinear(D2["w"], r=5, alpha=10.0)
    with torch.no_grad():
        l1.B.copy_(D1["Bd"])
        l2.B.copy_(D2["Bd"])
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
    hp = {k: float(np.float32(v)) for k, v in hp.items()}
    opt = FusedAdapterAdamW([l1, l2], lr=hp["lr"], betas=(hp["beta1"], hp["beta2"]), eps=hp["eps"],
                            weight_decay=hp["weight_decay"])
    params = [l1.A, l1.B, l2.A, l2.B]

    # (a) backward through both layers lands in the flat gradient buffer
    grad_ptrs = [p.grad.data_ptr() for p in params]
    opt.zero_grad()
    l2(l1(D1["Xd"])).float().square().mean().backward()
    assert [p.grad.data_ptr() for p in params] == grad_ptrs
    assert all(bool(torch.any(p.grad != 0)) for p in params)
    assert int(torch.count_nonzero(opt.flat_grad)) == sum(int(torch.count_nonzero(p.grad)) for p in params)

    # (b) seeded gradients, three steps
    rng = np.random.default_rng(7)
    state = [(f64(p.detach()), np.zeros(p.shape), np.zeros(p.shape)) for p in params]
    for step in range(1, 4):
        grads = [rng.normal(size=tuple(p.shape)).astype(np.float32) * 0.1 for p in params]
        opt.zero_grad()
        with torch.no_grad():
            for p, g in zip(params, grads):
                p.grad.copy_(torch.from_numpy(g))
        opt.step()
        for i, p in enumerate(params):
            assert opt.flat.data_ptr() <= p.data_ptr() < opt.flat.data_ptr() + opt.flat.numel() * 4
            pr, mr, vr = oracle_optim.adamw_step(state[i][0], grads[i], state[i][1], state[i][2], step=step, **hp)
            tol = step * 2.0 ** -23 * np.abs(pr) + 32 * 2.0 ** -24 * hp["lr"] * step
            assert np.all(np.abs(f64(p.detach()) - pr) <= tol), (step, i)
            state[i] = (pr, mr, vr)

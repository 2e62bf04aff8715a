"""The layer as a torch module: autograd glue over the C-ABI calls, nothing else.

`LPLoRAFunction` is Figure 1 of the ModuLoRA paper with the three library calls in place of
its PyTorch lines: forward = modulora_fwd, backward = modulora_bwd_input (the weight is
re-materialized from the codes, nothing but codes, scales and zeros is kept) plus
modulora_bwd_lora for the adapter factors.  `ModuLoRALinear` holds the frozen quantized
weight and the trainable adapter (A [d_in][r], B [r][d_out], fp32; the paper's B and A^T).
All arithmetic runs in the HIP kernels; this file only reshapes, keeps tensors alive for the
backward pass and hands pointers over.
"""
from __future__ import annotations

import math
from typing import Optional

import torch

from . import binding as b


def _calls(w):
    """(forward, input gradient, adapter gradients, activation dtype) for the kind of frozen weight:
    the bfloat16 integer-zero-point layer or the paper-literal binary16 one (b.QWeightF16)."""
    if isinstance(w, b.QWeightF16):
        return b.modulora_f16_fwd, b.modulora_f16_bwd_input, b.modulora_f16_bwd_lora, torch.float16
    return b.modulora_fwd, b.modulora_bwd_input, b.modulora_bwd_lora, torch.bfloat16


class LPLoRAFunction(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x: torch.Tensor, A: Optional[torch.Tensor], B: Optional[torch.Tensor], w, lora_scale: float):
        x2 = x.reshape(-1, w.d_in)
        if not x2.is_contiguous():
            x2 = x2.contiguous()
        y, xa = _calls(w)[0](w, x2, A, B, lora_scale)
        ctx.w, ctx.lora_scale, ctx.x_shape = w, lora_scale, x.shape
        ctx.save_for_backward(x2, A, B, xa)       # activations and adapter only: no weight copy
        return y.view(*x.shape[:-1], w.d_out)

    @staticmethod
    def backward(ctx, grad_y: torch.Tensor):
        x2, A, B, xa = ctx.saved_tensors
        w, s = ctx.w, ctx.lora_scale
        _, bwd_input, bwd_lora, act_dtype = _calls(w)
        dy = grad_y.reshape(-1, w.d_out)
        if dy.dtype != act_dtype:
            dy = dy.to(act_dtype)
        if not dy.is_contiguous():
            dy = dy.contiguous()
        dx, t = bwd_input(w, dy, A, B, s)
        dA = dB = None
        if A is not None and (ctx.needs_input_grad[1] or ctx.needs_input_grad[2]):
            dA, dB = bwd_lora(x2, dy, A, B, s, XA=xa, dYBt=t)
        return dx.view(ctx.x_shape), dA, dB, None, None


class ModuLoRALinear(torch.nn.Module):
    """y = x What^T + (alpha / r) (x A) B with What frozen in 2/3/4-bit group-quantized form.
    `w` is a b.QWeight (bfloat16 activations, integer zero points) or a b.QWeightF16 (the paper's
    own convention: binary16 activations, added float zero point, bias inside `w`)."""

    def __init__(self, w, r: int = 8, alpha: float = 16.0, device: str = "cuda"):
        super().__init__()
        self.w = w
        self.r = r
        self.lora_scale = float(alpha) / r if r else 0.0
        if r:
            # the usual LoRA start: the factor next to the output is zero, so the layer starts
            # as the plain quantized one (Section 3.1: the adapter then learns the correction)
            self.A = torch.nn.Parameter(torch.randn(w.d_in, r, device=device) / math.sqrt(w.d_in))
            self.B = torch.nn.Parameter(torch.zeros(r, w.d_out, device=device))
        else:
            self.register_parameter("A", None)
            self.register_parameter("B", None)

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        return LPLoRAFunction.apply(x, self.A, self.B, self.w, self.lora_scale)

    def reserve_workspace(self, tokens: int) -> None:
        """Size the binding's cached scratch buffer of the current stream for `tokens` rows now, so
        that no allocation happens later (call it on the capture stream before a HIP graph capture)."""
        query = b.modulora_f16_workspace_bytes if isinstance(self.w, b.QWeightF16) else b.modulora_workspace_bytes
        b.reserve_workspace(self.w.device, query(self.w, int(tokens), self.r))


class FusedAdapterAdamW:
    """AdamW (the optimizer of the paper's Appendix hyper-parameter tables) over the adapter
    factors of many `ModuLoRALinear` modules with one kernel launch per step.

    All A and B are moved into one flat float32 buffer (each starting on a 16-byte boundary) and
    become views of it; their `.grad` become views of a second flat buffer, into which autograd
    accumulates in place.  `step()` is a single `modulora_adamw` call over the whole buffer;
    `zero_grad()` clears the flat gradient (never sets `.grad` to None, which would detach it).
    """

    def __init__(self, modules, lr: float = 3e-4, betas=(0.9, 0.999), eps: float = 1e-8, weight_decay: float = 0.0):
        params = [p for m in modules for p in (m.A, m.B) if p is not None]
        assert params, "no trainable adapter factors"
        dev = params[0].device
        offsets, total = [], 0
        for p in params:
            assert p.dtype == torch.float32 and p.device == dev
            offsets.append(total)
            total += (p.numel() + 3) // 4 * 4
        self.flat = torch.zeros(total, dtype=torch.float32, device=dev)
        self.flat_grad = torch.zeros_like(self.flat)
        self.exp_avg = torch.zeros_like(self.flat)
        self.exp_avg_sq = torch.zeros_like(self.flat)
        with torch.no_grad():
            for p, off in zip(params, offsets):
                view = self.flat[off:off + p.numel()].view(p.shape)
                view.copy_(p.data)
                p.data = view
                p.grad = self.flat_grad[off:off + p.numel()].view(p.shape)
        self.params = params
        self.lr, self.betas, self.eps, self.weight_decay = lr, betas, eps, weight_decay
        self.steps = 0

    def zero_grad(self) -> None:
        self.flat_grad.zero_()

    def step(self) -> None:
        self.steps += 1
        b.modulora_adamw(self.flat, self.flat_grad, self.exp_avg, self.exp_avg_sq, self.lr, self.betas[0],
                         self.betas[1], self.eps, self.weight_decay, self.steps)

"""Helpers for the GPU parity tests: move a synthetic layer to the device, widen GPU
outputs to float64, and the two comparison bars."""
import numpy as np
import torch

from paper_2309_16119_amd import binding as b

REL_LINF = 2e-2     # the stated bar: max|gpu - ref| <= 2e-2 * max|ref|, per output tensor


def bf16_dev(bits_u16: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits_u16.view(np.int16)).cuda().view(torch.bfloat16)


def to_device(L: dict) -> dict:
    D = dict(L)
    D["w"] = b.QWeight.from_numpy(L["qweight"], L["scales"], L["zeros"], L["K"], L["N"], L["bits"], L["group"])
    D["Xd"] = bf16_dev(L["X"])
    D["dYd"] = bf16_dev(L["dY"])
    D["Ad"] = torch.from_numpy(L["A"]).cuda() if L["r"] else None
    D["Bd"] = torch.from_numpy(L["B"]).cuda() if L["r"] else None
    return D


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def bits16(t: torch.Tensor) -> np.ndarray:
    return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)


def oracle_args(L):
    return (L["qweight"], L["scales"], L["zeros"], L["K"], L["N"], L["bits"], L["group"])


def assert_bar(name, got, ref):
    """The stated parity bar.  An identically-zero reference demands an exact zero."""
    scale = np.abs(ref).max() if ref.size else 0.0
    err = np.abs(got - ref).max() if ref.size else 0.0
    if scale == 0.0:
        assert err == 0.0, "%s: reference is zero, got max %g" % (name, err)
    else:
        assert err <= REL_LINF * scale, "%s: max err %g > %g * %g" % (name, err, REL_LINF, scale)
    return err / scale if scale else 0.0


def assert_tight(name, got, ref, out_bf16, K_sum, extra_abs=0.0):
    """A bound derived from the arithmetic, far tighter than the stated bar, so that a
    dropped or mis-scaled small term cannot hide: one bfloat16 rounding of the output
    (2^-9 relative, when out_bf16) plus fp32 accumulation over K_sum terms, plus the
    hi/lo bf16 split of the adapter operands (about 2^-16 relative to the adapter term,
    covered by the accumulation allowance)."""
    scale = np.abs(ref).max()
    rel = (2.0 ** -8 if out_bf16 else 2.0 ** -20)
    tol = rel * np.abs(ref) + (4e-7 * np.sqrt(K_sum) + 2e-5) * scale + extra_abs
    bad = np.abs(got - ref) > tol
    assert not bad.any(), "%s: %d elements off, worst %g (ref scale %g)" % (
        name, int(bad.sum()), float(np.abs(got - ref).max()), scale)

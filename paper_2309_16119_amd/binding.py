"""ctypes binding of libmodulora.so -- argument marshalling only.

Every function here has the name of the C entry point it calls
(include/modulora.h) and does nothing but turn torch tensors into device
pointers, allocate outputs and the workspace with torch, pass torch's current
stream, and raise on a non-zero status.  All arithmetic of the layer runs in
the HIP kernels; there is no CPU or PyTorch fallback: if the shared library
cannot be loaded the import of this module fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
# MODULORA_LIB may point at another build of the same library (e.g. one compiled with other flags)
LIB_PATH = os.environ.get("MODULORA_LIB") or os.path.join(_PKG, "libmodulora.so")

OK = 0
STATUS_NAMES = {
    0: "MODULORA_OK", 1: "MODULORA_ERR_NULL", 2: "MODULORA_ERR_SHAPE", 3: "MODULORA_ERR_BITS",
    4: "MODULORA_ERR_GROUP", 5: "MODULORA_ERR_ALIGN", 6: "MODULORA_ERR_RANK",
    7: "MODULORA_ERR_WORKSPACE", 8: "MODULORA_ERR_HIP", 9: "MODULORA_ERR_HYPER",
}


class modulora_qweight(ctypes.Structure):
    _fields_ = [
        ("d_in", ctypes.c_int32), ("d_out", ctypes.c_int32),
        ("bits", ctypes.c_int32), ("group_size", ctypes.c_int32),
        ("qweight", ctypes.c_void_p), ("scales", ctypes.c_void_p), ("zeros", ctypes.c_void_p),
    ]


class modulora_qweight_f16(ctypes.Structure):
    _fields_ = [
        ("d_in", ctypes.c_int32), ("d_out", ctypes.c_int32),
        ("bits", ctypes.c_int32), ("group_size", ctypes.c_int32),
        ("qweight", ctypes.c_void_p), ("scales", ctypes.c_void_p), ("zeros", ctypes.c_void_p), ("bias", ctypes.c_void_p),
    ]


class modulora_kernel_time(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 64), ("launches", ctypes.c_int32), ("total_ms", ctypes.c_float)]


class ModuloraError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (%s)" % (where, STATUS_NAMES.get(status, status), modulora_status_string(status)))


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        # nothing built yet: build in-tree (needs hipcc); never fall back to other code
        from .build import build_library
        build_library()
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
    qp = ctypes.POINTER(modulora_qweight)
    lib.modulora_status_string.restype = ctypes.c_char_p
    lib.modulora_status_string.argtypes = [ctypes.c_int]
    lib.modulora_workspace_bytes.restype = sz
    lib.modulora_workspace_bytes.argtypes = [qp, i32, i32]
    lib.modulora_dequant.restype = ctypes.c_int
    lib.modulora_dequant.argtypes = [qp, vp, vp]
    lib.modulora_fwd.restype = ctypes.c_int
    lib.modulora_fwd.argtypes = [qp, vp, i32, vp, vp, i32, f32, vp, vp, vp, sz, vp]
    lib.modulora_fwd_static.restype = ctypes.c_int
    lib.modulora_fwd_static.argtypes = [qp, vp, i32, vp, vp, i32, f32, vp, vp, vp]
    lib.modulora_bwd_input.restype = ctypes.c_int
    lib.modulora_bwd_input.argtypes = [qp, vp, i32, vp, vp, i32, f32, vp, vp, vp, sz, vp]
    lib.modulora_bwd_lora.restype = ctypes.c_int
    lib.modulora_bwd_lora.argtypes = [i32, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, sz, vp]
    qh = ctypes.POINTER(modulora_qweight_f16)
    lib.modulora_f16_workspace_bytes.restype = sz
    lib.modulora_f16_workspace_bytes.argtypes = [qh, i32, i32]
    lib.modulora_f16_dequant.restype = ctypes.c_int
    lib.modulora_f16_dequant.argtypes = [qh, vp, vp]
    lib.modulora_f16_fwd.restype = ctypes.c_int
    lib.modulora_f16_fwd.argtypes = [qh, vp, i32, vp, vp, i32, f32, vp, vp, vp, sz, vp]
    lib.modulora_f16_bwd_input.restype = ctypes.c_int
    lib.modulora_f16_bwd_input.argtypes = [qh, vp, i32, vp, vp, i32, f32, vp, vp, vp, sz, vp]
    lib.modulora_f16_bwd_lora.restype = ctypes.c_int
    lib.modulora_f16_bwd_lora.argtypes = [i32, i32, i32, i32, f32, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, sz, vp]
    lib.modulora_quantize_rtn.restype = ctypes.c_int
    lib.modulora_quantize_rtn.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, vp]
    lib.modulora_adamw.restype = ctypes.c_int
    lib.modulora_adamw.argtypes = [vp, vp, vp, vp, sz, f32, f32, f32, f32, f32, i32, vp]
    lib.modulora_bench_read.restype = ctypes.c_int
    lib.modulora_bench_read.argtypes = [vp, sz, vp, vp]
    lib.modulora_profile_begin.restype = ctypes.c_int
    lib.modulora_profile_begin.argtypes = []
    lib.modulora_profile_end.restype = ctypes.c_int
    lib.modulora_profile_end.argtypes = [ctypes.POINTER(modulora_kernel_time), i32, ctypes.POINTER(i32)]
    return lib


lib = _load()


# ----------------------------------------------------------------------------- helpers
def _ptr(t: Optional[torch.Tensor]) -> ctypes.c_void_p:
    if t is None:
        return ctypes.c_void_p(0)
    assert t.is_contiguous(), "tensors must be contiguous"
    return ctypes.c_void_p(t.data_ptr())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


class QWeight:
    """The frozen quantized weight on the device: packed codes, scales and zeros.

    qweight int32 [d_in*bits/32][d_out] (the uint32 words, reinterpreted),
    scales float16 [d_in/g][d_out], zeros uint8 [d_in/g][d_out].
    """

    def __init__(self, qweight: torch.Tensor, scales: torch.Tensor, zeros: torch.Tensor,
                 d_in: int, d_out: int, bits: int, group_size: int):
        assert qweight.dtype == torch.int32 and scales.dtype == torch.float16 and zeros.dtype == torch.uint8
        self.qweight, self.scales, self.zeros = qweight, scales, zeros
        self.d_in, self.d_out, self.bits, self.group_size = d_in, d_out, bits, group_size

    @classmethod
    def from_numpy(cls, qweight_u32, scales_u16, zeros_u8, d_in, d_out, bits, group_size, device="cuda"):
        """Copy host arrays (uint32 words, binary16 bit patterns, uint8) to the device."""
        import numpy as np
        q = torch.from_numpy(np.ascontiguousarray(qweight_u32).view(np.int32)).to(device)
        s = torch.from_numpy(np.ascontiguousarray(scales_u16).view(np.float16)).to(device)
        z = torch.from_numpy(np.ascontiguousarray(zeros_u8)).to(device)
        return cls(q, s, z, d_in, d_out, bits, group_size)

    def c_struct(self) -> modulora_qweight:
        return modulora_qweight(self.d_in, self.d_out, self.bits, self.group_size,
                                self.qweight.data_ptr(), self.scales.data_ptr(), self.zeros.data_ptr())

    @property
    def device(self):
        return self.qweight.device


_workspaces: dict = {}


def _workspace(device, nbytes: int) -> Optional[torch.Tensor]:
    """Scratch memory for one call: a cached tensor per (device, current stream), so that calls
    sharing a buffer are ordered on one stream as the library requires.  A request larger than
    the cached buffer gets a new one; the old ones stay alive until the process ends, because a
    HIP graph captured earlier may still hold their addresses.  torch memory is 256-byte aligned.
    Callers that capture graphs can size the buffer first with reserve_workspace()."""
    if nbytes == 0:
        return None
    key = (torch.device(device), torch.cuda.current_stream(device).cuda_stream)
    held = _workspaces.setdefault(key, [])
    if not held or held[-1].numel() < nbytes:
        held.append(torch.empty(nbytes, dtype=torch.uint8, device=device))
    return held[-1]


def reserve_workspace(device, nbytes: int) -> None:
    """Make the cached scratch buffer of (device, current stream) at least `nbytes` large now, e.g.
    before a HIP graph capture (allocating during capture would tie the buffer to the graph's pool)."""
    _workspace(device, int(nbytes))


def _check(status: int, where: str):
    if status != OK:
        raise ModuloraError(status, where)


# ----------------------------------------------------------------------------- entry points
def modulora_status_string(status: int) -> str:
    return lib.modulora_status_string(int(status)).decode()


def modulora_workspace_bytes(w: QWeight, M: int, r: int) -> int:
    st = w.c_struct()
    return int(lib.modulora_workspace_bytes(ctypes.byref(st), M, r))


def modulora_dequant(w: QWeight, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """What [d_out][d_in] bfloat16 (test-only weight materialization)."""
    if out is None:
        out = torch.empty((w.d_out, w.d_in), dtype=torch.bfloat16, device=w.device)
    st = w.c_struct()
    _check(lib.modulora_dequant(ctypes.byref(st), _ptr(out), _stream()), "modulora_dequant")
    return out


def modulora_fwd(w: QWeight, X: torch.Tensor, A: Optional[torch.Tensor], B: Optional[torch.Tensor],
                 lora_scale: float, Y: Optional[torch.Tensor] = None, XA: Optional[torch.Tensor] = None,
                 want_XA: bool = True):
    """Y = X What^T + lora_scale (X A) B.  Returns (Y bf16 [M][d_out], XA fp32 [M][r] or None)."""
    assert X.dtype == torch.bfloat16 and X.dim() == 2 and X.shape[1] == w.d_in
    M = X.shape[0]
    r = 0 if A is None else A.shape[1]
    if r:
        assert A.dtype == torch.float32 and B.dtype == torch.float32
        assert tuple(A.shape) == (w.d_in, r) and tuple(B.shape) == (r, w.d_out)
    if Y is None:
        Y = torch.empty((M, w.d_out), dtype=torch.bfloat16, device=X.device)
    if XA is None and want_XA and r:
        XA = torch.empty((M, r), dtype=torch.float32, device=X.device)
    nbytes = modulora_workspace_bytes(w, M, r)
    ws = _workspace(X.device, nbytes)
    st = w.c_struct()
    _check(lib.modulora_fwd(ctypes.byref(st), _ptr(X), M, _ptr(A), _ptr(B), r, float(lora_scale),
                            _ptr(Y), _ptr(XA), _ptr(ws), nbytes, _stream()), "modulora_fwd")
    return Y, XA


STATIC_SCRATCH_BYTES = 16 << 20


def modulora_fwd_static(w: QWeight, X: torch.Tensor, A: Optional[torch.Tensor], B: Optional[torch.Tensor],
                        lora_scale: float, Y: torch.Tensor, XA: Optional[torch.Tensor] = None):
    """modulora_fwd on the library's own static scratch: the caller passes every buffer (Y, and XA
    if wanted), this wrapper allocates nothing either."""
    assert X.dtype == torch.bfloat16 and X.dim() == 2 and X.shape[1] == w.d_in
    M = X.shape[0]
    r = 0 if A is None else A.shape[1]
    assert Y.dtype == torch.bfloat16 and tuple(Y.shape) == (M, w.d_out)
    st = w.c_struct()
    _check(lib.modulora_fwd_static(ctypes.byref(st), _ptr(X), M, _ptr(A), _ptr(B), r, float(lora_scale),
                                   _ptr(Y), _ptr(XA), _stream()), "modulora_fwd_static")
    return Y, XA


def modulora_bwd_input(w: QWeight, dY: torch.Tensor, A: Optional[torch.Tensor], B: Optional[torch.Tensor],
                       lora_scale: float, dX: Optional[torch.Tensor] = None,
                       dYBt: Optional[torch.Tensor] = None, want_dYBt: bool = True):
    """dX = dY What + lora_scale (dY B^T) A^T.  Returns (dX bf16 [M][d_in], dYBt fp32 [M][r] or None)."""
    assert dY.dtype == torch.bfloat16 and dY.dim() == 2 and dY.shape[1] == w.d_out
    M = dY.shape[0]
    r = 0 if A is None else A.shape[1]
    if r:
        assert A.dtype == torch.float32 and B.dtype == torch.float32
        assert tuple(A.shape) == (w.d_in, r) and tuple(B.shape) == (r, w.d_out)
    if dX is None:
        dX = torch.empty((M, w.d_in), dtype=torch.bfloat16, device=dY.device)
    if dYBt is None and want_dYBt and r:
        dYBt = torch.empty((M, r), dtype=torch.float32, device=dY.device)
    nbytes = modulora_workspace_bytes(w, M, r)
    ws = _workspace(dY.device, nbytes)
    st = w.c_struct()
    _check(lib.modulora_bwd_input(ctypes.byref(st), _ptr(dY), M, _ptr(A), _ptr(B), r, float(lora_scale),
                                  _ptr(dX), _ptr(dYBt), _ptr(ws), nbytes, _stream()), "modulora_bwd_input")
    return dX, dYBt


def modulora_bwd_lora(X: torch.Tensor, dY: torch.Tensor, A: torch.Tensor, B: torch.Tensor, lora_scale: float,
                      XA: Optional[torch.Tensor] = None, dYBt: Optional[torch.Tensor] = None,
                      dA: Optional[torch.Tensor] = None, dB: Optional[torch.Tensor] = None,
                      accumulate: bool = False):
    """dA = s X^T (dY B^T), dB = s (X A)^T dY.  Returns (dA fp32 [d_in][r], dB fp32 [r][d_out])."""
    M, d_in = X.shape
    d_out = dY.shape[1]
    r = A.shape[1]
    assert X.dtype == torch.bfloat16 and dY.dtype == torch.bfloat16 and dY.shape[0] == M
    assert tuple(A.shape) == (d_in, r) and tuple(B.shape) == (r, d_out)
    if dA is None:
        assert not accumulate
        dA = torch.empty((d_in, r), dtype=torch.float32, device=X.device)
    if dB is None:
        assert not accumulate
        dB = torch.empty((r, d_out), dtype=torch.float32, device=X.device)
    shape = modulora_qweight(d_in, d_out, 4, 32, 0, 0, 0)
    nbytes = int(lib.modulora_workspace_bytes(ctypes.byref(shape), M, r))
    ws = _workspace(X.device, nbytes)
    _check(lib.modulora_bwd_lora(d_in, d_out, M, r, float(lora_scale), _ptr(X), _ptr(dY), _ptr(A), _ptr(B),
                                 _ptr(XA), _ptr(dYBt), _ptr(dA), _ptr(dB), 1 if accumulate else 0,
                                 _ptr(ws), nbytes, _stream()), "modulora_bwd_lora")
    return dA, dB


# ----------------------------------------------------------------------------- paper-literal variant
class QWeightF16:
    """The frozen weight in the paper's own convention (eq. (2)): packed codes, binary16 scales,
    binary16 zero points that are added, optional binary16 bias [d_out]."""

    def __init__(self, qweight: torch.Tensor, scales: torch.Tensor, zeros: torch.Tensor, bias: Optional[torch.Tensor],
                 d_in: int, d_out: int, bits: int, group_size: int):
        assert qweight.dtype == torch.int32 and scales.dtype == torch.float16 and zeros.dtype == torch.float16
        assert bias is None or bias.dtype == torch.float16
        self.qweight, self.scales, self.zeros, self.bias = qweight, scales, zeros, bias
        self.d_in, self.d_out, self.bits, self.group_size = d_in, d_out, bits, group_size

    @classmethod
    def from_numpy(cls, qweight_u32, scales_u16, zeros_u16, bias_u16, d_in, d_out, bits, group_size, device="cuda"):
        import numpy as np
        q = torch.from_numpy(np.ascontiguousarray(qweight_u32).view(np.int32)).to(device)
        s = torch.from_numpy(np.ascontiguousarray(scales_u16).view(np.float16)).to(device)
        z = torch.from_numpy(np.ascontiguousarray(zeros_u16).view(np.float16)).to(device)
        b = None if bias_u16 is None else torch.from_numpy(np.ascontiguousarray(bias_u16).view(np.float16)).to(device)
        return cls(q, s, z, b, d_in, d_out, bits, group_size)

    def c_struct(self) -> modulora_qweight_f16:
        return modulora_qweight_f16(self.d_in, self.d_out, self.bits, self.group_size, self.qweight.data_ptr(),
                                    self.scales.data_ptr(), self.zeros.data_ptr(),
                                    0 if self.bias is None else self.bias.data_ptr())

    @property
    def device(self):
        return self.qweight.device


def modulora_f16_workspace_bytes(w: QWeightF16, M: int, r: int) -> int:
    st = w.c_struct()
    return int(lib.modulora_f16_workspace_bytes(ctypes.byref(st), M, r))


def modulora_f16_dequant(w: QWeightF16, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """What [d_out][d_in] float16 (test-only weight materialization)."""
    if out is None:
        out = torch.empty((w.d_out, w.d_in), dtype=torch.float16, device=w.device)
    st = w.c_struct()
    _check(lib.modulora_f16_dequant(ctypes.byref(st), _ptr(out), _stream()), "modulora_f16_dequant")
    return out


def _f16_call(fn, name, w: QWeightF16, act: torch.Tensor, width_in: int, width_out: int, A, B, lora_scale, out, P, want_P):
    assert act.dtype == torch.float16 and act.dim() == 2 and act.shape[1] == width_in
    M = act.shape[0]
    r = 0 if A is None else A.shape[1]
    if r:
        assert A.dtype == torch.float32 and B.dtype == torch.float32
        assert tuple(A.shape) == (w.d_in, r) and tuple(B.shape) == (r, w.d_out)
    if out is None:
        out = torch.empty((M, width_out), dtype=torch.float16, device=act.device)
    if P is None and want_P and r:
        P = torch.empty((M, r), dtype=torch.float32, device=act.device)
    nbytes = modulora_f16_workspace_bytes(w, M, r)
    ws = _workspace(act.device, nbytes)
    st = w.c_struct()
    _check(fn(ctypes.byref(st), _ptr(act), M, _ptr(A), _ptr(B), r, float(lora_scale), _ptr(out), _ptr(P), _ptr(ws), nbytes,
              _stream()), name)
    return out, P


def modulora_f16_fwd(w: QWeightF16, X, A, B, lora_scale: float, Y=None, XA=None, want_XA: bool = True):
    """Y = X What^T + bias + lora_scale (X A) B.  Returns (Y fp16 [M][d_out], XA fp32 [M][r] or None)."""
    return _f16_call(lib.modulora_f16_fwd, "modulora_f16_fwd", w, X, w.d_in, w.d_out, A, B, lora_scale, Y, XA, want_XA)


def modulora_f16_bwd_input(w: QWeightF16, dY, A, B, lora_scale: float, dX=None, dYBt=None, want_dYBt: bool = True):
    """dX = dY What + lora_scale (dY B^T) A^T.  Returns (dX fp16 [M][d_in], dYBt fp32 [M][r] or None)."""
    return _f16_call(lib.modulora_f16_bwd_input, "modulora_f16_bwd_input", w, dY, w.d_out, w.d_in, A, B, lora_scale, dX, dYBt,
                     want_dYBt)


def modulora_f16_bwd_lora(X: torch.Tensor, dY: torch.Tensor, A: torch.Tensor, B: torch.Tensor, lora_scale: float,
                          XA: Optional[torch.Tensor] = None, dYBt: Optional[torch.Tensor] = None,
                          dA: Optional[torch.Tensor] = None, dB: Optional[torch.Tensor] = None, accumulate: bool = False):
    """dA = s X^T (dY B^T), dB = s (X A)^T dY from float16 X, dY."""
    M, d_in = X.shape
    d_out = dY.shape[1]
    r = A.shape[1]
    assert X.dtype == torch.float16 and dY.dtype == torch.float16 and dY.shape[0] == M
    assert tuple(A.shape) == (d_in, r) and tuple(B.shape) == (r, d_out)
    if dA is None:
        assert not accumulate
        dA = torch.empty((d_in, r), dtype=torch.float32, device=X.device)
    if dB is None:
        assert not accumulate
        dB = torch.empty((r, d_out), dtype=torch.float32, device=X.device)
    shape = modulora_qweight_f16(d_in, d_out, 4, 32, 0, 0, 0, 0)
    nbytes = int(lib.modulora_f16_workspace_bytes(ctypes.byref(shape), M, r))
    ws = _workspace(X.device, nbytes)
    _check(lib.modulora_f16_bwd_lora(d_in, d_out, M, r, float(lora_scale), _ptr(X), _ptr(dY), _ptr(A), _ptr(B),
                                     _ptr(XA), _ptr(dYBt), _ptr(dA), _ptr(dB), 1 if accumulate else 0,
                                     _ptr(ws), nbytes, _stream()), "modulora_f16_bwd_lora")
    return dA, dB


def modulora_quantize_rtn(W: torch.Tensor, bits: int, group_size: int) -> "QWeight":
    """Round-to-nearest group quantization of W float32 [d_out][d_in] into a QWeight."""
    assert W.dtype == torch.float32 and W.dim() == 2
    d_out, d_in = W.shape
    W = W.contiguous()
    # an invalid shape: let the library name the error (it validates on the host before touching
    # any pointer), instead of sizing allocations by it
    probe = modulora_qweight(d_in, d_out, bits, group_size, 0, 0, 0)
    if lib.modulora_workspace_bytes(ctypes.byref(probe), 1, 1) == 0:
        _check(lib.modulora_quantize_rtn(_ptr(W), d_in, d_out, bits, group_size, 0, 0, 0, _stream()),
               "modulora_quantize_rtn")
        raise AssertionError("unreachable: invalid shape accepted")
    G = d_in // group_size
    q = torch.empty((d_in * bits // 32, d_out), dtype=torch.int32, device=W.device)
    sc = torch.empty((G, d_out), dtype=torch.float16, device=W.device)
    z = torch.empty((G, d_out), dtype=torch.uint8, device=W.device)
    _check(lib.modulora_quantize_rtn(_ptr(W), d_in, d_out, bits, group_size, _ptr(q), _ptr(sc), _ptr(z), _stream()),
           "modulora_quantize_rtn")
    return QWeight(q, sc, z, d_in, d_out, bits, group_size)


def modulora_adamw(param: torch.Tensor, grad: torch.Tensor, exp_avg: torch.Tensor, exp_avg_sq: torch.Tensor,
                   lr: float, beta1: float, beta2: float, eps: float, weight_decay: float, step: int) -> None:
    """One AdamW step, in place, on flat float32 buffers of equal length."""
    n = param.numel()
    for t in (param, grad, exp_avg, exp_avg_sq):
        assert t.dtype == torch.float32 and t.numel() == n and t.device == param.device
    _check(lib.modulora_adamw(_ptr(param), _ptr(grad), _ptr(exp_avg), _ptr(exp_avg_sq), n, float(lr), float(beta1),
                              float(beta2), float(eps), float(weight_decay), int(step), _stream()), "modulora_adamw")


BENCH_READ_SINK_WORDS = 2048


def modulora_bench_read(buf: torch.Tensor, sink: Optional[torch.Tensor] = None) -> torch.Tensor:
    """One plain streaming read of `buf` by the library's hand-written read kernel (benchmark hook)."""
    if sink is None:
        sink = torch.empty(BENCH_READ_SINK_WORDS, dtype=torch.int32, device=buf.device)
    assert sink.numel() >= BENCH_READ_SINK_WORDS and sink.dtype == torch.int32
    _check(lib.modulora_bench_read(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink), _stream()),
           "modulora_bench_read")
    return sink


def modulora_profile_begin() -> None:
    _check(lib.modulora_profile_begin(), "modulora_profile_begin")


def modulora_profile_end(capacity: int = 64) -> dict:
    """Returns {kernel name: (launches, total_ms)} for the kernels launched since profile_begin."""
    arr = (modulora_kernel_time * capacity)()
    n = ctypes.c_int32(0)
    _check(lib.modulora_profile_end(arr, capacity, ctypes.byref(n)), "modulora_profile_end")
    return {arr[i].name.decode(): (int(arr[i].launches), float(arr[i].total_ms)) for i in range(n.value)}

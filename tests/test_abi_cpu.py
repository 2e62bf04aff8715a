"""CPU-only checks of the C ABI: the library loads, exports every symbol the header
declares, and rejects bad arguments on the host before any HIP call is made.
No kernel is launched here."""
import ctypes
import os
import re

import pytest

from paper_2309_16119_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "modulora.h")

FAKE = 0x10000          # a non-NULL, 256-byte aligned address that is never dereferenced
ODD = FAKE + 4          # misaligned


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(modulora_[a-z_]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    names = declared_functions()
    for required in ("modulora_fwd", "modulora_bwd_input", "modulora_bwd_lora", "modulora_dequant",
                     "modulora_workspace_bytes", "modulora_status_string"):
        assert required in names


@pytest.mark.parametrize("name", declared_functions())
def test_library_exports_symbol(name):
    assert hasattr(b.lib, name), name


def qw(d_in=4096, d_out=4096, bits=3, group=128, q=FAKE, s=FAKE, z=FAKE):
    return b.modulora_qweight(d_in, d_out, bits, group, q, s, z)


def fwd(w, X=FAKE, M=16, A=FAKE, B=FAKE, r=8, Y=FAKE, XA=0, ws=FAKE, wsb=1 << 30):
    return b.lib.modulora_fwd(ctypes.byref(w), X, M, A, B, r, 2.0, Y, XA, ws, wsb, None)


def bwd(w, dY=FAKE, M=16, A=FAKE, B=FAKE, r=8, dX=FAKE, T=0, ws=FAKE, wsb=1 << 30):
    return b.lib.modulora_bwd_input(ctypes.byref(w), dY, M, A, B, r, 2.0, dX, T, ws, wsb, None)


def test_status_strings():
    for code in range(0, 10):
        assert b.modulora_status_string(code)
    assert "unknown" in b.modulora_status_string(99)


@pytest.mark.parametrize("call", [fwd, bwd])
def test_rejections_fwd_and_bwd_input(call):
    assert call(qw(bits=5)) == 3
    assert call(qw(bits=1)) == 3
    assert call(qw(group=100)) == 4           # not a multiple of 32
    assert call(qw(group=96)) == 4            # multiple of 32 that does not divide d_in
    assert call(qw(group=0)) == 4
    assert call(qw(d_in=4100)) == 2           # not a multiple of 32
    assert call(qw(d_out=4100)) == 2          # not a multiple of 8
    assert call(qw(d_in=0)) == 2
    assert call(qw(q=0)) == 1
    assert call(qw(s=0)) == 1
    assert call(qw(z=ODD)) == 5
    assert call(qw(), M=0) == 2
    assert call(qw(), M=-3) == 2
    assert call(qw(), r=65) == 6
    assert call(qw(), r=-1) == 6
    assert call(qw(), A=0) == 6               # r > 0 needs A and B
    assert call(qw(), B=ODD) == 5
    assert call(qw(), ws=0) == 7
    assert call(qw(), ws=FAKE + 16) == 7      # workspace must be 256-byte aligned
    assert call(qw(), wsb=16) == 7
    if call is fwd:
        assert call(qw(), X=0) == 1 and call(qw(), Y=0) == 1 and call(qw(), X=ODD) == 5
    else:
        assert call(qw(), dY=0) == 1 and call(qw(), dX=0) == 1 and call(qw(), dX=ODD) == 5


def test_null_layer_pointer():
    assert b.lib.modulora_fwd(None, FAKE, 1, None, None, 0, 1.0, FAKE, None, None, 0, None) == 1
    assert b.lib.modulora_dequant(None, FAKE, None) == 1
    assert b.lib.modulora_dequant(ctypes.byref(qw()), None, None) == 1
    assert b.lib.modulora_dequant(ctypes.byref(qw(bits=7)), FAKE, None) == 3


def test_rejections_bwd_lora():
    def call(d_in=4096, d_out=4096, M=16, r=8, X=FAKE, dY=FAKE, A=FAKE, B=FAKE, dA=FAKE, dB=FAKE,
             ws=FAKE, wsb=1 << 30):
        return b.lib.modulora_bwd_lora(d_in, d_out, M, r, 2.0, X, dY, A, B, None, None, dA, dB, 0, ws, wsb, None)
    assert call(d_in=33) == 2
    assert call(d_out=12) == 2
    assert call(M=0) == 2
    assert call(r=0) == 6                      # the adapter gradients need r >= 1
    assert call(r=70) == 6
    assert call(X=0) == 1 and call(dA=0) == 1 and call(dB=0) == 1
    assert call(dY=ODD) == 5
    assert call(A=0) == 6
    assert call(ws=0) == 7
    assert call(wsb=100) == 7


def test_rejections_quantize_rtn():
    def call(W=FAKE, d_in=4096, d_out=4096, bits=3, group=128, q=FAKE, s=FAKE, z=FAKE):
        return b.lib.modulora_quantize_rtn(W, d_in, d_out, bits, group, q, s, z, None)
    assert call(W=0) == 1 and call(q=0) == 1 and call(s=0) == 1 and call(z=0) == 1
    assert call(W=ODD) == 5 and call(q=ODD) == 5
    assert call(bits=5) == 3 and call(group=48) == 4 and call(group=96) == 4
    assert call(d_in=100) == 2 and call(d_out=12) == 2


def test_rejections_adamw():
    def call(p=FAKE, g=FAKE, m=FAKE, v=FAKE, n=1024, lr=1e-3, b1=0.9, b2=0.999, eps=1e-8, wd=0.01, step=1):
        return b.lib.modulora_adamw(p, g, m, v, n, lr, b1, b2, eps, wd, step, None)
    assert call(p=0) == 1 and call(g=0) == 1 and call(m=0) == 1 and call(v=0) == 1
    assert call(p=ODD) == 5 and call(v=ODD) == 5
    assert call(n=0) == 2
    assert call(step=0) == 9 and call(lr=-1.0) == 9 and call(b1=1.0) == 9 and call(b2=-0.1) == 9
    assert call(eps=0.0) == 9 and call(wd=-1.0) == 9 and call(lr=float("nan")) == 9 and call(lr=float("inf")) == 9


def test_workspace_bytes():
    w = qw()
    # r = 0 at M = 32: 16 tiles of 128 x 256, each cut into 8 slices of the contraction (more than
    # the streaming kernels' scratch for two passes of 16 rows)
    assert b.lib.modulora_workspace_bytes(ctypes.byref(w), 32, 0) == 16 * 8 * 128 * 256 * 4
    # r = 0 at M = 512: 2 x 16 tiles of 256 x 256, each cut into 8 slices of the contraction
    # that leave fp32 partial tiles
    assert b.lib.modulora_workspace_bytes(ctypes.byref(w), 512, 0) == 32 * 8 * 256 * 256 * 4
    n8 = b.lib.modulora_workspace_bytes(ctypes.byref(w), 512, 8)
    n16 = b.lib.modulora_workspace_bytes(ctypes.byref(w), 512, 16)
    assert 0 < n8 < n16 and n8 % 256 == 0
    assert b.lib.modulora_workspace_bytes(ctypes.byref(qw(bits=9)), 512, 8) == 0
    assert b.lib.modulora_workspace_bytes(ctypes.byref(w), 0, 8) == 0
    assert b.lib.modulora_workspace_bytes(None, 1, 1) == 0


def test_profile_api_without_launches():
    b.modulora_profile_begin()
    assert b.modulora_profile_end() == {}


# ---- the paper-literal variant (binary16 zero points and activations, bias) ----------------
def qh(d_in=4096, d_out=4096, bits=3, group=128, q=FAKE, s=FAKE, z=FAKE, bias=0):
    return b.modulora_qweight_f16(d_in, d_out, bits, group, q, s, z, bias)


def f16_fwd(w, X=FAKE, M=16, A=FAKE, B=FAKE, r=8, Y=FAKE, XA=0, ws=FAKE, wsb=1 << 30):
    return b.lib.modulora_f16_fwd(ctypes.byref(w), X, M, A, B, r, 2.0, Y, XA, ws, wsb, None)


def f16_bwd(w, dY=FAKE, M=16, A=FAKE, B=FAKE, r=8, dX=FAKE, T=0, ws=FAKE, wsb=1 << 30):
    return b.lib.modulora_f16_bwd_input(ctypes.byref(w), dY, M, A, B, r, 2.0, dX, T, ws, wsb, None)


@pytest.mark.parametrize("call", [f16_fwd, f16_bwd])
def test_rejections_of_the_f16_calls(call):
    assert call(qh(bits=5)) == 3
    assert call(qh(group=100)) == 4
    assert call(qh(d_in=4100)) == 2
    assert call(qh(d_out=4100)) == 2
    assert call(qh(q=0)) == 1
    assert call(qh(z=ODD)) == 5
    assert call(qh(bias=ODD)) == 5
    assert call(qh(), M=0) == 2
    assert call(qh(), r=65) == 6
    assert call(qh(), A=0) == 6
    assert call(qh(), ws=0) == 7
    assert call(qh(), wsb=16) == 7
    assert call(qh(), ws=FAKE + 16) == 7
    # 4096 tokens without adapter are exactly 256 whole tiles and need no scratch (valid; no GPU here,
    # so the launch itself may fail); 16 or 20 tokens take the streaming kernels, whose slices meet
    # in the workspace
    assert call(qh(), M=4096, r=0, A=0, B=0, ws=0, wsb=0) in (0, 8)
    assert call(qh(), M=16, r=0, A=0, B=0, ws=0, wsb=0) == 7
    assert call(qh(), M=20, r=0, A=0, B=0, ws=0, wsb=0) == 7


def test_f16_workspace_query_and_dequant_rejections():
    w = qh()
    with_adapter = b.lib.modulora_f16_workspace_bytes(ctypes.byref(w), 512, 8)
    without = b.lib.modulora_f16_workspace_bytes(ctypes.byref(w), 512, 0)
    assert with_adapter > without >= 0            # r = 0 still needs the tile kernel's scratch for partial tiles
    assert with_adapter % 256 == 0 and without % 256 == 0
    assert b.lib.modulora_f16_workspace_bytes(ctypes.byref(qh(bits=7)), 512, 8) == 0
    assert b.lib.modulora_f16_dequant(ctypes.byref(w), 0, None) == 1
    assert b.lib.modulora_f16_dequant(ctypes.byref(w), ODD, None) == 5
    bl = b.lib.modulora_f16_bwd_lora
    assert bl(4096, 4096, 16, 0, 2.0, FAKE, FAKE, FAKE, FAKE, 0, 0, FAKE, FAKE, 0, FAKE, 1 << 30, None) == 6
    assert bl(4096, 4100, 16, 8, 2.0, FAKE, FAKE, FAKE, FAKE, 0, 0, FAKE, FAKE, 0, FAKE, 1 << 30, None) == 2
    assert bl(4096, 4096, 16, 8, 2.0, FAKE, 0, FAKE, FAKE, 0, 0, FAKE, FAKE, 0, FAKE, 1 << 30, None) == 1
    assert bl(4096, 4096, 16, 8, 2.0, FAKE, FAKE, FAKE, FAKE, 0, 0, FAKE, FAKE, 0, 0, 0, None) == 7


def test_bench_read_hook_rejections():
    f = b.lib.modulora_bench_read
    assert f(0, 1024, FAKE, None) == 1
    assert f(FAKE, 1024, 0, None) == 1
    assert f(ODD, 1024, FAKE, None) == 5
    assert f(FAKE, 0, FAKE, None) == 2
    assert f(FAKE, 1000, FAKE, None) == 2        # not a multiple of 16


def test_static_scratch_forward_rejections():
    """Host-side checks of modulora_fwd_static: the same argument errors as modulora_fwd, and a
    request beyond the library's static scratch is refused before anything touches the GPU."""
    def f(w, X=FAKE, M=16, A=FAKE, B=FAKE, r=8, Y=FAKE, XA=0):
        return b.lib.modulora_fwd_static(ctypes.byref(w), X, M, A, B, r, 2.0, Y, XA, None)
    assert f(qw(bits=5)) == 3
    assert f(qw(), X=0) == 1
    assert f(qw(), X=ODD) == 5
    assert f(qw(), r=65) == 6
    assert f(qw(), M=0) == 2
    # 30000 tokens at rank 64 need about 19 MB of adapter operands: more than the 16 MiB array
    assert f(qw(), M=30000, r=64) == 7
    assert b.STATIC_SCRATCH_BYTES == 16 << 20

"""The C-ABI library loads, exports every symbol the header declares, and rejects bad arguments on
the host before any launch (so these run without a GPU)."""
import ctypes as C
import os
import re

import pytest

import paper_2411_11038_amd as ef

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _ensure_built():
    if not os.path.exists(ef.lib_path()):
        from paper_2411_11038_amd import build
        build.build()


def test_library_exports_every_declared_symbol():
    _ensure_built()
    hdr = open(os.path.join(ROOT, "include", "efqat.h")).read()
    declared = sorted(set(re.findall(r"\b(efqat_[a-z0-9_]+)\s*\(", hdr)))
    assert declared, "no declarations found"
    L = C.CDLL(ef.lib_path())
    for name in declared:
        assert hasattr(L, name), f"{name} declared in efqat.h but not exported"
    assert sorted(ef.EXPORTS) == declared


def test_version_strerror_k_from_ratio():
    _ensure_built()
    L = ef.lib()
    assert L.efqat_version() == 200
    assert L.efqat_strerror(0) == b"ok"
    for code in range(-9, 0):
        assert L.efqat_strerror(code) not in (b"", b"unknown error code")
    assert L.efqat_strerror(-99) == b"unknown error code"
    assert ef.k_from_ratio(3072, 1, 20) == 153 and ef.k_from_ratio(768, 1, 20) == 38
    assert ef.k_from_ratio(11008, 1, 100) == 110 and ef.k_from_ratio(4096, 1, 50) == 81
    assert ef.k_from_ratio(256, 0, 1) == 0 and ef.k_from_ratio(256, 1, 1) == 256
    assert ef.k_from_ratio(256, 2, 1) == -1 and ef.k_from_ratio(-1, 1, 2) == -1 and ef.k_from_ratio(8, 1, 0) == -1


def test_argument_validation_needs_no_device():
    _ensure_built()
    L = ef.lib()
    fake = 0x1000          # non-NULL, 256-aligned; never dereferenced because validation fails first
    # fakequant
    assert L.efqat_fakequant_fwd(None, 0, 4, 4, 0, 8, 1, fake, fake, fake, fake, None, fake, 1 << 20, None) == -1
    assert L.efqat_fakequant_fwd(fake, 0, 0, 4, 0, 8, 1, fake, fake, fake, fake, None, fake, 1 << 20, None) == -2
    assert L.efqat_fakequant_fwd(fake, 0, 4, 4, 0, 9, 1, fake, fake, fake, fake, None, fake, 1 << 20, None) == -3
    assert L.efqat_fakequant_fwd(fake, 0, 4, 4, 0, 1, 1, fake, fake, fake, fake, None, fake, 1 << 20, None) == -3
    assert L.efqat_fakequant_fwd(fake, 7, 4, 4, 0, 8, 1, fake, fake, fake, fake, None, fake, 1 << 20, None) == -8
    assert L.efqat_fakequant_fwd(fake, 0, 4, 4, 5, 8, 1, fake, fake, fake, fake, None, fake, 1 << 20, None) == -5
    assert L.efqat_fakequant_fwd(fake, 0, 4, 4, 0, 8, 1, fake, fake, fake, fake, None, fake, 16, None) == -6
    assert L.efqat_fakequant_fwd(fake, 0, 4, 4, 0, 8, 1, fake, fake, fake, fake, None, fake + 8, 1 << 20, None) == -9
    assert L.efqat_fakequant_fwd(fake, 0, 4, 4, 0, 8, 1, fake, None, fake, fake, None, fake, 1 << 20, None) == -1
    # select
    assert L.efqat_channel_select(fake, 8, 4, 9, None, fake, fake, 1 << 20, None) == -4
    assert L.efqat_channel_select(fake, 8, 4, -1, None, fake, fake, 1 << 20, None) == -4
    assert L.efqat_channel_select(fake, 0, 4, 0, None, fake, fake, 1 << 20, None) == -2
    assert L.efqat_channel_select(None, 8, 4, 2, None, fake, fake, 1 << 20, None) == -1
    assert L.efqat_channel_select(fake, 8, 4, 2, None, None, fake, 1 << 20, None) == -1
    assert L.efqat_channel_select(fake, 8, 4, 2, None, fake, fake, 8, None) == -6
    assert L.efqat_network_select(fake, fake, 2, 8, 9, fake, fake, fake, 1 << 20, None) == -4
    assert L.efqat_network_select(fake, None, 2, 8, 3, fake, fake, fake, 1 << 20, None) == -1
    assert L.efqat_layer_select(fake, fake, 4, 5, None, fake, fake, fake, 1 << 20, None) == -4
    assert L.efqat_layer_select(fake, fake, 0, 0, None, fake, fake, fake, 1 << 20, None) == -2
    assert L.efqat_layer_select(fake, fake, 4, 2, None, None, fake, fake, 1 << 20, None) == -1
    assert L.efqat_layer_select(fake, fake, 4, 2, None, fake, fake, fake, 8, None) == -6
    # weight quantizer + select in one call
    def wqs(w=fake, c_out=8, block=4, bits=8, k=2, idx=fake, ws=fake, wsb=1 << 20, scale=fake):
        return L.efqat_weight_quant_select(w, c_out, block, bits, 1, scale, fake, fake, k, None, idx, ws, wsb, None)
    assert wqs(w=None) == -1 and wqs(idx=None) == -1 and wqs(scale=None) == -1
    assert wqs(c_out=0) == -2 and wqs(bits=9) == -3 and wqs(k=9) == -4 and wqs(wsb=8) == -6 and wqs(ws=fake + 8) == -9
    # select with the built-in scratch: argument errors come before anything touches a device
    assert L.efqat_channel_select_static(fake, 8, 4, 9, fake, None) == -4
    assert L.efqat_channel_select_static(fake, 0, 4, 0, fake, None) == -2
    assert L.efqat_channel_select_static(None, 8, 4, 2, fake, None) == -1
    assert L.efqat_channel_select_static(fake, 8, 4, 2, None, None) == -1
    assert L.efqat_channel_select_static(fake, 65537, 4, 2, fake, None) == -6      # beyond the built-in scratch
    assert L.efqat_channel_select_static(fake + 2, 8, 4, 2, fake, None) == -9
    # bias gradient
    assert L.efqat_bias_grad(None, 1, 0, 8, 8, fake, fake, 1 << 20, None) == -1
    assert L.efqat_bias_grad(fake, 1, 0, 0, 8, fake, fake, 1 << 20, None) == -2
    assert L.efqat_bias_grad(fake, 5, 0, 8, 8, fake, fake, 1 << 20, None) == -8
    assert L.efqat_bias_grad(fake, 1, 3, 8, 8, fake, fake, 1 << 20, None) == -5
    assert L.efqat_bias_grad(fake, 1, 0, 8, 8, fake, fake, 16, None) == -6
    assert L.efqat_bias_grad(fake, 1, 0, 8, 8, fake, fake + 4, 1 << 20, None) == -9

    # linear backward
    def lin(dy=fake, T=8, c_in=8, c_out=8, k=2, idx=fake, dw=fake, ws=fake, wsb=1 << 30, dyd=1, lay=0, sc=0):
        return L.efqat_linear_bwd(dy, dyd, lay, T, c_in, c_out, fake, fake, fake, 1, fake, fake, fake, fake, fake,
                                  fake, idx, k, fake, 1, dw, sc, fake, fake, fake, ws, wsb, None)
    assert lin(dy=None) == -1
    assert lin(T=0) == -2
    assert lin(k=9) == -4 and lin(k=-1) == -4
    assert lin(idx=None) == -1 and lin(dw=None) == -1
    assert lin(wsb=64) == -6
    assert lin(dyd=3) == -8
    assert lin(lay=2) == -5 and lin(sc=2) == -5
    assert lin(ws=fake + 16) == -9
    assert lin(dy=fake + 2) == -9

    # weight operand made beforehand
    need = L.efqat_linear_bwd_weight_operand_bytes(384, 192, 384, 1, 0)
    assert need == 192 * 384 * 2 + 256                 # bf16 [c_in][c_out] and a zero page
    assert L.efqat_linear_bwd_weight_operand_bytes(8192, 4096, 11008, 1, 0) == 0     # reads the int8 codes instead
    assert L.efqat_linear_bwd_weight_operand_bytes(0, 192, 384, 1, 0) == 0
    def wop(codes=fake, sw=fake, T=384, op=fake, opb=need, dyd=1, lay=0):
        return L.efqat_linear_bwd_weight_operand(codes, sw, T, 192, 384, dyd, lay, op, opb, None)
    assert wop(codes=None) == -1 and wop(sw=None) == -1 and wop(op=None) == -1
    assert wop(T=0) == -2
    assert wop(opb=need - 1) == -6
    assert wop(op=fake + 64) == -9
    assert wop(dyd=5) == -8 and wop(lay=3) == -5
    def lin_ex(wop_=None, step=None, dxk=0, ws=fake, wsb=1 << 30, dy=fake, w=fake, dw=fake, c_in=8, xc=fake, wc=fake,
               lay=0, k=2):
        return L.efqat_linear_bwd_ex(dy, 1, lay, 8, c_in, 8, xc, fake, fake, 1, fake, fake, wc, fake, w, fake, fake, k,
                                     fake, 1, dw, 0, fake, fake, fake, wop_, step, dxk, ws, wsb, None, None)
    assert lin_ex(dy=None) == -1
    assert lin_ex(wop_=fake + 64) == -9
    assert lin_ex(wsb=64) == -6 and lin_ex(wop_=fake, wsb=64) == -6
    assert lin_ex(dxk=4) == -5 and lin_ex(dxk=-1) == -5
    assert lin_ex(wop_=fake, dxk=2) == -5              # the prepared operand belongs to the default kernel choice
    # operands that the chosen kernels copy 16 bytes at a time: found misaligned before anything is launched
    assert lin_ex(c_in=16, xc=fake + 8) == -9          # token-major dW product reads the codes as they lie
    assert lin_ex(c_in=16, dxk=2, wc=fake + 8) == -9   # dX product on the int8 weight codes
    assert lin_ex(c_in=16, lay=1, xc=fake + 8) == -9 and lin_ex(c_in=16, lay=1, wc=fake + 8, k=0) == -9
    assert L.efqat_linear_bwd_workspace_bytes_ex(8, 16, 8, 2, 1, 0, 7) == 0
    assert (L.efqat_linear_bwd_workspace_bytes_ex(1024, 512, 640, 64, 1, 0, 2)
            != L.efqat_linear_bwd_workspace_bytes_ex(1024, 512, 640, 64, 1, 0, 1))   # no bf16 W_q^T copy with INT8

    # fused optimizer step
    from paper_2411_11038_amd.binding import OptStep
    def st(momentum=0.0, mom_w=None, b1=0.9, b2=0.999, eps=1e-8, m=fake, v=fake, t=fake):
        return C.byref(OptStep(0.1, momentum, 0.0, mom_w, 0.01, b1, b2, eps, m, v, t))
    assert lin_ex(step=st(momentum=0.9)) == -1         # momentum without a buffer
    assert lin_ex(step=st(m=None)) == -1 and lin_ex(step=st(v=None)) == -1 and lin_ex(step=st(t=None)) == -1
    assert lin_ex(step=st(), w=None) == -1
    assert lin_ex(step=st(b1=1.0)) == -5 and lin_ex(step=st(b2=-0.1)) == -5 and lin_ex(step=st(eps=-1.0)) == -5
    assert lin_ex(step=st(t=fake + 2)) == -9
    assert lin_ex(step=st(), dw=None, wsb=64) == -6    # gradients are optional with the step: valid up to the workspace check
    assert lin_ex(dw=None) == -1                       # ... and required without it

    # conv backward
    def conv(N=1, H=4, W=4, c_in=8, c_out=8, KH=3, KW=3, stride=1, pad=1, k=2, wsb=1 << 30):
        return L.efqat_conv_bwd(fake, 1, 0, N, H, W, c_in, c_out, KH, KW, stride, pad, fake, fake, fake, 1, fake,
                                fake, fake, fake, fake, fake, fake, k, fake, 1, fake, 0, fake, fake, fake, fake,
                                wsb, None)
    assert conv(stride=0) == -2 and conv(pad=-1) == -2 and conv(H=1, pad=0) == -2
    assert conv(k=9) == -4
    assert conv(wsb=64) == -6
    def conv_ex(step=None, dxk=0, wsb=1 << 30):
        return L.efqat_conv_bwd_ex(fake, 1, 0, 1, 4, 4, 8, 8, 3, 3, 1, 1, fake, fake, fake, 1, fake, fake, fake, fake,
                                   fake, fake, fake, 2, fake, 1, fake, 0, fake, fake, fake, step, dxk, fake, wsb, None, None)
    assert conv_ex(dxk=9) == -5 and conv_ex(wsb=64) == -6 and conv_ex(step=st(m=None)) == -1


def test_workspace_queries_are_host_only_and_monotone():
    _ensure_built()
    L = ef.lib()
    a = L.efqat_linear_bwd_workspace_bytes(12288, 768, 3072, 0, 1, 0)
    b = L.efqat_linear_bwd_workspace_bytes(12288, 768, 3072, 153, 1, 0)
    c = L.efqat_linear_bwd_workspace_bytes(12288, 768, 3072, 3072, 1, 0)
    assert 0 < a < b and a < c                       # not monotone in k: k == C_out needs no gathered copy
    assert L.efqat_linear_bwd_workspace_bytes(0, 768, 3072, 0, 1, 0) == 0
    assert L.efqat_conv_bwd_workspace_bytes(64, 14, 14, 256, 256, 3, 3, 1, 1, 64, 1, 0) > 0
    assert L.efqat_channel_select_workspace_bytes(11008) >= 11008 * 8
    assert L.efqat_fakequant_fwd_workspace_bytes(12288, 768, 0) >= 8192
    assert L.efqat_bias_grad_workspace_bytes(12288, 3072, 0) >= (12288 // 64) * 3072 * 4
    assert L.efqat_bias_grad_workspace_bytes(12288, 3072, 1) >= 3072 * 4
    assert L.efqat_layer_select_workspace_bytes(48) >= 48 * 8


def test_product_path_has_no_oracle_or_cpu_fallback():
    pkg = os.path.join(ROOT, "paper_2411_11038_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.replace("no oracle", ""), f"{f} mentions the oracle"
    # missing library must raise, not fall back
    import paper_2411_11038_amd.binding as b
    saved, b._LIB = b._LIB, None
    real = b.lib_path
    b.lib_path = lambda: "/nonexistent/libefqat.so"
    try:
        with pytest.raises(FileNotFoundError):
            b.lib()
    finally:
        b.lib_path, b._LIB = real, saved

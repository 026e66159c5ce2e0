"""ctypes loader and thin wrappers for libefqat.so (see include/efqat.h for the contract)."""
from __future__ import annotations

import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
F32, BF16 = 0, 1
ACT_PER_TENSOR_ASYM, W_PER_ROW_SYM = 0, 1
DY_TOKEN_MAJOR, DY_CHANNEL_MAJOR = 0, 1

EXPORTS = [
    "efqat_version", "efqat_strerror", "efqat_k_from_ratio",
    "efqat_fakequant_fwd_workspace_bytes", "efqat_fakequant_fwd",
    "efqat_channel_select_workspace_bytes", "efqat_channel_select", "efqat_channel_select_static",
    "efqat_weight_quant_select_workspace_bytes", "efqat_weight_quant_select",
    "efqat_network_select_workspace_bytes", "efqat_network_select",
    "efqat_layer_select_workspace_bytes", "efqat_layer_select",
    "efqat_bias_grad_workspace_bytes", "efqat_bias_grad",
    "efqat_linear_bwd_workspace_bytes", "efqat_linear_bwd_workspace_bytes_ex", "efqat_linear_bwd", "efqat_linear_bwd_ex",
    "efqat_linear_bwd_weight_operand_bytes", "efqat_linear_bwd_weight_operand",
    "efqat_conv_bwd_workspace_bytes", "efqat_conv_bwd_workspace_bytes_ex", "efqat_conv_bwd", "efqat_conv_bwd_ex",
    "efqat_linear_fwd_workspace_bytes", "efqat_linear_fwd",
    "efqat_profile_enable", "efqat_profile_read",
]


class OptStep(C.Structure):
    """efqat_opt_step of include/efqat.h."""
    _fields_ = [("lr_w", C.c_float), ("momentum", C.c_float), ("weight_decay", C.c_float), ("mom_w", C.c_void_p),
                ("lr_s", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("adam_m", C.c_void_p), ("adam_v", C.c_void_p), ("adam_t", C.c_void_p)]


class EfqatError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {lib().efqat_strerror(code).decode()} ({code})")


def lib_path() -> str:
    return os.path.join(HERE, "lib", "libefqat.so")


_LIB = None


def lib():
    """Load libefqat.so (built by paper_2411_11038_amd/build.py).  Raises if it is missing."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} not built: run `python -m paper_2411_11038_amd.build`")
    L = C.CDLL(path)
    i64, sz, vp, ci = C.c_int64, C.c_size_t, C.c_void_p, C.c_int
    L.efqat_version.restype = ci
    L.efqat_strerror.restype = C.c_char_p
    L.efqat_strerror.argtypes = [ci]
    L.efqat_k_from_ratio.restype = i64
    L.efqat_k_from_ratio.argtypes = [i64, i64, i64]
    L.efqat_fakequant_fwd_workspace_bytes.restype = sz
    L.efqat_fakequant_fwd_workspace_bytes.argtypes = [i64, i64, ci]
    L.efqat_fakequant_fwd.restype = ci
    L.efqat_fakequant_fwd.argtypes = [vp, ci, i64, i64, ci, ci, ci, vp, vp, vp, vp, vp, vp, sz, vp]
    L.efqat_channel_select_workspace_bytes.restype = sz
    L.efqat_channel_select_workspace_bytes.argtypes = [i64]
    L.efqat_channel_select.restype = ci
    L.efqat_channel_select.argtypes = [vp, i64, i64, i64, vp, vp, vp, sz, vp]
    L.efqat_channel_select_static.restype = ci
    L.efqat_channel_select_static.argtypes = [vp, i64, i64, i64, vp, vp]
    L.efqat_weight_quant_select_workspace_bytes.restype = sz
    L.efqat_weight_quant_select_workspace_bytes.argtypes = [i64]
    L.efqat_weight_quant_select.restype = ci
    L.efqat_weight_quant_select.argtypes = [vp, i64, i64, ci, ci, vp, vp, vp, i64, vp, vp, vp, sz, vp]
    L.efqat_network_select_workspace_bytes.restype = sz
    L.efqat_network_select_workspace_bytes.argtypes = [i64]
    L.efqat_network_select.restype = ci
    L.efqat_network_select.argtypes = [vp, vp, i64, i64, i64, vp, vp, vp, sz, vp]
    L.efqat_layer_select_workspace_bytes.restype = sz
    L.efqat_layer_select_workspace_bytes.argtypes = [i64]
    L.efqat_layer_select.restype = ci
    L.efqat_layer_select.argtypes = [vp, vp, i64, i64, vp, vp, vp, vp, sz, vp]
    L.efqat_bias_grad_workspace_bytes.restype = sz
    L.efqat_bias_grad_workspace_bytes.argtypes = [i64, i64, ci]
    L.efqat_bias_grad.restype = ci
    L.efqat_bias_grad.argtypes = [vp, ci, ci, i64, i64, vp, vp, sz, vp]
    bwd_common = [vp, vp, vp, ci, vp, vp] + [vp, vp, vp, vp] + [vp, i64] + [vp, ci, vp, ci, vp, vp, vp]
    L.efqat_linear_bwd_workspace_bytes.restype = sz
    L.efqat_linear_bwd_workspace_bytes.argtypes = [i64, i64, i64, i64, ci, ci]
    L.efqat_linear_bwd_workspace_bytes_ex.restype = sz
    L.efqat_linear_bwd_workspace_bytes_ex.argtypes = [i64, i64, i64, i64, ci, ci, ci]
    L.efqat_linear_bwd.restype = ci
    L.efqat_linear_bwd.argtypes = [vp, ci, ci, i64, i64, i64] + bwd_common + [vp, sz, vp]
    L.efqat_linear_bwd_ex.restype = ci
    L.efqat_linear_bwd_ex.argtypes = ([vp, ci, ci, i64, i64, i64] + bwd_common + [vp, C.POINTER(OptStep), ci]
                                      + [vp, sz, vp, vp])
    L.efqat_linear_bwd_weight_operand_bytes.restype = sz
    L.efqat_linear_bwd_weight_operand_bytes.argtypes = [i64, i64, i64, ci, ci]
    L.efqat_linear_bwd_weight_operand.restype = ci
    L.efqat_linear_bwd_weight_operand.argtypes = [vp, vp, i64, i64, i64, ci, ci, vp, sz, vp]
    L.efqat_conv_bwd_workspace_bytes.restype = sz
    L.efqat_conv_bwd_workspace_bytes.argtypes = [i64] * 10 + [ci, ci]
    L.efqat_conv_bwd_workspace_bytes_ex.restype = sz
    L.efqat_conv_bwd_workspace_bytes_ex.argtypes = [i64] * 10 + [ci, ci, ci]
    L.efqat_conv_bwd.restype = ci
    L.efqat_conv_bwd.argtypes = [vp, ci, ci] + [i64] * 9 + bwd_common + [vp, sz, vp]
    L.efqat_conv_bwd_ex.restype = ci
    L.efqat_conv_bwd_ex.argtypes = [vp, ci, ci] + [i64] * 9 + bwd_common + [C.POINTER(OptStep), ci] + [vp, sz, vp, vp]
    L.efqat_linear_fwd_workspace_bytes.restype = sz
    L.efqat_linear_fwd_workspace_bytes.argtypes = [i64, i64, i64]
    L.efqat_linear_fwd.restype = ci
    L.efqat_linear_fwd.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, vp, ci, vp, sz, vp]
    L.efqat_profile_enable.restype = ci
    L.efqat_profile_enable.argtypes = [ci]
    L.efqat_profile_read.restype = ci
    L.efqat_profile_read.argtypes = [ci, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    _LIB = L
    return L


# ------------------------------------------------------------------ marshalling helpers
def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _p(t):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("tensor must live on the GPU")
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _ws(nbytes: int, like: torch.Tensor) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=like.device)


def _check(rc: int, where: str):
    if rc != 0:
        raise EfqatError(rc, where)


def profile_enable(on: bool) -> None:
    _check(lib().efqat_profile_enable(int(bool(on))), "efqat_profile_enable")


PROF_DX, PROF_DW, PROF_FWD, PROF_PREP, PROF_FINISH, PROF_QUANT_ACT, PROF_QUANT_W, PROF_IMPORTANCE, PROF_TOPK, \
    PROF_BIAS, PROF_CLASSES = range(11)


def profile_read(which: int):
    """(total ms, brackets) of kernel class `which` (PROF_*) since profile_enable(True)."""
    ms, n = C.c_double(0.0), C.c_int64(0)
    _check(lib().efqat_profile_read(which, C.byref(ms), C.byref(n)), "efqat_profile_read")
    return ms.value, n.value


def k_from_ratio(c_out: int, num: int, den: int) -> int:
    return int(lib().efqat_k_from_ratio(c_out, num, den))


def fakequant_fwd(x: torch.Tensor, mode: int, bits: int, init_minmax: bool = True, scale=None,
                  zero_point=None, want_xq: bool = False, ws=None, out=None):
    """Returns dict(codes, clip_bits, scale, zero_point, xq).  x is [rows, cols] (leading dims are
    flattened into rows; a conv weight [C_out, KH, KW, C_in] is rows = C_out).  `out` may carry
    preallocated codes / clip_bits / xq tensors."""
    L = lib()
    cols = x.shape[-1] if mode == ACT_PER_TENSOR_ASYM else x[0].numel()
    rows = x.numel() // cols
    dev = x.device
    out = out or {}
    if scale is None:
        scale = out.get("scale")
    if scale is None:
        scale = torch.empty(1 if mode == ACT_PER_TENSOR_ASYM else rows, dtype=torch.float32, device=dev)
    if zero_point is None:
        zero_point = out.get("zero_point")
    if zero_point is None and mode == ACT_PER_TENSOR_ASYM:
        zero_point = torch.empty(1, dtype=torch.float32, device=dev)
    codes = out.get("codes")
    if codes is None:
        codes = torch.empty(x.shape, dtype=torch.uint8 if mode == ACT_PER_TENSOR_ASYM else torch.int8, device=dev)
    clip = out.get("clip_bits")
    if clip is None:
        clip = torch.empty((rows, (cols + 31) // 32), dtype=torch.int32, device=dev)
    xq = out.get("xq")
    if xq is None and want_xq:
        xq = torch.empty(x.shape, dtype=torch.bfloat16, device=dev)
    if ws is None:
        ws = _ws(L.efqat_fakequant_fwd_workspace_bytes(rows, cols, mode), x)
    rc = L.efqat_fakequant_fwd(_p(x), _dt(x), rows, cols, mode, bits, int(bool(init_minmax)), _p(scale),
                               _p(zero_point), _p(codes), _p(clip), _p(xq), _p(ws), ws.numel(), _stream())
    _check(rc, "efqat_fakequant_fwd")
    return dict(codes=codes, clip_bits=clip, scale=scale, zero_point=zero_point, xq=xq)


def channel_select(w: torch.Tensor, k: int, want_scores: bool = True, ws=None, out=None):
    """Returns (idx int32[k], scores float64[c_out] or None).  w is [c_out, ...] fp32."""
    L = lib()
    c_out = w.shape[0]
    block = w[0].numel()
    out = out or {}
    scores = out.get("scores")
    if scores is None and want_scores:
        scores = torch.empty(c_out, dtype=torch.float64, device=w.device)
    idx = out.get("idx")
    if idx is None:
        idx = torch.empty(max(k, 0), dtype=torch.int32, device=w.device)
    if ws is None:
        ws = _ws(L.efqat_channel_select_workspace_bytes(c_out), w)
    rc = L.efqat_channel_select(_p(w), c_out, block, k, _p(scores), _p(idx) if k > 0 else None, _p(ws),
                                ws.numel(), _stream())
    _check(rc, "efqat_channel_select")
    return idx, scores


def weight_quant_select(w: torch.Tensor, bits: int, k: int, init_minmax: bool = True, scale=None, ws=None, out=None):
    """efqat_weight_quant_select: fake-quant of the fp32 weights w [c_out, ...] and channel selection in one call.
    Returns dict(codes, clip_bits, scale, scores, idx).  `out` may carry preallocated tensors (same keys)."""
    L = lib()
    c_out = w.shape[0]
    block = w[0].numel()
    dev = w.device
    out = out or {}
    if scale is None:
        scale = out.get("scale")
    if scale is None:
        scale = torch.empty(c_out, dtype=torch.float32, device=dev)
    codes = out.get("codes")
    if codes is None:
        codes = torch.empty(w.shape, dtype=torch.int8, device=dev)
    clip = out.get("clip_bits")
    if clip is None:
        clip = torch.empty((c_out, (block + 31) // 32), dtype=torch.int32, device=dev)
    scores = out.get("scores")
    if scores is None:
        scores = torch.empty(c_out, dtype=torch.float64, device=dev)
    idx = out.get("idx")
    if idx is None:
        idx = torch.empty(max(k, 0), dtype=torch.int32, device=dev)
    if ws is None:
        ws = _ws(L.efqat_weight_quant_select_workspace_bytes(c_out), w)
    rc = L.efqat_weight_quant_select(_p(w), c_out, block, bits, int(bool(init_minmax)), _p(scale), _p(codes), _p(clip),
                                     k, _p(scores), _p(idx) if k > 0 else None, _p(ws), ws.numel(), _stream())
    _check(rc, "efqat_weight_quant_select")
    return dict(codes=codes, clip_bits=clip, scale=scale, scores=scores, idx=idx)


def channel_select_static(w: torch.Tensor, k: int, out=None):
    """efqat_channel_select_static: the same selection with the library's built-in scratch (no workspace, no scores
    output).  `out`: preallocated int32[k].  Returns idx."""
    c_out = w.shape[0]
    block = w[0].numel()
    idx = out if out is not None else torch.empty(max(k, 0), dtype=torch.int32, device=w.device)
    rc = lib().efqat_channel_select_static(_p(w), c_out, block, k, _p(idx) if k > 0 else None, _stream())
    _check(rc, "efqat_channel_select_static")
    return idx


def network_select(scores: torch.Tensor, layer_off: torch.Tensor, k_total: int, ws=None):
    """Returns (idx int32[k_total] of layer-local channel indices, k_per_layer int32[n_layers])."""
    L = lib()
    total = scores.numel()
    n_layers = layer_off.numel() - 1
    idx = torch.empty(max(k_total, 0), dtype=torch.int32, device=scores.device)
    kpl = torch.empty(n_layers, dtype=torch.int32, device=scores.device)
    if ws is None:
        ws = _ws(L.efqat_network_select_workspace_bytes(total), scores)
    rc = L.efqat_network_select(_p(scores), _p(layer_off), n_layers, total, k_total,
                                _p(idx) if k_total > 0 else None, _p(kpl), _p(ws), ws.numel(), _stream())
    _check(rc, "efqat_network_select")
    return idx, kpl


DX_KERNEL_AUTO, DX_KERNEL_BF16, DX_KERNEL_INT8, DX_KERNEL_BF16_PINNED = 0, 1, 2, 3


def layer_select(scores: torch.Tensor, layer_off: torch.Tensor, k_layers: int, ws=None):
    """EfQAT-LWPN.  Returns (layer_idx int32[k_layers], k_per_layer int32[n_layers], layer_scores double[n_layers])."""
    L = lib()
    n_layers = layer_off.numel() - 1
    lidx = torch.empty(max(k_layers, 0), dtype=torch.int32, device=scores.device)
    kpl = torch.empty(n_layers, dtype=torch.int32, device=scores.device)
    ls = torch.empty(n_layers, dtype=torch.float64, device=scores.device)
    if ws is None:
        ws = _ws(L.efqat_layer_select_workspace_bytes(n_layers), scores)
    rc = L.efqat_layer_select(_p(scores), _p(layer_off), n_layers, k_layers, _p(ls),
                              _p(lidx) if k_layers > 0 else None, _p(kpl), _p(ws), ws.numel(), _stream())
    _check(rc, "efqat_layer_select")
    return lidx, kpl, ls


def bias_grad(dy: torch.Tensor, dy_layout=DY_TOKEN_MAJOR, ws=None, out=None):
    """db[c] = sum over tokens of dY.  dy: [T, c_out] (token major; leading dims are flattened) or [c_out, T]."""
    L = lib()
    if dy_layout == DY_TOKEN_MAJOR:
        c_out = dy.shape[-1]
        T = dy.numel() // c_out
    else:
        c_out = dy.shape[0]
        T = dy.numel() // c_out
    db = out if out is not None else torch.empty(c_out, dtype=torch.float32, device=dy.device)
    if ws is None:
        ws = _ws(L.efqat_bias_grad_workspace_bytes(T, c_out, dy_layout), dy)
    rc = L.efqat_bias_grad(_p(dy), _dt(dy), dy_layout, T, c_out, _p(db), _p(ws), ws.numel(), _stream())
    _check(rc, "efqat_bias_grad")
    return db


def _bwd_outputs(x, w, k, dx_dtype, scatter):
    dev = x.device
    c_out = w.shape[0]
    dx = torch.empty(x.shape, dtype=dx_dtype, device=dev)
    if scatter:
        dw = torch.zeros(w.shape, dtype=torch.float32, device=dev)
        ds_w = torch.zeros(c_out, dtype=torch.float32, device=dev)
    else:
        dw = torch.empty((k,) + tuple(w.shape[1:]), dtype=torch.float32, device=dev)
        ds_w = torch.empty(k, dtype=torch.float32, device=dev)
    ds_x = torch.empty(1, dtype=torch.float32, device=dev)
    dz_x = torch.empty(1, dtype=torch.float32, device=dev)
    return dx, dw, ds_w, ds_x, dz_x


def _step_struct(step):
    """dict(lr_w, momentum=0, weight_decay=0, mom_w=None, lr_s, beta1=0.9, beta2=0.999, eps=1e-8, adam_m, adam_v,
    adam_t) -> OptStep"""
    return OptStep(float(step["lr_w"]), float(step.get("momentum", 0.0)), float(step.get("weight_decay", 0.0)),
                   _p(step.get("mom_w")), float(step["lr_s"]), float(step.get("beta1", 0.9)),
                   float(step.get("beta2", 0.999)), float(step.get("eps", 1e-8)), _p(step["adam_m"]),
                   _p(step["adam_v"]), _p(step["adam_t"]))


def linear_bwd_weight_operand(w_codes, s_w, T, dy_dtype=BF16, dy_layout=DY_TOKEN_MAJOR, out=None):
    """The bf16 W_q^T operand of the dX product, made ahead of efqat_linear_bwd_prepared (argument w_operand of
    linear_bwd).  Returns a uint8 tensor, or None when the layer's dX product reads the int8 codes themselves."""
    L = lib()
    c_out, c_in = w_codes.shape
    need = L.efqat_linear_bwd_weight_operand_bytes(T, c_in, c_out, dy_dtype, dy_layout)
    if need == 0:
        return None
    if out is None:
        out = torch.empty(need, dtype=torch.uint8, device=w_codes.device)
    rc = L.efqat_linear_bwd_weight_operand(_p(w_codes), _p(s_w), T, c_in, c_out, dy_dtype, dy_layout, _p(out),
                                           out.numel(), _stream())
    _check(rc, "efqat_linear_bwd_weight_operand")
    return out


def linear_bwd(dy, x_codes, x_clip, x, s_x, z_x, w_codes, w_clip, w, s_w, idx, dy_layout=DY_TOKEN_MAJOR,
               dx_dtype=None, scatter=False, ws=None, out=None, step=None, w_operand=None, dx_kernel=DX_KERNEL_AUTO,
               side_stream=None):
    """Backward of one quantized linear layer restricted to the rows idx.  Returns
    dict(dx, dw, ds_w, ds_x, dz_x).  `out` may carry preallocated outputs (same keys).
    step: dict for the fused optimizer step (see _step_struct): w and s_w are then updated in place.
    w_operand: the tensor made by linear_bwd_weight_operand for these weights.
    dx_kernel: DX_KERNEL_* (tests and measurements).
    side_stream: a torch.cuda.Stream on which the weight-gradient branch may run beside the dX product.
    Any of the four routes the call to efqat_linear_bwd_ex."""
    L = lib()
    T, c_in = x_codes.shape
    c_out = w_codes.shape[0]
    k = 0 if idx is None else int(idx.numel())
    dx_dtype = dx_dtype or (torch.bfloat16 if dy.dtype == torch.bfloat16 else torch.float32)
    if out is None:
        dx, dw, ds_w, ds_x, dz_x = _bwd_outputs(x, w, k, dx_dtype, scatter)
    else:
        dx, dw, ds_w, ds_x, dz_x = out["dx"], out["dw"], out["ds_w"], out["ds_x"], out["dz_x"]
    if ws is None:
        ws = _ws(L.efqat_linear_bwd_workspace_bytes_ex(T, c_in, c_out, k, _dt(dy), dy_layout, dx_kernel), x)
    args = (_p(dy), _dt(dy), dy_layout, T, c_in, c_out, _p(x_codes), _p(x_clip), _p(x), _dt(x),
            _p(s_x), _p(z_x), _p(w_codes), _p(w_clip), _p(w), _p(s_w),
            _p(idx) if k > 0 else None, k, _p(dx), _dt(dx), _p(dw) if k > 0 and dw is not None else None,
            int(bool(scatter)), _p(ds_w) if k > 0 and ds_w is not None else None, _p(ds_x), _p(dz_x))
    if step is None and w_operand is None and dx_kernel == DX_KERNEL_AUTO and side_stream is None:
        rc = L.efqat_linear_bwd(*args, _p(ws), ws.numel(), _stream())
    else:
        st = _step_struct(step) if step is not None else None
        rc = L.efqat_linear_bwd_ex(*args, _p(w_operand), C.byref(st) if st is not None else None, dx_kernel,
                                   _p(ws), ws.numel(), _stream(), side_stream.cuda_stream if side_stream else None)
    _check(rc, "efqat_linear_bwd")
    return dict(dx=dx, dw=dw, ds_w=ds_w, ds_x=ds_x, dz_x=dz_x)


def linear_fwd(x_codes, s_x, z_x, w_codes, s_w, y_dtype=torch.bfloat16, ws=None, out=None):
    """Low-precision forward Y = X_q W_q^T from the integer codes (int8 matrix cores).  Returns y [T, c_out]."""
    L = lib()
    T, c_in = x_codes.shape
    c_out = w_codes.shape[0]
    y = out if out is not None else torch.empty((T, c_out), dtype=y_dtype, device=x_codes.device)
    if ws is None:
        ws = _ws(L.efqat_linear_fwd_workspace_bytes(T, c_in, c_out), x_codes)
    rc = L.efqat_linear_fwd(_p(x_codes), _p(s_x), _p(z_x), _p(w_codes), _p(s_w), T, c_in, c_out, _p(y), _dt(y),
                            _p(ws), ws.numel(), _stream())
    _check(rc, "efqat_linear_fwd")
    return y


def conv_bwd(dy, x_codes, x_clip, x, s_x, z_x, w_codes, w_clip, w, s_w, idx, stride=1, pad=0,
             dy_layout=DY_TOKEN_MAJOR, dx_dtype=None, scatter=False, ws=None, out=None, step=None,
             dx_kernel=DX_KERNEL_AUTO, side_stream=None):
    """Backward of one quantized conv layer (x NHWC, w OHWI) restricted to output channels idx."""
    L = lib()
    N, H, W, c_in = x_codes.shape
    c_out, KH, KW, _ = w_codes.shape
    k = 0 if idx is None else int(idx.numel())
    dx_dtype = dx_dtype or (torch.bfloat16 if dy.dtype == torch.bfloat16 else torch.float32)
    if out is None:
        dx, dw, ds_w, ds_x, dz_x = _bwd_outputs(x, w, k, dx_dtype, scatter)
    else:
        dx, dw, ds_w, ds_x, dz_x = out["dx"], out["dw"], out["ds_w"], out["ds_x"], out["dz_x"]
    if ws is None:
        ws = _ws(L.efqat_conv_bwd_workspace_bytes_ex(N, H, W, c_in, c_out, KH, KW, stride, pad, k, _dt(dy), dy_layout,
                                                     dx_kernel), x)
    args = (_p(dy), _dt(dy), dy_layout, N, H, W, c_in, c_out, KH, KW, stride, pad, _p(x_codes),
            _p(x_clip), _p(x), _dt(x), _p(s_x), _p(z_x), _p(w_codes), _p(w_clip), _p(w), _p(s_w),
            _p(idx) if k > 0 else None, k, _p(dx), _dt(dx), _p(dw) if k > 0 and dw is not None else None,
            int(bool(scatter)), _p(ds_w) if k > 0 and ds_w is not None else None, _p(ds_x), _p(dz_x))
    if step is None and dx_kernel == DX_KERNEL_AUTO and side_stream is None:
        rc = L.efqat_conv_bwd(*args, _p(ws), ws.numel(), _stream())
    else:
        st = _step_struct(step) if step is not None else None
        rc = L.efqat_conv_bwd_ex(*args, C.byref(st) if st is not None else None, dx_kernel, _p(ws), ws.numel(),
                                 _stream(), side_stream.cuda_stream if side_stream else None)
    _check(rc, "efqat_conv_bwd")
    return dict(dx=dx, dw=dw, ds_w=ds_w, ds_x=ds_x, dz_x=dz_x)

"""GPU parity at the full sizes of the workload configs, in the launch configuration bench.py times (preallocated
outputs and workspace, bf16 activations and gradients, bf16 dX, min/max-initialised quantizers), against the complete
fp64 oracle: every element of dX and dW, every dS_w, and dS_x / dZ_x against the oracle's own sums."""
import functools

import numpy as np
import pytest
import torch

import paper_2411_11038_amd as ef
from oracle import efqat_oracle as orc
from workloads import synth

from bwd_checks import check_backward
from gpu_util import act_tensor, clip_words, dev, host, pack_mask, report

pytestmark = pytest.mark.gpu


@functools.lru_cache(maxsize=2)
def _linear_data(seed, T, c_in, c_out):
    return synth.linear_layer(seed, T, c_in, c_out, act_dtype="bf16")


def _run_linear_layer(X, W, dY, w_bits, num, den, layout):
    """One layer the way bench.py runs it: quantize, select, backward into preallocated buffers."""
    T, c_in = X.shape
    c_out = W.shape[0]
    xd, wd = act_tensor(X, "bf16"), dev(W)
    fx = ef.fakequant_fwd(xd, ef.ACT_PER_TENSOR_ASYM, 8, init_minmax=True)
    fw = ef.fakequant_fwd(wd, ef.W_PER_ROW_SYM, w_bits, init_minmax=True)
    k = ef.k_from_ratio(c_out, num, den)
    idx, scores = ef.channel_select(wd, k)
    dyh = dY if layout == 0 else np.ascontiguousarray(dY.T)
    e = lambda shape, dt: torch.empty(shape, dtype=dt, device="cuda")
    out = dict(dx=e((T, c_in), torch.bfloat16), dw=e((max(k, 1), c_in), torch.float32), ds_w=e(max(k, 1), torch.float32),
               ds_x=e(1, torch.float32), dz_x=e(1, torch.float32))
    ws = e(max(ef.lib().efqat_linear_bwd_workspace_bytes(T, c_in, c_out, k, ef.BF16, layout), 256), torch.uint8)
    ef.linear_bwd(act_tensor(dyh, "bf16"), fx["codes"], fx["clip_bits"], xd, fx["scale"], fx["zero_point"],
                  fw["codes"], fw["clip_bits"], wd, fw["scale"], idx if k else None, dy_layout=layout, ws=ws, out=out)
    torch.cuda.synchronize()
    return fx, fw, idx, scores, out, k


def _check_forward(X, W, fx, fw, idx, scores, ref, sx, zx, sw, k):
    assert fx["scale"].item() == float(sx) and fx["zero_point"].item() == float(zx)
    assert np.array_equal(fw["scale"].cpu().numpy(), sw)
    assert np.array_equal(fx["codes"].cpu().numpy(), ref["x_codes"].astype(np.uint8))
    assert np.array_equal(fw["codes"].cpu().numpy(), ref["w_codes"].astype(np.int8))
    assert np.array_equal(clip_words(fx["clip_bits"]), pack_mask(ref["x_mask"].reshape(-1, ref["x_mask"].shape[-1])))
    assert np.array_equal(clip_words(fw["clip_bits"]), pack_mask(ref["w_mask"].reshape(W.shape[0], -1)))
    imp = orc.channel_importance(W)
    np.testing.assert_allclose(scores.cpu().numpy(), imp, rtol=1e-12)
    idx_ref = orc.top_k_channels(imp, k)
    assert np.array_equal(idx.cpu().numpy().astype(np.int64), idx_ref)
    return idx_ref


def _full_linear_case(seed, T, c_in, c_out, w_bits, frac, layout):
    X, W, dY = _linear_data(seed, T, c_in, c_out)
    num, den = frac
    fx, fw, idx, scores, out, k = _run_linear_layer(X, W, dY, w_bits, num, den, layout)
    sx, zx = orc.act_qparams_minmax(X, 8)
    sw = orc.weight_scale_minmax(W, w_bits)
    idx_ref = orc.top_k_channels(orc.channel_importance(W), k)
    ref = orc.linear_bwd(dY, X, sx, zx, 8, W, sw, w_bits, idx_ref)
    _check_forward(X, W, fx, fw, idx, scores, ref, sx, zx, sw, k)
    if k:
        out = dict(out, dw=out["dw"][:k], ds_w=out["ds_w"][:k])
    check_backward(out, ref, idx, idx_ref, X, W, (sx, zx, sw), "bf16", False, True)


# ---------------------------------------------------------------- config 2: BERT-base FFN pair, every fraction it names
@pytest.mark.parametrize("frac", [(0, 1), (1, 20), (1, 4), (1, 1)], ids=lambda f: "r%d-%d" % f)
@pytest.mark.parametrize("layer", [0, 1])
def test_cfg2_bert_ffn_full(layer, frac):
    cfg = synth.CFG2
    name, T, c_in, c_out = cfg["layers"][layer]
    _full_linear_case(cfg["seed"] + layer, T, c_in, c_out, 8, frac, 0)


@pytest.mark.parametrize("layer", [0, 1])
def test_cfg2_bert_ffn_full_channel_major(layer):
    cfg = synth.CFG2
    name, T, c_in, c_out = cfg["layers"][layer]
    _full_linear_case(cfg["seed"] + layer, T, c_in, c_out, 8, (1, 20), 1)


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("layer", [0, 1])
def test_cfg2_bias_grad_full(layer, layout):
    cfg = synth.CFG2
    name, T, c_in, c_out = cfg["layers"][layer]
    _, _, dY = _linear_data(cfg["seed"] + layer, T, c_in, c_out)
    dyh = dY if layout == 0 else np.ascontiguousarray(dY.T)
    db = ef.bias_grad(act_tensor(dyh, "bf16"), dy_layout=layout)
    torch.cuda.synchronize()
    ref = orc.bias_grad(dY)
    scale = np.sqrt((dY.astype(np.float64) ** 2).sum(axis=0))
    r = float(np.max(np.abs(host(db) - ref) / scale))
    report("bias gradient max err / column l2 %.2e (bound 1e-5)" % r)
    assert r <= 1e-5


# ---------------------------------------------------------------- config 3: the four linears of a BERT-base encoder
# layer (the 12 layers of the stack repeat these shapes), both weight bit widths the config names
@pytest.mark.parametrize("w_bits,frac", [(4, (1, 20)), (8, (1, 20)), (4, (1, 4))], ids=["W4A8_r5", "W8A8_r5", "W4A8_r25"])
@pytest.mark.parametrize("layer", [0, 1, 2, 3])
def test_cfg3_encoder_linears_full(layer, w_bits, frac):
    cfg = synth.CFG3
    name, T, c_in, c_out = cfg["layers"][layer]
    _full_linear_case(cfg["seed"] + layer, T, c_in, c_out, w_bits, frac, 0)


# ---------------------------------------------------------------- config 4: ResNet-50-shaped convolutions
@pytest.mark.parametrize("frac", [(1, 20), (1, 4), (1, 1)], ids=lambda f: "r%d-%d" % f)
@pytest.mark.parametrize("which", ["conv", "conv1x1"])
def test_cfg4_resnet_conv_full(which, frac):
    cfg = synth.CFG4
    g = cfg[which]
    X, W, dY = synth.conv_layer(cfg["seed"] + (which == "conv1x1"), g["N"], g["H"], g["W"], g["c_in"], g["c_out"],
                                g["kh"], g["kw"], g["stride"], g["pad"], act_dtype="bf16")
    xd, wd = act_tensor(X, "bf16"), dev(W)
    fx = ef.fakequant_fwd(xd, ef.ACT_PER_TENSOR_ASYM, 8, init_minmax=True)
    fw = ef.fakequant_fwd(wd, ef.W_PER_ROW_SYM, 4, init_minmax=True)
    k = ef.k_from_ratio(g["c_out"], *frac)
    idx, scores = ef.channel_select(wd, k)
    out = ef.conv_bwd(act_tensor(dY, "bf16"), fx["codes"], fx["clip_bits"], xd, fx["scale"], fx["zero_point"],
                      fw["codes"], fw["clip_bits"], wd, fw["scale"], idx, stride=g["stride"], pad=g["pad"])
    torch.cuda.synchronize()
    sx, zx = orc.act_qparams_minmax(X, 8)
    sw = orc.weight_scale_minmax(W, 4)
    idx_ref = orc.top_k_channels(orc.channel_importance(W), k)
    ref = orc.conv_bwd(dY, X, sx, zx, 8, W, sw, 4, idx_ref, g["stride"], g["pad"])
    _check_forward(X, W, fx, fw, idx, scores, ref, sx, zx, sw, k)
    check_backward(out, ref, idx, idx_ref, X, W, (sx, zx, sw), "bf16", False, True)


# ---------------------------------------------------------------- config 5: LLM-sized MLP pair, the headline of bench.py
@pytest.mark.parametrize("frac", [(1, 100), (1, 4), (1, 1)], ids=lambda f: "r%d-%d" % f)
@pytest.mark.parametrize("layer", [0, 1])
def test_cfg5_llm_mlp_full(layer, frac):
    cfg = synth.CFG5
    name, T, c_in, c_out = cfg["layers"][layer]
    _full_linear_case(cfg["seed"] + layer, T, c_in, c_out, 4, frac, 0)


@pytest.mark.parametrize("layer", [0, 1])
def test_cfg5_llm_mlp_full_channel_major(layer):
    cfg = synth.CFG5
    name, T, c_in, c_out = cfg["layers"][layer]
    _full_linear_case(cfg["seed"] + layer, T, c_in, c_out, 4, (1, 20), 1)

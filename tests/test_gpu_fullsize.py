"""GPU parity at the full sizes of the workload configs, in the launch configuration bench.py times
(preallocated outputs, token-major bf16 dY, min/max-initialised quantizers).  Where the fp64 oracle
finishes in seconds the comparison is complete; for the LLM-sized layers it is done on sampled output
rows that the oracle computes one by one, plus reduction properties that hold at any size."""
import numpy as np
import pytest
import torch

import paper_2411_11038_amd as ef
from oracle import efqat_oracle as orc
from workloads import synth

from gpu_util import act_tensor, assert_max_err, clip_words, dev, host, pack_mask

pytestmark = pytest.mark.gpu


def _gpu_layer(X, W, dY, kind, a_bits, w_bits, num, den, dx_dtype=None, layout=0):
    xd, wd = act_tensor(X, kind), dev(W)
    fx = ef.fakequant_fwd(xd, ef.ACT_PER_TENSOR_ASYM, a_bits, init_minmax=True)
    fw = ef.fakequant_fwd(wd, ef.W_PER_ROW_SYM, w_bits, init_minmax=True)
    k = ef.k_from_ratio(W.shape[0], num, den)
    idx, scores = ef.channel_select(wd, k)
    dyh = dY if layout == 0 else np.ascontiguousarray(dY.T)
    out = ef.linear_bwd(act_tensor(dyh, kind), fx["codes"], fx["clip_bits"], xd, fx["scale"], fx["zero_point"],
                        fw["codes"], fw["clip_bits"], wd, fw["scale"], idx if k else None, dx_dtype=dx_dtype,
                        dy_layout=layout)
    torch.cuda.synchronize()
    return fx, fw, idx, scores, out


def _check_forward(X, W, fx, fw, idx, scores, a_bits, w_bits, k):
    sx, zx = orc.act_qparams_minmax(X, a_bits)
    sw = orc.weight_scale_minmax(W, w_bits)
    assert fx["scale"].item() == float(sx) and fx["zero_point"].item() == float(zx)
    assert np.array_equal(fw["scale"].cpu().numpy(), sw)
    xc, xm, Xq = orc.fakequant_act(X, sx, zx, a_bits)
    wc, wm, Wq = orc.fakequant_weight(W, sw, w_bits)
    assert np.array_equal(fx["codes"].cpu().numpy(), xc.astype(np.uint8))
    assert np.array_equal(fw["codes"].cpu().numpy(), wc.astype(np.int8))
    assert np.array_equal(clip_words(fx["clip_bits"]), pack_mask(xm))
    assert np.array_equal(clip_words(fw["clip_bits"]), pack_mask(wm))
    imp = orc.channel_importance(W)
    np.testing.assert_allclose(scores.cpu().numpy(), imp, rtol=1e-12)
    idx_ref = orc.top_k_channels(imp, k)
    assert np.array_equal(idx.cpu().numpy().astype(np.int64), idx_ref)
    return sx, zx, sw, xc, xm, Xq, wc, wm, Wq, idx_ref


@pytest.mark.parametrize("layer", [0, 1])
@pytest.mark.parametrize("frac", [(1, 4), (1, 20)])
def test_cfg2_bert_ffn_full(layer, frac):
    cfg = synth.CFG2
    name, T, c_in, c_out = cfg["layers"][layer]
    X, W, dY = synth.linear_layer(cfg["seed"] + layer, T, c_in, c_out, act_dtype="bf16")
    num, den = frac
    k = orc.k_from_ratio(c_out, num, den)
    fx, fw, idx, scores, out = _gpu_layer(X, W, dY, "bf16", 8, 8, num, den)
    sx, zx, sw, xc, xm, Xq, wc, wm, Wq, idx_ref = _check_forward(X, W, fx, fw, idx, scores, 8, 8, k)
    dY64 = dY.astype(np.float64)
    dXq = dY64 @ Wq
    dX = np.where(xm, dXq, 0.0)
    assert_max_err(host(out["dx"]), dX, 2e-2, "dX")
    dS_x, dZ_x = orc.grad_act_qparams(dXq, X, xc, xm, sx, zx)
    g = np.where(xm, (xc - float(zx)) - X.astype(np.float64) / float(sx), xc - float(zx))
    l2 = np.sqrt(np.sum((dXq * g) ** 2))
    assert abs(out["ds_x"].item() - dS_x) <= 2e-2 * l2
    l2z = float(sx) * np.sqrt(np.sum(dXq[~xm] ** 2))
    assert abs(out["dz_x"].item() - dZ_x) <= 2e-2 * l2z + 1e-30
    dWq = dY64[:, idx_ref].T @ Xq
    dW = np.where(wm[idx_ref], dWq, 0.0)
    assert_max_err(host(out["dw"]), dW, 2e-4, "dW")           # bf16 dY and integer codes are exact in bf16
    dS_w = orc.grad_weight_scale(dWq, W[idx_ref], wc[idx_ref], wm[idx_ref], sw[idx_ref])
    gw = np.where(wm[idx_ref], wc[idx_ref] - W[idx_ref].astype(np.float64) / sw[idx_ref, None], wc[idx_ref])
    row_l2 = np.sqrt(np.sum((dWq * gw) ** 2, axis=1))
    assert np.all(np.abs(host(out["ds_w"]) - dS_w) <= 1e-3 * row_l2 + 1e-30)


@pytest.mark.parametrize("layer", [0, 1])
@pytest.mark.parametrize("layout", [0, 1])
def test_cfg2_bias_grad_full(layer, layout):
    cfg = synth.CFG2
    name, T, c_in, c_out = cfg["layers"][layer]
    _, _, dY = synth.linear_layer(cfg["seed"] + layer, T, c_in, c_out, act_dtype="bf16")
    dyh = dY if layout == 0 else np.ascontiguousarray(dY.T)
    db = ef.bias_grad(act_tensor(dyh, "bf16"), dy_layout=layout)
    torch.cuda.synchronize()
    ref = orc.bias_grad(dY)
    scale = np.sqrt((dY.astype(np.float64) ** 2).sum(axis=0))
    assert np.max(np.abs(host(db) - ref) / scale) <= 1e-5


@pytest.mark.parametrize("layer,w_bits", [(0, 4), (1, 8)])
def test_cfg3_attention_projections_full(layer, w_bits):
    cfg = synth.CFG3
    name, T, c_in, c_out = cfg["layers"][layer]               # qkv 768->2304, out 768->768
    X, W, dY = synth.linear_layer(cfg["seed"] + layer, T, c_in, c_out, act_dtype="bf16")
    k = orc.k_from_ratio(c_out, 1, 20)
    fx, fw, idx, scores, out = _gpu_layer(X, W, dY, "bf16", 8, w_bits, 1, 20)
    sx, zx, sw, xc, xm, Xq, wc, wm, Wq, idx_ref = _check_forward(X, W, fx, fw, idx, scores, 8, w_bits, k)
    dY64 = dY.astype(np.float64)
    assert_max_err(host(out["dx"]), np.where(xm, dY64 @ Wq, 0.0), 2e-2, "dX")
    assert_max_err(host(out["dw"]), np.where(wm[idx_ref], dY64[:, idx_ref].T @ Xq, 0.0), 2e-4, "dW")


@pytest.mark.parametrize("which", ["conv", "conv1x1"])
def test_cfg4_resnet_conv_full(which):
    cfg = synth.CFG4
    g = cfg[which]
    X, W, dY = synth.conv_layer(cfg["seed"] + (which == "conv1x1"), g["N"], g["H"], g["W"], g["c_in"], g["c_out"],
                                g["kh"], g["kw"], g["stride"], g["pad"], act_dtype="bf16")
    xd, wd = act_tensor(X, "bf16"), dev(W)
    fx = ef.fakequant_fwd(xd, ef.ACT_PER_TENSOR_ASYM, 8, init_minmax=True)
    fw = ef.fakequant_fwd(wd, ef.W_PER_ROW_SYM, 4, init_minmax=True)
    k = ef.k_from_ratio(g["c_out"], 1, 4)
    idx, _ = ef.channel_select(wd, k)
    out = ef.conv_bwd(act_tensor(dY, "bf16"), fx["codes"], fx["clip_bits"], xd, fx["scale"], fx["zero_point"],
                      fw["codes"], fw["clip_bits"], wd, fw["scale"], idx, stride=g["stride"], pad=g["pad"])
    torch.cuda.synchronize()
    sx, zx = orc.act_qparams_minmax(X, 8)
    sw = orc.weight_scale_minmax(W, 4)
    idx_ref = orc.top_k_channels(orc.channel_importance(W), k)
    ref = orc.conv_bwd(dY, X, sx, zx, 8, W, sw, 4, idx_ref, g["stride"], g["pad"])
    assert np.array_equal(idx.cpu().numpy().astype(np.int64), idx_ref)
    assert np.array_equal(fx["codes"].cpu().numpy().astype(np.int64), ref["x_codes"])
    assert np.array_equal(fw["codes"].cpu().numpy().astype(np.int64), ref["w_codes"])
    assert_max_err(host(out["dx"]), ref["dX"], 2e-2, "dX")
    assert_max_err(host(out["dw"]), ref["dW"][idx_ref], 2e-4, "dW")
    l2 = np.sqrt(np.sum(ref["dXq"] ** 2)) * 0.5
    assert abs(out["ds_x"].item() - ref["dS_x"]) <= 2e-2 * l2


@pytest.mark.parametrize("layer", [0, 1])
def test_cfg5_llm_mlp_sampled(layer):
    cfg = synth.CFG5
    name, T, c_in, c_out = cfg["layers"][layer]
    X, W, dY = synth.linear_layer(cfg["seed"] + layer, T, c_in, c_out, act_dtype="bf16")
    num, den = 1, 10
    k = orc.k_from_ratio(c_out, num, den)
    fx, fw, idx, scores, out = _gpu_layer(X, W, dY, "bf16", 8, 4, num, den, dx_dtype=torch.float32)
    sx, zx, sw, xc, xm, Xq, wc, wm, Wq, idx_ref = _check_forward(X, W, fx, fw, idx, scores, 8, 4, k)
    rng = np.random.default_rng(5)
    rows = np.sort(rng.choice(T, 64, replace=False)); rows[0] = 0; rows[-1] = T - 1
    dx = out["dx"].cpu().numpy().astype(np.float64)
    dXq_rows = dY[rows].astype(np.float64) @ Wq
    assert_max_err(dx[rows], np.where(xm[rows], dXq_rows, 0.0), 2e-2, "dX rows")
    sel = np.sort(rng.choice(k, 64, replace=False)); sel[0] = 0; sel[-1] = k - 1
    ch = idx_ref[sel]
    dWq_rows = dY[:, ch].astype(np.float64).T @ Xq
    dw = out["dw"].cpu().numpy().astype(np.float64)
    assert_max_err(dw[sel], np.where(wm[ch], dWq_rows, 0.0), 2e-4, "dW rows")
    dS_w = orc.grad_weight_scale(dWq_rows, W[ch], wc[ch], wm[ch], sw[ch])
    gw = np.where(wm[ch], wc[ch] - W[ch].astype(np.float64) / sw[ch, None], wc[ch])
    row_l2 = np.sqrt(np.sum((dWq_rows * gw) ** 2, axis=1))
    assert np.all(np.abs(out["ds_w"].cpu().numpy().astype(np.float64)[sel] - dS_w) <= 1e-3 * row_l2)
    # reduction property: dS_x equals the sum of (dX_q * g) over the GPU's own fp32 dX_q (sampled rows above
    # tie it to the oracle); g comes from the oracle's codes.  The few clipped elements (min/max init can clip
    # the extreme value when both range ends round away from each other) get their dX_q from the oracle.
    q = xc - float(zx)
    gterm = np.where(xm, q - X.astype(np.float64) / float(sx), q)
    ct, ci = np.nonzero(~xm)
    assert ct.size < 64
    dxq_clip = np.array([float(dY[t].astype(np.float64) @ Wq[:, i]) for t, i in zip(ct, ci)])
    ref_sum = float(np.sum(dx * gterm)) + float(np.sum(dxq_clip * q[ct, ci]))
    l2 = np.sqrt(np.sum((dx * gterm) ** 2))
    assert abs(out["ds_x"].item() - ref_sum) <= 1e-3 * l2
    ref_dz = -float(sx) * float(np.sum(dxq_clip))
    assert abs(out["dz_x"].item() - ref_dz) <= 2e-2 * abs(ref_dz) + 1e-30
    assert not dx[ct, ci].any()

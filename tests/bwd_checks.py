"""Comparison of one backward call of the HIP library with the oracle's result, shared by the GPU parity tests.

Bounds (each measured error / scale ratio is printed, see gpu_util.report):

  dX, dW     max|err| <= 2e-2 max|ref| for products whose operands were rounded to bf16 (the stated bound); dW from a
             bf16 dY has exact operands (bf16 values, integers |code - Z_x| <= 255) and only differs by the order of
             the fp32 sums: 2e-4.
  dS_x, dZ_x sums of dX_q * g over all activations.  Every dX_q carries the rounding of the bf16 weight operand
             S_w * code (and of a dY that arrived in fp32): relative error uniform within half an ulp of an 8-bit
             significand, i.e. rms eps = 2^-8 / sqrt(3) * E[1/m] ~ 1.6e-3 per rounded factor (m = significand in
             [1, 2)), independent between weights.  The error of the sum is therefore about eps times the l2 norm of
             its summands.  Measured over the 118 cases of tests/test_gpu_parity.py: <= 5.5e-3 (dS_x), <= 7e-3 (dZ_x);
             QP_SUM_TOL = 1e-2 is about six standard deviations and twice the worst case seen.  For dZ_x, a sum over
             the few clipped elements only, the scale uses for every element the larger of its |dX_q| and the rms
             |dX_q| of the layer, because a single dX_q that is small by cancellation still carries the rounding
             error of its un-cancelled terms.
  dS_w[c]    sum_j dW_q[c][j] * g[c][j], g = code - w / S_w.  With exact operands (bf16 dY) two things are left: the
             fp32 rounding of the quotient w / S_w (|w / S_w| < 128: at most 2^-18 absolute, the subtraction from the
             code is exact), worth at most 2^-18 sum_j |dW_q[c][j]|, and fp32 accumulation, 1e-5 of the row's l2
             scale (the bound stated for fp32 reductions).  Measured: <= 0.45 of the first term alone.  With a dY
             that was rounded to bf16 the summands carry eps as above: QP_SUM_TOL of the row's l2 scale (measured
             <= 4.5e-3).
"""
import numpy as np

from gpu_util import assert_max_err, assert_rms_err, host, report

GEMM_TOL = 2e-2      # bf16 operands, fp32 accumulation (stated bound)
GEMM_RMS = 5e-3      # one bf16 rounding per W_q / fp32-dY element: rms 1.6e-3 per factor, plus the bf16 output
EXACT_TOL = 2e-4     # bf16 dY and integer codes are exact in bf16: only the order of the fp32 sums differs
QP_SUM_TOL = 1e-2    # sums whose terms carry bf16 operand rounding, relative to the l2 norm of the terms
QP_FP32_TOL = 1e-5   # fp32 reductions of exact terms, relative to the l2 norm of the terms
QUOT_ULP = 2.0 ** -18  # fp32 rounding of w / S_w, |w / S_w| < 128


def qparam_x_scales(ref, X, sx, zx):
    """(g, l2 of the dS_x summands, scale of the dZ_x sum) from the oracle's result."""
    z = np.rint(float(zx))
    q = ref["x_codes"] - z
    xm = ref["x_mask"]
    g = np.where(xm, q - np.asarray(X, dtype=np.float64) / float(sx), q)
    l2 = np.sqrt(np.sum((ref["dXq"] * g) ** 2))
    rms2 = float(np.mean(ref["dXq"] ** 2))
    clipped = ref["dXq"][~xm]
    l2z = float(sx) * np.sqrt(np.sum(np.maximum(clipped ** 2, rms2)))
    return g, l2, l2z


def check_qparams_x(ds_x, dz_x, ref, X, sx, zx, what=""):
    g, l2, l2z = qparam_x_scales(ref, X, sx, zx)
    n_clip = int((~ref["x_mask"]).sum())
    r_sx = abs(ds_x - ref["dS_x"]) / max(l2, 1e-300)
    r_zx = abs(dz_x - ref["dZ_x"]) / l2z if n_clip else 0.0
    report("%sdS_x err/l2 %.2e  dZ_x err/scale %.2e  (n=%d, clipped=%d; bound %.0e)"
           % (what, r_sx, r_zx, g.size, n_clip, QP_SUM_TOL))
    assert r_sx <= QP_SUM_TOL, (ds_x, ref["dS_x"], l2)
    assert r_zx <= QP_SUM_TOL, (dz_x, ref["dZ_x"], l2z)
    if n_clip == 0:
        assert dz_x == 0.0


def check_ds_w(dsw, ref, idx_ref, W, sw, exact_operands, what=""):
    """dsw: the k values of the GPU, in the order of idx_ref."""
    k = len(idx_ref)
    shape2 = (ref["dW"].shape[0], -1)
    dw_ref = ref["dW"].reshape(shape2)
    wm = ref["w_mask"].reshape(shape2)[idx_ref]
    wc = ref["w_codes"].reshape(shape2)[idx_ref].astype(np.float64)
    W2 = np.asarray(W).reshape(shape2)[idx_ref].astype(np.float64)
    gw = np.where(wm, wc - W2 / np.asarray(sw)[idx_ref, None].astype(np.float64), wc)
    # error scale per row: the larger of the l2 size of the row's actual summands dW_q * g (un-masked dW_q from the
    # oracle) and of the summands with every |dW_q| replaced by the row's largest gradient entry (zero when the whole
    # row is clipped; the other is small when the large entries of g meet small entries of dW_q)
    dwq = np.asarray(ref["dWq_sel"], dtype=np.float64).reshape(k, -1)
    l2_sum = np.sqrt(np.sum((dwq * gw) ** 2, axis=1))
    l2_max = np.sqrt(np.sum((np.abs(dw_ref[idx_ref]).max(axis=1, keepdims=True) * gw) ** 2, axis=1))
    row_l2 = np.maximum(l2_sum, l2_max)
    quot = QUOT_ULP * np.sum(np.abs(dwq), axis=1)
    err = np.abs(np.asarray(dsw, dtype=np.float64) - ref["dS_w"][idx_ref])
    tol = QP_FP32_TOL if exact_operands else QP_SUM_TOL
    bound = tol * row_l2 + quot
    r_l2 = float(np.max(np.maximum(err - quot, 0.0) / np.maximum(row_l2, 1e-300)))
    r_q = float(np.max(err / np.maximum(quot, 1e-300)))
    report("%sdS_w max (err - quotient term)/row_l2 %.2e (bound %.0e)  max err/quotient term %.2e  (%s operands, k=%d, n=%d)"
           % (what, r_l2, tol, r_q, "exact" if exact_operands else "rounded", k, dwq.shape[1]))
    assert np.all(err <= bound + 1e-30), (float(err.max()), float(row_l2.min()))


def check_backward(out, ref, idx, idx_ref, X, W, qp, kind, scatter, dx_is_bf16, shape_w=None):
    sx, zx, sw = qp
    k = len(idx_ref)
    assert idx.cpu().numpy().tolist() == np.asarray(idx_ref).tolist()
    # ---- dX: masked entries are exactly zero, the rest within the bf16-MFMA bound
    dx = host(out["dx"]).reshape(ref["dX"].shape)
    assert not dx[~ref["x_mask"]].any()
    assert_max_err(dx, ref["dX"], GEMM_TOL, "dX")
    assert_rms_err(dx, ref["dX"], GEMM_RMS + (4e-3 if dx_is_bf16 else 0.0), "dX rms")
    check_qparams_x(out["ds_x"].item(), out["dz_x"].item(), ref, X, sx, zx)
    if k == 0:
        return
    # ---- dW rows idx (+ frozen rows untouched in scatter mode)
    tol = EXACT_TOL if kind == "bf16" else GEMM_TOL
    dw = host(out["dw"]).astype(np.float64)
    dsw = host(out["ds_w"]).astype(np.float64)
    dw_ref = ref["dW"].reshape(ref["dW"].shape[0], -1)
    if scatter:
        dw = dw.reshape(dw_ref.shape)
        frozen = np.setdiff1d(np.arange(dw_ref.shape[0]), idx_ref)
        assert not dw[frozen].any() and not dsw[frozen].any()
        dw = dw[idx_ref]; dsw = dsw[idx_ref]
    else:
        dw = dw.reshape(-1, dw_ref.shape[1])[:k]
        dsw = dsw[:k]
    wm = ref["w_mask"].reshape(dw_ref.shape)[idx_ref]
    assert not dw[~wm].any()
    assert_max_err(dw, dw_ref[idx_ref], tol, "dW")
    check_ds_w(dsw, ref, idx_ref, W, sw, kind == "bf16")

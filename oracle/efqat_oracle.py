"""CPU oracle for the EfQAT backward hot path (arXiv 2411.11038).

TEST INFRASTRUCTURE ONLY.  A plain, slow, fp64 NumPy implementation of what the
paper defines, used to check the HIP library.  It shares no code with the HIP
path and must never be imported by it; only tests, the smoke check and the
benchmark's cpu_baseline leg call it.

What is fixed by the paper and what is a reading of it:
  * Eq. 1 (asymmetric activation quantizer), Eq. 2 (its scale / zero point from a
    range), Eq. 4 (symmetric weight scale), Eq. 5 (the two backward products),
    Eq. 6 (block importance = mean magnitude), Alg. 1 (weight gradient only for
    the unfrozen rows `id`), Sec. 3.4 (k = floor(r * C_out)) are written out as
    printed.
  * Eq. 3 as printed has its two bounds swapped (it would be a constant); it is
    read as clamp(round(W/S_w), -(2^(b-1)-1), +(2^(b-1)-1)), the range Eq. 4's
    denominator implies.
  * round-to-nearest is taken with ties to even.
  * The integer code is decided on the single-precision quotient x/s (inputs are
    fp32 or bf16 values, scales are fp32); everything after the codes is fp64.
  * The paper trains S_x, Z_x, S_w with the straight-through estimator but prints
    no formula for their gradients.  They are derived here by differentiating
    Eq. 1 / Eq. 3 with d round(u)/du := 1 (see grad_* below).  These functions are
    pinned by finite differences of that surrogate and by autograd, not by a
    formula in the paper.
  * Optimizer step of Alg. 1: the unfrozen weight rows keep the full-precision run's
    optimizer (SGD with momentum in the paper's CNN experiments), the quantization
    parameters are always trained with Adam (Sec. 4 "Setup").  The paper gives no betas
    or eps (the caller passes them) and does not say what happens to the Adam state of a
    frozen channel; it is read here as: one Adam state and step count per channel, which
    advance only in the steps that update that channel.
  * Non-integer Z_x and degenerate ranges (max == min, all-zero weight row) are
    this build's reading only: parity unpinned by the paper for those two cases.

Shapes follow the paper's Linear convention Y = X_q W_q^T with W [C_out, C_in];
conv tensors are NHWC (activations) and OHWI (weights).
"""
from __future__ import annotations

import numpy as np

F32 = np.float32


# --------------------------------------------------------------------------
# Quantizer parameters
# --------------------------------------------------------------------------
def act_qparams_minmax(X: np.ndarray, bits: int = 8):
    """Eq. 2 with the MinMax observer range [alpha, beta] = [min X, max X] (Sec. 4,
    PTQ baseline).  Returns (S_x, Z_x) as fp32 numbers; each operation is a
    single-precision operation because S_x decides integer codes downstream."""
    x = np.asarray(X, dtype=F32)
    alpha, beta = F32(x.min()), F32(x.max())
    qmax = F32(2 ** bits - 1)
    s = F32(F32(beta - alpha) / qmax)
    if not (s > 0):  # beta == alpha: reading for the degenerate range
        s = F32(1.0)
    z = F32(0.0) - F32(np.rint(F32(alpha / s)))
    return s, F32(z)


def weight_scale_minmax(W: np.ndarray, bits: int = 8) -> np.ndarray:
    """Eq. 4 per output channel (row): S_w[c] = max_j |W[c, j]| / (2^(b-1) - 1)."""
    w = np.asarray(W, dtype=F32).reshape(W.shape[0], -1)
    qw = F32(2 ** (bits - 1) - 1)
    s = (np.abs(w).max(axis=1).astype(F32) / qw).astype(F32)
    s[~(s > 0)] = F32(1.0)  # all-zero row: reading for the degenerate range
    return s


# --------------------------------------------------------------------------
# Fake-quant forward
# --------------------------------------------------------------------------
def fakequant_act(X: np.ndarray, S_x, Z_x, bits: int = 8):
    """Eq. 1.  Returns (codes int64, in-range mask bool, X_q fp64).

    mask is true where the un-clamped code round(X/S_x)+Z_x lies in the closed
    interval [0, 2^b - 1] (a value exactly on a bound is not clipped)."""
    x = np.asarray(X, dtype=F32)
    s = F32(S_x)
    z = np.rint(np.float64(Z_x))
    qmax = float(2 ** bits - 1)
    q32 = (x / s).astype(F32)                       # correctly rounded fp32 quotient
    c = np.rint(q32.astype(np.float64)) + z         # un-clamped code
    mask = (c >= 0.0) & (c <= qmax)
    codes = np.minimum(np.maximum(c, 0.0), qmax)
    Xq = np.float64(s) * (codes - z)
    return codes.astype(np.int64), mask, Xq


def fakequant_weight(W: np.ndarray, S_w: np.ndarray, bits: int = 8):
    """Eq. 3 (bounds un-swapped), Z_w = 0, one scale per output channel.
    Returns (codes int64, in-range mask bool, W_q fp64), shaped like W."""
    w = np.asarray(W, dtype=F32)
    s = np.asarray(S_w, dtype=F32).reshape((-1,) + (1,) * (w.ndim - 1))
    qw = float(2 ** (bits - 1) - 1)
    v32 = (w / s).astype(F32)
    r = np.rint(v32.astype(np.float64))
    mask = np.abs(r) <= qw
    codes = np.minimum(np.maximum(r, -qw), qw)
    Wq = s.astype(np.float64) * codes
    return codes.astype(np.int64), mask, Wq


# --------------------------------------------------------------------------
# Importance and selection
# --------------------------------------------------------------------------
def channel_importance(W: np.ndarray) -> np.ndarray:
    """Eq. 6 with one block per output channel: I[c] = mean_j |W[c, j]| over all
    C_in (x kh x kw) entries of the master weights."""
    w = np.asarray(W, dtype=np.float64).reshape(W.shape[0], -1)
    return np.abs(w).sum(axis=1) / w.shape[1]


def k_from_ratio(c_out: int, num: int, den: int) -> int:
    """Sec. 3.4: floor(r * C_out) rows are updated, r = num/den, in integers."""
    return (int(c_out) * int(num)) // int(den)


def top_k_channels(importance: np.ndarray, k: int) -> np.ndarray:
    """Top-K (Sec. 3.2): the k largest importances; equal scores go to the lower
    index; the result is returned in ascending index order."""
    I = np.asarray(importance, dtype=np.float64)
    c = np.arange(I.shape[0])
    order = np.lexsort((c, -I))          # primary: I descending, secondary: index ascending
    return np.sort(order[:k]).astype(np.int64)


def network_top_k(importances, k_total: int):
    """EfQAT-CWPN (Table 2): one Top-K over the channel importances of all layers
    together; returns the per-layer ascending index lists.  Ties go to the earlier
    layer, then the lower channel index."""
    sizes = [len(i) for i in importances]
    flat = np.concatenate([np.asarray(i, dtype=np.float64) for i in importances])
    sel = top_k_channels(flat, k_total)
    out, base = [], 0
    for n in sizes:
        s = sel[(sel >= base) & (sel < base + n)] - base
        out.append(s.astype(np.int64))
        base += n
    return out


def layer_top_k(weights, k_layers: int):
    """EfQAT-LWPN (Table 2): the block is a whole layer, its importance the mean |w| over
    all of the layer's weights (Eq. 6 with one block per layer); the k_layers most
    important layers are unfrozen entirely, the others frozen entirely.  Returns the
    ascending list of unfrozen layers and the per-layer channel count (C_out or 0).
    Ties go to the earlier layer."""
    imp = np.array([np.mean(np.abs(np.asarray(w, dtype=np.float64))) for w in weights])
    sel = top_k_channels(imp, k_layers)
    chosen = set(int(i) for i in sel)
    k_per_layer = np.array([np.asarray(w).shape[0] if l in chosen else 0 for l, w in enumerate(weights)],
                           dtype=np.int64)
    return sel, k_per_layer, imp


def bias_grad(dY):
    """Gradient of a bias added per output channel, Y = X_q W_q^T + b: db[c] = sum_t dY[t, c].
    Biases stay unfrozen whatever the update fraction (Sec. 3.4, Alg. 1 optimizer step)."""
    d = np.asarray(dY, dtype=np.float64)
    return d.reshape(-1, d.shape[-1]).sum(axis=0)


def sgd_step_rows(W, idx, dW_rows, lr_w, momentum=0.0, weight_decay=0.0, mom_w=None):
    """Optimizer step of Alg. 1 on the unfrozen weight channels only.  The network parameters keep the
    optimizer of the full-precision run (Sec. 4 "Setup"), which is SGD with momentum and weight decay in
    the paper's CNN experiments; frozen rows and their momentum buffers stay as they are:
        g = dW + wd * W;  buf = mu * buf + g (if mu != 0);  W -= lr_w * buf
    Returns new copies (W, mom_w) in fp64."""
    W = np.array(W, dtype=np.float64)
    mw = None if mom_w is None else np.array(mom_w, dtype=np.float64)
    idx = np.asarray(idx, dtype=np.int64)
    g = np.asarray(dW_rows, dtype=np.float64) + weight_decay * W[idx]
    if momentum != 0.0:
        mw[idx] = momentum * mw[idx] + g
        g = mw[idx]
    W[idx] = W[idx] - lr_w * g
    return W, mw


def adam_step_rows(S_w, idx, dS_w_rows, lr, m, v, t, beta1=0.9, beta2=0.999, eps=1e-8):
    """Optimizer step of Alg. 1 on the weight scales of the unfrozen channels.  Quantization parameters are
    always trained with Adam (Sec. 4 "Setup"); a frozen channel's scale is not updated (Sec. 3.2,
    "Quantization Granularity"), so every channel carries its own first / second moment and its own step
    count t[c], and only the channels in idx advance:
        t += 1;  m = b1 m + (1 - b1) g;  v = b2 v + (1 - b2) g^2
        S -= lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps)
    (Adam as published, with bias correction, no weight decay; the paper names no betas or eps, the
    defaults of the Adam paper are the caller's to pass).  Returns new copies (S_w, m, v, t)."""
    S = np.array(S_w, dtype=np.float64)
    m = np.array(m, dtype=np.float64); v = np.array(v, dtype=np.float64)
    t = np.array(t, dtype=np.int64)
    idx = np.asarray(idx, dtype=np.int64)
    g = np.asarray(dS_w_rows, dtype=np.float64)
    t[idx] += 1
    m[idx] = beta1 * m[idx] + (1.0 - beta1) * g
    v[idx] = beta2 * v[idx] + (1.0 - beta2) * g * g
    m_hat = m[idx] / (1.0 - np.power(float(beta1), t[idx]))
    v_hat = v[idx] / (1.0 - np.power(float(beta2), t[idx]))
    S[idx] = S[idx] - lr * m_hat / (np.sqrt(v_hat) + eps)
    return S, m, v, t


# --------------------------------------------------------------------------
# Quantizer-parameter gradients (derived; see module header)
# --------------------------------------------------------------------------
def grad_act_qparams(dXq, X, codes, mask, S_x, Z_x):
    """d/dS_x and d/dZ_x of X_q = S_x * (clamp(round(X/S_x) + Z_x, 0, Q) - Z_x) with the
    straight-through estimator.  In range:  dX_q/dS_x = round(X/S_x) - X/S_x,
    dX_q/dZ_x = 0.  Clipped:  dX_q/dS_x = code - Z_x,  dX_q/dZ_x = -S_x."""
    s = np.float64(F32(S_x))
    z = np.rint(np.float64(Z_x))
    x = np.asarray(X, dtype=np.float64)
    q = codes.astype(np.float64) - z
    g = np.where(mask, q - x / s, q)
    dS = float(np.sum(dXq * g))
    dZ = float(np.sum(np.where(mask, 0.0, -s) * dXq))
    return dS, dZ


def grad_weight_scale(dWq_rows, W_rows, codes_rows, mask_rows, S_w_rows):
    """d/dS_w[c] of W_q[c,:] = S_w[c] * clamp(round(W[c,:]/S_w[c]), -Q, Q) under STE:
    in range code - W/S_w, clipped code.  One value per given row."""
    n = dWq_rows.shape[0]
    s = np.asarray(S_w_rows, dtype=np.float64).reshape(n, -1)
    w = np.asarray(W_rows, dtype=np.float64).reshape(n, -1)
    c = codes_rows.astype(np.float64).reshape(n, -1)
    m = mask_rows.reshape(n, -1)
    g = np.where(m, c - w / s, c)
    return np.sum(dWq_rows.reshape(n, -1) * g, axis=1)


# --------------------------------------------------------------------------
# Linear forward (Sec. 3.1, "Computational Bottleneck of QAT Schemes")
# --------------------------------------------------------------------------
def linear_fwd(X, S_x, Z_x, a_bits, W, S_w, w_bits):
    """Y = X_q W_q^T with the fake-quantised operands of Eq. 1 / Eq. 3 (PyTorch Linear convention)."""
    _, _, Xq = fakequant_act(X, S_x, Z_x, a_bits)
    _, _, Wq = fakequant_weight(W, S_w, w_bits)
    return Xq @ Wq.T


# --------------------------------------------------------------------------
# Linear backward (Eq. 5, Alg. 1 backward step)
# --------------------------------------------------------------------------
def linear_bwd(dY, X, S_x, Z_x, a_bits, W, S_w, w_bits, idx):
    """Backward of Y = X_q W_q^T for one layer, weight gradient restricted to the
    rows in `idx` (ascending list of unfrozen output channels).

    Returns dict with
      dX   [T, C_in]      = (dY W_q) masked by the activation clip mask (STE)
      dXq  [T, C_in]      = dY W_q                         (Eq. 5 left, all channels)
      dW   [C_out, C_in]  rows idx = (dY^T X_q)[idx] masked by the weight clip mask,
                          other rows zero                  (Alg. 1; Eq. 5 right restricted)
      dS_w [C_out]        rows idx only, others zero       (Sec. 3.2, quantization granularity)
      dS_x, dZ_x          scalars
    """
    dY = np.asarray(dY, dtype=np.float64)
    idx = np.asarray(idx, dtype=np.int64)
    xc, xm, Xq = fakequant_act(X, S_x, Z_x, a_bits)
    wc, wm, Wq = fakequant_weight(W, S_w, w_bits)

    dXq = dY @ Wq                                   # all output channels, always
    dX = np.where(xm, dXq, 0.0)
    dS_x, dZ_x = grad_act_qparams(dXq, X, xc, xm, S_x, Z_x)

    c_out, c_in = W.shape
    dW = np.zeros((c_out, c_in), dtype=np.float64)
    dS_w = np.zeros(c_out, dtype=np.float64)
    dWq_sel = np.zeros((idx.size, c_in), dtype=np.float64)
    if idx.size:
        dWq_sel = dY[:, idx].T @ Xq                 # step 1-2 of Sec. 4 "Practical Speedups"
        dW[idx] = np.where(wm[idx], dWq_sel, 0.0)   # step 3: rows written back
        dS_w[idx] = grad_weight_scale(dWq_sel, W[idx], wc[idx], wm[idx], np.asarray(S_w)[idx])
    # dWq_sel: the un-masked rows idx of the weight gradient (an intermediate, handed out for error scales in tests)
    return dict(dX=dX, dXq=dXq, dW=dW, dS_w=dS_w, dS_x=dS_x, dZ_x=dZ_x, dWq_sel=dWq_sel,
                x_codes=xc, x_mask=xm, w_codes=wc, w_mask=wm)


# --------------------------------------------------------------------------
# Convolution backward (same two contractions, Eq. 8 shapes)
# --------------------------------------------------------------------------
def conv_out_size(n_in: int, k: int, stride: int, pad: int) -> int:
    return (n_in + 2 * pad - k) // stride + 1


def conv_bwd(dY, X, S_x, Z_x, a_bits, W, S_w, w_bits, idx, stride=1, pad=0):
    """Backward of the convolution Y[n,ho,wo,co] = sum_{kh,kw,ci}
    X_q[n, ho*s+kh-p, wo*s+kw-p, ci] * W_q[co,kh,kw,ci] (zero outside the image).

    X is NHWC, W is OHWI, dY is [N, Ho, Wo, C_out].  Same outputs as linear_bwd with
    dW / masks shaped like W.  The sums over (kh, kw) are written as a loop over
    kernel taps; the sum over channels / pixels inside each tap is a matrix product.
    """
    dY = np.asarray(dY, dtype=np.float64)
    idx = np.asarray(idx, dtype=np.int64)
    N, H, Wd, c_in = X.shape
    c_out, KH, KW, _ = W.shape
    Ho, Wo = conv_out_size(H, KH, stride, pad), conv_out_size(Wd, KW, stride, pad)
    assert dY.shape == (N, Ho, Wo, c_out)
    xc, xm, Xq = fakequant_act(X, S_x, Z_x, a_bits)
    wc, wm, Wq = fakequant_weight(W, S_w, w_bits)

    # zero-padded copies so every tap is a plain strided slice
    Xp = np.zeros((N, H + 2 * pad, Wd + 2 * pad, c_in), dtype=np.float64)
    Xp[:, pad:pad + H, pad:pad + Wd, :] = Xq
    dXp = np.zeros_like(Xp)
    dWq_sel = np.zeros((idx.size, KH, KW, c_in), dtype=np.float64)
    dY2 = dY.reshape(-1, c_out)
    dYsel = dY2[:, idx]
    for kh in range(KH):
        for kw in range(KW):
            hs = slice(kh, kh + (Ho - 1) * stride + 1, stride)
            ws = slice(kw, kw + (Wo - 1) * stride + 1, stride)
            # input gradient: every output channel contributes
            dXp[:, hs, ws, :] += (dY2 @ Wq[:, kh, kw, :]).reshape(N, Ho, Wo, c_in)
            # weight gradient: only the unfrozen output channels
            if idx.size:
                dWq_sel[:, kh, kw, :] = dYsel.T @ Xp[:, hs, ws, :].reshape(-1, c_in)
    dXq = dXp[:, pad:pad + H, pad:pad + Wd, :]
    dX = np.where(xm, dXq, 0.0)
    dS_x, dZ_x = grad_act_qparams(dXq, X, xc, xm, S_x, Z_x)

    dW = np.zeros(W.shape, dtype=np.float64)
    dS_w = np.zeros(c_out, dtype=np.float64)
    if idx.size:
        dW[idx] = np.where(wm[idx], dWq_sel, 0.0)
        dS_w[idx] = grad_weight_scale(dWq_sel, W[idx], wc[idx], wm[idx], np.asarray(S_w)[idx])
    return dict(dX=dX, dXq=dXq, dW=dW, dS_w=dS_w, dS_x=dS_x, dZ_x=dZ_x, dWq_sel=dWq_sel,
                x_codes=xc, x_mask=xm, w_codes=wc, w_mask=wm)


# --------------------------------------------------------------------------
# Operation-count model (Eq. 7 / Eq. 8), used only for reporting
# --------------------------------------------------------------------------
def ops_bwd_linear(c_in: int, c_out: int, k: int) -> int:
    """Eq. 7: multiply-accumulates per token, C_in*k (weight grad) + C_in*C_out."""
    return c_in * k + c_in * c_out


def ops_bwd_conv(c_in: int, c_out: int, k: int, ksize: int, h_out: int, w_out: int) -> int:
    """Eq. 8: per image, k^2 C_in (k_sel + C_out) H_out W_out."""
    return ksize * ksize * c_in * (k + c_out) * h_out * w_out

"""Pins for the CPU oracle: closed forms, invariants, brute force, finite differences
and library routines (torch autograd / conv2d), none of which re-use the oracle's own
formulas.  CPU only."""
import os

import numpy as np
import pytest
import torch

from oracle import efqat_oracle as orc
from workloads import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    out = []
    for line in open(os.path.join(GOLD, name)):
        line = line.split("#")[0].strip()
        if line:
            out.append([int(t) for t in line.split()])
    return out


# ------------------------------------------------------------------ Eq. 1 / Eq. 2
def test_act_on_grid_roundtrip_and_clip():
    S, Z, bits = 0.125, 10.0, 8          # power-of-two scale: every product below is exact
    q = np.arange(256, dtype=np.float64)
    x = (S * (q - Z)).astype(np.float32)
    codes, mask, xq = orc.fakequant_act(x, S, Z, bits)
    assert np.array_equal(codes, q.astype(np.int64))
    assert mask.all()                    # includes both bounds: on-bound is not clipped
    assert np.array_equal(xq, x.astype(np.float64))
    lo = np.float32(S * (-1 - Z)); hi = np.float32(S * (256 - Z))
    codes, mask, xq = orc.fakequant_act(np.array([lo, hi, -1e30, 1e30], np.float32), S, Z, bits)
    assert codes.tolist() == [0, 255, 0, 255] and not mask.any()
    assert xq.tolist() == [S * (0 - Z), S * (255 - Z), S * (0 - Z), S * (255 - Z)]


def test_act_ties_round_to_even():
    S = 0.25
    x = np.array([0.5, 1.5, 2.5, 3.5, -0.5, -1.5, 6.5], np.float32) * np.float32(S)
    codes, mask, _ = orc.fakequant_act(x, S, 8.0, 8)
    assert codes.tolist() == [8 + 0, 8 + 2, 8 + 2, 8 + 4, 8 - 0, 8 - 2, 8 + 6]
    assert mask.all()


@pytest.mark.parametrize("bits", [4, 8])
def test_act_minmax_init_closed_form(bits):
    Q = 2 ** bits - 1
    S = 0.0625
    x = (S * (np.arange(Q + 1) - 37.0)).astype(np.float32)      # range spans exactly Q steps
    s, z = orc.act_qparams_minmax(x, bits)
    assert s == np.float32(S) and z == 37.0
    codes, mask, _ = orc.fakequant_act(x, s, z, bits)
    assert codes[0] == 0 and codes[-1] == Q and mask.all()


def test_act_minmax_random_extremes():
    x = synth.normal(11, 0, (64, 33)).astype(np.float32)
    s, z = orc.act_qparams_minmax(x, 8)
    assert abs(float(s) - (float(x.max()) - float(x.min())) / 255.0) <= 1e-6 * float(s)
    codes, mask, xq = orc.fakequant_act(x, s, z, 8)
    assert codes.flat[x.argmin()] == 0
    assert codes.flat[x.argmax()] >= 254
    # quantization error of in-range values is at most half a step
    assert np.all(np.abs(xq - x)[mask] <= 0.5 * float(s) * (1 + 1e-6))
    assert z == np.rint(z)


def test_degenerate_ranges_reading():
    s, z = orc.act_qparams_minmax(np.full((4, 4), 3.0, np.float32), 8)
    assert s == 1.0 and z == -3.0
    sw = orc.weight_scale_minmax(np.zeros((3, 5), np.float32), 8)
    assert np.all(sw == 1.0)
    codes, mask, wq = orc.fakequant_weight(np.zeros((3, 5), np.float32), sw, 8)
    assert not codes.any() and mask.all() and not wq.any()


# ------------------------------------------------------------------ Eq. 3 / Eq. 4
@pytest.mark.parametrize("bits", [4, 8])
def test_weight_symmetric_properties(bits):
    Q = 2 ** (bits - 1) - 1
    W = synth.normal(5, 1, (16, 24), std=0.02).astype(np.float32)
    sw = orc.weight_scale_minmax(W, bits)
    assert np.allclose(sw, np.abs(W).max(1) / Q, rtol=1e-6)
    c, m, wq = orc.fakequant_weight(W, sw, bits)
    c2, m2, wq2 = orc.fakequant_weight(-W, sw, bits)
    assert np.array_equal(c2, -c) and np.array_equal(m2, m) and np.array_equal(wq2, -wq)
    assert m.all()                                   # min/max scale clips nothing
    am = np.abs(W).argmax(1)
    assert np.all(np.abs(c[np.arange(16), am]) == Q)  # extreme lands on the last level
    assert np.abs(c).max() <= Q
    assert np.all(np.abs(wq - W) <= 0.5 * sw[:, None] * (1 + 1e-6))


def test_weight_on_grid_and_clip():
    sw = np.array([0.5, 0.25], np.float32)
    W = np.array([[3.0, -3.5, 4.0, 3.25, 0.25], [1.75, -1.75, 2.0, -0.125, 0.375]], np.float32)
    c, m, wq = orc.fakequant_weight(W, sw, 4)        # Q = 7
    assert c.tolist() == [[6, -7, 7, 6, 0], [7, -7, 7, 0, 2]]
    assert m.tolist() == [[True, True, False, True, True], [True, True, False, True, True]]
    assert wq.tolist() == [[3.0, -3.5, 3.5, 3.0, 0.0], [1.75, -1.75, 1.75, 0.0, 0.5]]


# ------------------------------------------------------------------ Eq. 6, Top-K, k
def test_importance_is_mean_abs():
    W = np.array([[1, -2, 3, -4], [0, 0, 0, 8], [-1, -1, -1, -1]], np.float32)
    assert orc.channel_importance(W).tolist() == [2.5, 2.0, 1.0]
    W4 = W.reshape(3, 2, 2, 1)                       # conv block = all of (kh, kw, ci)
    assert orc.channel_importance(W4).tolist() == [2.5, 2.0, 1.0]


def test_k_table_from_paper_formula():
    for c_out, num, den, k in _rows("k_table.txt"):
        assert orc.k_from_ratio(c_out, num, den) == k


def _brute_topk(I, k):
    chosen, used = [], set()
    for _ in range(k):
        best = None
        for c in range(len(I)):
            if c in used:
                continue
            if best is None or I[c] > I[best]:       # strict: earlier index wins ties
                best = c
        used.add(best); chosen.append(best)
    return sorted(chosen)


def test_topk_bruteforce_and_ties():
    rng = np.random.default_rng(3)
    for n in (1, 2, 7, 33):
        I = rng.integers(0, 5, size=n).astype(np.float64)     # many exact ties
        for k in {0, 1, n // 2, max(n - 1, 0), n}:
            assert orc.top_k_channels(I, k).tolist() == _brute_topk(I, k)
    I = np.array([1.0, 3.0, 3.0, 2.0, 3.0])
    assert orc.top_k_channels(I, 2).tolist() == [1, 2]
    assert orc.top_k_channels(I, 4).tolist() == [1, 2, 3, 4]
    assert orc.top_k_channels(I, 0).tolist() == []


def test_network_topk_balances_across_layers():
    a = np.array([0.1, 0.9, 0.5]); b = np.array([0.7, 0.2]); c = np.array([0.05, 0.06])
    sel = orc.network_top_k([a, b, c], 3)
    assert [s.tolist() for s in sel] == [[1, 2], [0], []]      # third layer fully frozen
    sel = orc.network_top_k([a, b, c], 7)
    assert [s.tolist() for s in sel] == [[0, 1, 2], [0, 1], [0, 1]]


def test_layer_topk_lwpn():
    # Table 2, LWPN: whole layers are the blocks.  Layers of different shapes; importances set by
    # construction (constant |w| per layer), so the ranking is known without the oracle.
    rng = np.random.default_rng(5)
    mags = [0.3, 0.9, 0.1, 0.9, 0.5]
    shapes = [(4, 6), (3, 5), (8, 2), (2, 9), (5, 5)]
    ws = [m * rng.choice([-1.0, 1.0], size=sh) for m, sh in zip(mags, shapes)]
    sel, kpl, imp = orc.layer_top_k(ws, 3)
    np.testing.assert_allclose(imp, mags, rtol=1e-15)
    assert list(sel) == [1, 3, 4]                       # 0.9, 0.9 (tie -> both), then 0.5
    assert list(kpl) == [0, 3, 0, 2, 5]
    sel, kpl, _ = orc.layer_top_k(ws, 1)
    assert list(sel) == [1] and list(kpl) == [0, 3, 0, 0, 0]   # tie goes to the earlier layer
    sel, kpl, _ = orc.layer_top_k(ws, 0)
    assert len(sel) == 0 and not kpl.any()
    sel, kpl, _ = orc.layer_top_k(ws, 5)
    assert list(kpl) == [4, 3, 8, 2, 5]
    # the layer importance is the mean over all weights = mean of the channel means (equal block sizes)
    w = rng.normal(size=(7, 11))
    _, _, imp = orc.layer_top_k([w], 1)
    assert abs(imp[0] - orc.channel_importance(w).mean()) < 1e-15


def test_bias_grad_is_gradient_of_bias():
    # db is the derivative of sum(dY * (Y0 + b)) with respect to b: check by exact finite differences
    # (the function is linear in b) and against torch autograd of a broadcast add.
    rng = np.random.default_rng(6)
    dY = rng.normal(size=(37, 5))
    db = orc.bias_grad(dY)
    for c in range(5):
        e = np.zeros(5); e[c] = 1.0
        np.testing.assert_allclose(np.sum(dY * (0.0 + e[None, :])), db[c], rtol=1e-13)
    y0 = torch.zeros(37, 5, dtype=torch.float64)
    b = torch.zeros(5, dtype=torch.float64, requires_grad=True)
    (y0 + b).backward(torch.from_numpy(dY))
    np.testing.assert_allclose(db, b.grad.numpy(), rtol=1e-13)
    # conv-shaped dY [N, Ho, Wo, C]: sum over every axis but the channel
    d4 = rng.normal(size=(2, 3, 4, 5))
    np.testing.assert_allclose(orc.bias_grad(d4), d4.sum(axis=(0, 1, 2)), rtol=1e-13)


@pytest.mark.parametrize("momentum,wd", [(0.0, 0.0), (0.9, 0.0), (0.9, 5e-4), (0.0, 1e-2)])
def test_sgd_step_rows_matches_torch_sgd_on_the_unfrozen_rows(momentum, wd):
    # torch.optim.SGD over a parameter that holds only the unfrozen rows (two steps, so the momentum buffer is used);
    # frozen rows must come back untouched
    rng = np.random.default_rng(11)
    W = rng.normal(size=(9, 5))
    idx = np.array([1, 4, 7])
    pw = torch.tensor(W[idx], dtype=torch.float64, requires_grad=True)
    opt_w = torch.optim.SGD([pw], lr=0.1, momentum=momentum, weight_decay=wd)
    mw = np.zeros_like(W) if momentum else None
    Wc = W.copy()
    for step in range(2):
        dW = rng.normal(size=(3, 5))
        pw.grad = torch.tensor(dW)
        opt_w.step()
        Wc, mw = orc.sgd_step_rows(Wc, idx, dW, 0.1, momentum, wd, mw)
    np.testing.assert_allclose(Wc[idx], pw.detach().numpy(), rtol=1e-13, atol=1e-15)
    frozen = np.setdiff1d(np.arange(9), idx)
    assert np.array_equal(Wc[frozen], W[frozen])
    if momentum:
        assert not mw[frozen].any()


@pytest.mark.parametrize("betas,eps", [((0.9, 0.999), 1e-8), ((0.8, 0.95), 1e-6)])
def test_adam_step_rows_matches_torch_adam_on_the_unfrozen_rows(betas, eps):
    # Quantization parameters are trained with Adam (Sec. 4 "Setup").  torch.optim.Adam over a parameter that holds
    # only the unfrozen scales, five steps with the same idx (every selected channel then has the optimizer's own step
    # count); frozen channels and their state must come back untouched
    rng = np.random.default_rng(12)
    S = rng.uniform(0.5, 1.5, size=9)
    idx = np.array([0, 3, 4, 8])
    ps = torch.tensor(S[idx], dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([ps], lr=1e-2, betas=betas, eps=eps)
    Sc, m, v, t = S.copy(), np.zeros(9), np.zeros(9), np.zeros(9, dtype=np.int64)
    for step in range(5):
        g = rng.normal(size=4) * 10.0 ** rng.integers(-3, 2)
        ps.grad = torch.tensor(g)
        opt.step()
        Sc, m, v, t = orc.adam_step_rows(Sc, idx, g, 1e-2, m, v, t, betas[0], betas[1], eps)
    np.testing.assert_allclose(Sc[idx], ps.detach().numpy(), rtol=1e-12, atol=1e-15)
    st = opt.state[ps]
    np.testing.assert_allclose(m[idx], st["exp_avg"].numpy(), rtol=1e-12, atol=1e-300)
    np.testing.assert_allclose(v[idx], st["exp_avg_sq"].numpy(), rtol=1e-12, atol=1e-300)
    frozen = np.setdiff1d(np.arange(9), idx)
    assert np.array_equal(Sc[frozen], S[frozen]) and not m[frozen].any() and not v[frozen].any()
    assert t[idx].tolist() == [5] * 4 and not t[frozen].any()


def test_adam_step_rows_with_a_changing_selection_is_one_adam_per_channel():
    # The selected set changes between steps (channel importance is re-evaluated, Sec. 3.2 "Freezing Frequency"): a
    # channel's scale, moments and step count move only in the steps that select it, i.e. every channel behaves like a
    # torch.optim.Adam of its own that is stepped only then
    rng = np.random.default_rng(13)
    C = 6
    S = rng.uniform(0.5, 1.5, size=C)
    ps = [torch.tensor([S[c]], dtype=torch.float64, requires_grad=True) for c in range(C)]
    opts = [torch.optim.Adam([p], lr=3e-3) for p in ps]
    Sc, m, v, t = S.copy(), np.zeros(C), np.zeros(C), np.zeros(C, dtype=np.int64)
    picks = [[0, 2, 5], [2, 3], [0, 1, 2, 3, 4, 5], [5], [1, 2]]
    for idx in picks:
        g = rng.normal(size=len(idx))
        for j, c in enumerate(idx):
            ps[c].grad = torch.tensor([g[j]])
            opts[c].step()
        Sc, m, v, t = orc.adam_step_rows(Sc, np.array(idx), g, 3e-3, m, v, t)
    np.testing.assert_allclose(Sc, np.array([p.item() for p in ps]), rtol=1e-12)
    assert t.tolist() == [sum(c in p for p in picks) for c in range(C)]


def test_ops_model_golden():
    rows = _rows("ops_bound.txt")
    for r in rows:
        if len(r) == 5:
            c_in, c_out, num, den, ops = r
            k = orc.k_from_ratio(c_out, num, den)
            assert orc.ops_bwd_linear(c_in, c_out, k) == ops
            assert ops * den <= (den + num) * c_in * c_out
        else:
            ks, c_in, c_out, num, den, ho, wo, ops = r
            k = orc.k_from_ratio(c_out, num, den)
            assert orc.ops_bwd_conv(c_in, c_out, k, ks, ho, wo) == ops
    # r = 0 is exactly half of r = 1 (the 2x bound)
    assert 2 * orc.ops_bwd_linear(768, 3072, 0) == orc.ops_bwd_linear(768, 3072, 3072)


# ------------------------------------------------------------------ Eq. 5: the two products
def _tiny_layer(seed=7, T=5, c_in=4, c_out=3, shrink=1.0, a_bits=8, w_bits=8):
    X, W, dY = synth.linear_layer(seed, T, c_in, c_out, act_dtype="f32", w_std=0.5)
    sx, zx = orc.act_qparams_minmax(X, a_bits)
    sw = orc.weight_scale_minmax(W, w_bits)
    return X, W, dY, np.float32(sx * np.float32(shrink)), zx, (sw * np.float32(shrink)).astype(np.float32)


def test_eq5_bruteforce_triple_loop():
    X, W, dY, sx, zx, sw = _tiny_layer()
    out = orc.linear_bwd(dY, X, sx, zx, 8, W, sw, 8, np.arange(3))
    _, _, Xq = orc.fakequant_act(X, sx, zx, 8)
    _, _, Wq = orc.fakequant_weight(W, sw, 8)
    T, c_in = X.shape; c_out = W.shape[0]
    for t in range(T):
        for i in range(c_in):
            acc = 0.0
            for c in range(c_out):
                acc += float(dY[t, c]) * Wq[c, i]
            assert abs(acc - out["dXq"][t, i]) < 1e-12
    for c in range(c_out):
        for i in range(c_in):
            acc = 0.0
            for t in range(T):
                acc += float(dY[t, c]) * Xq[t, i]
            assert abs(acc - out["dW"][c, i]) < 1e-12      # min/max init: nothing masked


def test_eq5_is_gradient_of_forward_by_finite_differences():
    # L = <dY, Xq Wq^T> is bilinear, so central differences are exact up to rounding.
    X, W, dY, sx, zx, sw = _tiny_layer(seed=8)
    out = orc.linear_bwd(dY, X, sx, zx, 8, W, sw, 8, np.arange(3))
    _, _, Xq = orc.fakequant_act(X, sx, zx, 8)
    _, _, Wq = orc.fakequant_weight(W, sw, 8)
    L = lambda a, b: float(np.sum(dY.astype(np.float64) * (a @ b.T)))
    h = 1e-3
    for t in range(X.shape[0]):
        for i in range(X.shape[1]):
            E = np.zeros_like(Xq); E[t, i] = h
            fd = (L(Xq + E, Wq) - L(Xq - E, Wq)) / (2 * h)
            assert abs(fd - out["dXq"][t, i]) < 1e-8
    for c in range(W.shape[0]):
        for i in range(W.shape[1]):
            E = np.zeros_like(Wq); E[c, i] = h
            fd = (L(Xq, Wq + E) - L(Xq, Wq - E)) / (2 * h)
            assert abs(fd - out["dW"][c, i]) < 1e-8


# ------------------------------------------------------------------ STE masks and qparam grads
def _torch_ste_linear(X, W, dY, sx, zx, sw, a_bits, w_bits):
    """Library pin: torch autograd through the usual straight-through construction
    u + (round(u) - u).detach().  Nothing here comes from the oracle."""
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True)
    Xt, Wt, St, Zt, Swt = t(X), t(W), t(sx), t(zx), t(sw)
    ste = lambda u: u + (torch.round(u) - u).detach()
    Qa, Qw = 2 ** a_bits - 1, 2 ** (w_bits - 1) - 1
    Xq = St * (torch.clamp(ste(Xt / St) + ste(Zt), 0, Qa) - ste(Zt))
    Wq = Swt[:, None] * torch.clamp(ste(Wt / Swt[:, None]), -Qw, Qw)
    L = (torch.tensor(np.asarray(dY, dtype=np.float64)) * (Xq @ Wq.T)).sum()
    L.backward()
    return Xt.grad.numpy(), Wt.grad.numpy(), St.grad.item(), Zt.grad.item(), Swt.grad.numpy()


@pytest.mark.parametrize("shrink,a_bits,w_bits", [(1.0, 8, 8), (0.6, 8, 8), (0.7, 8, 4), (0.5, 4, 4)])
def test_backward_matches_autograd_of_ste_surrogate(shrink, a_bits, w_bits):
    X, W, dY, sx, zx, sw = _tiny_layer(seed=21, T=9, c_in=7, c_out=6, shrink=shrink,
                                       a_bits=a_bits, w_bits=w_bits)
    out = orc.linear_bwd(dY, X, sx, zx, a_bits, W, sw, w_bits, np.arange(6))
    gX, gW, gS, gZ, gSw = _torch_ste_linear(X, W, dY, sx, zx, sw, a_bits, w_bits)
    if shrink < 1.0:
        assert (~out["x_mask"]).any() and (~out["w_mask"]).any()   # clipped branch exercised
    np.testing.assert_allclose(out["dX"], gX, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(out["dW"], gW, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(out["dS_w"], gSw, rtol=1e-9, atol=1e-10)
    assert abs(out["dS_x"] - gS) <= 1e-9 * max(1.0, abs(gS))
    assert abs(out["dZ_x"] - gZ) <= 1e-9 * max(1.0, abs(gZ))


def test_qparam_grads_by_finite_differences_of_surrogate():
    # Freeze the rounding residual delta = round(X/S) - X/S at the base point and
    # differentiate S' * (clamp(X/S' + delta + Z', 0, Q) - Z') numerically.
    X, W, dY, sx, zx, sw = _tiny_layer(seed=33, T=8, c_in=6, c_out=5, shrink=0.6)
    out = orc.linear_bwd(dY, X, sx, zx, 8, W, sw, 8, np.arange(5))
    X64, W64, dY64 = X.astype(np.float64), W.astype(np.float64), dY.astype(np.float64)
    s0, z0, sw0 = float(sx), float(zx), sw.astype(np.float64)
    dlt = np.rint((X / sx).astype(np.float32).astype(np.float64)) - X64 / s0
    dltw = np.rint((W / sw[:, None]).astype(np.float32).astype(np.float64)) - W64 / sw0[:, None]
    _, _, Wq = orc.fakequant_weight(W, sw, 8)
    _, _, Xq = orc.fakequant_act(X, sx, zx, 8)

    def L_act(s, z):
        xq = s * (np.clip(X64 / s + dlt + z, 0, 255) - z)
        return float(np.sum(dY64 * (xq @ Wq.T)))

    def L_w(swv):
        wq = swv[:, None] * np.clip(W64 / swv[:, None] + dltw, -127, 127)
        return float(np.sum(dY64 * (Xq @ wq.T)))

    h = 1e-7
    fdS = (L_act(s0 + h, z0) - L_act(s0 - h, z0)) / (2 * h)
    fdZ = (L_act(s0, z0 + 1e-4) - L_act(s0, z0 - 1e-4)) / 2e-4
    assert abs(fdS - out["dS_x"]) <= 1e-5 * max(1.0, abs(fdS))
    assert abs(fdZ - out["dZ_x"]) <= 1e-6 * max(1.0, abs(fdZ))
    for c in range(5):
        e = np.zeros(5); e[c] = 1e-8
        fd = (L_w(sw0 + e) - L_w(sw0 - e)) / 2e-8
        assert abs(fd - out["dS_w"][c]) <= 1e-4 * max(1.0, abs(fd))


def test_ste_mask_identities():
    X, W, dY, sx, zx, sw = _tiny_layer(seed=4, T=12, c_in=9, c_out=8, shrink=0.7)
    out = orc.linear_bwd(dY, X, sx, zx, 8, W, sw, 8, np.arange(8))
    xm, wm = out["x_mask"], out["w_mask"]
    assert np.array_equal(out["dX"][xm], out["dXq"][xm]) and not out["dX"][~xm].any()
    assert not out["dW"][~wm].any()
    # min/max init: every mask is 1, so dX == dXq and dZ_x == 0
    X, W, dY, sx, zx, sw = _tiny_layer(seed=4, T=12, c_in=9, c_out=8)
    out = orc.linear_bwd(dY, X, sx, zx, 8, W, sw, 8, np.arange(8))
    if out["x_mask"].all():
        assert np.array_equal(out["dX"], out["dXq"]) and out["dZ_x"] == 0.0


# ------------------------------------------------------------------ restriction (Alg. 1)
def test_restriction_invariants():
    X, W, dY = synth.linear_layer(2, 40, 24, 32, act_dtype="bf16")
    sx, zx = orc.act_qparams_minmax(X, 8)
    sw = (orc.weight_scale_minmax(W, 4) * np.float32(0.8)).astype(np.float32)
    imp = orc.channel_importance(W)
    full = orc.linear_bwd(dY, X, sx, zx, 8, W, sw, 4, np.arange(32))
    for num, den in [(0, 1), (1, 20), (1, 4), (1, 2), (1, 1)]:
        k = orc.k_from_ratio(32, num, den)
        idx = orc.top_k_channels(imp, k)
        assert len(idx) == k and np.all(np.diff(idx) > 0)
        out = orc.linear_bwd(dY, X, sx, zx, 8, W, sw, 4, idx)
        frozen = np.setdiff1d(np.arange(32), idx)
        assert np.array_equal(out["dW"][idx], full["dW"][idx])
        assert not out["dW"][frozen].any() and not out["dS_w"][frozen].any()
        assert np.array_equal(out["dS_w"][idx], full["dS_w"][idx])
        # the input gradient and activation qparam grads do not depend on r
        assert np.array_equal(out["dX"], full["dX"])
        assert out["dS_x"] == full["dS_x"] and out["dZ_x"] == full["dZ_x"]
        if k == 0:
            assert not out["dW"].any()
        if k == 32:
            assert np.array_equal(out["dW"], full["dW"])
        # the kept rows are the most important ones
        if 0 < k < 32:
            assert imp[idx].min() >= imp[frozen].max()


# ------------------------------------------------------------------ convolution
def _conv_case(seed, N, H, Wd, c_in, c_out, kh, kw, stride, pad, shrink=1.0, w_bits=4):
    X, W, dY = synth.conv_layer(seed, N, H, Wd, c_in, c_out, kh, kw, stride, pad, act_dtype="f32",
                                w_std=0.3)
    sx, zx = orc.act_qparams_minmax(X, 8)
    sw = (orc.weight_scale_minmax(W, w_bits) * np.float32(shrink)).astype(np.float32)
    return X, W, dY, np.float32(sx * np.float32(shrink)), zx, sw


@pytest.mark.parametrize("stride,pad,kh,kw", [(1, 1, 3, 3), (2, 1, 3, 3), (1, 0, 1, 1), (2, 0, 2, 3)])
def test_conv_bruteforce_loops(stride, pad, kh, kw):
    X, W, dY, sx, zx, sw = _conv_case(50, 2, 5, 6, 3, 4, kh, kw, stride, pad)
    idx = np.array([1, 3])
    out = orc.conv_bwd(dY, X, sx, zx, 8, W, sw, 4, idx, stride, pad)
    _, _, Xq = orc.fakequant_act(X, sx, zx, 8)
    _, wm, Wq = orc.fakequant_weight(W, sw, 4)
    N, H, Wd, c_in = X.shape; c_out = W.shape[0]; _, Ho, Wo, _ = dY.shape
    dXq = np.zeros(X.shape); dWq = np.zeros(W.shape)
    for n in range(N):
        for ho in range(Ho):
            for wo in range(Wo):
                for co in range(c_out):
                    g = float(dY[n, ho, wo, co])
                    for a in range(kh):
                        for b in range(kw):
                            h = ho * stride + a - pad; w = wo * stride + b - pad
                            if 0 <= h < H and 0 <= w < Wd:
                                for ci in range(c_in):
                                    dXq[n, h, w, ci] += g * Wq[co, a, b, ci]
                                    dWq[co, a, b, ci] += g * Xq[n, h, w, ci]
    np.testing.assert_allclose(out["dXq"], dXq, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(out["dW"][idx], np.where(wm, dWq, 0)[idx], rtol=1e-12, atol=1e-12)
    assert not out["dW"][[0, 2]].any()


@pytest.mark.parametrize("stride,pad", [(1, 1), (2, 1)])
def test_conv_matches_torch_conv2d_autograd(stride, pad):
    X, W, dY, sx, zx, sw = _conv_case(51, 3, 7, 6, 5, 6, 3, 3, stride, pad, shrink=0.7)
    out = orc.conv_bwd(dY, X, sx, zx, 8, W, sw, 4, np.arange(6), stride, pad)
    assert (~out["x_mask"]).any() and (~out["w_mask"]).any()
    t = lambda a: torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True)
    Xt, Wt, St, Zt, Swt = t(X), t(W), t(sx), t(zx), t(sw)
    ste = lambda u: u + (torch.round(u) - u).detach()
    Xq = St * (torch.clamp(ste(Xt / St) + Zt, 0, 255) - Zt)
    Wq = Swt[:, None, None, None] * torch.clamp(ste(Wt / Swt[:, None, None, None]), -7, 7)
    Y = torch.nn.functional.conv2d(Xq.permute(0, 3, 1, 2), Wq.permute(0, 3, 1, 2), stride=stride,
                                   padding=pad)
    L = (Y.permute(0, 2, 3, 1) * torch.tensor(dY.astype(np.float64))).sum()
    L.backward()
    np.testing.assert_allclose(out["dX"], Xt.grad.numpy(), rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(out["dW"], Wt.grad.numpy(), rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(out["dS_w"], Swt.grad.numpy(), rtol=1e-9, atol=1e-9)
    assert abs(out["dS_x"] - St.grad.item()) <= 1e-9 * max(1.0, abs(St.grad.item()))
    assert abs(out["dZ_x"] - Zt.grad.item()) <= 1e-9 * max(1.0, abs(Zt.grad.item()))


def test_conv_1x1_equals_linear():
    X, W, dY, sx, zx, sw = _conv_case(52, 2, 4, 5, 6, 7, 1, 1, 1, 0, shrink=0.8)
    idx = np.array([0, 2, 5])
    oc = orc.conv_bwd(dY, X, sx, zx, 8, W, sw, 4, idx, 1, 0)
    ol = orc.linear_bwd(dY.reshape(-1, 7), X.reshape(-1, 6), sx, zx, 8, W.reshape(7, 6), sw, 4, idx)
    np.testing.assert_allclose(oc["dX"].reshape(-1, 6), ol["dX"], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oc["dW"].reshape(7, 6), ol["dW"], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oc["dS_w"], ol["dS_w"], rtol=1e-12, atol=1e-13)
    assert abs(oc["dS_x"] - ol["dS_x"]) < 1e-10 and abs(oc["dZ_x"] - ol["dZ_x"]) < 1e-10


# ------------------------------------------------------------------ planted mistakes are caught
def test_pins_catch_planted_mistakes(monkeypatch):
    """Each plausible slip, planted in the oracle on the CPU, must trip a pin above."""
    X, W, dY, sx, zx, sw = _tiny_layer(seed=21, T=9, c_in=7, c_out=6, shrink=0.6)
    ref = _torch_ste_linear(X, W, dY, sx, zx, sw, 8, 8)

    def differs():
        out = orc.linear_bwd(dY, X, sx, zx, 8, W, sw, 8, np.arange(6))
        return not (np.allclose(out["dX"], ref[0], rtol=1e-9, atol=1e-11)
                    and np.allclose(out["dW"], ref[1], rtol=1e-9, atol=1e-11)
                    and abs(out["dS_x"] - ref[2]) < 1e-8 * max(1, abs(ref[2]))
                    and abs(out["dZ_x"] - ref[3]) < 1e-8 * max(1, abs(ref[3]))
                    and np.allclose(out["dS_w"], ref[4], rtol=1e-8, atol=1e-9))

    assert not differs()
    good_act, good_w = orc.grad_act_qparams, orc.grad_weight_scale
    # wrong sign of the zero-point gradient
    monkeypatch.setattr(orc, "grad_act_qparams",
                        lambda *a: (good_act(*a)[0], -good_act(*a)[1]))
    assert differs()
    # dropped -X/S term in the scale gradient
    monkeypatch.setattr(orc, "grad_act_qparams",
                        lambda dXq, X_, c, m, s, z: (float(np.sum(dXq * (c - np.rint(float(z))))),
                                                     good_act(dXq, X_, c, m, s, z)[1]))
    assert differs()
    monkeypatch.setattr(orc, "grad_act_qparams", good_act)
    # weight-scale gradient ignoring the clip mask
    monkeypatch.setattr(orc, "grad_weight_scale",
                        lambda d, w, c, m, s: good_w(d, w, c, np.ones_like(m), s))
    assert differs()
    monkeypatch.setattr(orc, "grad_weight_scale", good_w)
    # floor rounding instead of nearest-even
    good_rint = np.rint
    monkeypatch.setattr(np, "rint", np.floor)
    try:
        bad = orc.fakequant_act(np.array([0.375], np.float32), 0.25, 0.0, 8)[0][0]
    finally:
        monkeypatch.setattr(np, "rint", good_rint)
    assert bad != orc.fakequant_act(np.array([0.375], np.float32), 0.25, 0.0, 8)[0][0]


def test_non_integer_zero_point_reading():
    """Reading (paper silent): the forward uses round(Z_x) and the gradient reaches Z_x
    through that round by STE.  Pinned only against autograd of that same reading."""
    X, W, dY, sx, zx, sw = _tiny_layer(seed=22, T=9, c_in=7, c_out=6, shrink=0.6)
    zf = np.float32(zx + 0.3)
    out = orc.linear_bwd(dY, X, sx, zf, 8, W, sw, 8, np.arange(6))
    ref = orc.linear_bwd(dY, X, sx, zx, 8, W, sw, 8, np.arange(6))
    assert np.array_equal(out["x_codes"], ref["x_codes"]) and out["dZ_x"] == ref["dZ_x"]
    gX, gW, gS, gZ, gSw = _torch_ste_linear(X, W, dY, sx, zf, sw, 8, 8)
    np.testing.assert_allclose(out["dX"], gX, rtol=1e-10, atol=1e-12)
    assert abs(out["dZ_x"] - gZ) <= 1e-9 * max(1.0, abs(gZ))


# ------------------------------------------------------------------ forward product (Sec. 3.1)
def test_forward_is_exact_integer_product_times_scales():
    X, W, dY, sx, zx, sw = _tiny_layer(seed=41, T=7, c_in=9, c_out=5, shrink=0.7, w_bits=4)
    Y = orc.linear_fwd(X, sx, zx, 8, W, sw, 4)
    xc, _, _ = orc.fakequant_act(X, sx, zx, 8)
    wc, _, _ = orc.fakequant_weight(W, sw, 4)
    z = int(np.rint(float(zx)))
    for t in range(7):
        for c in range(5):
            acc = 0
            for i in range(9):
                acc += (int(xc[t, i]) - z) * int(wc[c, i])          # exact integer sum
            assert abs(Y[t, c] - float(sx) * float(sw[c]) * acc) <= 1e-12 * max(1.0, abs(Y[t, c]))
    # Eq. 5 is the gradient of <dY, Y>: the backward pins above use the same forward
    out = orc.linear_bwd(dY, X, sx, zx, 8, W, sw, 4, np.arange(5))
    _, _, Wq = orc.fakequant_weight(W, sw, 4)
    np.testing.assert_allclose(out["dXq"], dY.astype(np.float64) @ Wq, rtol=1e-13)

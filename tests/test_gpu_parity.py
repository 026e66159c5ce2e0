"""GPU parity: the HIP library (through its C ABI) against the fp64 CPU oracle, element by
element on the same seeded inputs.  Integer results (codes, clip masks, indices) must be
bit-exact; bf16-MFMA gradients within max|err| <= 2e-2 * max|ref|; fp32 reductions within
1e-5 relative; the quantizer-parameter gradients within the bounds derived in bwd_checks.py."""
import numpy as np
import pytest
import torch

import paper_2411_11038_amd as ef
from oracle import efqat_oracle as orc
from workloads import synth

from bwd_checks import GEMM_TOL, check_backward
from gpu_util import (act_tensor, assert_max_err, assert_rms_err, clip_words, dev, host, pack_mask)

pytestmark = pytest.mark.gpu


# ---------------------------------------------------------------- fake-quant forward
@pytest.mark.parametrize("rows,cols", [(1, 1), (5, 7), (37, 100), (256, 256), (300, 768), (64, 4104), (3, 1031)])
@pytest.mark.parametrize("kind", ["f32", "bf16"])
@pytest.mark.parametrize("bits", [8, 4])
def test_fakequant_act_minmax(rows, cols, kind, bits):
    X = synth.normal(100 + rows, 0, (rows, cols))
    X = synth.as_bf16_values(X) if kind == "bf16" else X.astype(np.float32)
    s, z = orc.act_qparams_minmax(X, bits)
    codes, mask, xq = orc.fakequant_act(X, s, z, bits)
    out = ef.fakequant_fwd(act_tensor(X, kind), ef.ACT_PER_TENSOR_ASYM, bits, init_minmax=True, want_xq=True)
    torch.cuda.synchronize()
    assert out["scale"].item() == float(s) and out["zero_point"].item() == float(z)
    assert np.array_equal(out["codes"].cpu().numpy().astype(np.int64), codes)
    assert np.array_equal(clip_words(out["clip_bits"]), pack_mask(mask))
    assert_max_err(host(out["xq"]), xq, 2.0 ** -8, "xq")


@pytest.mark.parametrize("rows,cols", [(5, 7), (129, 200), (256, 256)])
@pytest.mark.parametrize("kind", ["f32", "bf16"])
def test_fakequant_act_given_params_clipping_and_ties(rows, cols, kind):
    X = synth.normal(7, 0, (rows, cols))
    X = synth.as_bf16_values(X) if kind == "bf16" else X.astype(np.float32)
    # exact ties and on-bound values: multiples of S/2 with S a power of two
    S, Z = np.float32(0.03125), np.float32(100.3)       # non-integer zero point: forward uses round(Z)
    X.flat[: min(40, X.size)] = (np.arange(min(40, X.size)) - 20.5) * 0.5 * S
    X.flat[-1] = S * (255 - 100); X.flat[-2] = S * (0 - 100); X.flat[-3] = S * (256 - 100)
    codes, mask, _ = orc.fakequant_act(X, S, Z, 8)
    assert (~mask).any() and mask.any()
    out = ef.fakequant_fwd(act_tensor(X, kind), ef.ACT_PER_TENSOR_ASYM, 8, init_minmax=False,
                           scale=dev(np.array([S])), zero_point=dev(np.array([Z])))
    torch.cuda.synchronize()
    assert np.array_equal(out["codes"].cpu().numpy().astype(np.int64), codes)
    assert np.array_equal(clip_words(out["clip_bits"]), pack_mask(mask))


@pytest.mark.parametrize("rows,cols", [(1, 1), (6, 5), (40, 100), (256, 256), (136, 200), (33, 1032)])
@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("shrink", [1.0, 0.7])
def test_fakequant_weight(rows, cols, bits, shrink):
    W = synth.normal(9 + cols, 1, (rows, cols), std=0.02).astype(np.float32)
    if rows > 3:
        W[2] = 0.0                                            # degenerate row
    sw = orc.weight_scale_minmax(W, bits)
    if shrink == 1.0:
        out = ef.fakequant_fwd(dev(W), ef.W_PER_ROW_SYM, bits, init_minmax=True, want_xq=True)
    else:
        sw = (sw * np.float32(shrink)).astype(np.float32)
        out = ef.fakequant_fwd(dev(W), ef.W_PER_ROW_SYM, bits, init_minmax=False, scale=dev(sw), want_xq=True)
    codes, mask, wq = orc.fakequant_weight(W, sw, bits)
    torch.cuda.synchronize()
    assert np.array_equal(out["scale"].cpu().numpy(), sw)
    assert np.array_equal(out["codes"].cpu().numpy().astype(np.int64), codes)
    assert np.array_equal(clip_words(out["clip_bits"]), pack_mask(mask))
    assert_max_err(host(out["xq"]), wq, 2.0 ** -8, "wq")
    if shrink < 1.0 and rows * cols > 100:
        assert (~mask).any()


# min/max initialisation of fp32 weights whose rows are whole mask words and at most 4096 long runs on the kernels that
# hold the row in registers: one case per variant (chunks per lane x wavefronts per row), ragged row counts, a zero row
@pytest.mark.parametrize("rows,cols", [(256, 256), (4097, 512), (5, 1024), (3, 2080), (7, 4096), (4100, 1056),
                                       (4098, 2080), (4099, 4096), (2, 32), (5, 4128), (3, 8192),
                                       (300, 11008), (4100, 16384), (9, 16416)])
@pytest.mark.parametrize("bits", [8, 4])
def test_fakequant_weight_minmax_rows_in_registers(rows, cols, bits):
    W = synth.normal(31 + rows + cols, 1, (rows, cols), std=0.02).astype(np.float32)
    W[rows // 2] = 0.0                                        # degenerate row
    W[0, cols - 1] = 3.0 * np.abs(W[0]).max()                 # the row's maximum sits in its last element
    sw = orc.weight_scale_minmax(W, bits)
    codes, mask, _ = orc.fakequant_weight(W, sw, bits)
    out = ef.fakequant_fwd(dev(W), ef.W_PER_ROW_SYM, bits, init_minmax=True)
    torch.cuda.synchronize()
    assert np.array_equal(out["scale"].cpu().numpy(), sw)
    assert np.array_equal(out["codes"].cpu().numpy().astype(np.int64), codes)
    assert np.array_equal(clip_words(out["clip_bits"]), pack_mask(mask))


def test_fakequant_conv_weight_ohwi():
    W = synth.normal(3, 1, (24, 3, 3, 16), std=0.05).astype(np.float32)
    sw = orc.weight_scale_minmax(W, 4)
    codes, mask, _ = orc.fakequant_weight(W, sw, 4)
    out = ef.fakequant_fwd(dev(W), ef.W_PER_ROW_SYM, 4, init_minmax=True)
    torch.cuda.synchronize()
    assert np.array_equal(out["scale"].cpu().numpy(), sw)
    assert np.array_equal(out["codes"].cpu().numpy().astype(np.int64), codes)
    assert np.array_equal(clip_words(out["clip_bits"]), pack_mask(mask.reshape(24, -1)))


# ---------------------------------------------------------------- importance + Top-K
@pytest.mark.parametrize("c_out,block", [(1, 1), (7, 5), (256, 256), (300, 77), (1030, 64), (3072, 768)])
def test_channel_select_matches_oracle(c_out, block):
    W = synth.normal(40 + c_out, 1, (c_out, block), std=0.02).astype(np.float32)
    if c_out >= 7:
        W[5] = W[1]; W[6] = -W[1]                              # exact ties: lower index must win
    imp = orc.channel_importance(W)
    Wd = dev(W)
    for k in sorted({0, 1, c_out // 20, c_out // 4, c_out - 1, c_out}):
        if k < 0:
            continue
        idx, scores = ef.channel_select(Wd, k)
        torch.cuda.synchronize()
        np.testing.assert_allclose(scores.cpu().numpy(), imp, rtol=1e-12, atol=0)
        assert idx.cpu().numpy().tolist() == orc.top_k_channels(imp, k).tolist(), (c_out, k)


def test_channel_select_all_equal_scores_picks_lowest_indices():
    W = np.full((200, 16), 0.5, np.float32)
    W[:, ::2] *= -1
    idx, _ = ef.channel_select(dev(W), 37)
    assert idx.cpu().numpy().tolist() == list(range(37))


def test_network_select_cwpn():
    shapes = [(64, 32), (48, 100), (200, 8), (16, 16)]
    scores, offs = [], [0]
    for i, (c, b) in enumerate(shapes):
        W = synth.normal(60 + i, 1, (c, b), std=0.02 * (1 + 0.3 * i)).astype(np.float32)
        scores.append(orc.channel_importance(W)); offs.append(offs[-1] + c)
    scores[2][:] = scores[2][0]                                 # one layer of all-equal scores
    flat = dev(np.concatenate(scores)); off_d = dev(np.array(offs, dtype=np.int64))
    for k_total in (0, 1, 40, 163, offs[-1]):
        idx, kpl = ef.network_select(flat, off_d, k_total)
        torch.cuda.synchronize()
        ref = orc.network_top_k(scores, k_total)
        assert kpl.cpu().numpy().tolist() == [len(r) for r in ref]
        assert idx.cpu().numpy().tolist() == np.concatenate(ref).astype(np.int64).tolist() if k_total else True


@pytest.mark.parametrize("n,spread_bits,k", [(1000, 9, 137), (3072, 3, 768), (5000, 20, 1), (14000, 13, 9000),
                                             (700, 0, 50), (11008, 30, 2752), (16384, 11, 16000), (16385, 12, 77),
                                             (40000, 17, 12345), (20000, 0, 300)])
def test_topk_on_scores_that_differ_only_in_their_low_bits(n, spread_bits, k):
    # keys whose highest differing bit is low: the first digit window is clamped to bits 0..7 or is followed by a
    # narrower last window; many exact ties (every value occurs several times), which must go to the lower index.
    # More than 3072 scores do not fit the registers of the block: up to 16384 are kept in LDS, more are re-read
    # from memory in every pass.
    base = np.float64(0.8171).view(np.uint64)
    r = synth.normal(900 + n, 0, (n,))
    low = (np.abs(r) * 1e6).astype(np.uint64) % np.uint64(1 << spread_bits) if spread_bits else np.zeros(n, np.uint64)
    scores = (base + low).view(np.float64)
    flat = dev(scores); off_d = dev(np.array([0, n], dtype=np.int64))
    idx, kpl = ef.network_select(flat, off_d, k)
    torch.cuda.synchronize()
    ref = orc.top_k_channels(scores, k)
    assert kpl.cpu().numpy().tolist() == [k]
    assert idx.cpu().numpy().tolist() == ref.astype(np.int64).tolist()


@pytest.mark.parametrize("n,k", [(300, 40), (2000, 999), (9000, 4500), (30000, 100)])
def test_topk_on_scores_spread_over_many_binades(n, k):
    # importances of very different magnitude (exponents differ): keys are ranked relative to the smallest one
    r = synth.normal(950 + n, 0, (n,))
    scores = np.abs(r) * 10.0 ** (np.arange(n) % 13 - 6)
    scores[7] = scores[3]; scores[n - 1] = 0.0
    flat = dev(scores); off_d = dev(np.array([0, n], dtype=np.int64))
    idx, kpl = ef.network_select(flat, off_d, k)
    torch.cuda.synchronize()
    assert idx.cpu().numpy().tolist() == orc.top_k_channels(scores, k).astype(np.int64).tolist()


def test_layer_select_lwpn():
    shapes = [(64, 32), (48, 100), (200, 8), (16, 16), (16, 16), (33, 7)]
    ws, scores, offs = [], [], [0]
    for i, (c, b) in enumerate(shapes):
        W = synth.normal(70 + i, 1, (c, b), std=0.02 * (1 + 0.25 * ((i * 5) % 4))).astype(np.float32)
        ws.append(W); scores.append(orc.channel_importance(W)); offs.append(offs[-1] + c)
    ws[4] = ws[3].copy(); scores[4] = scores[3].copy()           # two layers with identical importance
    flat = dev(np.concatenate(scores)); off_d = dev(np.array(offs, dtype=np.int64))
    for k_layers in (0, 1, 2, 3, 4, len(shapes)):
        lidx, kpl, ls = ef.layer_select(flat, off_d, k_layers)
        torch.cuda.synchronize()
        sel, kpl_ref, imp = orc.layer_top_k(ws, k_layers)
        np.testing.assert_allclose(ls.cpu().numpy(), imp, rtol=1e-12)
        assert lidx.cpu().numpy().tolist() == [int(v) for v in sel]
        assert kpl.cpu().numpy().tolist() == [int(v) for v in kpl_ref]


@pytest.mark.parametrize("trial", range(8))
def test_network_and_layer_select_on_random_networks(trial):
    """Seeded random networks (1 to 39 layers, some with identical rows or identical layers: ties) through the CWPN
    and LWPN selections, against the oracle."""
    rng = np.random.default_rng(31337 + trial)
    nl = int(rng.integers(1, 40))
    ws, scores, offs = [], [], [0]
    for i in range(nl):
        c, b = int(rng.integers(1, 700)), int(rng.integers(1, 64))
        W = synth.normal(1000 + trial * 50 + i, 1, (c, b), std=0.02 * (1 + 0.3 * (i % 4))).astype(np.float32)
        if rng.integers(0, 4) == 0:
            W[:] = W[0]
        ws.append(W)
    if nl > 2 and rng.integers(0, 2):
        ws[1] = ws[0].copy()
    for W in ws:
        scores.append(orc.channel_importance(W)); offs.append(offs[-1] + W.shape[0])
    flat = dev(np.concatenate(scores)); off_d = dev(np.array(offs, dtype=np.int64))
    total = offs[-1]
    for k_total in sorted({0, 1, total, int(rng.integers(0, total + 1)), int(rng.integers(0, total + 1))}):
        idx, kpl = ef.network_select(flat, off_d, k_total)
        torch.cuda.synchronize()
        ref = orc.network_top_k(scores, k_total)
        assert kpl.cpu().numpy().tolist() == [len(r) for r in ref]
        if k_total:
            assert idx.cpu().numpy().tolist() == np.concatenate(ref).astype(np.int64).tolist()
    for k_layers in sorted({0, 1, nl, int(rng.integers(0, nl + 1))}):
        lidx, kpl, ls = ef.layer_select(flat, off_d, k_layers)
        torch.cuda.synchronize()
        sel, kpl_ref, imp = orc.layer_top_k(ws, k_layers)
        np.testing.assert_allclose(ls.cpu().numpy(), imp, rtol=1e-12)
        assert lidx.cpu().numpy().tolist() == [int(v) for v in sel]
        assert kpl.cpu().numpy().tolist() == [int(v) for v in kpl_ref]


@pytest.mark.parametrize("shape,bits,num,den", [((3072, 768), 8, 1, 4), ((768, 3072), 4, 1, 20), ((256, 3, 3, 256), 4, 1, 4),
                                                 ((130, 70), 8, 1, 3), ((64, 20000), 8, 1, 2), ((11008, 4096), 4, 1, 100),
                                                 ((40, 96), 8, 0, 1)],
                         ids=lambda v: str(v))
def test_weight_quant_select_equals_the_two_calls(shape, bits, num, den):
    # one call for the weight side of a step (quantizer with the row in registers, which also sums |w|; Top-K) against
    # the separate entry points and the oracle; (130, 70) and (64, 20000) take the fall-back kernels
    W = synth.normal(333 + shape[0], 1, shape, std=0.02).astype(np.float32)
    W[5] = W[2]                                              # equal scores: the tie goes to the lower index
    wd = dev(W)
    k = ef.k_from_ratio(shape[0], num, den)
    one = ef.weight_quant_select(wd, bits, k)
    fw = ef.fakequant_fwd(wd.view(shape[0], -1), ef.W_PER_ROW_SYM, bits, init_minmax=True)
    idx, scores = ef.channel_select(wd, k)
    torch.cuda.synchronize()
    assert torch.equal(one["codes"].view(shape[0], -1), fw["codes"]) and torch.equal(one["clip_bits"], fw["clip_bits"])
    assert torch.equal(one["scale"], fw["scale"]) and torch.equal(one["idx"], idx)
    imp = orc.channel_importance(W)
    np.testing.assert_allclose(one["scores"].cpu().numpy(), imp, rtol=1e-12)
    np.testing.assert_allclose(scores.cpu().numpy(), imp, rtol=1e-12)
    assert one["idx"].cpu().numpy().tolist() == orc.top_k_channels(imp, k).tolist()
    sw = orc.weight_scale_minmax(W, bits)
    codes, mask, _ = orc.fakequant_weight(W, sw, bits)
    assert np.array_equal(one["scale"].cpu().numpy(), sw)
    assert np.array_equal(one["codes"].cpu().numpy().astype(np.int64), codes)
    assert np.array_equal(clip_words(one["clip_bits"]), pack_mask(mask.reshape(shape[0], -1)))
    # given scales (no initialisation): the scores come from the pass of their own
    two = ef.weight_quant_select(wd, bits, k, init_minmax=False, scale=dev((sw * np.float32(0.75)).astype(np.float32)))
    torch.cuda.synchronize()
    codes2, mask2, _ = orc.fakequant_weight(W, (sw * np.float32(0.75)).astype(np.float32), bits)
    assert np.array_equal(two["codes"].cpu().numpy().astype(np.int64), codes2)
    assert torch.equal(two["idx"], idx)


BIAS_CASES = [
    # T, c_out, kind, layout
    (517, 264, "bf16", 0), (517, 264, "f32", 0), (300, 77, "bf16", 0), (300, 77, "f32", 0), (1, 8, "bf16", 0),
    (2048, 1024, "bf16", 0), (517, 264, "bf16", 1), (9000, 5, "f32", 1), (300, 77, "f32", 1), (4096, 520, "bf16", 1),
]


@pytest.mark.parametrize("T,c_out,kind,layout", BIAS_CASES, ids=lambda v: str(v))
def test_bias_grad_matches_oracle(T, c_out, kind, layout):
    dY = synth.normal(900 + T + c_out, 3, (T, c_out), std=1.0)
    dY = synth.as_bf16_values(dY) if kind == "bf16" else dY.astype(np.float32)
    dy_host = dY if layout == ef.DY_TOKEN_MAJOR else np.ascontiguousarray(dY.T)
    db = ef.bias_grad(act_tensor(dy_host, kind), dy_layout=layout)
    torch.cuda.synchronize()
    ref = orc.bias_grad(dY)
    # fp32 partial sums over at most 256 terms per lane, then fp64: error relative to the size of a
    # random-sign sum, the l2 norm of the column
    scale = np.sqrt((np.asarray(dY, dtype=np.float64) ** 2).sum(axis=0))
    assert np.max(np.abs(db.cpu().numpy().astype(np.float64) - ref) / scale) <= 1e-5


# ---------------------------------------------------------------- linear backward
def _run_linear(X, W, dY, kind, a_bits, w_bits, shrink, num, den, layout, scatter, dx_dtype=None,
                dx_kernel=ef.DX_KERNEL_AUTO):
    T, c_in = X.shape; c_out = W.shape[0]
    xd, wd = act_tensor(X, kind), dev(W)
    fx = ef.fakequant_fwd(xd, ef.ACT_PER_TENSOR_ASYM, a_bits, init_minmax=True)
    fw = ef.fakequant_fwd(wd, ef.W_PER_ROW_SYM, w_bits, init_minmax=True)
    sx, zx = orc.act_qparams_minmax(X, a_bits)
    sw = orc.weight_scale_minmax(W, w_bits)
    if shrink != 1.0:
        sx = np.float32(sx * np.float32(shrink)); sw = (sw * np.float32(shrink)).astype(np.float32)
        fx = ef.fakequant_fwd(xd, ef.ACT_PER_TENSOR_ASYM, a_bits, init_minmax=False, scale=dev(np.array([sx])),
                              zero_point=dev(np.array([zx])))
        fw = ef.fakequant_fwd(wd, ef.W_PER_ROW_SYM, w_bits, init_minmax=False, scale=dev(sw))
    k = ef.k_from_ratio(c_out, num, den)
    assert k == orc.k_from_ratio(c_out, num, den)
    idx, _ = ef.channel_select(wd, k)
    idx_ref = orc.top_k_channels(orc.channel_importance(W), k)
    dy_host = dY if layout == ef.DY_TOKEN_MAJOR else np.ascontiguousarray(dY.T)
    out = ef.linear_bwd(act_tensor(dy_host, kind), fx["codes"], fx["clip_bits"], xd, fx["scale"], fx["zero_point"],
                        fw["codes"], fw["clip_bits"], wd, fw["scale"], idx if k else None, dy_layout=layout,
                        scatter=scatter, dx_dtype=dx_dtype, dx_kernel=dx_kernel)
    torch.cuda.synchronize()
    ref = orc.linear_bwd(dY, X, sx, zx, a_bits, W, sw, w_bits, idx_ref)
    return out, ref, idx, idx_ref, fx, fw, (sx, zx, sw)


LIN_CASES = [
    # T, c_in, c_out, kind, a_bits, w_bits, shrink, (num, den), layout, scatter
    (256, 256, 256, "f32", 8, 8, 1.0, (1, 4), 0, False),          # config 1, seed 0
    (256, 256, 256, "f32", 8, 8, 0.7, (1, 4), 0, True),
    (256, 256, 256, "f32", 8, 8, 1.0, (1, 4), 1, False),
    (300, 200, 136, "bf16", 8, 4, 0.7, (1, 4), 0, False),         # ragged tiles, several per dimension
    (300, 200, 136, "bf16", 8, 4, 0.7, (1, 4), 1, True),
    (517, 392, 264, "bf16", 8, 8, 0.8, (1, 2), 0, True),
    (129, 72, 40, "bf16", 8, 8, 1.0, (1, 1), 0, False),           # r = 100 %: full QAT backward
    (129, 72, 40, "bf16", 8, 8, 0.7, (0, 1), 0, False),           # r = 0: no weight gradient
    (130, 70, 43, "f32", 8, 4, 0.7, (1, 3), 0, False),            # nothing a multiple of 8
    (130, 70, 43, "bf16", 8, 4, 0.7, (1, 3), 1, False),
    (131, 70, 43, "f32", 4, 4, 0.6, (1, 3), 1, True),
    (1, 8, 8, "bf16", 8, 8, 1.0, (1, 1), 0, False),               # single token
    (1024, 768, 768, "bf16", 8, 8, 0.8, (1, 20), 0, False),       # BERT-width, split-K path
    (1024, 768, 768, "bf16", 8, 8, 0.8, (1, 20), 1, False),
    # c_in a multiple of 16 and token-major dY: weight gradient straight from the uint8 codes (LDS transpose reads)
    (300, 208, 136, "bf16", 8, 4, 0.7, (1, 4), 0, False),
    (517, 400, 264, "bf16", 8, 8, 0.8, (1, 2), 0, True),
    (300, 208, 136, "bf16", 8, 8, 0.7, (1, 1), 0, False),         # every channel: dY itself is the operand
    (300, 208, 130, "bf16", 8, 8, 0.7, (1, 1), 0, False),         # ... C_out not a multiple of 8: compacted copy
    (333, 272, 200, "f32", 8, 8, 0.7, (1, 1), 0, True),
    (70, 16, 24, "bf16", 8, 8, 1.0, (1, 3), 0, False),
    (2048, 512, 640, "bf16", 8, 8, 0.8, (1, 1), 0, False),        # several 256-wide tiles, split-K
    # channel-major bf16 dY, T % 8 == 0, c_in % 16 == 0: rows idx of dY gathered by the dW kernel's tile loads,
    # activation operand read from the uint8 codes as they lie
    (304, 208, 136, "bf16", 8, 4, 0.7, (1, 4), 1, False),         # tails in M (k = 34), N and K (304 = 4 * 64 + 48)
    (304, 208, 136, "bf16", 8, 8, 0.8, (1, 2), 1, True),
    (72, 16, 24, "bf16", 8, 8, 1.0, (1, 3), 1, False),
    (2048, 512, 640, "bf16", 8, 8, 0.8, (1, 1), 1, False),        # every channel; several tiles; split-K
    (1000, 768, 1096, "bf16", 8, 8, 0.8, (1, 20), 1, False),      # k = 54 of 1096
    (384, 256, 136, "bf16", 8, 8, 0.6, (1, 4), 1, False),         # whole 128 tiles: straight-line dX epilogue
    (256, 128, 136, "bf16", 8, 8, 0.6, (1, 4), 0, False),         # ... of the bf16-operand 128 x 128 kernel
    (256, 136, 128, "bf16", 4, 8, 0.6, (1, 4), 0, False),         # (C_in = 136: general epilogue, same kernel family)
]


@pytest.mark.parametrize("case", LIN_CASES, ids=lambda c: "T%d_%dx%d_%s_w%d_s%s_r%d-%d_L%d_sc%d" % (
    c[0], c[1], c[2], c[3], c[5], c[6], c[7][0], c[7][1], c[8], int(c[9])))
def test_linear_bwd_matches_oracle(case):
    T, c_in, c_out, kind, a_bits, w_bits, shrink, (num, den), layout, scatter = case
    seed = 0 if (T, c_in, c_out) == (256, 256, 256) else 1000 + T + c_in
    X, W, dY = synth.linear_layer(seed, T, c_in, c_out, act_dtype=kind)
    out, ref, idx, idx_ref, fx, fw, qp = _run_linear(X, W, dY, kind, a_bits, w_bits, shrink, num, den, layout,
                                                     scatter)
    assert np.array_equal(fx["codes"].cpu().numpy().astype(np.int64), ref["x_codes"])
    assert np.array_equal(fw["codes"].cpu().numpy().astype(np.int64), ref["w_codes"])
    assert np.array_equal(clip_words(fx["clip_bits"]), pack_mask(ref["x_mask"]))
    assert np.array_equal(clip_words(fw["clip_bits"]), pack_mask(ref["w_mask"]))
    check_backward(out, ref, idx, idx_ref, X, W, qp, kind, scatter, kind == "bf16", W.shape)


# (T, c_in, c_out, layout): the pinned 192-tile kernel, the 128-tile kernel with ragged edges, a padded C_out,
# and two layers whose dX product reads the int8 codes (no operand exists: the call must behave like the plain one)
PREPARED_CASES = [(384, 192, 384, 0), (300, 200, 136, 0), (129, 72, 43, 0), (2048, 512, 640, 0), (384, 256, 136, 1)]


@pytest.mark.parametrize("case", PREPARED_CASES, ids=lambda c: "T%d_%dx%d_L%d" % c)
def test_linear_bwd_with_weight_operand_made_beforehand_is_bit_identical(case):
    T, c_in, c_out, layout = case
    X, W, dY = synth.linear_layer(7000 + T, T, c_in, c_out, act_dtype="bf16")
    xd, wd = act_tensor(X, "bf16"), dev(W)
    fx = ef.fakequant_fwd(xd, ef.ACT_PER_TENSOR_ASYM, 8, init_minmax=True)
    fw = ef.fakequant_fwd(wd, ef.W_PER_ROW_SYM, 8, init_minmax=True)
    k = ef.k_from_ratio(c_out, 1, 4)
    idx, _ = ef.channel_select(wd, k)
    dyd = act_tensor(dY if layout == 0 else np.ascontiguousarray(dY.T), "bf16")
    args = (dyd, fx["codes"], fx["clip_bits"], xd, fx["scale"], fx["zero_point"], fw["codes"], fw["clip_bits"], wd,
            fw["scale"], idx)
    ref = ef.linear_bwd(*args, dy_layout=layout)
    op = ef.linear_bwd_weight_operand(fw["codes"], fw["scale"], T, ef.BF16, layout)
    need = ef.lib().efqat_linear_bwd_weight_operand_bytes(T, c_in, c_out, ef.BF16, layout)
    assert (op is None) == (need == 0)
    if op is None:                                       # nothing to prepare: any aligned pointer is ignored
        op = torch.zeros(256, dtype=torch.uint8, device=xd.device)
    else:
        # the operand is bf16(S_w[c] * code[c][i]) transposed, zero padded, followed by a zero page
        ldc = (c_out + 7) // 8 * 8
        got = op[:c_in * ldc * 2].view(torch.bfloat16).view(c_in, ldc).float().cpu().numpy()
        wq = (fw["scale"].cpu().numpy()[:, None] * fw["codes"].cpu().numpy().astype(np.float32))
        want = torch.from_numpy(wq.T.copy()).to(torch.bfloat16).float().numpy()
        assert np.array_equal(got[:, :c_out], want) and not got[:, c_out:].any()
        assert not op[-256:].any()
    out = ef.linear_bwd(*args, dy_layout=layout, w_operand=op)
    torch.cuda.synchronize()
    for key in ("dx", "dw", "ds_w", "ds_x", "dz_x"):
        a, b = out[key], ref[key]
        if a.dtype == torch.bfloat16:
            a, b = a.view(torch.int16), b.view(torch.int16)
        assert torch.equal(a, b), key


def _random_case(seed):
    """A seeded small layer with nothing aligned on purpose: shapes, dtypes, layout, fraction, scatter, bit widths."""
    rng = np.random.default_rng(9000 + seed)
    T = int(rng.integers(1, 420)); c_in = int(rng.integers(1, 330)); c_out = int(rng.integers(1, 330))
    if seed % 4 == 0:                                    # some whole-tile shapes as well
        T = 192 * int(rng.integers(1, 3)); c_in = 64 * int(rng.integers(1, 5))
    kind = "bf16" if rng.integers(0, 3) else "f32"
    layout = int(rng.integers(0, 2))
    num, den = [(0, 1), (1, 7), (1, 3), (1, 1), (1, 20)][int(rng.integers(0, 5))]
    return (T, c_in, c_out, kind, [8, 4][int(rng.integers(0, 2))], [8, 4][int(rng.integers(0, 2))],
            [1.0, 0.7, 0.5][int(rng.integers(0, 3))], (num, den), layout, bool(rng.integers(0, 2)))


# 67, 181, 317: rows of one to five weights that are all clipped (the masked gradient row is zero, dS_w is not)
@pytest.mark.parametrize("seed", list(range(24)) + [67, 181, 317])
def test_linear_bwd_random_shapes_match_oracle(seed):
    T, c_in, c_out, kind, a_bits, w_bits, shrink, (num, den), layout, scatter = _random_case(seed)
    X, W, dY = synth.linear_layer(5000 + seed, T, c_in, c_out, act_dtype=kind)
    out, ref, idx, idx_ref, fx, fw, qp = _run_linear(X, W, dY, kind, a_bits, w_bits, shrink, num, den, layout,
                                                     scatter)
    assert np.array_equal(fx["codes"].cpu().numpy().astype(np.int64), ref["x_codes"])
    assert np.array_equal(fw["codes"].cpu().numpy().astype(np.int64), ref["w_codes"])
    assert np.array_equal(clip_words(fx["clip_bits"]), pack_mask(ref["x_mask"]))
    assert np.array_equal(clip_words(fw["clip_bits"]), pack_mask(ref["w_mask"]))
    check_backward(out, ref, idx, idx_ref, X, W, qp, kind, scatter, kind == "bf16", W.shape)


# dX product with the weight operand read from the int8 codes (bf16 token-major dY, C_out % 8 == 0, C_in % 16 == 0):
# forced through the dx_kernel argument so that both tile sizes meet ragged edges in every dimension
DX8_CASES = [
    # T, c_in, c_out, a_bits, w_bits, shrink, (num, den), scatter
    (300, 208, 136, 8, 4, 0.7, (1, 4), False),      # 128 tile; K tail 136 % 64 = 8, N tail, M tail
    (517, 400, 264, 8, 8, 0.8, (1, 2), True),
    (70, 16, 24, 8, 8, 1.0, (1, 3), False),         # one partial stage, one partial tile
    (129, 144, 64, 8, 8, 0.7, (0, 1), False),       # exactly one full stage, r = 0
    (260, 128, 448, 8, 8, 0.8, (1, 20), False),     # seven full stages (pipelined loop + drain), full-width tile
    (2048, 512, 640, 8, 8, 0.8, (1, 1), False),     # 256 tile, everything a multiple of the tile
    (1100, 528, 200, 8, 4, 0.7, (1, 4), False),     # 256 tile with tails in M, N and K
    (1030, 768, 1096, 8, 8, 0.8, (1, 20), False),   # 256 tile, 17 full stages + tail
    (384, 256, 136, 8, 8, 0.6, (1, 4), False),      # whole 128 tiles: straight-line epilogue, clipped activations
    (1024, 512, 200, 4, 8, 0.6, (1, 4), True),      # whole 256 tiles, 4-bit activations (many clipped)
    # more than one round of 256 x 256 tiles on the 256 compute units
    (2048, 8704, 64, 8, 8, 0.7, (1, 4), False),     # 8 x 34 whole tiles, one K stage
    (2000, 8752, 72, 8, 4, 0.7, (1, 8), False),     # the same with ragged rows, a ragged last column tile and a K tail
]


@pytest.mark.parametrize("case", DX8_CASES, ids=lambda c: "T%d_%dx%d_w%d_r%d-%d" % (c[0], c[1], c[2], c[4],
                                                                                    c[6][0], c[6][1]))
def test_linear_bwd_int8_weight_operand(case):
    T, c_in, c_out, a_bits, w_bits, shrink, (num, den), scatter = case
    X, W, dY = synth.linear_layer(3000 + T + c_in, T, c_in, c_out, act_dtype="bf16")
    out, ref, idx, idx_ref, fx, fw, qp = _run_linear(X, W, dY, "bf16", a_bits, w_bits, shrink, num, den, 0, scatter,
                                                     dx_kernel=ef.DX_KERNEL_INT8)
    out2, *_ = _run_linear(X, W, dY, "bf16", a_bits, w_bits, shrink, num, den, 0, scatter, dx_kernel=ef.DX_KERNEL_BF16)
    check_backward(out, ref, idx, idx_ref, X, W, qp, "bf16", scatter, True, W.shape)
    # both kernels round S_w * code to bf16 once and accumulate in fp32; only the fp32 summation order differs, so
    # the bf16 outputs agree to an ulp or two of the largest element
    assert_max_err(host(out["dx"]), host(out2["dx"]), 8e-3, "dX int8-operand vs bf16-operand kernel")


# dX product by the 192 x 192 kernel with the pinned instruction order and the three-stage LDS ring, forced through
# the dx_kernel argument (the planner takes it only for large products): ragged edges in every dimension, K from a single
# 8-wide chunk to many stages, so that the pipelined loop, its drain and the zero-page tail all run
PINNED_CASES = [
    # T, c_in, c_out, kind, a_bits, w_bits, shrink, (num, den), layout, scatter
    (300, 208, 136, "bf16", 8, 4, 0.7, (1, 4), 0, False),     # 2 full stages + 8: drain only, tails in M and N
    (70, 16, 8, "bf16", 8, 8, 1.0, (1, 2), 0, False),         # one chunk of K
    (129, 144, 64, "bf16", 8, 8, 0.7, (0, 1), 0, False),      # exactly one stage, r = 0
    (192, 192, 192, "bf16", 8, 8, 0.8, (1, 4), 0, False),     # one exact tile, three stages
    (260, 200, 448, "bf16", 8, 8, 0.8, (1, 20), 0, False),    # seven stages: one trip of the pinned loop + drain
    (517, 392, 1096, "bf16", 8, 8, 0.8, (1, 8), 0, True),     # 17 stages + tail of 8; several tiles
    (400, 70, 645, "f32", 8, 4, 0.7, (1, 3), 0, False),       # nothing a multiple of 8: staged dY, scalar epilogue
    (520, 208, 840, "bf16", 8, 8, 0.8, (1, 4), 1, False),     # channel-major dY: transposed copy, then this kernel
    # bf16 in and out, T and C_in multiples of 192: the straight-line epilogue (several tiles, clipped activations)
    (384, 576, 264, "bf16", 8, 8, 0.6, (1, 4), 0, False),
    (576, 192, 1096, "bf16", 8, 4, 0.7, (1, 8), 0, True),
    (192, 384, 72, "bf16", 4, 8, 0.6, (1, 2), 0, False),      # 4-bit activations: many clipped elements
]


@pytest.mark.parametrize("case", PINNED_CASES, ids=lambda c: "T%d_%dx%d_%s_r%d-%d_L%d" % (
    c[0], c[1], c[2], c[3], c[7][0], c[7][1], c[8]))
def test_linear_bwd_pinned_dx_kernel(case):
    T, c_in, c_out, kind, a_bits, w_bits, shrink, (num, den), layout, scatter = case
    X, W, dY = synth.linear_layer(7000 + T + c_out, T, c_in, c_out, act_dtype=kind)
    out, ref, idx, idx_ref, fx, fw, qp = _run_linear(X, W, dY, kind, a_bits, w_bits, shrink, num, den, layout, scatter,
                                                     dx_kernel=ef.DX_KERNEL_BF16_PINNED)
    out2, *_ = _run_linear(X, W, dY, kind, a_bits, w_bits, shrink, num, den, layout, scatter,
                           dx_kernel=ef.DX_KERNEL_BF16)
    check_backward(out, ref, idx, idx_ref, X, W, qp, kind, scatter, kind == "bf16", W.shape)
    # same operands, same bf16 rounding, fp32 accumulation in the same K order: only the epilogue's output rounding
    # can differ, and not even that - the two kernels must agree exactly
    assert np.array_equal(host(out["dx"]), host(out2["dx"]))


def _close_fp32_update(got, want, old, name):
    """The kernel forms the optimizer update in fp32: each result carries a few units of rounding at the size of its
    operands (old value and step), which is more than a relative bound on the result where the two nearly cancel."""
    mag = np.abs(np.asarray(old, dtype=np.float64)) + np.abs(want - np.asarray(old, dtype=np.float64))
    bad = np.abs(got - want) > 2e-6 * np.abs(want) + 2.0 ** -22 * mag
    assert not bad.any(), (name, int(bad.sum()), float(np.abs(got - want).max()))


def _adam_state(c_out, seed, fresh):
    """Adam state of the weight scales: zeros before the first step, or moments and per-channel step counts as they
    would be after some earlier steps (channels unfrozen at different times have different counts)."""
    if fresh:
        return np.zeros(c_out, np.float32), np.zeros(c_out, np.float32), np.zeros(c_out, np.int32)
    m = synth.normal(seed, 7, (c_out,), std=0.05).astype(np.float32)
    v = (synth.normal(seed, 8, (c_out,), std=0.05) ** 2).astype(np.float32)
    t = (np.arange(c_out) * 7 % 23).astype(np.int32)
    return m, v, t


def _check_fused_step(W, S0, ii, plain, w2, s2, mom_w0, mw, adam0, adam_dev, hp):
    """Weights: SGD rule of the oracle on rows idx.  Scales: Adam rule of the oracle.  Everything else untouched."""
    c_out = W.shape[0]
    Wn, mwn = orc.sgd_step_rows(W, ii, host(plain["dw"]).reshape(len(ii), *W.shape[1:]), hp["lr_w"], hp["momentum"],
                                hp["weight_decay"], mom_w0 if hp["momentum"] else None)
    m0, v0, t0 = adam0
    Sn, mn, vn, tn = orc.adam_step_rows(S0, ii, host(plain["ds_w"]), float(np.float32(hp["lr_s"])), m0, v0, t0,
                                        float(np.float32(hp["beta1"])), float(np.float32(hp["beta2"])),
                                        float(np.float32(hp["eps"])))
    _close_fp32_update(host(w2).reshape(W.shape), Wn, W, "w")
    frozen = np.setdiff1d(np.arange(c_out), ii)
    assert np.array_equal(host(w2).reshape(W.shape)[frozen], W[frozen].astype(np.float64))
    if hp["momentum"]:
        _close_fp32_update(host(mw).reshape(W.shape), mwn, mom_w0, "mom_w")
        assert np.array_equal(host(mw).reshape(W.shape)[frozen], mom_w0[frozen].astype(np.float64))
    # Adam on the scales: the kernel forms the update in double precision from the fp32 inputs, so what is left is
    # the fp32 rounding of the stored moments and of the new scale (half an ulp each) and the accuracy of pow / sqrt
    md, vd, td = (host(t_) for t_ in adam_dev)
    # (relative to the operands of the final subtraction, old scale and step: the two may nearly cancel)
    errs = dict(s_w=np.max(np.abs(host(s2) - Sn) / (np.abs(S0) + np.abs(Sn - S0))),
                adam_m=np.max(np.abs(md[ii] - mn[ii]) / np.maximum(np.abs(mn[ii]), 1e-30)),
                adam_v=np.max(np.abs(vd[ii] - vn[ii]) / np.maximum(np.abs(vn[ii]), 1e-30)))
    print("fused step, relative errors (ulp of fp32 = 6e-8):", {k_: float("%.2e" % v_) for k_, v_ in errs.items()})
    assert errs["s_w"] <= 6.1e-8 and errs["adam_m"] <= 6.1e-8 and errs["adam_v"] <= 6.1e-8, errs
    assert np.array_equal(td, tn)
    assert np.array_equal(host(s2)[frozen], S0[frozen].astype(np.float64))
    assert np.array_equal(md[frozen], m0[frozen].astype(np.float64))
    assert np.array_equal(vd[frozen], v0[frozen].astype(np.float64))
    assert np.array_equal(td[frozen], t0[frozen])


# (453, 140, 232): a weight whose update nearly cancels it (found by a soak over random shapes)
@pytest.mark.parametrize("momentum,wd,fresh", [(0.0, 0.0, True), (0.9, 5e-4, False), (0.0, 5e-4, False)])
@pytest.mark.parametrize("shape", [(300, 208, 136), (260, 70, 43), (453, 140, 232)])
def test_linear_bwd_fused_optimizer_step(shape, momentum, wd, fresh):
    # the fused optimizer step must equal the plain call followed by the oracle's rules on the rows idx (SGD on the
    # weight rows, Adam on their scales: Sec. 4 "Setup"), and leave everything else untouched
    T, c_in, c_out = shape
    X, W, dY = synth.linear_layer(5100 + T, T, c_in, c_out, act_dtype="bf16")
    xd, wd_t, dyd = act_tensor(X, "bf16"), dev(W), act_tensor(dY, "bf16")
    fx = ef.fakequant_fwd(xd, ef.ACT_PER_TENSOR_ASYM, 8, init_minmax=True)
    fw = ef.fakequant_fwd(wd_t, ef.W_PER_ROW_SYM, 8, init_minmax=True)
    k = ef.k_from_ratio(c_out, 1, 4)
    idx, _ = ef.channel_select(wd_t, k)
    args = (dyd, fx["codes"], fx["clip_bits"], xd, fx["scale"], fx["zero_point"], fw["codes"], fw["clip_bits"])
    plain = ef.linear_bwd(*args, wd_t, fw["scale"], idx)
    torch.cuda.synchronize()
    S0 = fw["scale"].cpu().numpy()
    mom_w0 = synth.normal(77, 5, (c_out, c_in), std=0.01).astype(np.float32)
    adam0 = _adam_state(c_out, 79, fresh)
    w2, s2 = wd_t.clone(), fw["scale"].clone()
    mw = dev(mom_w0)
    adam_dev = tuple(dev(a_) for a_ in adam0)
    hp = dict(lr_w=0.05, momentum=momentum, weight_decay=wd, lr_s=1e-3, beta1=0.9, beta2=0.999, eps=1e-8)
    step = dict(hp, mom_w=mw if momentum else None, adam_m=adam_dev[0], adam_v=adam_dev[1], adam_t=adam_dev[2])
    fused = ef.linear_bwd(*args, w2, s2, idx, step=step)
    torch.cuda.synchronize()
    for key in ("dx", "dw", "ds_w", "ds_x", "dz_x"):
        assert torch.equal(plain[key], fused[key]), key
    ii = idx.cpu().numpy().astype(np.int64)
    _check_fused_step(W, S0, ii, plain, w2, s2, mom_w0, mw, adam0, adam_dev, hp)
    # gradients are optional outputs of the fused call
    w3, s3 = wd_t.clone(), fw["scale"].clone()
    adam3 = tuple(dev(a_) for a_ in adam0)
    mw3 = dev(mom_w0)
    out3 = dict(dx=fused["dx"], dw=None, ds_w=None, ds_x=fused["ds_x"], dz_x=fused["dz_x"])
    ef.linear_bwd(*args, w3, s3, idx, out=out3,
                  step=dict(hp, mom_w=mw3 if momentum else None, adam_m=adam3[0], adam_v=adam3[1], adam_t=adam3[2]))
    torch.cuda.synchronize()
    assert torch.equal(w3, w2) and torch.equal(s3, s2)
    for a_, b_ in zip(adam3, adam_dev):
        assert torch.equal(a_, b_)


def test_conv_bwd_fused_optimizer_step():
    N, H, Wd, c_in, c_out, kh, kw = 2, 7, 6, 16, 24, 3, 3
    X, W, dY = synth.conv_layer(5200, N, H, Wd, c_in, c_out, kh, kw, 1, 1, act_dtype="bf16")
    xd, wd_t, dyd = act_tensor(X, "bf16"), dev(W), act_tensor(dY, "bf16")
    fx = ef.fakequant_fwd(xd.view(-1, c_in), ef.ACT_PER_TENSOR_ASYM, 8, init_minmax=True)
    fw = ef.fakequant_fwd(wd_t.view(c_out, -1), ef.W_PER_ROW_SYM, 4, init_minmax=True)
    k = ef.k_from_ratio(c_out, 1, 3)
    idx, _ = ef.channel_select(wd_t, k)
    xc, wc = fx["codes"].view(X.shape), fw["codes"].view(W.shape)
    args = (dyd, xc, fx["clip_bits"], xd, fx["scale"], fx["zero_point"], wc, fw["clip_bits"])
    plain = ef.conv_bwd(*args, wd_t, fw["scale"], idx, stride=1, pad=1)
    torch.cuda.synchronize()
    S0 = fw["scale"].cpu().numpy()
    w2, s2 = wd_t.clone(), fw["scale"].clone()
    mom_w0 = synth.normal(78, 5, W.shape, std=0.01).astype(np.float32)
    adam0 = _adam_state(c_out, 80, False)
    mw = dev(mom_w0)
    adam_dev = tuple(dev(a_) for a_ in adam0)
    hp = dict(lr_w=0.05, momentum=0.9, weight_decay=1e-3, lr_s=1e-6, beta1=0.8, beta2=0.95, eps=1e-6)
    fused = ef.conv_bwd(*args, w2, s2, idx, stride=1, pad=1,
                        step=dict(hp, mom_w=mw, adam_m=adam_dev[0], adam_v=adam_dev[1], adam_t=adam_dev[2]))
    torch.cuda.synchronize()
    for key in ("dx", "dw", "ds_w", "ds_x", "dz_x"):
        assert torch.equal(plain[key], fused[key]), key
    ii = idx.cpu().numpy().astype(np.int64)
    _check_fused_step(W, S0, ii, plain, w2, s2, mom_w0, mw, adam0, adam_dev, hp)


def test_linear_bwd_dx_independent_of_fraction_and_fp32_dx():
    X, W, dY = synth.linear_layer(77, 260, 136, 200, act_dtype="bf16")
    outs = []
    for num, den in [(0, 1), (1, 20), (1, 1)]:
        out, ref, *_ = _run_linear(X, W, dY, "bf16", 8, 8, 0.8, num, den, 0, False, dx_dtype=torch.float32)
        outs.append(out)
        assert_max_err(host(out["dx"]), ref["dX"], GEMM_TOL, "dX fp32")
    for o in outs[1:]:
        assert torch.equal(o["dx"], outs[0]["dx"])                   # bitwise: dX does not depend on r
        assert o["ds_x"].item() == outs[0]["ds_x"].item() and o["dz_x"].item() == outs[0]["dz_x"].item()


def test_linear_bwd_is_deterministic():
    X, W, dY = synth.linear_layer(78, 512, 256, 264, act_dtype="bf16")
    a, *_ = _run_linear(X, W, dY, "bf16", 8, 8, 0.8, 1, 4, 0, False)
    b, *_ = _run_linear(X, W, dY, "bf16", 8, 8, 0.8, 1, 4, 0, False)
    for key in ("dx", "dw", "ds_w", "ds_x", "dz_x"):
        assert torch.equal(a[key], b[key]), key


# ---------------------------------------------------------------- conv backward
CONV_CASES = [
    # N, H, W, c_in, c_out, kh, kw, stride, pad, kind, w_bits, shrink, (num, den), layout, scatter
    (2, 7, 6, 16, 24, 3, 3, 1, 1, "bf16", 4, 0.7, (1, 4), 0, False),
    (2, 7, 6, 16, 24, 3, 3, 1, 1, "bf16", 4, 0.7, (1, 4), 1, True),
    (3, 9, 8, 12, 20, 3, 3, 2, 1, "f32", 4, 0.8, (1, 2), 0, False),
    (2, 8, 8, 24, 16, 1, 1, 1, 0, "bf16", 8, 0.7, (1, 4), 0, False),
    (2, 8, 8, 24, 16, 1, 1, 2, 0, "bf16", 8, 1.0, (1, 1), 0, False),
    (2, 6, 7, 10, 9, 2, 3, 2, 0, "f32", 4, 0.7, (1, 3), 1, False),
    (4, 14, 14, 64, 64, 3, 3, 1, 1, "bf16", 4, 0.8, (1, 20), 0, False),   # ResNet-like, several tiles
    (4, 14, 14, 64, 64, 3, 3, 1, 1, "bf16", 4, 0.8, (0, 1), 0, False),
    # stride 1 and C_out a multiple of 64: the dX operand is gathered inside the tile loads (no im2col matrix)
    (2, 9, 7, 32, 128, 3, 3, 1, 1, "bf16", 8, 0.8, (1, 4), 0, False),     # two K stages per tap
    (2, 9, 7, 32, 64, 2, 3, 1, 0, "bf16", 4, 0.7, (1, 2), 0, True),       # no padding: output smaller than input
    (2, 6, 10, 16, 64, 3, 3, 1, 2, "f32", 8, 0.8, (1, 4), 0, False),      # padding 2: output larger than input
    (2, 6, 10, 16, 64, 3, 1, 1, 1, "bf16", 8, 0.8, (1, 4), 1, False),     # channel-major dY, 3 x 1 kernel
    (5, 11, 13, 48, 192, 3, 3, 1, 1, "bf16", 8, 0.8, (1, 20), 0, False),  # several row tiles, ragged edge
    # C_in a multiple of 128 and token-major dY: the dW operand (codes) is gathered inside the tile loads
    (2, 7, 6, 128, 24, 3, 3, 1, 1, "bf16", 4, 0.7, (1, 4), 0, False),
    (3, 9, 8, 128, 40, 3, 3, 2, 1, "bf16", 8, 0.8, (1, 2), 0, True),      # stride 2
    (1, 5, 5, 256, 64, 2, 2, 1, 0, "f32", 8, 0.8, (1, 1), 0, False),      # image smaller than a 64-token stage
    (2, 6, 10, 128, 64, 3, 1, 1, 1, "bf16", 8, 0.8, (1, 1), 0, False),    # every channel: dY itself is the A operand
    (7, 10, 9, 128, 64, 3, 3, 1, 1, "bf16", 4, 0.8, (1, 4), 0, False),    # 630 tokens: split-K with a ragged last stage
    # 128 input pixels x 128 channels: whole tiles, the straight-line dX epilogue behind the implicit-im2col loop
    (2, 8, 8, 128, 64, 3, 3, 1, 1, "bf16", 8, 0.6, (1, 4), 0, False),
    (3, 8, 16, 256, 128, 3, 3, 1, 1, "bf16", 8, 0.6, (1, 2), 0, True),
]


@pytest.mark.parametrize("case", CONV_CASES, ids=lambda c: "N%d_%dx%d_%d-%d_k%dx%d_s%dp%d_%s_L%d" % (
    c[0], c[1], c[2], c[3], c[4], c[5], c[6], c[7], c[8], c[9], c[13]))
def test_conv_bwd_matches_oracle(case):
    _conv_case(case)


# strided convolutions stage an im2col matrix of dY; with dx_kernel = BF16_PINNED that matrix is the A operand of
# the 192 x 192 pinned-order kernel
@pytest.mark.parametrize("case", [CONV_CASES[2], CONV_CASES[4], CONV_CASES[5], CONV_CASES[14]],
                         ids=lambda c: "N%d_%dx%d_%d-%d_k%dx%d_s%dp%d_%s_L%d" % (
                             c[0], c[1], c[2], c[3], c[4], c[5], c[6], c[7], c[8], c[9], c[13]))
def test_conv_bwd_pinned_dx_kernel_on_im2col_matrix(case):
    assert case[7] == 2
    _conv_case(case, dx_kernel=ef.DX_KERNEL_BF16_PINNED)


def _random_conv_case(seed):
    """A seeded small convolution: image, channels, kernel, stride, padding, dtype, layout and fraction all drawn."""
    rng = np.random.default_rng(9500 + seed)
    kh, kw = int(rng.integers(1, 4)), int(rng.integers(1, 4))
    stride, pad = int(rng.integers(1, 3)), int(rng.integers(0, 3))
    H, Wd = int(rng.integers(kh, 13)), int(rng.integers(kw, 13))
    N = int(rng.integers(1, 5))
    c_in = [int(rng.integers(1, 90)), 128, 64][int(rng.integers(0, 3))]
    c_out = [int(rng.integers(1, 90)), 64, 128][int(rng.integers(0, 3))]
    kind = "bf16" if rng.integers(0, 3) else "f32"
    num, den = [(0, 1), (1, 7), (1, 3), (1, 1)][int(rng.integers(0, 4))]
    return (N, H, Wd, c_in, c_out, kh, kw, stride, pad, kind, [8, 4][int(rng.integers(0, 2))],
            [1.0, 0.7][int(rng.integers(0, 2))], (num, den), int(rng.integers(0, 2)), bool(rng.integers(0, 2)))


@pytest.mark.parametrize("seed", list(range(16)) + [44])
def test_conv_bwd_random_shapes_match_oracle(seed):
    _conv_case(_random_conv_case(seed))


def _conv_case(case, dx_kernel=ef.DX_KERNEL_AUTO):
    N, H, Wd, c_in, c_out, kh, kw, stride, pad, kind, w_bits, shrink, (num, den), layout, scatter = case
    X, W, dY = synth.conv_layer(4000 + H + c_in, N, H, Wd, c_in, c_out, kh, kw, stride, pad, act_dtype=kind)
    xd, wd = act_tensor(X, kind), dev(W)
    sx, zx = orc.act_qparams_minmax(X, 8)
    sw = orc.weight_scale_minmax(W, w_bits)
    sx = np.float32(sx * np.float32(shrink)); sw = (sw * np.float32(shrink)).astype(np.float32)
    fx = ef.fakequant_fwd(xd, ef.ACT_PER_TENSOR_ASYM, 8, init_minmax=False, scale=dev(np.array([sx])),
                          zero_point=dev(np.array([zx])))
    fw = ef.fakequant_fwd(wd, ef.W_PER_ROW_SYM, w_bits, init_minmax=False, scale=dev(sw))
    k = ef.k_from_ratio(c_out, num, den)
    idx, _ = ef.channel_select(wd, k)
    idx_ref = orc.top_k_channels(orc.channel_importance(W), k)
    dy_host = dY if layout == 0 else np.ascontiguousarray(np.moveaxis(dY, -1, 0))
    out = ef.conv_bwd(act_tensor(dy_host, kind), fx["codes"], fx["clip_bits"], xd, fx["scale"], fx["zero_point"],
                      fw["codes"], fw["clip_bits"], wd, fw["scale"], idx if k else None, stride=stride, pad=pad,
                      dy_layout=layout, scatter=scatter, dx_kernel=dx_kernel)
    torch.cuda.synchronize()
    ref = orc.conv_bwd(dY, X, sx, zx, 8, W, sw, w_bits, idx_ref, stride, pad)
    assert np.array_equal(fx["codes"].cpu().numpy().astype(np.int64), ref["x_codes"])
    assert np.array_equal(clip_words(fx["clip_bits"]), pack_mask(ref["x_mask"].reshape(-1, c_in)))
    assert np.array_equal(clip_words(fw["clip_bits"]), pack_mask(ref["w_mask"].reshape(c_out, -1)))
    check_backward(out, ref, idx, idx_ref, X, W, (sx, zx, sw), kind, scatter, kind == "bf16", W.shape)


# ---------------------------------------------------------------- low-precision forward (int8 matrix cores)
FWD_CASES = [
    (256, 256, 256, 8, 1.0, torch.float32),
    (300, 208, 136, 4, 0.7, torch.float32),
    (300, 200, 136, 4, 0.7, torch.bfloat16),        # c_in not a multiple of 16: padded operand copies
    (517, 392, 264, 8, 0.8, torch.bfloat16),
    (1, 16, 8, 8, 1.0, torch.float32),
    (1024, 768, 3072, 8, 1.0, torch.bfloat16),
]


@pytest.mark.parametrize("case", FWD_CASES, ids=lambda c: "T%d_%dx%d_w%d_s%s_%s" % (
    c[0], c[1], c[2], c[3], c[4], "f32" if c[5] == torch.float32 else "bf16"))
def test_linear_fwd_int8_matches_oracle(case):
    T, c_in, c_out, w_bits, shrink, ydt = case
    X, W, _ = synth.linear_layer(900 + T + c_in, T, c_in, c_out, act_dtype="bf16")
    sx, zx = orc.act_qparams_minmax(X, 8)
    sw = orc.weight_scale_minmax(W, w_bits)
    sx = np.float32(sx * np.float32(shrink)); sw = (sw * np.float32(shrink)).astype(np.float32)
    zx = np.float32(zx + 0.3)                                     # forward uses round(Z_x)
    xd, wd = act_tensor(X, "bf16"), dev(W)
    fx = ef.fakequant_fwd(xd, ef.ACT_PER_TENSOR_ASYM, 8, init_minmax=False, scale=dev(np.array([sx])),
                          zero_point=dev(np.array([zx])))
    fw = ef.fakequant_fwd(wd, ef.W_PER_ROW_SYM, w_bits, init_minmax=False, scale=dev(sw))
    y = ef.linear_fwd(fx["codes"], fx["scale"], fx["zero_point"], fw["codes"], fw["scale"], y_dtype=ydt)
    torch.cuda.synchronize()
    ref = orc.linear_fwd(X, sx, zx, 8, W, sw, w_bits)
    # exact integer accumulation; only the two fp32 scale multiplications (and the bf16 store) round
    assert_max_err(host(y), ref, 2e-6 if ydt == torch.float32 else 2.0 ** -8, "Y")
    if ydt == torch.float32:
        xc, _, _ = orc.fakequant_act(X, sx, zx, 8)
        wc, _, _ = orc.fakequant_weight(W, sw, w_bits)
        acc = (xc - int(np.rint(float(zx)))) @ wc.T                 # int64, exact
        got = y.cpu().numpy().astype(np.float64) / (float(sx) * sw.astype(np.float64)[None, :])
        assert np.abs(got - acc).max() <= 2e-6 * max(1.0, np.abs(acc).max())

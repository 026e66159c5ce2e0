#!/usr/bin/env python3
"""Benchmark of the EfQAT backward hot path on one MI355X.

One "step" = one pass of the whole hot path over one batch of synthetic input, for every layer of the workload:
activation statistic + fake-quant, weight statistic + fake-quant, channel importance + Top-K, then the restricted
backward (dX product with fused STE / S_x, Z_x gradients; gathered dW product; mask + S_w gradients).  The headline
value is the backward TFLOP/s at the headline update fraction, 2*T*C_in*(C_out + k) per layer (Eq. 7 of the paper
times 2*T), over the whole step time.

The headline workload is the largest single-GPU configuration (config 5, the LLM-sized MLP pair) at r = 25 %.  The
`roofline` object of the output line carries, besides the dominant kernel (the dX product) against the bf16 matrix-core
peak:
  kernels    every kernel class of the headline step: time per step, algorithmic flops and bytes, the roofline time
             max(flops / peak, bytes / bandwidth) and the fraction of it that was reached;
  sweep      the backward call alone at every update fraction the config names (and r = 0), with the speedup over the
             full (r = 100 %) backward - the quantity the paper reports - and the cost over r = 0 against k;
  workloads  the same sweep, compact, for the other configurations (config 2 BERT FFN pair, config 3 encoder linears
             at W4A8 and W8A8, config 4 ResNet convolutions) and for both layouts of dY.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import glob
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg5", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--w-bits", type=int, default=0, help="weight bit width (default: the config's first)")
    ap.add_argument("--fraction", default=None, help="headline update fraction num/den (default 1/4)")
    ap.add_argument("--dy-layout", type=int, default=0, help="0 token major [T,C_out], 1 channel major")
    ap.add_argument("--streams", type=int, default=0, choices=[0, 1, 2],
                    help="2: the weight-side calls of each layer run on a second stream, joined before its backward; "
                         "1: one stream; 0: two streams except for the small workloads (cfg1, cfg4), whose kernels are "
                         "shorter than the cross-stream joins cost")
    ap.add_argument("--dw-stream", type=int, default=-1, choices=[-1, 0, 1],
                    help="1: the backward calls get a second stream (side_stream) for their weight-gradient branch; "
                         "-1: only for the workload that gains from it (cfg5)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--no-attach", action="store_true",
                    help="leave out the compact blocks for the other configurations and the other dY layout")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain device copy of 256 MiB (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


_HOST_CACHE = {}


def host_tensors(synth, key, make):
    """Seeded host tensors are shared by the variants of one layer (layouts, weight bit widths)."""
    if key not in _HOST_CACHE:
        _HOST_CACHE[key] = make()
    return _HOST_CACHE[key]


class Layer:
    """Device buffers of one layer, all allocated up front (nothing is allocated in a timed region)."""

    def __init__(self, ef, torch, name, seed, T, c_in, c_out, act_dtype, a_bits, w_bits, layout, synth, fracs,
                 conv=None, row_sigma=0.0):
        self.name, self.c_in, self.c_out, self.conv = name, c_in, c_out, conv
        self.a_bits, self.w_bits, self.layout = a_bits, w_bits, layout
        L = ef.lib()
        dyd = 1 if act_dtype == "bf16" else 0
        self.dyd = dyd
        ks = sorted({ef.k_from_ratio(c_out, n_, d_) for (n_, d_) in fracs} | {c_out})
        if conv is None:
            X, W, dY = host_tensors(synth, ("lin", seed, T, c_in, c_out, act_dtype, row_sigma),
                                    lambda: synth.linear_layer(seed, T, c_in, c_out, act_dtype=act_dtype,
                                                               row_scale_sigma=row_sigma))
            self.T, self.T_in, self.taps = T, T, 1
            bwd_ws = [L.efqat_linear_bwd_workspace_bytes(T, c_in, c_out, k_, dyd, layout) for k_ in ks]
        else:
            g = conv
            X, W, dY = host_tensors(synth, ("conv", seed, tuple(sorted(g.items())), act_dtype),
                                    lambda: synth.conv_layer(seed, g["N"], g["H"], g["W"], c_in, c_out, g["kh"], g["kw"],
                                                             g["stride"], g["pad"], act_dtype=act_dtype))
            self.T = int(np.prod(dY.shape[:3]))         # output pixels
            self.T_in = int(np.prod(X.shape[:3]))       # input pixels
            self.taps = g["kh"] * g["kw"]
            bwd_ws = [L.efqat_conv_bwd_workspace_bytes(g["N"], g["H"], g["W"], c_in, c_out, g["kh"], g["kw"],
                                                       g["stride"], g["pad"], k_, dyd, layout) for k_ in ks]
        self.host = (X, W, dY)
        tdt = torch.bfloat16 if act_dtype == "bf16" else torch.float32
        self.x = torch.from_numpy(X).to(tdt).cuda()
        self.w = torch.from_numpy(W).cuda()
        dy_dev = torch.from_numpy(dY).to(tdt).cuda()
        # channel major: [C_out][T] (transposed on the device: the values are the same bits)
        self.dy = dy_dev if layout == 0 else dy_dev.reshape(-1, c_out).t().contiguous()
        del dy_dev
        dev = self.x.device
        e = lambda shape, dt: torch.empty(shape, dtype=dt, device=dev)
        block = self.taps * c_in                         # weights per output channel
        self.fx = dict(codes=e(X.shape, torch.uint8), clip_bits=e((self.T_in, (c_in + 31) // 32), torch.int32),
                       scale=e(1, torch.float32), zero_point=e(1, torch.float32))
        self.fw = dict(codes=e(W.shape, torch.int8), clip_bits=e((c_out, (block + 31) // 32), torch.int32),
                       scale=e(c_out, torch.float32))
        self.scores = e(c_out, torch.float64)
        self.idx_full = e(c_out, torch.int32)
        self.dx = e(X.shape, tdt)
        self.dw = e(W.shape, torch.float32)              # compact [k, ...] uses the first k rows
        self.ds_w = e(c_out, torch.float32)
        self.ds_x, self.dz_x = e(1, torch.float32), e(1, torch.float32)
        # the backward workspace is not monotone in k: size it for every update fraction that will be run
        need = max(bwd_ws + [L.efqat_fakequant_fwd_workspace_bytes(self.T_in, c_in, 0),
                             L.efqat_channel_select_workspace_bytes(c_out)])
        self.ws = torch.empty(need, dtype=torch.uint8, device=dev)
        # the weight-side calls (quantize W, select) get a workspace of their own: they may run on a second stream
        need_w = max(L.efqat_fakequant_fwd_workspace_bytes(c_out, block, 1), L.efqat_channel_select_workspace_bytes(c_out))
        self.ws_w = torch.empty(max(need_w, 256), dtype=torch.uint8, device=dev)
        # bf16 W_q^T operand of the dX product, when the layer uses one: made on the weight side of the step
        nop = 0 if conv is not None else L.efqat_linear_bwd_weight_operand_bytes(self.T, c_in, c_out, dyd, layout)
        self.w_op = torch.empty(nop, dtype=torch.uint8, device=dev) if nop else None

    def quant_x(self, ef, init=True):
        x2 = self.x.view(self.T_in, self.c_in)
        fx2 = dict(self.fx, codes=self.fx["codes"].view(self.T_in, self.c_in))
        ef.fakequant_fwd(x2, ef.ACT_PER_TENSOR_ASYM, self.a_bits, init, ws=self.ws, out=fx2)

    def quant_w(self, ef):
        w2 = self.w.view(self.c_out, -1)
        fw2 = dict(self.fw, codes=self.fw["codes"].view(self.c_out, -1))
        ef.fakequant_fwd(w2, ef.W_PER_ROW_SYM, self.w_bits, True, ws=self.ws_w, out=fw2)

    def quant_w_select(self, ef, k):
        """The weight side of a step in one call (one read of the master weights): codes, mask, scales, scores, idx."""
        idx = self.idx_full[:k]
        ef.weight_quant_select(self.w, self.w_bits, k, ws=self.ws_w,
                               out=dict(self.fw, scores=self.scores, idx=idx))
        return idx

    def prepare_w(self, ef):
        if self.w_op is not None:
            ef.linear_bwd_weight_operand(self.fw["codes"].view(self.c_out, -1), self.fw["scale"], self.T,
                                         self.dyd, self.layout, out=self.w_op)

    def forward_quant(self, ef):
        self.quant_x(ef)
        self.quant_w(ef)

    def requant_given(self, ef):
        """Quantise X and W again with the scales / zero point the buffers hold (no min/max initialisation)."""
        x2 = self.x.view(self.T_in, self.c_in)
        w2 = self.w.view(self.c_out, -1)
        fx2 = dict(self.fx, codes=self.fx["codes"].view(self.T_in, self.c_in))
        fw2 = dict(self.fw, codes=self.fw["codes"].view(self.c_out, -1))
        ef.fakequant_fwd(x2, ef.ACT_PER_TENSOR_ASYM, self.a_bits, False, ws=self.ws, out=fx2)
        ef.fakequant_fwd(w2, ef.W_PER_ROW_SYM, self.w_bits, False, ws=self.ws_w, out=fw2)

    def clipped_fraction(self, torch):
        """Share of the activation elements whose clip-mask bit is 0 (columns are a multiple of 32 in every workload)."""
        table = torch.tensor([bin(i).count("1") for i in range(256)], dtype=torch.int64, device=self.x.device)
        ones = int(table[self.fx["clip_bits"].view(torch.uint8).long()].sum().item())
        return 1.0 - ones / float(self.T_in * self.c_in)

    def select(self, ef, k):
        idx = self.idx_full[:k]
        ef.channel_select(self.w.view(self.c_out, -1), k, ws=self.ws_w, out=dict(scores=self.scores, idx=idx))
        return idx

    def backward(self, ef, idx, prepared=False, side=None, step=None):
        k = int(idx.numel())
        out = dict(dx=self.dx, dw=self.dw[:max(k, 1)], ds_w=self.ds_w[:max(k, 1)], ds_x=self.ds_x, dz_x=self.dz_x)
        if self.conv is None:
            ef.linear_bwd(self.dy, self.fx["codes"], self.fx["clip_bits"], self.x, self.fx["scale"],
                          self.fx["zero_point"], self.fw["codes"], self.fw["clip_bits"], self.w, self.fw["scale"],
                          idx if k else None, dy_layout=self.layout, ws=self.ws, out=out,
                          w_operand=self.w_op if prepared else None, side_stream=side, step=step)
        else:
            ef.conv_bwd(self.dy, self.fx["codes"], self.fx["clip_bits"], self.x, self.fx["scale"],
                        self.fx["zero_point"], self.fw["codes"], self.fw["clip_bits"], self.w, self.fw["scale"],
                        idx if k else None, stride=self.conv["stride"], pad=self.conv["pad"],
                        dy_layout=self.layout, ws=self.ws, out=out, side_stream=side, step=step)

    def flops(self, k):
        # Eq. 7 / Eq. 8 op counts (x2 for multiply + add): dX over every channel, dW over the k selected ones
        return 2.0 * self.T * self.c_in * self.taps * (self.c_out + k)

    # ---- algorithmic work of each kernel class for one call on this layer: (flops, HBM bytes).  Bytes are what the
    # operation must move once: inputs read once, outputs written once; e = bytes per activation element.
    def work(self, k):
        e = 2 if self.dyd else 4
        T, Ti, ci, co, taps = self.T, self.T_in, self.c_in, self.c_out, self.taps
        nw = taps * ci                                   # weights per output channel
        w = {}
        # dX product + fused epilogue: dY, the int8 weight codes, x / codes / mask in, dX out
        w["dx"] = (2.0 * T * ci * taps * co, T * co * e + co * nw + Ti * ci * (e + 1 + 0.125) + Ti * ci * e)
        # dW product: the k selected columns (rows) of dY, the uint8 codes, k x n fp32 out
        w["dw"] = (2.0 * T * nw * k, T * k * e + Ti * ci + k * nw * 4.0) if k else (0.0, 0.0)
        # compaction of the selected dY columns (token-major dY only): read them, write them once as bf16
        w["prep"] = (0.0, (T * k * e + T * k * 2.0) if (k and k < co and self.layout == 0) else 0.0)
        # second pass: mask, master weights and codes of the k rows in, dW out (dS_w, dS_x, dZ_x are scalars)
        w["finish"] = (0.0, k * nw * (4 + 1 + 0.125) + k * nw * 4.0)
        # activation statistic (one read) + quantizer (one read, codes and mask out)
        w["quant_act"] = (0.0, Ti * ci * e + Ti * ci * (e + 1 + 0.125))
        w["quant_w"] = (0.0, co * nw * (4 + 1 + 0.125))
        w["importance"] = (0.0, co * nw * 4.0)
        w["topk"] = (0.0, co * 8.0 + k * 4.0)
        return w


CLASSES = [("dx", 0), ("dw", 1), ("prep", 3), ("finish", 4), ("quant_act", 5), ("quant_w", 6), ("importance", 7),
           ("topk", 8)]


_DW_SIDE = {"stream": None}


def dw_side_stream(torch, on=True):
    """The stream handed to the backward calls as side_stream (one per process), or None when switched off."""
    if not on:
        return None
    if _DW_SIDE["stream"] is None:
        _DW_SIDE["stream"] = torch.cuda.Stream()
    return _DW_SIDE["stream"]


def dw_stream_default(workload):
    # measured: the LLM-sized layers gain 1 - 2 % from running the two products side by side; on the smaller
    # workloads the dX product is a single round of workgroups and the fork / join costs what the overlap gains
    return workload == "cfg5"


def make_step(torch, ef, layers, ks, streams, dw_side=False, act_init=True):
    """One step over `layers` with ks[i] selected channels each: quantize X and W, select, restricted backward.

    The weight-side call of a layer (quantize W, importance, Top-K: small kernels that leave most of the chip idle)
    do not depend on its activations, so with streams == 2 they are issued on a second stream of the same (default)
    priority and joined before the layer's backward, together with the bf16 weight operand of the dX product
    (efqat_linear_bwd_weight_operand, handed to efqat_linear_bwd_ex); ev_bwd keeps the next step from rewriting a
    layer's weight codes, operand and idx while this step's backward still reads them.
    streams == 1 issues everything on one stream through the plain entry points."""
    main_stream = torch.cuda.current_stream()
    side_stream = torch.cuda.Stream() if streams == 2 else None
    dw_stream = dw_side_stream(torch, dw_side)
    ev_w = [torch.cuda.Event() for _ in layers]
    ev_bwd = [torch.cuda.Event() for _ in layers]

    def step():
        for i, (l, k) in enumerate(zip(layers, ks)):
            if side_stream is None:
                l.quant_x(ef, act_init)
                idx = l.quant_w_select(ef, k)
            else:
                side_stream.wait_event(ev_bwd[i])
                with torch.cuda.stream(side_stream):
                    idx = l.quant_w_select(ef, k)
                    l.prepare_w(ef)                      # the bf16 W_q^T operand of the dX product, where one is used
                    ev_w[i].record(side_stream)
                l.quant_x(ef, act_init)
                main_stream.wait_event(ev_w[i])
            l.backward(ef, idx, prepared=side_stream is not None, side=dw_stream)
            if side_stream is not None:
                ev_bwd[i].record(main_stream)
    return step


def time_region(torch, fn, steps):
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def profiled(torch, ef, fn, steps):
    """`steps` more runs of fn with the library's HIP events around every kernel class (on the stream the kernels go
    to).  Returns {class: (ms per run, brackets per run)}.  A separate pass, because every event record costs a few
    microseconds on the stream."""
    ef.profile_enable(True)
    sec = time_region(torch, fn, steps)
    res = {}
    for name, which in CLASSES:
        ms, n = ef.profile_read(which)
        res[name] = (ms / steps, n / steps)
    ef.profile_enable(False)
    res["_ms_with_events"] = sec * 1e3
    return res


def kernel_rows(layers, ks, prof):
    """Per kernel class of one step: measured time against the roofline time of its algorithmic work."""
    rows = []
    for name, _ in CLASSES:
        fl = sum(l.work(k)[name][0] for l, k in zip(layers, ks))
        by = sum(l.work(k)[name][1] for l, k in zip(layers, ks))
        ms, n = prof[name]
        if n == 0:
            continue
        t_mfma = fl / (PEAK_BF16_TFLOPS * 1e12) * 1e3
        t_hbm = by / (PEAK_HBM_GBS * 1e9) * 1e3
        roof = max(t_mfma, t_hbm)
        row = dict(kernel=name, ms=round(ms, 5), launches=round(n, 2), gflop=round(fl / 1e9, 3), mbytes=round(by / 1e6, 3),
                   bound="mfma" if t_mfma >= t_hbm else "hbm", roof_ms=round(roof, 5),
                   frac=round(roof / ms, 4) if (ms > 0 and roof > 0) else None)
        if fl:
            row["tflops"] = round(fl / ms / 1e9, 1)
        if by:
            row["gbps"] = round(by / ms / 1e6, 1)
        if name == "topk":                               # one workgroup, latency bound: microseconds are the figure
            row = dict(kernel=name, ms=round(ms, 5), launches=round(n, 2), bound="latency")
        rows.append(row)
    return rows


def products_per_layer(torch, ef, layers, ks, steps):
    """The two product kernels layer by layer, each against its own roofline time max(flops / MFMA peak, bytes / HBM
    peak): a short-K product such as the 3072 -> 768 FFN layer moves more bytes in its epilogue than its flops cover."""
    for l in layers:
        l.forward_quant(ef)
    rows = []
    for l, k in zip(layers, ks):
        idx = l.select(ef, k)
        one = lambda: l.backward(ef, idx)
        for _ in range(3):
            one()
        pl = profiled(torch, ef, one, max(3, steps // 2))
        row = dict(layer=l.name, k=k)
        for name in ("dx", "dw"):
            fl, by = l.work(k)[name]
            ms, n = pl[name]
            if n == 0:
                continue
            t_m, t_h = fl / (PEAK_BF16_TFLOPS * 1e12) * 1e3, by / (PEAK_HBM_GBS * 1e9) * 1e3
            row[name] = dict(ms=round(ms, 5), tflops=round(fl / ms / 1e9, 1), mbytes=round(by / 1e6, 1),
                             bound="mfma" if t_m >= t_h else "hbm", roof_ms=round(max(t_m, t_h), 5),
                             frac=round(max(t_m, t_h) / ms, 4))
        rows.append(row)
    return rows


def sweep_backward(torch, ef, layers, fracs, steps, warmup, per_layer, side=False):
    """The backward call alone at every fraction: total time, speedup over r = 100 %, cost over r = 0 against k."""
    for l in layers:
        l.forward_quant(ef)
    fr = sorted(set(fracs) | {(0, 1), (1, 1)}, key=lambda f: f[0] / f[1])
    rows, times = [], {}
    for (n_, d_) in fr:
        kk = [ef.k_from_ratio(l.c_out, n_, d_) for l in layers]
        idxs = [l.select(ef, k) for l, k in zip(layers, kk)]

        def bwd(side=None):
            for l, idx in zip(layers, idxs):
                l.backward(ef, idx, side=side)
        timed = (lambda: bwd(dw_side_stream(torch))) if side else bwd
        for _ in range(max(2, warmup)):
            timed()
        t = time_region(torch, timed, max(3, steps))
        prof = profiled(torch, ef, bwd, max(3, steps // 2))      # per class: on one stream, nothing overlaps
        times[(n_, d_)] = t
        fl = sum(l.flops(k) for l, k in zip(layers, kk))
        row = dict(r="%d/%d" % (n_, d_), k=kk, ms=round(t * 1e3, 5), tflops=round(fl / t / 1e12, 1),
                   dx_ms=round(prof["dx"][0], 5), dw_ms=round(prof["dw"][0], 5), prep_ms=round(prof["prep"][0], 5),
                   finish_ms=round(prof["finish"][0], 5))
        if per_layer:
            lay = []
            for l, idx, k_ in zip(layers, idxs, kk):
                one = lambda: l.backward(ef, idx, side=dw_side_stream(torch, side))
                for _ in range(2):
                    one()
                tl = time_region(torch, one, max(3, steps))
                lay.append(dict(name=l.name, k=k_, ms=round(tl * 1e3, 5), tflops=round(l.flops(k_) / tl / 1e12, 1)))
            row["layers"] = lay
        rows.append(row)
    full, zero = times[(1, 1)], times[(0, 1)]
    for row, key in zip(rows, fr):
        row["speedup_vs_full"] = round(full / times[key], 4)
        row["ideal_speedup"] = round(sum(l.flops(l.c_out) for l in layers)
                                     / sum(l.flops(k) for l, k in zip(layers, row["k"])), 4)   # Eq. 7 / Eq. 8 op counts
        row["over_r0_ms"] = round((times[key] - zero) * 1e3, 5)
        ksum = sum(row["k"])
        row["over_r0_us_per_channel"] = round((times[key] - zero) * 1e6 / ksum, 4) if ksum else None
    return rows


def build_layers(ef, torch, synth, workload, w_bits, layout, fracs, row_sigma=0.0):
    cfg = {"cfg1": synth.CFG1, "cfg2": synth.CFG2, "cfg3": synth.CFG3, "cfg4": synth.CFG4, "cfg5": synth.CFG5}[workload]
    if "layers" in cfg:
        return [Layer(ef, torch, n, cfg["seed"] + i, T, ci, co, cfg["act_dtype"], cfg["a_bits"], w_bits, layout, synth,
                      fracs, row_sigma=row_sigma) for i, (n, T, ci, co) in enumerate(cfg["layers"])]
    return [Layer(ef, torch, n, cfg["seed"] + i, 0, cfg[n]["c_in"], cfg[n]["c_out"], cfg["act_dtype"], cfg["a_bits"],
                  w_bits, layout, synth, fracs, conv=cfg[n]) for i, n in enumerate(("conv", "conv1x1"))]


def describe(workload, layers, num, den, w_bits, a_bits, layout):
    return "%s: %s, r=%d/%d, W%dA%d, dY %s-major" % (
        workload, ", ".join("%s T=%d %d->%d" % (l.name, l.T, l.c_in, l.c_out) for l in layers), num, den, w_bits,
        a_bits, "token" if layout == 0 else "channel")


def compact_block(torch, ef, synth, workload, w_bits, layout, num, den, steps, warmup):
    """Step time at the headline fraction and the backward sweep for one more workload / layout (compact)."""
    cfg = {"cfg2": synth.CFG2, "cfg3": synth.CFG3, "cfg4": synth.CFG4, "cfg5": synth.CFG5}[workload]
    fracs = list(cfg["fractions"]) + [(num, den), (0, 1), (1, 1)]
    layers = build_layers(ef, torch, synth, workload, w_bits, layout, fracs)
    ks = [ef.k_from_ratio(l.c_out, num, den) for l in layers]
    streams = 1 if workload in ("cfg1", "cfg4") else 2
    step = make_step(torch, ef, layers, ks, streams, dw_stream_default(workload))
    for _ in range(warmup):
        step()
    sec = time_region(torch, step, steps)
    prof = profiled(torch, ef, make_step(torch, ef, layers, ks, 1), max(3, steps // 2))   # one stream: see main()
    flops = sum(l.flops(k) for l, k in zip(layers, ks))
    dx_fl = sum(l.work(k)["dx"][0] for l, k in zip(layers, ks))
    blk = dict(workload=describe(workload, layers, num, den, w_bits, cfg["a_bits"], layout), k=ks,
               step_ms=round(sec * 1e3, 5), tflops=round(flops / sec / 1e12, 1),
               dx_frac_of_mfma_peak=round(dx_fl / (prof["dx"][0] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
               kernels=kernel_rows(layers, ks, prof),
               products_per_layer=products_per_layer(torch, ef, layers, ks, steps),
               sweep=sweep_backward(torch, ef, layers, cfg["fractions"], steps, warmup, per_layer=False,
                                    side=dw_stream_default(workload)))
    if workload == "cfg3":
        blk["note"] = ("the four linears of one encoder layer; the 12 layers of the stack repeat exactly this work "
                       "(x12 in time and flops)")
    del layers, step
    torch.cuda.empty_cache()
    return blk


def measured_traffic(workload, layout):
    """HBM bytes per launch of the dX product kernel as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE: read
    from the tracked profile summaries (lines `TRAFFIC <workload> layout=<0|1> kernel=dx fetch_bytes=.. write_bytes=..`).
    None when no summary covers this workload: the counters cannot be read from inside this process."""
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md")) + glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        for line in open(path):
            m = re.match(r"\s*TRAFFIC\s+(\S+)\s+layout=(\d)\s+kernel=dx\s+fetch_bytes=([0-9.eE+]+)\s+write_bytes=([0-9.eE+]+)", line)
            if m and m.group(1) == workload and int(m.group(2)) == layout:
                return dict(fetch_bytes=float(m.group(3)), write_bytes=float(m.group(4)),
                            total_bytes=float(m.group(3)) + float(m.group(4)), source=os.path.relpath(path, ROOT))
    return None


def cpu_baseline(host_data, num, den, a_bits, w_bits):
    """The oracle, as it stands, on the host cores: whole steps (every layer, all tokens) of the headline workload.
    host_data: (name, c_out, conv geometry or None, (X, W, dY), flops(k)) per layer."""
    from oracle import efqat_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    # whole steps of the workload (not a sub-sample), repeated until about ten seconds have passed (at most 12 times)
    t0 = time.perf_counter()
    fl = 0.0
    reps = 0
    while reps < 12 and (reps == 0 or time.perf_counter() - t0 < 10.0):
        for name, c_out, conv, (X, W, dY), flops in host_data:
            sx, zx = orc.act_qparams_minmax(X, a_bits)
            sw = orc.weight_scale_minmax(W, w_bits)
            k = orc.k_from_ratio(c_out, num, den)
            idx = orc.top_k_channels(orc.channel_importance(W), k)
            if conv is None:
                orc.linear_bwd(dY, X, sx, zx, a_bits, W, sw, w_bits, idx)
            else:
                orc.conv_bwd(dY, X, sx, zx, a_bits, W, sw, w_bits, idx, stride=conv["stride"], pad=conv["pad"])
            fl += flops(k)
        reps += 1
    dt = time.perf_counter() - t0
    return dict(value=fl / dt / 1e12, unit="TFLOP/s", cores=int(threads), kind="oracle",
                sample="%d whole step(s) of the same workload (%s; all tokens; r=%d/%d; quantize, select, backward), "
                       "fp64 NumPy, %.1f s" % (reps, ", ".join(h[0] for h in host_data), num, den, dt))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path would shard by tokens, one all-reduce of dW[idx] per layer); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2411_11038_amd as ef
    from workloads import synth

    if not os.path.exists(ef.lib_path()):
        from paper_2411_11038_amd import build as b
        b.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = {"cfg1": synth.CFG1, "cfg2": synth.CFG2, "cfg3": synth.CFG3, "cfg4": synth.CFG4,
           "cfg5": synth.CFG5}[args.workload]     # cfg3: the four linears of one encoder layer (the stack repeats them 12x)
    w_bits = args.w_bits or (cfg["w_bits"] if isinstance(cfg["w_bits"], int) else cfg["w_bits"][0])
    if args.fraction:
        num, den = (int(t) for t in args.fraction.split("/"))
    else:
        num, den = 1, 4
    fracs = list(cfg["fractions"]) + [(num, den), (0, 1), (1, 1)]
    layers = build_layers(ef, torch, synth, args.workload, w_bits, args.dy_layout, fracs)
    ks = [ef.k_from_ratio(l.c_out, num, den) for l in layers]

    if args.dw_stream < 0:
        args.dw_stream = int(dw_stream_default(args.workload))
    if args.streams == 0:
        args.streams = 1 if args.workload in ("cfg1", "cfg4") else 2
    step = make_step(torch, ef, layers, ks, args.streams, bool(args.dw_stream))

    for _ in range(args.warmup):
        step()
    # the timed region: exactly --steps steps, nothing but the library's launches on the stream
    sec = time_region(torch, step, args.steps)
    # a second pass of the same steps with HIP events recorded by the library around every kernel class (on the stream
    # the kernels run on) gives the kernel durations of the roofline block.  This pass issues the step on ONE stream:
    # with the weight side on a second stream its small kernels queue behind the products that fill the chip, and the
    # time between their events would be that wait, not their own duration.
    prof = profiled(torch, ef, make_step(torch, ef, layers, ks, 1), args.steps)
    flops = sum(l.flops(k) for l, k in zip(layers, ks))
    value = flops / sec / 1e12

    # dominant kernel: the dX product (always the full C_out); algorithmic flops per launch
    dx_flops = sum(l.work(k)["dx"][0] for l, k in zip(layers, ks)) / len(layers)
    dx_avg_s = prof["dx"][0] / max(prof["dx"][1], 1e-9) / 1e3
    achieved = dx_flops / dx_avg_s / 1e12 if prof["dx"][1] else 0.0
    traffic = measured_traffic(args.workload, args.dy_layout)
    roofline = dict(bound="mfma", achieved=achieved, peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                    frac=achieved / PEAK_BF16_TFLOPS, traffic=traffic["total_bytes"] if traffic else None,
                    traffic_detail=traffic,
                    kernel="dX product with fused epilogue (k_gemm_dx8 / k_gemm_kk / k_gemm_nt by shape)",
                    algorithmic_flops_per_launch=dx_flops,
                    algorithmic_bytes_per_launch=sum(l.work(k)["dx"][1] for l, k in zip(layers, ks)) / len(layers),
                    avg_kernel_ms=dx_avg_s * 1e3, launches_per_step=prof["dx"][1],
                    ms_per_step_with_events=prof["_ms_with_events"],
                    peaks=dict(bf16_mfma_tflops=PEAK_BF16_TFLOPS, hbm_gbps=PEAK_HBM_GBS),
                    kernels=kernel_rows(layers, ks, prof))

    if not args.no_sweep:
        roofline["products_per_layer"] = products_per_layer(torch, ef, layers, ks, args.steps)
        roofline["sweep"] = sweep_backward(torch, ef, layers, cfg["fractions"], args.steps, args.warmup, per_layer=True,
                                           side=bool(args.dw_stream))

    # The backward call at the headline fraction on inputs of different structure (not part of `value`): a contiguous
    # block of channels (the best case for the compaction of dY columns; the selected set of i.i.d. rows is scattered,
    # the worst case) and scales shrunk to 0.7x after the min/max initialisation (a few per cent of the elements fall
    # outside the range, so the clip masks and dZ_x do real work).
    if not args.no_sweep:
        def time_bwd(lays, idxs):
            def bwd():
                for l, idx in zip(lays, idxs):
                    l.backward(ef, idx)
            for _ in range(10):                          # host-side set-up precedes every variant: let the clocks settle
                bwd()
            return round(time_region(torch, bwd, max(3, args.steps)) * 1e3, 5)
        for l in layers:
            l.forward_quant(ef)
        idx_sel = [l.select(ef, k) for l, k in zip(layers, ks)]
        variants = dict(r="%d/%d" % (num, den), selected_idx_ms=time_bwd(layers, idx_sel))
        idx_blk = [torch.arange(k, dtype=torch.int32, device="cuda") for k in ks]
        variants["contiguous_idx_ms"] = time_bwd(layers, idx_blk)
        for l in layers:
            l.fx["scale"].mul_(0.7)
            l.fw["scale"].mul_(0.7)
            l.requant_given(ef)
        variants["scales_x0p7_ms"] = time_bwd(layers, idx_sel)
        variants["scales_x0p7_clipped_activation_share"] = [round(l.clipped_fraction(torch), 5) for l in layers]
        for l in layers:
            l.forward_quant(ef)                          # back to the min/max scales
        # the step as it runs once S_x, Z_x are trained parameters: Eq. 2's min / max pass is an initialisation, the
        # headline step repeats it every time
        step_given = make_step(torch, ef, layers, ks, args.streams, bool(args.dw_stream), act_init=False)
        for _ in range(args.warmup):
            step_given()
        variants["step_with_given_activation_scales_ms"] = round(time_region(torch, step_given, args.steps) * 1e3, 5)
        roofline["variants"] = variants

    # low-precision forward (int8 matrix cores) and bias gradient of the same layers: not part of the step or of
    # `value` (the paper leaves the forward pass out of its timings; biases are always updated)
    if not args.no_sweep:
        extras = {}
        if all(l.conv is None for l in layers):
            ys = [torch.empty((l.T, l.c_out), dtype=l.x.dtype, device="cuda") for l in layers]
            fws = [torch.empty(max(ef.lib().efqat_linear_fwd_workspace_bytes(l.T, l.c_in, l.c_out), 256),
                               dtype=torch.uint8, device="cuda") for l in layers]

            def fwd_all():
                for l, y, w_ in zip(layers, ys, fws):
                    ef.linear_fwd(l.fx["codes"], l.fx["scale"], l.fx["zero_point"], l.fw["codes"], l.fw["scale"],
                                  ws=w_, out=y)
            for _ in range(3):
                fwd_all()
            ef.profile_enable(True)
            time_region(torch, fwd_all, max(3, args.steps // 2))
            kms, kn = ef.profile_read(ef.PROF_FWD)
            ef.profile_enable(False)
            ops = sum(2.0 * l.T * l.c_in * l.c_out for l in layers) / len(layers)
            extras["forward_int8"] = dict(kernel_ms=round(kms / max(kn, 1), 5), tops=round(ops / (kms / max(kn, 1)) / 1e9, 1),
                                          peak_tops=5000.0, frac=round(ops / (kms / max(kn, 1)) / 1e9 / 5000.0, 4),
                                          note="Y = X_q W_q^T from the 8-bit codes, v_mfma_i32_32x32x32_i8, per layer")
            del ys, fws
        dbs = [torch.empty(l.c_out, dtype=torch.float32, device="cuda") for l in layers]
        bws = [torch.empty(max(ef.lib().efqat_bias_grad_workspace_bytes(l.T, l.c_out, args.dy_layout), 256),
                           dtype=torch.uint8, device="cuda") for l in layers]

        def bias_all():
            for l, d_, w_ in zip(layers, dbs, bws):
                ef.bias_grad(l.dy, dy_layout=args.dy_layout, ws=w_, out=d_)
        for _ in range(3):
            bias_all()
        tb = time_region(torch, bias_all, max(3, args.steps // 2))
        nbytes = sum(l.dy.numel() * l.dy.element_size() for l in layers)
        extras["bias_grad"] = dict(ms=round(tb * 1e3, 5), gbps=round(nbytes / tb / 1e9, 1), peak_gbps=PEAK_HBM_GBS,
                                   frac=round(nbytes / tb / 1e9 / PEAK_HBM_GBS, 4),
                                   note="db = column sums of dY, all layers, two launches per layer")
        del dbs, bws

        # optimizer step of the unfrozen channels inside the backward call (SGD with momentum on the weight rows,
        # Adam on their scales) against the plain call; learning rates of 0 keep the weights as they are
        idxs = [l.select(ef, k) for l, k in zip(layers, ks)]
        steps_ = [dict(lr_w=0.0, momentum=0.9, weight_decay=5e-4, mom_w=torch.zeros_like(l.w), lr_s=0.0,
                       adam_m=torch.zeros(l.c_out, device="cuda"), adam_v=torch.zeros(l.c_out, device="cuda"),
                       adam_t=torch.zeros(l.c_out, dtype=torch.int32, device="cuda")) for l in layers]

        def bwd_plain():
            for l, idx in zip(layers, idxs):
                l.backward(ef, idx)

        def bwd_step():
            for l, idx, st_ in zip(layers, idxs, steps_):
                l.backward(ef, idx, step=st_)
        for _ in range(3):
            bwd_plain(); bwd_step()
        tp = time_region(torch, bwd_plain, max(3, args.steps // 2))
        ts = time_region(torch, bwd_step, max(3, args.steps // 2))
        upd = sum(k * l.c_in * l.taps * 4.0 * 5 for l, k in zip(layers, ks))   # dW, W and momentum read; W, momentum written
        extras["fused_optimizer_step"] = dict(backward_ms=round(tp * 1e3, 5), backward_with_step_ms=round(ts * 1e3, 5),
                                              unfused_update_mbytes=round(upd / 1e6, 1),
                                              note="SGD (momentum 0.9, weight decay) on rows idx of W and Adam on S_w[idx] "
                                                   "inside the pass that finishes dW; a separate update pass would move "
                                                   "unfused_update_mbytes through HBM")
        del steps_, idxs

        # network-level (CWPN) and layer-level (LWPN) selection over a BERT-base-sized stack: 12 encoder layers of
        # four linears, 82944 output channels
        louts = [2304, 768, 3072, 768] * 12
        off = torch.tensor([0] + list(torch.tensor(louts).cumsum(0).tolist()), dtype=torch.int64, device="cuda")
        g_ = torch.Generator(device="cuda"); g_.manual_seed(7)
        sc = torch.rand(int(off[-1].item()), generator=g_, device="cuda", dtype=torch.float64)
        ktot = sc.numel() // 4
        for _ in range(3):
            ef.network_select(sc, off, ktot); ef.layer_select(sc, off, len(louts) // 4)
        tn = time_region(torch, lambda: ef.network_select(sc, off, ktot), 10)
        tl = time_region(torch, lambda: ef.layer_select(sc, off, len(louts) // 4), 10)
        extras["network_select"] = dict(ms=round(tn * 1e3, 5), channels=sc.numel(), k_total=ktot, layers=len(louts),
                                        note="EfQAT-CWPN: one Top-K over the channels of all layers")
        extras["layer_select"] = dict(ms=round(tl * 1e3, 5), layers=len(louts), k_layers=len(louts) // 4,
                                      note="EfQAT-LWPN: Top-K over the layers' mean scores")
        roofline["extras"] = extras

    workload_name = describe(args.workload, layers, num, den, w_bits, cfg["a_bits"], args.dy_layout)
    # for the CPU baseline, run last (nothing here may keep a layer's device buffers alive)
    host_data = [(l.name, l.c_out, l.conv, l.host,
                  (lambda T, ci, taps, co: (lambda k: 2.0 * T * ci * taps * (co + k)))(l.T, l.c_in, l.taps, l.c_out))
                 for l in layers]
    del layers, step
    torch.cuda.empty_cache()

    # the other configurations and the other dY layout, compact
    if not args.no_attach and not args.no_sweep:
        blocks = []
        st, wu = max(5, args.steps // 2), max(5, args.warmup)
        plan = [(args.workload, w_bits, 1 - args.dy_layout)]
        for wl in ("cfg2", "cfg3", "cfg4"):
            if wl == args.workload:
                continue
            c = {"cfg2": synth.CFG2, "cfg3": synth.CFG3, "cfg4": synth.CFG4}[wl]
            for wb in ((c["w_bits"],) if isinstance(c["w_bits"], int) else c["w_bits"]):
                for lay in (0, 1):
                    plan.append((wl, wb, lay))
        last = None
        for wl, wb, lay in plan:
            if last is not None and last != wl:
                _HOST_CACHE.clear()                      # host tensors of a finished workload
            last = wl
            blocks.append(compact_block(torch, ef, synth, wl, wb, lay, num, den, st, wu))
        roofline["workloads"] = blocks
        _HOST_CACHE.clear()

    out = dict(metric="QAT backward time + TFLOP/s per layer vs update fraction; speedup over full bwd",
               value=value, unit="TFLOP/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
               ms_per_step=sec * 1e3, higher_is_better=True, scaling="weak", vs_baseline=None, dtype="bf16",
               data="synthetic",
               config=dict(workload=workload_name, k=ks,
                           step="fakequant(X,W) + select + restricted backward, every layer", streams=args.streams,
                           dw_side_stream=bool(args.dw_stream),
                           paper_context="paper: 1.44-1.64x whole-network backward speedup on A10/A100 (not this machine)"),
               roofline=roofline)
    if args.calibrate_copy:
        a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        b = torch.empty_like(a)
        a.fill_(1)
        for _ in range(5):
            b.copy_(a)                                  # reads 256 MiB, writes 256 MiB per launch
        torch.cuda.synchronize()
    # the oracle on the host cores comes last: the GPU idles meanwhile, and GPU timings taken right after such a pause
    # would see its clocks ramp up again
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(host_data, num, den, cfg["a_bits"], w_bits)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

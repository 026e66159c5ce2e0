"""The step that bench.py times, with the weight-side calls on a second stream, must produce exactly what the
same step on one stream produces (the one-stream calls are compared with the oracle elsewhere): a missing join or
a shared scratch buffer between the two streams would show up here as differing bits."""
import numpy as np
import pytest
import torch

import paper_2411_11038_amd as ef
from workloads import synth

import bench

pytestmark = pytest.mark.gpu

# (T, c_in, c_out) pairs: whole 192-tiles (the pinned dX kernel with the straight-line epilogue) and ragged sizes
SHAPES = [
    [("a", 384, 192, 384), ("b", 384, 384, 192)],
    [("a", 300, 200, 136), ("b", 300, 136, 200)],
]


def _layers(shapes, layout):
    fracs = [(1, 4), (1, 1)]
    return [bench.Layer(ef, torch, n, 77 + i, T, ci, co, "bf16", 8, 8, layout, synth, fracs)
            for i, (n, T, ci, co) in enumerate(shapes)]


def _snapshot(layers, ks):
    torch.cuda.synchronize()
    out = []
    for l, k in zip(layers, ks):
        out.append(dict(dx=l.dx.view(torch.int16).cpu().numpy().copy(), dw=l.dw[:k].cpu().numpy().copy(),
                        ds_w=l.ds_w[:k].cpu().numpy().copy(), ds_x=l.ds_x.cpu().numpy().copy(),
                        dz_x=l.dz_x.cpu().numpy().copy(), idx=l.idx_full[:k].cpu().numpy().copy(),
                        xc=l.fx["codes"].cpu().numpy().copy(), wc=l.fw["codes"].cpu().numpy().copy(),
                        sw=l.fw["scale"].cpu().numpy().copy()))
    return out


@pytest.mark.parametrize("shapes", SHAPES)
@pytest.mark.parametrize("layout", [0, 1])
def test_two_stream_step_equals_one_stream_step(shapes, layout):
    ks = [ef.k_from_ratio(co, 1, 4) for (_, _, _, co) in shapes]
    ref_layers = _layers(shapes, layout)
    bench.make_step(torch, ef, ref_layers, ks, 1)()
    ref = _snapshot(ref_layers, ks)
    layers = _layers(shapes, layout)
    step = bench.make_step(torch, ef, layers, ks, 2)
    for it in range(4):                                  # consecutive steps: the cross-step event is exercised too
        for l in layers:                                 # outputs of the previous step must not be what is compared
            l.dx.zero_(); l.dw.zero_(); l.ds_w.zero_(); l.ds_x.zero_(); l.dz_x.zero_()
        torch.cuda.synchronize()
        step()
        got = _snapshot(layers, ks)
        for a, b in zip(got, ref):
            for key in b:
                assert np.array_equal(a[key], b[key]), (it, key)

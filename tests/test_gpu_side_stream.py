"""The optional second stream of efqat_linear_bwd_ex / efqat_conv_bwd_ex: the weight-gradient branch runs beside the
dX product and is joined before the pass that finishes dW; results are bit-identical to the one-stream call, call
after call, and the fork / join can be captured in a HIP graph."""
import pytest
import torch

import paper_2411_11038_amd as ef
from workloads import synth

from gpu_util import act_tensor, dev

pytestmark = pytest.mark.gpu

KEYS = ("dx", "dw", "ds_w", "ds_x", "dz_x")


def _linear_setup(seed, T, c_in, c_out, frac, layout):
    X, W, dY = synth.linear_layer(seed, T, c_in, c_out, act_dtype="bf16")
    xd, wd = act_tensor(X, "bf16"), dev(W)
    dyd = act_tensor(dY if layout == 0 else dY.T.copy(), "bf16")
    fx = ef.fakequant_fwd(xd, ef.ACT_PER_TENSOR_ASYM, 8, init_minmax=True)
    fw = ef.fakequant_fwd(wd, ef.W_PER_ROW_SYM, 4, init_minmax=True)
    k = ef.k_from_ratio(c_out, *frac)
    idx, _ = ef.channel_select(wd, k)

    def call(side, ws=None, out=None):
        return ef.linear_bwd(dyd, fx["codes"], fx["clip_bits"], xd, fx["scale"], fx["zero_point"], fw["codes"],
                             fw["clip_bits"], wd, fw["scale"], idx if k else None, dy_layout=layout, side_stream=side,
                             ws=ws, out=out)
    return call, k


@pytest.mark.parametrize("layout", [0, 1])
@pytest.mark.parametrize("shape,frac", [((1024, 768, 768), (1, 20)), ((300, 208, 136), (1, 4)), ((2048, 512, 1024), (1, 1)),
                                        ((520, 208, 264), (0, 1)), ((130, 70, 43), (1, 3))])
def test_linear_bwd_with_a_second_stream_is_bit_identical(shape, frac, layout):
    call, k = _linear_setup(91 + layout, *shape, frac, layout)
    ref = call(None)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    for rep in range(3):                                 # back to back: the library's events are used again at once
        got = call(side)
    torch.cuda.synchronize()
    for key in KEYS:
        if k or key in ("dx", "ds_x", "dz_x"):
            assert torch.equal(ref[key], got[key]), key


def test_conv_bwd_with_a_second_stream_is_bit_identical():
    N, H, W, c_in, c_out = 4, 10, 9, 128, 64
    X, Wt, dY = synth.conv_layer(17, N, H, W, c_in, c_out, 3, 3, 1, 1, act_dtype="bf16")
    xd, wd, dyd = act_tensor(X, "bf16"), dev(Wt), act_tensor(dY, "bf16")
    fx = ef.fakequant_fwd(xd, ef.ACT_PER_TENSOR_ASYM, 8, init_minmax=True)
    fw = ef.fakequant_fwd(wd, ef.W_PER_ROW_SYM, 4, init_minmax=True)
    idx, _ = ef.channel_select(wd, 16)
    call = lambda side: ef.conv_bwd(dyd, fx["codes"], fx["clip_bits"], xd, fx["scale"], fx["zero_point"], fw["codes"],
                                    fw["clip_bits"], wd, fw["scale"], idx, stride=1, pad=1, side_stream=side)
    ref = call(None)
    side = torch.cuda.Stream()
    got = call(side)
    got = call(side)
    torch.cuda.synchronize()
    for key in KEYS:
        assert torch.equal(ref[key], got[key]), key


def test_second_stream_fork_and_join_replay_from_a_graph():
    T, c_in, c_out = 1024, 256, 512
    call, k = _linear_setup(5, T, c_in, c_out, (1, 4), 0)
    e = lambda shape, dt: torch.empty(shape, dtype=dt, device="cuda")
    out = dict(dx=e((T, c_in), torch.bfloat16), dw=e((k, c_in), torch.float32), ds_w=e(k, torch.float32),
               ds_x=e(1, torch.float32), dz_x=e(1, torch.float32))
    ws = e(ef.lib().efqat_linear_bwd_workspace_bytes(T, c_in, c_out, k, ef.BF16, 0), torch.uint8)
    ref = {key: t.clone() for key, t in call(None).items()}
    side = torch.cuda.Stream()
    cap = torch.cuda.Stream()
    cap.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(cap):
        call(side, ws, out)                              # first use outside the capture: the events are made here
    torch.cuda.current_stream().wait_stream(cap)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call(side, ws, out)
    for rep in range(3):
        for t in out.values():
            t.zero_()
        ws.random_(0, 255)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for key in KEYS:
            assert torch.equal(ref[key], out[key]), (rep, key)

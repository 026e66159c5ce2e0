"""The library's launches can be captured in a HIP graph (no allocation, no memset, no synchronisation inside the
calls) and replays reproduce the eager results bit for bit, also with other work in between."""
import numpy as np
import pytest
import torch

import paper_2411_11038_amd as ef
from workloads import synth

from gpu_util import act_tensor, dev

pytestmark = pytest.mark.gpu


def test_backward_step_replays_from_a_graph():
    T, c_in, c_out = 520, 208, 264
    X, W, dY = synth.linear_layer(4242, T, c_in, c_out, act_dtype="bf16")
    xd, wd, dyd = act_tensor(X, "bf16"), dev(W), act_tensor(dY, "bf16")
    k = ef.k_from_ratio(c_out, 1, 4)
    L = ef.lib()
    e = lambda shape, dt: torch.empty(shape, dtype=dt, device="cuda")
    fx = dict(codes=e((T, c_in), torch.uint8), clip_bits=e((T, (c_in + 31) // 32), torch.int32),
              scale=e(1, torch.float32), zero_point=e(1, torch.float32))
    fw = dict(codes=e((c_out, c_in), torch.int8), clip_bits=e((c_out, (c_in + 31) // 32), torch.int32),
              scale=e(c_out, torch.float32))
    sel = dict(scores=e(c_out, torch.float64), idx=e(k, torch.int32))
    out = dict(dx=e((T, c_in), torch.bfloat16), dw=e((k, c_in), torch.float32), ds_w=e(k, torch.float32),
               ds_x=e(1, torch.float32), dz_x=e(1, torch.float32))
    db = e(c_out, torch.float32)
    need = max(L.efqat_linear_bwd_workspace_bytes(T, c_in, c_out, k, 1, 0),
               L.efqat_fakequant_fwd_workspace_bytes(T, c_in, 0), L.efqat_channel_select_workspace_bytes(c_out),
               L.efqat_bias_grad_workspace_bytes(T, c_out, 0))
    ws = e(need, torch.uint8)

    def step():
        ef.fakequant_fwd(xd, ef.ACT_PER_TENSOR_ASYM, 8, True, ws=ws, out=fx)
        ef.fakequant_fwd(wd, ef.W_PER_ROW_SYM, 8, True, ws=ws, out=fw)
        ef.channel_select(wd, k, ws=ws, out=sel)
        ef.linear_bwd(dyd, fx["codes"], fx["clip_bits"], xd, fx["scale"], fx["zero_point"], fw["codes"],
                      fw["clip_bits"], wd, fw["scale"], sel["idx"], ws=ws, out=out)
        ef.bias_grad(dyd, ws=ws, out=db)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (*out.values(), db, fx["codes"], fw["codes"], sel["idx"])]

    step()
    ref = snapshot()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                       # warm-up on the capture stream (first-launch attributes)
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for rep in range(3):
        for t in (*out.values(), db):
            t.zero_()                                # eager work between the replays
        ws.random_(0, 255)                           # the workspace carries nothing from one call to the next
        torch.cuda.synchronize()
        g.replay()
        got = snapshot()
        for a, b in zip(ref, got):
            assert torch.equal(a, b), rep

"""The entry point that allocates nothing (efqat_channel_select_static: its scratch is a device array inside the
library) against the plain entry point it is a variant of, through the C ABI: two calls in a row on the same GPU,
the second on a smaller input, so that whatever the first call left in the shared scratch is still there."""
import numpy as np
import pytest
import torch

import paper_2411_11038_amd as ef
from workloads import synth

from gpu_util import dev

pytestmark = pytest.mark.gpu


def _both(W, k):
    """(idx of the plain call, idx of the static call) for the same weights, straight through the library's symbols."""
    L = ef.lib()
    wd = dev(W)
    c_out, block = W.shape[0], int(np.prod(W.shape[1:]))
    stream = torch.cuda.current_stream().cuda_stream
    ws = torch.empty(L.efqat_channel_select_workspace_bytes(c_out), dtype=torch.uint8, device="cuda")
    idx_a = torch.full((max(k, 1),), -1, dtype=torch.int32, device="cuda")
    idx_b = torch.full((max(k, 1),), -1, dtype=torch.int32, device="cuda")
    rc = L.efqat_channel_select(wd.data_ptr(), c_out, block, k, None, idx_a.data_ptr(), ws.data_ptr(), ws.numel(),
                                stream)
    assert rc == 0
    rc = L.efqat_channel_select_static(wd.data_ptr(), c_out, block, k, idx_b.data_ptr(), stream)
    assert rc == 0
    torch.cuda.synchronize()
    return idx_a.cpu().numpy()[:k], idx_b.cpu().numpy()[:k]


def test_static_select_equals_plain_select_on_two_calls_in_a_row():
    # first call: 3072 channels (BERT FFN width), duplicated rows so that ties are decided too
    W1 = synth.normal(611, 1, (3072, 768), std=0.02).astype(np.float32)
    W1[100] = W1[7]; W1[2000] = W1[7]
    a, b = _both(W1, 768)
    assert np.array_equal(a, b) and len(set(b.tolist())) == 768 and np.all(np.diff(b) > 0)
    # second call: fewer channels and another row length; the scratch still holds 3072 scores of the first call
    W2 = synth.normal(612, 1, (200, 3, 3, 24), std=0.02).astype(np.float32)
    a, b = _both(W2, 50)
    assert np.array_equal(a, b) and np.all(np.diff(b) > 0)
    # and k = C_out, k = 0 (nothing written)
    a, b = _both(W2, 200)
    assert np.array_equal(a, np.arange(200)) and np.array_equal(b, np.arange(200))
    a, b = _both(W2, 0)
    assert a.size == 0 and b.size == 0


def test_static_select_rejects_more_channels_than_its_scratch_holds():
    L = ef.lib()
    w = torch.zeros(8, dtype=torch.float32, device="cuda")
    idx = torch.zeros(8, dtype=torch.int32, device="cuda")
    assert L.efqat_channel_select_static(w.data_ptr(), 65537, 1, 1, idx.data_ptr(), None) == -6

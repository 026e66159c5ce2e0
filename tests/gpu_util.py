"""Helpers shared by the GPU parity tests: host<->device conversion and tolerance checks.
Holds no arithmetic of the method."""
import numpy as np
import torch


def report(line):
    """Measured error figures: printed (pytest shows them with -s / -rP) and, when EFQAT_ERR_REPORT names a file,
    appended there with the id of the running test."""
    import os
    print(line)
    path = os.environ.get("EFQAT_ERR_REPORT")
    if path:
        with open(path, "a") as f:
            f.write("%s :: %s\n" % (os.environ.get("PYTEST_CURRENT_TEST", "?"), line))


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def act_tensor(a32, kind):
    """fp32 numpy (bf16-representable when kind == 'bf16') -> device tensor of that dtype."""
    return dev(a32, torch.bfloat16 if kind == "bf16" else torch.float32)


def pack_mask(mask2d):
    """bool [rows, cols] -> uint32 [rows, ceil(cols/32)], bit j%32 of word j/32 (1 = in range)."""
    rows, cols = mask2d.shape
    wpr = (cols + 31) // 32
    b = np.packbits(mask2d.astype(np.uint8), axis=1, bitorder="little")
    pad = wpr * 4 - b.shape[1]
    if pad:
        b = np.concatenate([b, np.zeros((rows, pad), np.uint8)], axis=1)
    return np.ascontiguousarray(b).view(np.uint32)


def host(t):
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy().astype(np.float64)
    return t.cpu().numpy()


def clip_words(t):
    return t.cpu().numpy().view(np.uint32)


def assert_max_err(got, ref, rel, what):
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    scale = np.abs(ref).max() if ref.size else 0.0
    err = np.abs(got - ref).max() if ref.size else 0.0
    assert err <= rel * scale + 1e-30, f"{what}: max|err| {err:.3e} > {rel:g} * max|ref| {scale:.3e}"


def assert_rms_err(got, ref, rel, what):
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    if not ref.size:
        return
    e = np.sqrt(np.mean((got - ref) ** 2)); s = np.sqrt(np.mean(ref ** 2))
    assert e <= rel * s + 1e-30, f"{what}: rms err {e:.3e} > {rel:g} * rms ref {s:.3e}"

"""Helpers for the GPU parity tests: device upload, packing, error metrics (no method arithmetic)."""
import numpy as np


def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need a GPU"
    return torch


def to_dev(a):
    torch = torch_cuda()
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    return torch.from_numpy(a).cuda()


def pack_layer(goq, q):
    """canonical dict (numpy) -> packed device buffer (torch uint8)."""
    torch = torch_cuda()
    out, inn = q["codes"].shape
    nbytes = goq.packed_bytes(q["bw"], out, inn)
    packed = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    dev = [to_dev(q[k]) for k in ("codes", "pattern", "signs", "c1", "c2")]
    goq.pack(q["bw"], out, inn, *dev, packed)
    torch.cuda.synchronize()
    return packed


def a16_errors(y, ref, x, what_abs=None):
    """(i) max |y - ref| / max(|ref|, 1e-2 rms(ref));  (ii) backward error vs sum |x||W^| if given."""
    y = np.asarray(y, np.float64)
    ref = np.asarray(ref, np.float64)
    rms = np.sqrt(np.mean(ref ** 2))
    e1 = np.max(np.abs(y - ref) / np.maximum(np.abs(ref), 1e-2 * rms + 1e-300))
    e2 = None
    if what_abs is not None:
        scale = np.abs(np.asarray(x, np.float64)) @ what_abs.T
        e2 = np.max(np.abs(y - ref) / np.maximum(scale, 1e-300))
    return e1, e2

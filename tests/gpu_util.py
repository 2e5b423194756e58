"""Helpers for the GPU parity tests: move arrays to the device, call the C ABI through the
binding, bring bytes back.  No arithmetic of the method lives here."""
import numpy as np


def torch_mod():
    import torch
    return torch


def to_dev(x, bf16=False):
    """float32 numpy array -> device tensor (float32, or bfloat16 via RNE bits)."""
    torch = torch_mod()
    import synthetic_inputs as si
    if bf16:
        bits = si.to_bf16_bits(x).reshape(-1)
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16), bits
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32).reshape(-1)).cuda(), None


def dev_bytes(t):
    return t.detach().cpu().numpy().tobytes()


def out_to_numpy(t):
    """x_hat device tensor -> float32 array, or uint16 bit patterns for bfloat16."""
    torch = torch_mod()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def bytes_to_dev(b):
    torch = torch_mod()
    arr = np.frombuffer(bytes(b), dtype=np.uint8).copy()
    if arr.size == 0:
        return torch.empty(0, dtype=torch.uint8, device="cuda")
    return torch.from_numpy(arr).cuda()


def first_mismatch(a, b):
    a = np.frombuffer(a, dtype=np.uint8)
    b = np.frombuffer(b, dtype=np.uint8)
    if a.size != b.size:
        return "sizes %d vs %d" % (a.size, b.size)
    bad = np.nonzero(a != b)[0]
    if bad.size == 0:
        return None
    i = int(bad[0])
    return "%d of %d bytes differ, first at %d: %d vs %d" % (bad.size, a.size, i, a[i], b[i])

"""accept_compress_noalloc (the entry point for callers that cannot allocate) against
accept_compress: same header and payload bytes, on two calls in a row, the second with a
smaller input, so that whatever the first call left in the library's scratch is still there."""
import ctypes

import numpy as np
import pytest

import synthetic_inputs as si

from gpu_util import dev_bytes, first_mismatch, to_dev, torch_mod

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def A():
    torch = torch_mod()
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2311_05827_amd as pkg
    return pkg


def both_ways(A, d, xd, alpha):
    """(header, payload) bytes from accept_compress and from accept_compress_noalloc."""
    torch = torch_mod()
    h1, p1, w1 = A.alloc_outputs(d, xd.device)
    h2, p2, _ = A.alloc_outputs(d, xd.device)
    for t in (h1, p1, h2, p2):
        t.fill_(0xA5)
    torch.cuda.synchronize()
    A.accept_compress(d, xd, alpha_prev=alpha, header=h1, payload=p1, workspace=w1)
    before = torch.cuda.memory_allocated()
    A.accept_compress_noalloc(d, xd, alpha, h2, p2)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    return (dev_bytes(h1), dev_bytes(p1)), (dev_bytes(h2), dev_bytes(p2))


CASES = [
    # (scheme, k, channels, bf16, first shape, second, smaller shape)
    ("U", 8, 0, False, (16, 100003), (3, 8455)),
    ("U", 3, 0, False, (9, 70001), (2, 4099)),
    ("U", 6, 64, False, (12, 64 * 3136), (4, 64 * 784)),
    ("U", 4, 32, True, (8, 32 * 1024), (2, 32 * 512)),
    ("U", 5, 7, False, (5, 7 * 33), (3, 7 * 9)),       # short unaligned segments
    ("M", 2, 0, False, (64, 40004), (21, 4100)),
    ("M", 4, 0, False, (40, 50000), (8, 1028)),
    ("M", 3, 0, True, (24, 16384), (13, 2056)),
    ("M", 6, 0, False, (16, 9000), (5, 1003)),
]


@pytest.mark.parametrize("scheme,k,channels,bf16,big,small", CASES)
def test_two_calls_in_a_row_second_smaller(A, scheme, k, channels, bf16, big, small):
    torch = torch_mod()
    for call, shape in enumerate((big, small)):
        n, m = shape
        print("noalloc", scheme, "k", k, "C", channels, "bf16", bf16, "call", call, "shape", shape, flush=True)
        kind = "grad_outliers" if scheme == "U" else "relu_lognormal"
        x = si.make_shape(kind, (n, m), 900 + 10 * k + call)
        xd, _ = to_dev(x, bf16)
        tcode = A.BF16 if bf16 else A.F32
        if scheme == "U":
            d = A.make_desc(A.UNIFORM, k, n, m, channels=channels, in_dtype=tcode)
            alpha = None
        else:
            d = A.make_desc(A.MBQ, k, n, m, in_dtype=tcode, t=2)
            alpha = A.accept_mbq_init(d, xd)
            torch.cuda.synchronize()
        (h1, p1), (h2, p2) = both_ways(A, d, xd, alpha)
        assert h1 == h2, "header: " + str(first_mismatch(h1, h2))
        mm = first_mismatch(p1, p2)
        assert mm is None, "payload: " + mm


def test_limits_and_bad_arguments(A):
    lib = A.binding.lib
    V = ctypes.c_void_p
    good = A.make_desc(A.UNIFORM, 4, 4, 4)
    assert lib.accept_compress_noalloc(ctypes.byref(good), None, None, None, None, None) == 1
    assert lib.accept_compress_noalloc(ctypes.byref(good), V(0x1008), None, V(0x2000), V(0x3000), None) == 1
    # more (row, channel) partial maxima than the built-in scratch holds: refused, nothing launched
    huge = A.make_desc(A.UNIFORM, 4, 1024, 1024 * 512, channels=1024)
    assert A.accept_workspace_size(huge) > (1 << 20)
    assert lib.accept_compress_noalloc(ctypes.byref(huge), V(0x1000), None, V(0x2000), V(0x3000), None) == 2

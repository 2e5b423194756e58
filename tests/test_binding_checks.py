"""The binding refuses tensors that do not fit the descriptor before any pointer reaches the
library (the C functions take no capacities).  Runs without a GPU: the checks only look at the
tensors' metadata, so stand-ins that say they live on the device are enough, and the library
call itself is replaced by a recorder that must never be reached."""
import pytest

import paper_2311_05827_amd as A
from paper_2311_05827_amd import binding as B


class FakeTensor:
    """Metadata of a device tensor: dtype, element count, device flag, contiguity."""

    def __init__(self, dtype, numel, cuda=True, contiguous=True):
        import torch
        self.dtype = dtype
        self._numel = numel
        self.is_cuda = cuda
        self._contig = contiguous
        self._esize = torch.empty(0, dtype=dtype).element_size()
        self.device = "cuda:0"

    def numel(self):
        return self._numel

    def element_size(self):
        return self._esize

    def is_contiguous(self):
        return self._contig

    def data_ptr(self):
        raise AssertionError("a rejected call must not take a pointer")


@pytest.fixture()
def no_library_calls(monkeypatch):
    class Recorder:
        def __getattr__(self, name):
            real = getattr(B_REAL_LIB, name)
            if name in ("accept_packed_size", "accept_workspace_size", "accept_status_string"):
                return real
            def forbidden(*a, **k):
                raise AssertionError("library entry point %s reached with bad arguments" % name)
            return forbidden
    global B_REAL_LIB
    B_REAL_LIB = B.lib
    monkeypatch.setattr(B, "lib", Recorder())
    monkeypatch.setattr(B, "_stream_handle", lambda: None)
    yield


def bufs(desc, torch, shrink_header=0, shrink_payload=0, shrink_workspace=0):
    hb, pb = A.accept_packed_size(desc)
    wb = A.accept_workspace_size(desc)
    return (FakeTensor(torch.uint8, hb - shrink_header), FakeTensor(torch.uint8, pb - shrink_payload),
            FakeTensor(torch.uint8, wb - shrink_workspace))


def test_compress_rejects_wrong_dtype_short_or_host_tensors(no_library_calls):
    import torch
    n, m = 8, 1024
    d = A.make_desc(A.UNIFORM, 4, n, m)
    h, p, w = bufs(d, torch)
    with pytest.raises(A.AcceptError) as e:  # a bf16 tensor with a float32 descriptor
        A.accept_compress(d, FakeTensor(torch.bfloat16, n * m), header=h, payload=p, workspace=w)
    assert e.value.status == B.INVALID_ARG
    with pytest.raises(A.AcceptError) as e:  # a last, smaller batch
        A.accept_compress(d, FakeTensor(torch.float32, n * m - 1), header=h, payload=p, workspace=w)
    assert e.value.status == B.BUFFER_TOO_SMALL
    with pytest.raises(A.AcceptError):
        A.accept_compress(d, FakeTensor(torch.float32, n * m, cuda=False), header=h, payload=p, workspace=w)
    with pytest.raises(A.AcceptError):
        A.accept_compress(d, FakeTensor(torch.float32, n * m, contiguous=False), header=h, payload=p, workspace=w)
    with pytest.raises(TypeError):
        A.accept_compress(d, FakeTensor(torch.float16, n * m), header=h, payload=p, workspace=w)


@pytest.mark.parametrize("which", ["header", "payload", "workspace"])
def test_compress_rejects_small_output_buffers(no_library_calls, which):
    import torch
    n, m = 16, 4096
    for d in (A.make_desc(A.UNIFORM, 5, n, m, channels=8), A.make_desc(A.MBQ, 3, n, m)):
        h, p, w = bufs(d, torch, **{"shrink_" + which: 1})
        alpha = FakeTensor(torch.float32, d.bits)
        with pytest.raises(A.AcceptError) as e:
            A.accept_compress(d, FakeTensor(torch.float32, n * m), alpha_prev=alpha, header=h, payload=p, workspace=w)
        assert e.value.status == B.BUFFER_TOO_SMALL


def test_mbq_needs_k_previous_coefficients(no_library_calls):
    import torch
    n, m = 16, 4096
    d = A.make_desc(A.MBQ, 4, n, m)
    h, p, w = bufs(d, torch)
    x = FakeTensor(torch.float32, n * m)
    with pytest.raises(A.AcceptError) as e:
        A.accept_compress(d, x, alpha_prev=FakeTensor(torch.float32, 3), header=h, payload=p, workspace=w)
    assert e.value.status == B.BUFFER_TOO_SMALL
    with pytest.raises(A.AcceptError):
        A.accept_compress(d, x, alpha_prev=None, header=h, payload=p, workspace=w)
    with pytest.raises(A.AcceptError):
        A.accept_compress(d, x, alpha_prev=FakeTensor(torch.bfloat16, 4), header=h, payload=p, workspace=w)
    with pytest.raises(A.AcceptError):
        A.accept_compress_noalloc(d, x, FakeTensor(torch.float32, 2), h, p)
    with pytest.raises(A.AcceptError):
        A.accept_mbq_compress_first(d, FakeTensor(torch.float32, n * m - 8), header=h, payload=p, workspace=w)
    with pytest.raises(A.AcceptError):
        A.accept_mbq_init(d, x, alpha0=FakeTensor(torch.float32, 3), workspace=w)


def test_decompress_rejects_small_or_mistyped_buffers(no_library_calls):
    import torch
    n, m = 8, 2048
    d = A.make_desc(A.UNIFORM, 3, n, m, out_dtype=A.BF16)
    h, p, _ = bufs(d, torch)
    with pytest.raises(A.AcceptError) as e:
        A.accept_decompress(d, h, p, out=FakeTensor(torch.float32, n * m))   # descriptor says bfloat16
    assert e.value.status == B.INVALID_ARG
    with pytest.raises(A.AcceptError) as e:
        A.accept_decompress(d, h, p, out=FakeTensor(torch.bfloat16, n * m - 1))
    assert e.value.status == B.BUFFER_TOO_SMALL
    h2, p2, _ = bufs(d, torch, shrink_payload=1)
    with pytest.raises(A.AcceptError):
        A.accept_decompress(d, h2, p2, out=FakeTensor(torch.bfloat16, n * m))
    bad = A.make_desc(A.UNIFORM, 9, n, m)
    with pytest.raises(A.AcceptError):
        A.accept_decompress(bad, h, p, out=FakeTensor(torch.float32, n * m))

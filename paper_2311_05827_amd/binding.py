"""ctypes binding of libaccept.so: argument marshalling only.

Every step of the compression path runs in the library's HIP kernels; this module turns
PyTorch device tensors into pointers, allocates the output buffers with ``torch.empty`` and
passes the current HIP stream.  Function names follow the C ABI (include/accept.h).  There
is no CPU fallback: if the shared library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libaccept.so")

UNIFORM, MBQ = 0, 1
F32, BF16 = 0, 1
ROUND_NEAREST_EVEN, ROUND_STOCHASTIC = 0, 1
LAYOUT_PACKED, LAYOUT_BATCH, LAYOUT_UNENCODED = 0, 1, 2
MAX_STAGES = 8

STATUS_NAMES = {0: "ACCEPT_OK", 1: "ACCEPT_ERR_INVALID_ARG", 2: "ACCEPT_ERR_UNSUPPORTED",
                3: "ACCEPT_ERR_BUFFER_TOO_SMALL", 4: "ACCEPT_ERR_HIP"}


class AcceptError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__("%s: %s (%s)" % (where, STATUS_NAMES.get(self.status, self.status),
                                          status_string(self.status)))


class Desc(ctypes.Structure):
    """Mirror of accept_desc."""
    _fields_ = [
        ("scheme", ctypes.c_int32), ("bits", ctypes.c_int32),
        ("in_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
        ("n", ctypes.c_int64), ("m", ctypes.c_int64), ("channels", ctypes.c_int64),
        ("rounding", ctypes.c_int32), ("layout", ctypes.c_int32),
        ("seed", ctypes.c_uint64), ("t", ctypes.c_int64),
    ]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "libaccept.so is not built (%s). Run `python -m paper_2311_05827_amd.build`; "
            "there is no CPU fallback." % LIB_PATH)
    # PyTorch first: it brings its own copy of the HIP runtime, and the library and PyTorch must
    # share one (they exchange stream handles and device pointers).  The dynamic loader gives
    # the library whichever copy is already in the process, so the order of the two loads decides.
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    P, V, I = ctypes.POINTER, ctypes.c_void_p, ctypes.c_int
    sz = P(ctypes.c_size_t)
    lib.accept_packed_size.argtypes = [P(Desc), sz, sz]
    lib.accept_workspace_size.argtypes = [P(Desc), sz]
    lib.accept_compress.argtypes = [P(Desc), V, V, V, V, V, V]
    lib.accept_decompress.argtypes = [P(Desc), V, V, V, V]
    lib.accept_compress_noalloc.argtypes = [P(Desc), V, V, V, V, V]
    lib.accept_mbq_init.argtypes = [P(Desc), V, V, V, V]
    lib.accept_mbq_compress_first.argtypes = [P(Desc), V, V, V, V, V]
    lib.accept_compress_timed.argtypes = [P(Desc), V, V, V, V, V, V, P(ctypes.c_float), P(I)]
    lib.accept_decompress_timed.argtypes = [P(Desc), V, V, V, V, P(ctypes.c_float), P(I)]
    lib.accept_stage_name.argtypes = [P(Desc), I, I]
    lib.accept_stage_name.restype = ctypes.c_char_p
    lib.accept_bits_schedule.argtypes = [I, I]
    lib.accept_bits_schedule.restype = I
    lib.accept_status_string.argtypes = [I]
    lib.accept_status_string.restype = ctypes.c_char_p
    lib.accept_version.argtypes = []
    lib.accept_version.restype = ctypes.c_char_p
    for name in ("accept_packed_size", "accept_workspace_size", "accept_compress", "accept_decompress",
                 "accept_compress_noalloc", "accept_mbq_init", "accept_mbq_compress_first", "accept_compress_timed", "accept_decompress_timed"):
        getattr(lib, name).restype = I
    return lib


lib = _load()


def status_string(status):
    return lib.accept_status_string(int(status)).decode()


def version():
    return lib.accept_version().decode()


def _check(st, where):
    if st != 0:
        raise AcceptError(st, where)


def make_desc(scheme, bits, n, m, channels=0, in_dtype=F32, out_dtype=F32, rounding=0, seed=0, t=0,
              layout=LAYOUT_PACKED):
    return Desc(int(scheme), int(bits), int(in_dtype), int(out_dtype), int(n), int(m), int(channels),
                int(rounding), int(layout), int(seed), int(t))


def accept_packed_size(desc):
    h, p = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(lib.accept_packed_size(ctypes.byref(desc), ctypes.byref(h), ctypes.byref(p)), "accept_packed_size")
    return h.value, p.value


def accept_workspace_size(desc):
    b = ctypes.c_size_t(0)
    _check(lib.accept_workspace_size(ctypes.byref(desc), ctypes.byref(b)), "accept_workspace_size")
    return b.value


def accept_bits_schedule(direction, lr_changes_so_far):
    return lib.accept_bits_schedule(int(direction), int(lr_changes_so_far))


def accept_stage_name(desc, is_decompress, i):
    s = lib.accept_stage_name(ctypes.byref(desc), int(is_decompress), int(i))
    return s.decode() if s else None


# ---------------------------------------------------------------------- device-side calls
def _torch():
    import torch
    return torch


def _stream_handle():
    return ctypes.c_void_p(_torch().cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def dtype_code(t):
    torch = _torch()
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError("unsupported dtype %s (float32 or bfloat16)" % t.dtype)


def alloc_outputs(desc, device):
    """header (uint8, 4-byte sized), payload (uint8) and workspace (uint8, zero-filled as the
    library asks of a fresh workspace) device buffers."""
    torch = _torch()
    hb, pb = accept_packed_size(desc)
    wb = accept_workspace_size(desc)
    header = torch.empty(hb, dtype=torch.uint8, device=device)
    payload = torch.empty(max(pb, 1), dtype=torch.uint8, device=device)[:pb]
    workspace = torch.zeros(wb, dtype=torch.uint8, device=device)
    return header, payload, workspace


# ---- argument checks before any pointer reaches the library --------------------------------
# The C functions take no capacities: a tensor that is smaller than the descriptor says, or of
# another element type, would make a kernel read or write outside it.  Everything is checked
# here, on the host, and refused with the status code the C header reserves for it.
INVALID_ARG, BUFFER_TOO_SMALL = 1, 3


def _nbytes(t):
    return t.numel() * t.element_size()


def _check_tensor(t, where, what, dtype_is=None, min_elems=None, min_bytes=None):
    if t is None:
        raise AcceptError(INVALID_ARG, "%s: %s is missing" % (where, what))
    if not t.is_cuda:
        raise AcceptError(INVALID_ARG, "%s: %s is not a device tensor" % (where, what))
    if not t.is_contiguous():
        raise AcceptError(INVALID_ARG, "%s: %s is not contiguous" % (where, what))
    if dtype_is is not None and dtype_code(t) != dtype_is:
        raise AcceptError(INVALID_ARG, "%s: %s has dtype %s, the descriptor says %s"
                          % (where, what, t.dtype, "bfloat16" if dtype_is == BF16 else "float32"))
    if min_elems is not None and t.numel() < min_elems:
        raise AcceptError(BUFFER_TOO_SMALL, "%s: %s has %d elements, %d needed" % (where, what, t.numel(), min_elems))
    if min_bytes is not None and _nbytes(t) < min_bytes:
        raise AcceptError(BUFFER_TOO_SMALL, "%s: %s has %d bytes, %d needed" % (where, what, _nbytes(t), min_bytes))


def _check_compress_args(where, desc, x, alpha_prev, header, payload, workspace, need_alpha):
    hb, pb = accept_packed_size(desc)  # raises on a bad descriptor
    _check_tensor(x, where, "x", dtype_is=desc.in_dtype, min_elems=desc.n * desc.m)
    _check_tensor(header, where, "header", min_bytes=hb)
    _check_tensor(payload, where, "payload", min_bytes=pb)
    if workspace is not None:
        _check_tensor(workspace, where, "workspace", min_bytes=accept_workspace_size(desc))
    if need_alpha and desc.scheme == MBQ:
        _check_tensor(alpha_prev, where, "alpha_prev", dtype_is=F32, min_elems=desc.bits)


def accept_compress(desc, x, alpha_prev=None, header=None, payload=None, workspace=None):
    """Enqueue compression of the device tensor x on the current stream.

    Returns (header, payload) uint8 device tensors (allocated here unless passed in)."""
    if header is None or payload is None or workspace is None:
        h, p, w = alloc_outputs(desc, x.device)
        header = h if header is None else header
        payload = p if payload is None else payload
        workspace = w if workspace is None else workspace
    _check_compress_args("accept_compress", desc, x, alpha_prev, header, payload, workspace, True)
    st = lib.accept_compress(ctypes.byref(desc), _ptr(x), _ptr(alpha_prev), _ptr(header), _ptr(payload),
                             _ptr(workspace), _stream_handle())
    _check(st, "accept_compress")
    return header, payload


def accept_compress_noalloc(desc, x, alpha_prev, header, payload):
    """accept_compress on the library's built-in scratch: the caller passes every buffer and
    nothing is allocated, here or in the library."""
    _check_compress_args("accept_compress_noalloc", desc, x, alpha_prev, header, payload, None, True)
    st = lib.accept_compress_noalloc(ctypes.byref(desc), _ptr(x), _ptr(alpha_prev), _ptr(header), _ptr(payload),
                                     _stream_handle())
    _check(st, "accept_compress_noalloc")
    return header, payload


def accept_decompress(desc, header, payload, out=None):
    """Enqueue decompression on the current stream; returns the flat x_hat device tensor."""
    torch = _torch()
    hb, pb = accept_packed_size(desc)
    _check_tensor(header, "accept_decompress", "header", min_bytes=hb)
    _check_tensor(payload, "accept_decompress", "payload", min_bytes=pb)
    if out is None:
        dt = torch.bfloat16 if desc.out_dtype == BF16 else torch.float32
        out = torch.empty(desc.n * desc.m, dtype=dt, device=payload.device)
    _check_tensor(out, "accept_decompress", "out", dtype_is=desc.out_dtype, min_elems=desc.n * desc.m)
    st = lib.accept_decompress(ctypes.byref(desc), _ptr(header), _ptr(payload), _ptr(out), _stream_handle())
    _check(st, "accept_decompress")
    return out


def accept_mbq_init(desc, x, alpha0=None, workspace=None):
    torch = _torch()
    accept_packed_size(desc)
    _check_tensor(x, "accept_mbq_init", "x", dtype_is=desc.in_dtype, min_elems=desc.n * desc.m)
    if alpha0 is None:
        alpha0 = torch.empty(desc.bits, dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = torch.zeros(accept_workspace_size(desc), dtype=torch.uint8, device=x.device)
    _check_tensor(alpha0, "accept_mbq_init", "alpha0", dtype_is=F32, min_elems=desc.bits)
    _check_tensor(workspace, "accept_mbq_init", "workspace", min_bytes=accept_workspace_size(desc))
    st = lib.accept_mbq_init(ctypes.byref(desc), _ptr(x), _ptr(alpha0), _ptr(workspace), _stream_handle())
    _check(st, "accept_mbq_init")
    return alpha0


def accept_mbq_compress_first(desc, x, header=None, payload=None, workspace=None):
    """Batch 0 of an epoch: residue initialisation; returns (header, payload) like accept_compress."""
    if header is None or payload is None or workspace is None:
        h, p, w = alloc_outputs(desc, x.device)
        header = h if header is None else header
        payload = p if payload is None else payload
        workspace = w if workspace is None else workspace
    _check_compress_args("accept_mbq_compress_first", desc, x, None, header, payload, workspace, False)
    st = lib.accept_mbq_compress_first(ctypes.byref(desc), _ptr(x), _ptr(header), _ptr(payload), _ptr(workspace),
                                       _stream_handle())
    _check(st, "accept_mbq_compress_first")
    return header, payload


def accept_compress_timed(desc, x, alpha_prev, header, payload, workspace):
    """Measurement variant: returns {stage name: milliseconds}; synchronises."""
    _check_compress_args("accept_compress_timed", desc, x, alpha_prev, header, payload, workspace, True)
    ms = (ctypes.c_float * MAX_STAGES)()
    ns = ctypes.c_int(0)
    st = lib.accept_compress_timed(ctypes.byref(desc), _ptr(x), _ptr(alpha_prev), _ptr(header), _ptr(payload),
                                   _ptr(workspace), _stream_handle(), ms, ctypes.byref(ns))
    _check(st, "accept_compress_timed")
    return [(accept_stage_name(desc, 0, i), float(ms[i])) for i in range(ns.value)]


def accept_decompress_timed(desc, header, payload, out):
    hb, pb = accept_packed_size(desc)
    _check_tensor(header, "accept_decompress_timed", "header", min_bytes=hb)
    _check_tensor(payload, "accept_decompress_timed", "payload", min_bytes=pb)
    _check_tensor(out, "accept_decompress_timed", "out", dtype_is=desc.out_dtype, min_elems=desc.n * desc.m)
    ms = (ctypes.c_float * MAX_STAGES)()
    ns = ctypes.c_int(0)
    st = lib.accept_decompress_timed(ctypes.byref(desc), _ptr(header), _ptr(payload), _ptr(out), _stream_handle(),
                                     ms, ctypes.byref(ns))
    _check(st, "accept_decompress_timed")
    return [(accept_stage_name(desc, 1, i), float(ms[i])) for i in range(ns.value)]

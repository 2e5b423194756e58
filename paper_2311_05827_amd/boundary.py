"""Training-loop glue around the compression library: state, schedules, autograd.

Nothing here computes: compression, decompression and the residue initialisation all run in
libaccept's kernels.  This module only keeps what the paper's scheme carries from batch to
batch and wires it into PyTorch:

* the adaptive bit widths (forward 2 -> 3 -> 4, one step per learning-rate change; backward
  8 -> 4 at the first change; paragraphs after eq. (biased error) and after the
  stochastic-rounding equation),
* the multi-bit coefficients alpha and the batch index t of eq. (alpha update); batch 0 of
  every epoch is compressed by the residue method itself (paragraph "Forward Quantizer"),
* the straight-through estimator for the quantizer's gradient (the equation after the
  bit-width paragraph): the backward pass hands the gradient on unchanged, or, when a
  backward compressor is given, after its own uniform compress/decompress round trip, as it
  would arrive over the link.
"""
from __future__ import annotations

from . import binding as B


class BitWidthController:
    """Bit width as a function of the number of learning-rate changes seen so far."""

    def __init__(self, direction):
        assert direction in (0, 1)  # 0 forward (features), 1 backward (gradients)
        self.direction = direction
        self.lr_changes = 0

    def on_lr_change(self):
        self.lr_changes += 1

    @property
    def bits(self):
        return B.accept_bits_schedule(self.direction, self.lr_changes)


class ForwardCompressor:
    """Scheme M at one partition boundary: owns alpha, t and the device buffers."""

    def __init__(self, n, m, in_dtype=B.F32, out_dtype=B.F32, controller=None):
        self.n, self.m = int(n), int(m)
        self.in_dtype, self.out_dtype = in_dtype, out_dtype
        self.controller = controller or BitWidthController(0)
        self.t = 0
        self.alpha = None       # device tensor of k floats
        self._k = None
        self._bufs = None

    def start_epoch(self):
        """Batch 0 of an epoch re-initialises alpha from the data (residue method)."""
        self.t = 0
        self.alpha = None

    def _desc(self, k):
        return B.make_desc(B.MBQ, k, self.n, self.m, in_dtype=self.in_dtype, out_dtype=self.out_dtype, t=self.t)

    def compress(self, x):
        """x: flat contiguous device tensor of n*m elements.  Returns (desc, header, payload);
        the header's first k floats become alpha of the next batch (device-side copy, no
        synchronisation)."""
        k = self.controller.bits
        if self._k != k:             # the width changed: buffers and alpha have a new shape
            self._k, self._bufs, self.alpha = k, None, None
        d = self._desc(k)
        if self._bufs is None:
            self._bufs = B.alloc_outputs(d, x.device)
        header, payload, ws = self._bufs
        if self.alpha is None:
            # batch 0 of an epoch: B^0 and alpha^0 of the residue method are what is sent; the
            # search among the previous batch's levels starts with the next batch
            B.accept_mbq_compress_first(d, x, header=header, payload=payload, workspace=ws)
        else:
            B.accept_compress(d, x, alpha_prev=self.alpha, header=header, payload=payload, workspace=ws)
        self.alpha = header[: 4 * k].view(_torch().float32).clone()
        self.t += 1
        return d, header, payload

    def decompress(self, d, header, payload, out=None):
        return B.accept_decompress(d, header, payload, out=out)

    def transmitted_bytes(self):
        k = self.controller.bits
        h, p = B.accept_packed_size(self._desc(k))
        return h + p


class BackwardCompressor:
    """Scheme U at one partition boundary; stochastic rounding as in the paper by default."""

    def __init__(self, n, m, in_dtype=B.F32, out_dtype=B.F32, controller=None, stochastic=True, seed=0, channels=0):
        self.n, self.m = int(n), int(m)
        self.in_dtype, self.out_dtype = in_dtype, out_dtype
        self.controller = controller or BitWidthController(1)
        self.stochastic = stochastic
        self.seed = int(seed)
        self.channels = int(channels)
        self.calls = 0
        self._k = None
        self._bufs = None

    def _desc(self, k):
        return B.make_desc(B.UNIFORM, k, self.n, self.m, channels=self.channels, in_dtype=self.in_dtype,
                           out_dtype=self.out_dtype,
                           rounding=B.ROUND_STOCHASTIC if self.stochastic else B.ROUND_NEAREST_EVEN,
                           seed=self.seed + self.calls)

    def compress(self, g):
        k = self.controller.bits
        if self._k != k:
            self._k, self._bufs = k, None
        d = self._desc(k)
        if self._bufs is None:
            self._bufs = B.alloc_outputs(d, g.device)
        header, payload, ws = self._bufs
        B.accept_compress(d, g, header=header, payload=payload, workspace=ws)
        self.calls += 1     # a fresh random stream for every gradient tensor
        return d, header, payload

    def decompress(self, d, header, payload, out=None):
        return B.accept_decompress(d, header, payload, out=out)

    def transmitted_bytes(self):
        h, p = B.accept_packed_size(self._desc(self.controller.bits))
        return h + p


def _torch():
    import torch
    return torch


def boundary(x, forward, backward=None):
    """Pass a feature tensor through the partition boundary.

    Forward: x is compressed and decompressed by `forward` (what the next device receives).
    Backward: straight-through estimator; with `backward` given, the incoming gradient first
    takes that compressor's round trip (what the previous device receives)."""
    torch = _torch()

    class _Boundary(torch.autograd.Function):
        @staticmethod
        def forward(ctx, inp):
            flat = inp.contiguous().view(-1)
            d, header, payload = forward.compress(flat)
            out = forward.decompress(d, header, payload)
            return out.view(inp.shape)

        @staticmethod
        def backward(ctx, grad):
            if backward is None:
                return grad
            flat = grad.contiguous().view(-1)
            d, header, payload = backward.compress(flat)
            return backward.decompress(d, header, payload).view(grad.shape)

    return _Boundary.apply(x)

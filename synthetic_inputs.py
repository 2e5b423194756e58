"""Seeded synthetic tensors that stand in for partition-boundary activations and gradients.

This module holds no arithmetic of the compression method: it only draws random tensors
with the shapes and value distributions of the benchmark configurations.  Both the CPU
oracle's tests and the GPU tests/bench take their inputs from here, so the two sides see
the same numbers without sharing any code of the method itself.

Every generator uses ``numpy.random.default_rng(seed)`` and draws in the order written
in its body; results are float32 C-contiguous arrays of shape ``(n, ...)``.  The paper's
own tensors (outputs of MobileNetV2 / a 5-layer CNN on CIFAR10, MNIST, UCI-HAR; section
"The Large Amount of Transmission Data") are not available; these tensors take their
place.
"""
from __future__ import annotations

import numpy as np

# name -> (shape, kind, seed).  "act" tensors are post-ReLU features, "grad" tensors are
# signed gradients, "hidden" is a heavy-tailed transformer hidden state.
CONFIGS = {
    "cfg1_act": ((4, 64, 32, 32), "relu_normal", 0),
    "cfg2_grad": ((4, 64, 32, 32), "grad_outliers", 1),
    "cfg3_act": ((32, 128, 56, 56), "relu_lognormal", 2),
    "cfg4_act": ((64, 256, 56, 56), "relu_lognormal_chgain", 3),
    "cfg4_grad": ((64, 256, 56, 56), "grad", 4),
    "cfg5_hidden": ((16, 509, 768), "student_t3", 5),
    "cfg5_grad": ((16, 509, 768), "grad", 6),
}


def _normal(rng, shape):
    return rng.standard_normal(shape, dtype=np.float32)


def relu_normal(shape, seed):
    """max(z, 0), z ~ N(0,1): about half exact zeros, the rest half-normal."""
    rng = np.random.default_rng(seed)
    z = _normal(rng, shape)
    return np.maximum(z, np.float32(0.0))


def grad(shape, seed, sigma=1e-3):
    """Signed gradients z * sigma, z ~ N(0,1)."""
    rng = np.random.default_rng(seed)
    return _normal(rng, shape) * np.float32(sigma)


def grad_outliers(shape, seed, sigma=1e-3, p_out=1e-3, sigma_out=1e-1):
    """N(0, sigma) with a Bernoulli(p_out) fraction replaced by N(0, sigma_out) draws."""
    rng = np.random.default_rng(seed)
    g = _normal(rng, shape) * np.float32(sigma)
    mask = rng.random(shape, dtype=np.float32) < np.float32(p_out)
    out = _normal(rng, shape) * np.float32(sigma_out)
    return np.where(mask, out, g).astype(np.float32)


def relu_lognormal(shape, seed, p_zero=0.6, mu=-1.0, sigma=1.0):
    """Bernoulli(p_zero) exact zeros, the rest lognormal exp(mu + sigma z)."""
    rng = np.random.default_rng(seed)
    zero = rng.random(shape, dtype=np.float32) < np.float32(p_zero)
    v = np.exp(np.float32(mu) + np.float32(sigma) * _normal(rng, shape))
    v[zero] = np.float32(0.0)
    return v.astype(np.float32)


def relu_lognormal_chgain(shape, seed, p_zero=0.6, mu=-1.0, sigma=1.0, gain_sigma=0.5):
    """relu_lognormal times a per-channel (dimension 1) gain exp(gain_sigma * z_c)."""
    rng = np.random.default_rng(seed)
    zero = rng.random(shape, dtype=np.float32) < np.float32(p_zero)
    v = np.exp(np.float32(mu) + np.float32(sigma) * _normal(rng, shape))
    v[zero] = np.float32(0.0)
    gain = np.exp(np.float32(gain_sigma) * _normal(rng, (shape[1],)))
    bshape = (1, shape[1]) + (1,) * (len(shape) - 2)
    v *= gain.reshape(bshape)
    return v.astype(np.float32)


def student_t3(shape, seed):
    """Heavy-tailed hidden states, Student-t with 3 degrees of freedom."""
    rng = np.random.default_rng(seed)
    return rng.standard_t(3.0, size=shape).astype(np.float32)


_KINDS = {
    "relu_normal": relu_normal,
    "grad_outliers": grad_outliers,
    "relu_lognormal": relu_lognormal,
    "relu_lognormal_chgain": relu_lognormal_chgain,
    "grad": grad,
    "student_t3": student_t3,
}


def make(name):
    """Return the named configuration's tensor (float32, C-contiguous)."""
    shape, kind, seed = CONFIGS[name]
    return np.ascontiguousarray(_KINDS[kind](shape, seed), dtype=np.float32)


def make_shape(kind, shape, seed):
    """Return a tensor of an arbitrary shape drawn with one of the recipes above."""
    return np.ascontiguousarray(_KINDS[kind](tuple(shape), seed), dtype=np.float32)


def as_nm(x):
    """Leading ("batch") dimension n and m = product of the remaining dimensions."""
    n = int(x.shape[0])
    m = int(x.size // n) if n else 0
    return n, m


def to_bf16_bits(x):
    """Round-to-nearest-even bfloat16 image of a float32 array, as raw uint16 bits.

    A storage-format conversion of the *input*, not part of the method (finite values only).
    """
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)

"""GPU parity on the five benchmark configurations' own tensors, at their full sizes and in
the launch configuration the benchmark times.

Every cell compares the WHOLE output with the oracle: header and payload bit for bit, decoded
values bit for bit (scheme U: one float32 multiply) or within 1e-6 * sum|alpha| (scheme M, whose
header sums are reduced in another order).  One test per cell, so that a failure names it and
no test runs for long."""
import numpy as np
import pytest

import synthetic_inputs as si
from oracle import accept_oracle as orc

from gpu_util import dev_bytes, first_mismatch, out_to_numpy, to_dev, torch_mod

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def A():
    torch = torch_mod()
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2311_05827_amd as pkg
    return pkg


_cache = {}


def tensor(name):
    if name not in _cache:
        _cache.clear()  # one big tensor at a time
        _cache[name] = si.make(name)
    return _cache[name]


def check_uniform_full(A, name, k, channels=0, in_bf16=False):
    torch = torch_mod()
    x = tensor(name)
    n, m = si.as_nm(x)
    print("whole tensor", name, "U k", k, "C", channels, "bf16", in_bf16, flush=True)
    xd, bits = to_dev(x, in_bf16)
    d = A.make_desc(A.UNIFORM, k, n, m, channels=channels, in_dtype=A.BF16 if in_bf16 else A.F32,
                    out_dtype=A.BF16 if in_bf16 else A.F32)
    header, payload = A.accept_compress(d, xd)
    xh = A.accept_decompress(d, header, payload)
    torch.cuda.synchronize()
    oh, op = orc.uniform_compress(bits if in_bf16 else x, k, n, m, channels, in_bf16)
    assert dev_bytes(header) == oh
    mm = first_mismatch(dev_bytes(payload), op.tobytes())
    assert mm is None, mm
    ref = orc.uniform_decompress(oh, op, k, n, m, channels, in_bf16)
    got = out_to_numpy(xh)
    assert got.tobytes() == ref.tobytes()
    if not in_bf16:
        # what the paper's rule guarantees at any size: half a step per element, zeros stay zero
        C = max(channels, 1)
        s = np.frombuffer(oh, dtype="<f4").astype(np.float64)
        bound = np.broadcast_to((s * (0.5 + 2e-5)).reshape(1, C, 1), (n, C, m // C)).reshape(-1)
        xf = x.reshape(-1)
        assert np.all(np.abs(got.astype(np.float64) - xf.astype(np.float64)) <= bound)
        assert np.all(got[xf == 0] == 0)


def check_mbq_full(A, name, k, t=1, view=None):
    torch = torch_mod()
    x = tensor(name)
    n, m = view if view else si.as_nm(x)
    print("whole tensor", name, "M k", k, "as", n, "x", m, flush=True)
    xd, _ = to_dev(x)
    d = A.make_desc(A.MBQ, k, n, m, t=t)
    a0 = A.accept_mbq_init(d, xd)
    torch.cuda.synchronize()
    alpha = a0.cpu().numpy()
    exp0, _ = orc.mbq_residue_init(x, k)
    assert np.all(np.abs(alpha - exp0) <= 1e-6 * np.abs(exp0).sum())
    header, payload = A.accept_compress(d, xd, alpha_prev=a0)
    xh = A.accept_decompress(d, header, payload)
    torch.cuda.synchronize()
    oh, op = orc.mbq_compress(x, k, n, m, alpha, t)  # the oracle starts from the GPU's alpha0 bits
    mm = first_mismatch(dev_bytes(payload), op.tobytes())
    assert mm is None, mm
    gh = np.frombuffer(dev_bytes(header), dtype="<f4")
    ohf = np.frombuffer(oh, dtype="<f4")
    scale = float(np.abs(ohf[:k]).sum())
    herr = float(np.max(np.abs(gh.astype(np.float64) - ohf.astype(np.float64))))
    assert herr <= 1e-6 * scale, (gh, ohf)
    ref = orc.mbq_decompress(oh, op, k, n, m)
    got = xh.cpu().numpy()
    verr = float(np.max(np.abs(got.astype(np.float64) - ref.astype(np.float64))))
    print("  header error %.3g, value error %.3g, in units of 1e-6*sum|alpha|: %.4f %.4f"
          % (herr, verr, herr / (1e-6 * scale), verr / (1e-6 * scale)), flush=True)
    assert verr <= 1e-6 * scale
    # bias correction: the output keeps the input's mean
    assert abs(float(got.astype(np.float64).mean()) - float(x.astype(np.float64).mean())) <= 2e-6 * scale
    # batch 0 of an epoch on the same tensor: B^0 bit-exact for the GPU's alpha^0, header within tolerance
    h0, p0 = A.accept_mbq_compress_first(d, xd)
    torch.cuda.synchronize()
    g0 = np.frombuffer(dev_bytes(h0), dtype="<f4")
    assert g0[:k].tobytes() == alpha.tobytes()
    o0, _ = orc.mbq_compress_first(x, k, n, m)
    o0f = np.frombuffer(o0, dtype="<f4")
    assert np.all(np.abs(g0.astype(np.float64) - o0f.astype(np.float64)) <= 1e-6 * np.abs(o0f[:k]).sum()), (g0, o0f)
    mm = first_mismatch(dev_bytes(p0), orc.mbq_pack(orc.mbq_residue_signs(x, g0[:k]), k, n, m).tobytes())
    assert mm is None, mm


# ---- config 1: 4x64x32x32 post-ReLU activation, 8-bit round trip (and the forward widths)
def test_config1_uniform_k8(A):
    check_uniform_full(A, "cfg1_act", 8)


@pytest.mark.parametrize("k", [2, 3, 4])
def test_config1_mbq(A, k):
    check_mbq_full(A, "cfg1_act", k)                      # n = 4: the row group is padded to 8
    check_mbq_full(A, "cfg1_act", k, view=(256, 1024))


# ---- config 2: gradient with 0.1 % outliers (the max-abs rule's hard case), 4 and 2 bits
@pytest.mark.parametrize("k", [4, 2])
def test_config2_uniform(A, k):
    check_uniform_full(A, "cfg2_grad", k)


# ---- config 3: 32x128x56x56, widths 2..8
@pytest.mark.parametrize("k", [2, 3, 4, 5, 6, 7, 8])
def test_config3_uniform(A, k):
    check_uniform_full(A, "cfg3_act", k)


@pytest.mark.parametrize("k", [2, 3, 4])
def test_config3_mbq(A, k):
    check_mbq_full(A, "cfg3_act", k)


# ---- config 4: 64x256x56x56, fp32 and bf16, per tensor and per channel, 4/6/8 bits; gradient
@pytest.mark.parametrize("in_bf16", [False, True])
@pytest.mark.parametrize("channels", [0, 256])
@pytest.mark.parametrize("k", [4, 6, 8])
def test_config4_activation_uniform(A, k, channels, in_bf16):
    check_uniform_full(A, "cfg4_act", k, channels, in_bf16)


@pytest.mark.parametrize("k", [2, 3, 4])
def test_config4_activation_mbq(A, k):
    check_mbq_full(A, "cfg4_act", k)


@pytest.mark.parametrize("channels", [0, 256])
@pytest.mark.parametrize("k", [4, 6, 8])
def test_config4_gradient(A, k, channels):
    check_uniform_full(A, "cfg4_grad", k, channels)


# ---- config 5: 16x509x768, straddling widths, hidden states and gradients
@pytest.mark.parametrize("k", [3, 5, 6, 7])
@pytest.mark.parametrize("name", ["cfg5_hidden", "cfg5_grad"])
def test_config5_uniform(A, name, k):
    check_uniform_full(A, name, k)


def test_config5_mbq(A):
    check_mbq_full(A, "cfg5_hidden", 3)

"""GPU parity for the comparison layouts (the paper's batch-pair backward layout and the
one-byte-per-value "w/o enc." forms): payload and header bit-exact for scheme U, payload
bit-exact and header within 1e-6 * sum|alpha| for scheme M; decoded values bit-exact when the
decoder is fed the oracle's bytes."""
import numpy as np
import pytest

import synthetic_inputs as si
from oracle import accept_oracle as orc
from gpu_util import bytes_to_dev, dev_bytes, first_mismatch, out_to_numpy, to_dev, torch_mod

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def A():
    torch = torch_mod()
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2311_05827_amd as pkg
    return pkg


def run_uniform(A, x, k, n, m, layout, channels=0, in_bf16=False, out_bf16=False, rounding=0, seed=0):
    torch = torch_mod()
    print("case U layout", layout, "k", k, "n", n, "m", m, "C", channels, "bf16", in_bf16, out_bf16, "rnd", rounding,
          flush=True)
    xd, bits = to_dev(x, in_bf16)
    d = A.make_desc(A.UNIFORM, k, n, m, channels=channels, in_dtype=A.BF16 if in_bf16 else A.F32,
                    out_dtype=A.BF16 if out_bf16 else A.F32, rounding=rounding, seed=seed, layout=layout)
    assert A.accept_packed_size(d) == orc.packed_size(orc.SCHEME_UNIFORM, k, n, m, channels, layout)
    header, payload = A.accept_compress(d, xd)
    xh = A.accept_decompress(d, header, payload)
    torch.cuda.synchronize()
    oh, op = orc.uniform_compress(bits if in_bf16 else x, k, n, m, channels, in_bf16, rounding, seed, layout)
    assert dev_bytes(header) == oh
    mm = first_mismatch(dev_bytes(payload), op.tobytes())
    assert mm is None, "payload differs: " + mm
    oxh = orc.uniform_decompress(oh, op, k, n, m, channels, out_bf16, layout)
    assert out_to_numpy(xh).tobytes() == oxh.tobytes()


@pytest.mark.parametrize("k", [2, 4, 8])
def test_uniform_batch_layout(A, k):
    for (n, m), C in [((6, 8200), 0), ((7, 1028), 4), ((5, 333), 0), ((1, 9), 3), ((16, 4 * 4099), 4099), ((3, 1), 0)]:
        x = si.make_shape("grad_outliers", (n, m), 300 + k + n)
        run_uniform(A, x, k, n, m, A.LAYOUT_BATCH, channels=C)
    x = si.make_shape("student_t3", (9, 2052), 310 + k)
    run_uniform(A, x, k, 9, 2052, A.LAYOUT_BATCH, in_bf16=True, out_bf16=True)
    run_uniform(A, x, k, 9, 2052, A.LAYOUT_BATCH, rounding=A.ROUND_STOCHASTIC, seed=77)


@pytest.mark.parametrize("k", [2, 3, 4, 5, 6, 7, 8])
def test_uniform_unencoded_layout(A, k):
    for (n, m), C in [((3, 8455), 0), ((4, 1028), 4), ((1, 1), 0), ((1, 7), 0), ((5, 35), 5)]:
        x = si.make_shape("student_t3", (n, m), 320 + k + m)
        run_uniform(A, x, k, n, m, A.LAYOUT_UNENCODED, channels=C)
    x = si.make_shape("grad", (2, 4102), 330 + k)
    run_uniform(A, x, k, 2, 4102, A.LAYOUT_UNENCODED, in_bf16=True, out_bf16=True)
    run_uniform(A, x, k, 2, 4102, A.LAYOUT_UNENCODED, rounding=A.ROUND_STOCHASTIC, seed=5)


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5, 8])
def test_mbq_unencoded_layout(A, k):
    torch = torch_mod()
    for n, m in [(8, 2055), (19, 40004), (3, 5), (1, 1), (16, 3000)]:
        for in_bf16 in ([False, True] if m == 3000 else [False]):
            print("case M unencoded k", k, "n", n, "m", m, "bf16", in_bf16, flush=True)
            x = si.make_shape("relu_lognormal", (n, m), 340 + k + n)
            xd, bits = to_dev(x, in_bf16)
            xin = orc.widen_bf16(bits) if in_bf16 else x.reshape(-1)
            alpha, _ = orc.mbq_residue_init(xin, k)
            d = A.make_desc(A.MBQ, k, n, m, t=2, in_dtype=A.BF16 if in_bf16 else A.F32,
                            out_dtype=A.BF16 if in_bf16 else A.F32, layout=A.LAYOUT_UNENCODED)
            assert A.accept_packed_size(d) == orc.packed_size(orc.SCHEME_MBQ, k, n, m, 0, orc.LAYOUT_UNENCODED)
            header, payload = A.accept_compress(d, xd, alpha_prev=torch.from_numpy(alpha).cuda())
            torch.cuda.synchronize()
            oh, op = orc.mbq_compress(bits if in_bf16 else x, k, n, m, alpha, 2, in_bf16, orc.LAYOUT_UNENCODED)
            mm = first_mismatch(dev_bytes(payload), op.tobytes())
            assert mm is None, "payload differs: " + mm
            gh = np.frombuffer(dev_bytes(header), dtype="<f4")
            ohf = np.frombuffer(oh, dtype="<f4")
            scale = float(np.sum(np.abs(ohf[:k])))
            assert np.all(np.abs(gh.astype(np.float64) - ohf.astype(np.float64)) <= 1e-6 * scale), (gh, ohf)
            xh = A.accept_decompress(d, bytes_to_dev(oh), bytes_to_dev(op.tobytes()))
            torch.cuda.synchronize()
            oxh = orc.mbq_decompress(oh, op, k, n, m, in_bf16, orc.LAYOUT_UNENCODED)
            assert out_to_numpy(xh).tobytes() == oxh.tobytes()
            # the packed layout of the same call carries the same header
            dp = A.make_desc(A.MBQ, k, n, m, t=2, in_dtype=A.BF16 if in_bf16 else A.F32)
            hp, _ = A.accept_compress(dp, xd, alpha_prev=torch.from_numpy(alpha).cuda())
            torch.cuda.synchronize()
            ghp = np.frombuffer(dev_bytes(hp), dtype="<f4")
            assert np.all(np.abs(ghp.astype(np.float64) - gh.astype(np.float64)) <= 2e-6 * scale)

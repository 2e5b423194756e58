"""Seeded random geometries: every path (vector / scalar, per-tensor / per-channel in all
three range modes, partial row groups, all widths and dtypes) against the oracle."""
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


def divisors(v):
    return [d for d in range(1, v + 1) if v % d == 0]


def test_uniform_random_geometries(A):
    torch = torch_mod()
    rng = np.random.default_rng(20231105)
    kinds = ["relu_normal", "grad_outliers", "student_t3", "relu_lognormal_chgain"]
    for case in range(120):
        n = int(rng.integers(1, 40))
        m = int(rng.choice([rng.integers(1, 64), rng.integers(64, 3000), 8 * rng.integers(1, 1500),
                            1024 * rng.integers(1, 24)]))
        k = int(rng.integers(2, 9))
        C = int(rng.choice([0] + divisors(m)[:: max(1, len(divisors(m)) // 6)])) if case % 2 else 0
        in_bf16, out_bf16 = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        rounding = int(rng.integers(0, 2)) if case % 5 == 0 else 0
        seed = int(rng.integers(0, 2 ** 62))
        kind = kinds[case % 4]
        shape = (n, C, m // C) if C > 1 else (n, m)
        if kind == "relu_lognormal_chgain" and C <= 1:
            kind = "relu_normal"
        x = si.make_shape(kind, shape, 5000 + case)
        print("case", case, "n", n, "m", m, "k", k, "C", C, "bf16", in_bf16, out_bf16, "rnd", rounding, flush=True)
        xd, bits = to_dev(x, in_bf16)
        d = A.make_desc(A.UNIFORM, k, n, m, channels=C, in_dtype=A.BF16 if in_bf16 else A.F32,
                        out_dtype=A.BF16 if out_bf16 else A.F32, rounding=rounding, seed=seed)
        header, payload = A.accept_compress(d, xd)
        xh = A.accept_decompress(d, header, payload)
        torch.cuda.synchronize()
        oh, op = orc.uniform_compress(bits if in_bf16 else x, k, n, m, C, in_bf16, rounding, seed)
        assert dev_bytes(header) == oh, case
        mm = first_mismatch(dev_bytes(payload), op.tobytes())
        assert mm is None, (case, mm)
        ref = orc.uniform_decompress(oh, op, k, n, m, C, out_bf16)
        assert out_to_numpy(xh).tobytes() == ref.tobytes(), case


def test_uniform_random_tiled_geometries(A):
    """Per-channel geometries over several 8192-element tiles, drawn so that every way of
    finding an element's range is hit: long segments with the ranges finished tile by tile
    (whole tiles, few rows) or by the U1b kernel, short aligned segments, unaligned segments,
    one element per segment (channels-last)."""
    torch = torch_mod()
    rng = np.random.default_rng(20231107)
    for case in range(72):
        flavour = case % 6
        if flavour == 0:      # whole tiles, segments >= 2048: ranges per tile
            seg = 2048 * int(rng.integers(1, 6)) + 512 * int(rng.integers(0, 4)) * (case % 12 == 0)
            C = int(rng.integers(2, 9))
            n = 8192 // np.gcd(8192, C * seg) * int(rng.integers(1, 4))
        elif flavour == 1:    # long segments, not whole tiles
            seg = 4 * int(rng.integers(128, 2000))
            C, n = int(rng.integers(2, 7)), int(rng.integers(1, 9))
        elif flavour == 2:    # short aligned segments
            seg = 8 * int(rng.integers(1, 60))
            C, n = int(rng.integers(2, 40)), int(rng.integers(8, 60))
        elif flavour == 3:    # segments no vector respects
            seg = int(rng.integers(1, 50)) * 2 + 1
            C, n = int(rng.integers(2, 40)), int(rng.integers(8, 80))
        elif flavour == 4:    # channels-last, rows of whole vectors
            seg, C, n = 1, 8 * int(rng.integers(1, 40)), int(rng.integers(30, 900))
        else:                 # channels-last, rows that no vector divides
            seg, C, n = 1, int(rng.integers(3, 200)) | 1, int(rng.integers(30, 500))
        n, C, seg = int(n), int(C), int(seg)
        m = C * seg
        k = int(rng.integers(2, 9))
        bf = bool(rng.integers(0, 2))
        rounding = 1 if case % 9 == 0 else 0
        x = si.make_shape("relu_lognormal_chgain" if seg > 1 else "grad", (n, C, seg) if seg > 1 else (n, C), 8000 + case)
        if seg == 1:
            x = np.ascontiguousarray(x * (np.float32(2.0) ** rng.integers(-8, 8, C).astype(np.float32))[None, :], np.float32)
        print("case", case, "n", n, "C", C, "seg", seg, "k", k, "bf16", bf, "rnd", rounding, "N", n * m, flush=True)
        xd, bits = to_dev(x, bf)
        d = A.make_desc(A.UNIFORM, k, n, m, channels=C, in_dtype=A.BF16 if bf else A.F32,
                        out_dtype=A.BF16 if bf else A.F32, rounding=rounding, seed=case)
        header, payload = A.accept_compress(d, xd)
        xh = A.accept_decompress(d, header, payload)
        torch.cuda.synchronize()
        oh, op = orc.uniform_compress(bits if bf else x, k, n, m, C, bf, rounding, case)
        assert dev_bytes(header) == oh, case
        mm = first_mismatch(dev_bytes(payload), op.tobytes())
        assert mm is None, (case, mm)
        assert out_to_numpy(xh).tobytes() == orc.uniform_decompress(oh, op, k, n, m, C, bf).tobytes(), case


def test_mbq_random_geometries(A):
    torch = torch_mod()
    rng = np.random.default_rng(20231106)
    for case in range(80):
        n = int(rng.integers(1, 70))
        m = int(rng.choice([rng.integers(1, 40), rng.integers(40, 2000), 4 * rng.integers(1, 1200),
                            8 * rng.integers(1, 900)]))
        k = int(rng.choice([1, 2, 2, 3, 3, 4, 4, 5, 6, 8]))
        t = int(rng.integers(0, 120))
        in_bf16, out_bf16 = bool(rng.integers(0, 4) == 0), bool(rng.integers(0, 4) == 0)
        x = si.make_shape(["relu_normal", "student_t3", "relu_lognormal"][case % 3], (n, m), 7000 + case)
        print("case", case, "n", n, "m", m, "k", k, "t", t, "bf16", in_bf16, out_bf16, flush=True)
        xd, bits = to_dev(x, in_bf16)
        xin = orc.widen_bf16(bits) if in_bf16 else x.reshape(-1)
        if case % 4 == 3:
            # close levels: several thresholds share a bucket, the encoder's general path
            alpha = (np.float32(np.abs(xin).mean() + 1e-3) * np.array([1.0, 0.97, 0.03, 0.02, 0.011, 0.01, 0.005, 0.004],
                                                                     np.float32))[:k]
        else:
            alpha, _ = orc.mbq_residue_init(xin, k)
        d = A.make_desc(A.MBQ, k, n, m, in_dtype=A.BF16 if in_bf16 else A.F32,
                        out_dtype=A.BF16 if out_bf16 else A.F32, t=t)
        header, payload = A.accept_compress(d, xd, alpha_prev=torch.from_numpy(np.ascontiguousarray(alpha)).cuda())
        torch.cuda.synchronize()
        oh, op = orc.mbq_compress(bits if in_bf16 else x, k, n, m, alpha, t, in_bf16)
        mm = first_mismatch(dev_bytes(payload), op.tobytes())
        assert mm is None, (case, mm)
        gh = np.frombuffer(dev_bytes(header), dtype="<f4")
        ohf = np.frombuffer(oh, dtype="<f4")
        scale = float(np.abs(ohf[:k]).sum())
        assert np.all(np.abs(gh.astype(np.float64) - ohf.astype(np.float64)) <= 1e-6 * scale), (case, gh, ohf)
        xh = A.accept_decompress(d, bytes_to_dev(oh), bytes_to_dev(op.tobytes()))
        torch.cuda.synchronize()
        assert out_to_numpy(xh).tobytes() == orc.mbq_decompress(oh, op, k, n, m, out_bf16).tobytes(), case

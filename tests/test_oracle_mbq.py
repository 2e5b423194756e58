"""Pins for the oracle's scheme M (multi-bit quantization + batch bit planes)."""
import itertools

import numpy as np
import pytest

from oracle import accept_oracle as orc


def test_worked_encoder_example(golden_kv):
    """Paragraph "Forward Encoder": bits 0,0,1,1,0,1,1,0 along the batch -> byte 54."""
    kv = golden_kv("worked_examples.txt")
    bits = [int(b) for b in kv["encoder_bits"].split()]
    assert orc.mbq_pack(np.array(bits), 1, 8, 1).tolist() == [int(kv["encoder_byte"])]
    # the full example: 8 x 1 x 1 x 1 x 4 -> 1 x 1 x 1 x 1 x 4, k innermost.  Put the
    # printed bits on plane 2 and different bits on the other planes.
    planes = [[1, 0, 0, 0, 0, 0, 0, 0], [0, 0, 0, 0, 0, 0, 0, 1], bits, [1, 1, 1, 1, 0, 0, 0, 0]]
    code = np.zeros(8, dtype=np.int64)
    for p, pb in enumerate(planes):
        code |= np.array(pb) << p
    out = orc.mbq_pack(code, 4, 8, 1)
    assert out.shape == (4,)
    assert out.tolist() == [128, 1, 54, 240]
    assert orc.mbq_unpack(out, 4, 8, 1).tolist() == code.tolist()


@pytest.mark.parametrize("k", [1, 2, 3, 4, 8])
@pytest.mark.parametrize("n,m", [(8, 1), (16, 5), (3, 7), (9, 4), (1, 1), (64, 33)])
def test_pack_against_numpy_packbits(k, n, m):
    rng = np.random.default_rng(k * 100 + n * 7 + m)
    code = rng.integers(0, 2 ** k, size=(n, m))
    G = (n + 7) // 8
    bits = np.zeros((G * 8, m, k), dtype=np.uint8)
    for p in range(k):
        bits[:n, :, p] = (code >> p) & 1
    exp = np.packbits(bits.reshape(G, 8, m, k), axis=1).reshape(-1)
    got = orc.mbq_pack(code, k, n, m)
    assert got.size == orc.packed_size(orc.SCHEME_MBQ, k, n, m)[1]
    assert got.tobytes() == exp.tobytes()
    assert orc.mbq_unpack(got, k, n, m).tolist() == code.reshape(-1).tolist()


def test_levels_for_k2_are_the_four_sign_combinations():
    """P = {+-a1 +-a2} ("Forward Quantizer")."""
    a = np.array([0.75, 0.25], dtype=np.float32)
    lv, order, tau = orc.mbq_levels(a)
    assert lv.tolist() == [-1.0, -0.5, 0.5, 1.0]
    # pattern bit j = 1 <-> +alpha_j
    assert order.tolist() == [0b00, 0b10, 0b01, 0b11]
    assert tau.tolist() == [-0.75, 0.0, 0.75]
    # ties between equal levels are ordered by pattern
    lv, order, _ = orc.mbq_levels(np.array([0.5, 0.5], dtype=np.float32))
    assert lv.tolist() == [-1.0, 0.0, 0.0, 1.0] and order.tolist() == [0, 1, 2, 3]


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_assign_is_nearest_level_brute_force(k):
    rng = np.random.default_rng(k)
    alpha = np.sort(rng.uniform(0.05, 1.0, k))[::-1].astype(np.float32)
    x = rng.standard_normal(3000).astype(np.float32)
    code = orc.mbq_assign(x, alpha)
    # brute force: every pattern's level in float64, nearest by absolute distance
    pats = np.arange(2 ** k)
    lv = np.array([sum((1 if (p >> j) & 1 else -1) * float(alpha[j]) for j in range(k)) for p in pats])
    d = np.abs(x.astype(np.float64)[:, None] - lv[None, :])
    best = d.min(axis=1)
    chosen = d[np.arange(x.size), code]
    srt = np.sort(d, axis=1)
    clear = (srt[:, 1] - srt[:, 0]) > 1e-5  # away from exact ties
    assert clear.mean() > 0.99
    assert np.all(chosen[clear] == best[clear])
    assert np.all(chosen <= best + 1e-5)
    # a value equal to a level decodes to that level
    x2 = lv.astype(np.float32)
    code2 = orc.mbq_assign(x2, alpha)
    lv32 = np.array([np.float32(v) for v in lv])
    assert np.allclose(lv32[code2], x2, atol=1e-6)
    # an exact midpoint goes to the lower level; NaN goes to the lowest level
    lvs, order, tau = orc.mbq_levels(alpha)
    assert orc.mbq_assign(tau, alpha).tolist() == order[:-1].tolist()
    assert orc.mbq_assign(np.array([np.nan], np.float32), alpha).tolist() == [int(order[0])]


@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_alpha_solution_is_the_least_squares_minimiser(k):
    """eq. (alpha solution): compare with numpy.linalg.lstsq on the explicit +-1 matrix,
    check the normal equations, and the closed form at k = 1."""
    rng = np.random.default_rng(20 + k)
    x = rng.standard_normal(4000).astype(np.float32)
    alpha_prev = (np.array([0.9, 0.45, 0.22, 0.11][:k])).astype(np.float32)
    code = orc.mbq_assign(x, alpha_prev)
    G, h, Sb, Sx = orc.mbq_stats(x, code, k)
    B = np.stack([2.0 * ((code >> p) & 1) - 1.0 for p in range(k)], axis=1)
    assert np.array_equal(G, B.T @ B)
    assert np.allclose(h, B.T @ x.astype(np.float64), rtol=1e-12, atol=1e-9)
    assert np.array_equal(Sb, B.sum(axis=0)) and Sx == pytest.approx(float(x.astype(np.float64).sum()))
    a_t, cur = orc.mbq_alpha_update(alpha_prev, G, h, 5, x.size)
    ref = np.linalg.lstsq(B, x.astype(np.float64), rcond=None)[0]
    assert np.allclose(cur, ref, rtol=1e-10, atol=1e-12)
    resid = x.astype(np.float64) - B @ cur
    assert np.abs(B.T @ resid).max() < 1e-8 * x.size
    assert np.linalg.norm(resid) <= np.linalg.norm(x.astype(np.float64) - B @ alpha_prev.astype(np.float64)) + 1e-12
    b = orc.beta(5)
    assert np.allclose(a_t, b * alpha_prev + (1 - b) * ref, rtol=1e-6)
    if k == 1:
        assert cur[0] == pytest.approx(float(np.sum(B[:, 0] * x)) / x.size)


def test_singular_gram_keeps_previous_alpha():
    x = np.full(64, 5.0, dtype=np.float32)  # every element takes the top level: planes equal
    alpha_prev = np.array([1.0, 0.5], dtype=np.float32)
    code = orc.mbq_assign(x, alpha_prev)
    G, h, Sb, Sx = orc.mbq_stats(x, code, 2)
    a_t, cur = orc.mbq_alpha_update(alpha_prev, G, h, 3, x.size)
    assert cur.tolist() == [1.0, 0.5] and a_t.tolist() == [1.0, 0.5]


@pytest.mark.parametrize("k", [2, 3, 4])
@pytest.mark.parametrize("n,m", [(16, 50), (5, 33), (8, 8)])
def test_bias_correction_preserves_the_mean(k, n, m):
    """eq. (biased error): after subtracting E[n_q] the output has the input's mean."""
    rng = np.random.default_rng(k + n + m)
    x = np.maximum(rng.standard_normal((n, m)), 0).astype(np.float32)
    alpha0, _ = orc.mbq_residue_init(x, k)
    hdr, pay = orc.mbq_compress(x, k, n, m, alpha0, t=1)
    assert len(hdr) == 4 * (k + 1) and pay.size == ((n + 7) // 8) * m * k
    xh = orc.mbq_decompress(hdr, pay, k, n, m)
    assert float(xh.astype(np.float64).mean()) == pytest.approx(float(x.astype(np.float64).mean()), abs=2e-6)
    # every output + m_q is one of the 2^k levels of the transmitted alpha
    h = np.frombuffer(hdr, dtype="<f4")
    lv, _, _ = orc.mbq_levels(h[:k])
    back = (xh.astype(np.float64) + float(h[k]))
    assert np.all(np.min(np.abs(back[:, None] - lv[None, :].astype(np.float64)), axis=1) < 1e-6)
    # error of each element is at most half the widest gap (inside the level range) + bias
    inside = (x >= lv[0]) & (x <= lv[-1])
    gap = float(np.max(np.diff(lv.astype(np.float64))))
    # assignment used alpha0's levels; bound with both tables' gaps and the alpha drift
    lv0, _, _ = orc.mbq_levels(alpha0)
    gap0 = float(np.max(np.diff(lv0.astype(np.float64))))
    drift = float(np.sum(np.abs(h[:k].astype(np.float64) - alpha0.astype(np.float64))))
    inside0 = (x.reshape(-1) >= lv0[0]) & (x.reshape(-1) <= lv0[-1])
    err = np.abs(xh.astype(np.float64) - x.reshape(-1).astype(np.float64))
    assert np.all(err[inside0] <= gap0 / 2 + drift + abs(float(h[k])) + 1e-6)
    assert inside.any() and gap > 0


@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_residue_init_closed_forms(k):
    rng = np.random.default_rng(40 + k)
    x = rng.standard_normal(2000).astype(np.float32)
    alpha, code = orc.mbq_residue_init(x, k)
    assert alpha[0] == np.float32(np.mean(np.abs(x.astype(np.float64))))
    rho = x.astype(np.float64)
    prev = np.linalg.norm(rho)
    for j in range(k):
        b = np.where((code >> j) & 1, 1.0, -1.0)
        assert np.all(b == np.where(rho >= 0, 1.0, -1.0))
        # alpha_j is the least-squares coefficient for this sign vector: scan neighbours
        f = lambda a: np.sum((rho - a * b) ** 2)
        a = float(alpha[j])
        assert f(a) <= f(a * 1.01) and f(a) <= f(a * 0.99)
        rho = rho - a * b
        assert np.linalg.norm(rho) <= prev + 1e-12
        prev = np.linalg.norm(rho)
    # sign(0) = +1
    _, c0 = orc.mbq_residue_init(np.zeros(4, np.float32), 1)
    assert c0.tolist() == [1, 1, 1, 1]


def test_decompress_brute_force_tiny():
    """x_hat = B alpha - m_q element by element with Python floats, all 2-bit patterns on an
    n = 3 (padded group) tensor."""
    alpha = np.array([0.5, 0.125], dtype=np.float32)
    mq = np.float32(0.0625)
    hdr = np.array([0.5, 0.125, 0.0625], dtype="<f4").tobytes()
    for pats in itertools.product(range(4), repeat=3):
        code = np.array(pats)
        pay = orc.mbq_pack(code, 2, 3, 1)
        xh = orc.mbq_decompress(hdr, pay, 2, 3, 1)
        exp = [((0.5 if p & 1 else -0.5) + (0.125 if p & 2 else -0.125)) - 0.0625 for p in pats]
        assert xh.tolist() == exp


def test_bf16_input_equals_widened_input():
    rng = np.random.default_rng(77)
    x = np.maximum(rng.standard_normal((8, 64)), 0).astype(np.float32)
    bits = orc.narrow_bf16(x)
    a0, _ = orc.mbq_residue_init(orc.widen_bf16(bits), 3)
    h1, p1 = orc.mbq_compress(bits, 3, 8, 64, a0, 2, in_bf16=True)
    h2, p2 = orc.mbq_compress(orc.widen_bf16(bits), 3, 8, 64, a0, 2)
    assert h1 == h2 and p1.tobytes() == p2.tobytes()


@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_batch0_compress_pins(k):
    """Batch 0 ("Forward Quantizer": B^0, alpha^0 from the residue method are what is sent).
    Pins: a Python-float brute force of the residue recurrence on a tiny tensor; the decoded
    tensor keeps the input's mean (the header's m_q is the mean error of B^0 alpha^0); every
    decoded value is the chosen level minus m_q; for k = 1 the decoded magnitudes are mean|x|."""
    rng = np.random.default_rng(300 + k)
    n, m = 11, 37
    x = (rng.standard_normal((n, m)) * 0.7).astype(np.float32)
    x[0, :5] = 0.0  # sign(0) = +1
    hdr, pay = orc.mbq_compress_first(x, k, n, m)
    h = np.frombuffer(hdr, dtype="<f4")
    alpha = h[:k]
    # brute force, element by element, in Python floats (float64)
    codes = []
    for v in x.reshape(-1).tolist():
        rho, c = float(v), 0
        for j in range(k):
            s = 1.0 if rho >= 0.0 else -1.0
            c |= (1 if s > 0 else 0) << j
            rho -= s * float(alpha[j])
        codes.append(c)
    assert orc.mbq_unpack(pay, k, n, m).tolist() == codes
    assert orc.mbq_residue_signs(x, alpha).tolist() == codes
    assert pay.size == ((n + 7) // 8) * m * k and len(hdr) == 4 * (k + 1)
    xh = orc.mbq_decompress(hdr, pay, k, n, m)
    assert abs(float(xh.astype(np.float64).mean()) - float(x.astype(np.float64).mean())) <= 2e-7 * float(np.abs(alpha).sum())
    lv = [sum((1.0 if (c >> j) & 1 else -1.0) * float(alpha[j]) for j in range(k)) for c in codes]
    assert np.allclose(xh, np.array(lv) - float(h[k]), rtol=0, atol=1e-6)
    if k == 1:
        assert alpha[0] == np.float32(np.mean(np.abs(x.astype(np.float64))))
    # the same alpha^0 as the stand-alone initialisation, and a usable alpha_prev for batch 1
    a0, _ = orc.mbq_residue_init(x, k)
    assert a0.tobytes() == alpha.tobytes()

"""Pins for the oracle's scheme U (uniform max-abs quantizer + dense bit stream).

None of these tests re-types the oracle's formulas with the same primitives: expected
values come from integer rules worked out by hand, Python string formatting of bits,
numpy.packbits, the paper's printed ranges, or invariants the mathematics fixes.
"""
import itertools

import numpy as np
import pytest

from oracle import accept_oracle as orc

KS = [2, 3, 4, 5, 6, 7, 8]


def rhe_half(j):
    """round-half-to-even of j/2 using integers only."""
    if j % 2 == 0:
        return j // 2
    lo = (j - 1) // 2
    return lo if lo % 2 == 0 else lo + 1


def bitstring_bytes(codes, k):
    """Independent packer: write every code as k binary digits, cut into bytes."""
    s = "".join(format(int(c), "0{}b".format(k)) for c in codes)
    s += "0" * (-len(s) % 8)
    return np.array([int(s[i:i + 8], 2) for i in range(0, len(s), 8)], dtype=np.uint8)


def expected_code(q, k):
    return (q & 0xFF) if k == 8 else q + 2 ** (k - 1)


@pytest.mark.parametrize("k", KS)
def test_brute_force_tiny_tensors_with_ties(k):
    """All tensors of length 1..4 over an alphabet of exactly representable multiples of
    s/2 (so every odd multiple is an exact tie).  With c = L*2^e both s and 1/s are exact,
    so the expected integers follow from integer arithmetic alone."""
    L = 2 ** (k - 1) - 1
    e = -3
    s = 2.0 ** e
    # j counts halves of a step; always include +-2L so that max|x| = L*s
    js = sorted(set([2 * L, -2 * L, 0, 1, -1, 3, -3, 2 * L - 1, -(2 * L - 1), 2, 5 if 5 <= 2 * L else 1]))
    for length in (1, 2, 3, 4):
        for combo in itertools.product(js, repeat=length):
            if max(abs(j) for j in combo) != 2 * L:
                continue
            x = np.array([j * s / 2 for j in combo], dtype=np.float32)
            hdr, pay = orc.uniform_compress(x, k, 1, length)
            assert np.frombuffer(hdr, dtype="<f4")[0] == np.float32(s)
            q = [rhe_half(j) for j in combo]
            exp = bitstring_bytes([expected_code(v, k) for v in q], k)
            assert pay.tobytes() == exp.tobytes(), (k, combo)
            back = orc.uniform_decompress(hdr, pay, k, 1, length)
            assert back.tolist() == [v * s for v in q]


@pytest.mark.parametrize("k", KS)
def test_stream_matches_packbits_and_special_cases(k):
    """pack_stream against numpy.packbits (an independent big-endian bit packer), and the
    two layouts the paper itself describes: k=8 raw bytes, k=4 two codes per byte."""
    rng = np.random.default_rng(100 + k)
    for N in (1, 7, 8, 9, 31, 32, 33, 63, 64, 65, 257, 1000):
        u = rng.integers(0, 2 ** k, size=N).astype(np.uint64)
        got = orc.pack_stream(u, k)
        bits = ((u[:, None] >> np.arange(k - 1, -1, -1, dtype=np.uint64)[None, :]) & np.uint64(1)).astype(np.uint8)
        assert got.tobytes() == np.packbits(bits.reshape(-1)).tobytes()
        assert got.size == (N * k + 7) // 8
        assert orc.unpack_stream(got, k, N).tolist() == u.tolist()
        if k == 8:
            assert got.tolist() == u.tolist()
        if k == 4 and N % 2 == 0:
            assert got.tolist() == ((u[0::2] << np.uint64(4)) | u[1::2]).tolist()
    # unused low bits of the last byte are zero
    got = orc.pack_stream(np.full(3, 2 ** k - 1, dtype=np.uint64), k)
    tail_bits = (-3 * k) % 8
    assert int(got[-1]) & ((1 << tail_bits) - 1) == 0


def test_k4_code_range_is_the_papers(golden_kv):
    """Adding 8 maps [-8,7] onto [0,15] ("Backward Encoder")."""
    kv = golden_kv("worked_examples.txt")
    lo, hi = [int(v) for v in kv["uniform_k4_code_range"].split()]
    q = np.arange(-8, 8)
    u = orc.uniform_codes(q, 4)
    assert int(u.min()) == lo and int(u.max()) == hi
    assert (u.astype(np.int64) - q).tolist() == [int(kv["uniform_k4_offset"])] * 16
    # k = 8 is transmitted as it is: the int8 two's-complement byte
    q8 = np.arange(-128, 128)
    assert orc.uniform_codes(q8, 8).astype(np.uint8).view(np.int8).tolist() == q8.tolist()


@pytest.mark.parametrize("k", KS)
@pytest.mark.parametrize("kind", ["normal", "relu", "heavy"])
def test_round_trip_error_at_most_half_a_step(k, kind):
    rng = np.random.default_rng(7 * k + len(kind))
    x = rng.standard_normal(5000).astype(np.float32)
    if kind == "relu":
        x = np.maximum(x, 0)
    if kind == "heavy":
        x = rng.standard_t(3, 5000).astype(np.float32) * np.float32(1e-3)
    hdr, pay = orc.uniform_compress(x, k, 50, 100)
    s = float(np.frombuffer(hdr, dtype="<f4")[0])
    L = 2 ** (k - 1) - 1
    c = float(np.abs(x).max())
    assert s == pytest.approx(c / L, rel=1e-6)
    xh = orc.uniform_decompress(hdr, pay, k, 50, 100)
    assert np.all(np.abs(xh.astype(np.float64) - x.astype(np.float64)) <= s * (0.5 + 2e-5))
    # zero stays zero; the extreme values take the extreme codes; codes stay in range
    q = orc.uniform_decode(pay, k, x.size)
    assert np.all(xh[x == 0] == 0)
    assert abs(int(q[np.argmax(np.abs(x))])) == L
    assert q.min() >= -L and q.max() <= L
    # the quantizer is monotone
    order = np.argsort(x, kind="stable")
    assert np.all(np.diff(q[order]) >= 0)


@pytest.mark.parametrize("k", KS)
def test_representable_values_reconstruct_exactly(k):
    """x = fl32(q*s) for every q in [-L, L] comes back bit for bit."""
    L = 2 ** (k - 1) - 1
    for c in (1.0, 0.37, 3.1e-4, 1234.5):
        s = np.float32(c) / np.float32(L)
        qs = np.arange(-L, L + 1)
        x = (qs.astype(np.float32) * s).astype(np.float32)
        hdr, pay = orc.uniform_compress(x, k, 1, x.size)
        if np.frombuffer(hdr, dtype="<f4")[0] != s:
            continue  # fl32(L*s) != c: this c is not itself representable as L*s
        assert orc.uniform_decode(pay, k, x.size).tolist() == qs.tolist()
        assert orc.uniform_decompress(hdr, pay, k, 1, x.size).tobytes() == x.tobytes()


def test_all_zero_and_tiny_ranges():
    for x in (np.zeros(40, np.float32), np.full(40, 1e-40, np.float32), np.full(40, 2.0 ** -101, np.float32)):
        for k in KS:
            hdr, pay = orc.uniform_compress(x, k, 4, 10)
            assert np.frombuffer(hdr, dtype="<f4")[0] == 0.0
            assert orc.uniform_decode(pay, k, 40).tolist() == [0] * 40
            assert orc.uniform_decompress(hdr, pay, k, 4, 10).tolist() == [0.0] * 40
    x = np.full(8, 2.0 ** -100, np.float32)
    hdr, pay = orc.uniform_compress(x, 4, 1, 8)
    assert np.frombuffer(hdr, dtype="<f4")[0] > 0
    assert orc.uniform_decode(pay, 4, 8).tolist() == [7] * 8


@pytest.mark.parametrize("k", [4, 6, 8])
def test_per_channel_reduces_to_per_tensor_on_each_channel(k):
    """Per-channel ranges must equal the per-tensor scheme applied to each channel slice
    on its own (special case that reduces to the paper's per-tensor rule)."""
    rng = np.random.default_rng(3)
    n, C, inner = 3, 5, 12
    x = rng.standard_normal((n, C, inner)).astype(np.float32) * np.arange(1, C + 1, dtype=np.float32)[None, :, None]
    hdr, pay = orc.uniform_compress(x, k, n, C * inner, channels=C)
    s = np.frombuffer(hdr, dtype="<f4")
    q = orc.uniform_decode(pay, k, x.size).reshape(n, C, inner)
    xh = orc.uniform_decompress(hdr, pay, k, n, C * inner, channels=C).reshape(n, C, inner)
    for ch in range(C):
        sl = np.ascontiguousarray(x[:, ch, :])
        h1, p1 = orc.uniform_compress(sl, k, n, inner)
        assert np.frombuffer(h1, dtype="<f4")[0] == s[ch]
        assert orc.uniform_decode(p1, k, sl.size).tolist() == q[:, ch, :].reshape(-1).tolist()
        assert orc.uniform_decompress(h1, p1, k, n, inner).tolist() == xh[:, ch, :].reshape(-1).tolist()


def test_bf16_io_against_torch_casts():
    """bf16 input is widened exactly; bf16 output is the RNE cast: both checked against
    PyTorch's own bfloat16 conversions (a different implementation)."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(5)
    x = rng.standard_normal(4096).astype(np.float32)
    t = torch.from_numpy(x).to(torch.bfloat16)
    bits = t.view(torch.int16).numpy().view(np.uint16)
    assert orc.narrow_bf16(x).tolist() == bits.tolist()
    assert orc.widen_bf16(bits).tolist() == t.to(torch.float32).numpy().tolist()
    hdr, pay = orc.uniform_compress(bits, 6, 64, 64, in_bf16=True)
    h2, p2 = orc.uniform_compress(orc.widen_bf16(bits), 6, 64, 64)
    assert hdr == h2 and pay.tobytes() == p2.tobytes()
    out16 = orc.uniform_decompress(hdr, pay, 6, 64, 64, out_bf16=True)
    out32 = orc.uniform_decompress(hdr, pay, 6, 64, 64)
    assert out16.tolist() == torch.from_numpy(out32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).tolist()


# ---------------------------------------------------------------- stochastic rounding
def test_counter_uniform_matches_splitmix64_vectors(golden_rows, golden_kv):
    seed = int(golden_kv("splitmix64_vectors.txt")["seed"])
    vec = [int(r[0]) for r in golden_rows("splitmix64_vectors.txt") if len(r) == 1]
    assert len(vec) == 5
    u = orc.counter_uniform(seed, np.arange(5))
    assert u.tolist() == [(z >> 40) / 2.0 ** 24 for z in vec]
    assert np.all((u >= 0) & (u < 1))


@pytest.mark.parametrize("k", [4, 8])
def test_stochastic_rounding_is_floor_or_ceil_and_unbiased(k):
    """Paper's rule: floor(v)+1 w.p. v-floor(v) ("Backward Quantizer"): each code is one of
    the two neighbours, the mean over seeds approaches v (within 4 sigma), no code leaves
    the k-bit range, and the same seed gives the same stream."""
    rng = np.random.default_rng(11)
    x = (rng.standard_normal(512) * 0.3).astype(np.float32)
    L = 2 ** (k - 1) - 1
    c = np.abs(x).max()
    v = x.astype(np.float64) * (L / float(c))
    S = 400
    acc = np.zeros(x.size)
    for seed in range(S):
        hdr, pay = orc.uniform_compress(x, k, 8, 64, rounding=1, seed=seed)
        q = orc.uniform_decode(pay, k, x.size)
        assert np.all((q >= np.floor(v) - 1e-3 - 1) & (q <= np.floor(v) + 1 + 1e-3))
        assert np.all(np.abs(q - v) < 1 + 1e-4)
        assert q.min() >= -2 ** (k - 1) and q.max() <= L
        acc += q
    frac = v - np.floor(v)
    sigma = np.sqrt(np.maximum(frac * (1 - frac), 1e-12) / S)
    assert np.all(np.abs(acc / S - v) <= 4.5 * sigma + 1e-4)
    a = orc.uniform_compress(x, k, 8, 64, rounding=1, seed=9)
    b = orc.uniform_compress(x, k, 8, 64, rounding=1, seed=9)
    assert a[1].tobytes() == b[1].tobytes()
    assert a[1].tobytes() != orc.uniform_compress(x, k, 8, 64, rounding=1, seed=10)[1].tobytes()

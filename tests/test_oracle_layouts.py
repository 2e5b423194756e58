"""Oracle pins for the payload layouts beside the packed ones: the paper's own backward
layout (codes of neighbouring batch entries share a byte) and the "w/o enc." forms."""
import numpy as np
import pytest

from oracle import accept_oracle as orc


@pytest.mark.parametrize("k", [2, 4, 8])
@pytest.mark.parametrize("n,m", [(2, 1), (4, 3), (5, 7), (9, 4), (1, 5)])
def test_batch_layout_matches_packbits_and_inverts(k, n, m):
    """Independent packer: write every code as k bits, most significant first, lay the
    8/k batch neighbours of a column side by side and let numpy.packbits cut bytes."""
    rng = np.random.default_rng(100 * k + 10 * n + m)
    u = rng.integers(0, 2 ** k, size=(n, m)).astype(np.uint64)
    per = 8 // k
    G = (n + per - 1) // per
    pad = np.zeros((G * per, m), dtype=np.uint64)
    pad[:n] = u
    bits = ((pad[:, :, None] >> np.arange(k - 1, -1, -1, dtype=np.uint64)) & np.uint64(1)).astype(np.uint8)
    ref = np.packbits(bits.reshape(G, per, m, k).transpose(0, 2, 1, 3).reshape(-1))  # [g][j][entry][bit]
    got = orc.pack_batch(u, k, n, m)
    assert got.tolist() == ref.tolist()
    assert got.size == orc.packed_size(orc.SCHEME_UNIFORM, k, n, m, layout=orc.LAYOUT_BATCH)[1]
    assert orc.unpack_batch(got, k, n, m).tolist() == u.reshape(-1).tolist()


def test_batch_layout_k4_is_the_papers_halving():
    """"Backward Encoder": at k = 4 the codes q + 8 lie in [0, 15] and two tensors along the
    first dimension become one, n/2 x w x h x c bytes; at k = 8 g_q goes out as it is."""
    n, m = 6, 5
    x = np.linspace(-1.0, 1.0, n * m, dtype=np.float32)
    h4, p4 = orc.uniform_compress(x, 4, n, m, layout=orc.LAYOUT_BATCH)
    assert p4.size == (n // 2) * m
    q = orc.uniform_decode(p4, 4, n * m, orc.LAYOUT_BATCH, n, m).reshape(n, m)
    assert q.min() == -7 and q.max() == 7          # max|x| maps to +-7; -8 is never produced by symmetric data
    assert (p4.reshape(n // 2, m) >> 4).tolist() == (q[0::2] + 8).tolist()   # first entry of a pair: high nibble
    assert (p4.reshape(n // 2, m) & 15).tolist() == (q[1::2] + 8).tolist()
    h8, p8 = orc.uniform_compress(x, 8, n, m, layout=orc.LAYOUT_BATCH)
    _, d8 = orc.uniform_compress(x, 8, n, m)
    _, u8 = orc.uniform_compress(x, 8, n, m, layout=orc.LAYOUT_UNENCODED)
    assert p8.tolist() == d8.tolist() == u8.tolist()  # one byte per value either way
    # same values whatever the layout
    a = orc.uniform_decompress(h4, p4, 4, n, m, layout=orc.LAYOUT_BATCH)
    hd, pd = orc.uniform_compress(x, 4, n, m)
    assert hd == h4
    assert a.tobytes() == orc.uniform_decompress(hd, pd, 4, n, m).tobytes()


@pytest.mark.parametrize("k", [2, 3, 4, 5, 8])
def test_unencoded_uniform_is_int8_of_q(k):
    x = (np.random.default_rng(k).standard_normal(77) * 3).astype(np.float32)
    c = orc.uniform_range(x, 7, 11)
    s, r = orc.uniform_scale(c, k)
    q = orc.uniform_quantize(x, r, k, 7, 11)
    h, p = orc.uniform_compress(x, k, 7, 11, layout=orc.LAYOUT_UNENCODED)
    assert p.dtype == np.uint8 and p.size == 77
    assert p.view(np.int8).tolist() == q.tolist()
    hd, pd = orc.uniform_compress(x, k, 7, 11)
    assert orc.uniform_decompress(h, p, k, 7, 11, layout=orc.LAYOUT_UNENCODED).tobytes() == \
        orc.uniform_decompress(hd, pd, k, 7, 11).tobytes()


@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_unencoded_mbq_is_plus_minus_one_bytes(k):
    """"w/o enc.": each binary base is an 8-bit integer; B alpha - m_q is the same x_hat."""
    n, m = 9, 13
    x = np.random.default_rng(40 + k).standard_normal(n * m).astype(np.float32)
    alpha, _ = orc.mbq_residue_init(x, k)
    h, p = orc.mbq_compress(x, k, n, m, alpha, 3, layout=orc.LAYOUT_UNENCODED)
    assert p.size == n * m * k == orc.packed_size(orc.SCHEME_MBQ, k, n, m, layout=orc.LAYOUT_UNENCODED)[1]
    b = p.view(np.int8).reshape(n * m, k)
    assert set(np.unique(b).tolist()) <= {-1, 1}
    hp, pp = orc.mbq_compress(x, k, n, m, alpha, 3)
    assert h == hp                                     # the header does not depend on the layout
    code = orc.mbq_unpack(pp, k, n, m)
    assert ((b > 0).astype(np.int64) << np.arange(k)).sum(axis=1).tolist() == code.tolist()
    # B alpha computed directly from the +-1 bytes (float64) agrees with the dequantizer's float32 sum
    xh = orc.mbq_decompress(h, p, k, n, m, layout=orc.LAYOUT_UNENCODED)
    assert xh.tobytes() == orc.mbq_decompress(hp, pp, k, n, m).tobytes()
    hdr = np.frombuffer(h, "<f4")
    direct = b.astype(np.float64) @ hdr[:k].astype(np.float64) - float(hdr[k])
    assert np.all(np.abs(direct - xh) <= 1e-6 * np.abs(hdr[:k]).sum())

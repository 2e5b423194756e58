"""GPU parity beyond 2^31 elements: every index computation in the kernels is 64-bit.

The tensors are too large for a whole-tensor oracle run, so the oracle recomputes sampled
8-element groups (around the 2^31 boundary, at both ends, and at random) one by one."""
import numpy as np
import pytest

from oracle import accept_oracle as orc

from gpu_util import dev_bytes, torch_mod

pytestmark = pytest.mark.gpu

BIG = (1 << 31) + 2 * 8192 + 13  # past the 32-bit boundary, ragged tail


@pytest.fixture(scope="module")
def A():
    torch = torch_mod()
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2311_05827_amd as pkg
    return pkg


def big_tensor(N, seed):
    rng = np.random.default_rng(seed)
    block = rng.standard_normal(1 << 24, dtype=np.float32)
    x = np.tile(block, (N + block.size - 1) // block.size)[:N]
    # make the copies differ, and put the extreme value past the 2^31 boundary
    x[1 << 30:] *= np.float32(0.5)
    x[(1 << 31):] *= np.float32(1.5)
    x[(1 << 31) + 37] = np.float32(-9.0)
    return x


def sampled_groups(N, seed):
    rng = np.random.default_rng(seed)
    G = N // 8
    near = np.arange((1 << 31) // 8 - 16, (1 << 31) // 8 + 16)
    g = np.concatenate([rng.integers(0, G, size=20000), near, np.arange(0, 8), np.arange(G - 8, G)])
    return np.unique(g[(g >= 0) & (g < G)])


def test_uniform_beyond_2_31_elements(A):
    torch = torch_mod()
    N, k = BIG, 3
    print("building", N, "elements", flush=True)
    x = big_tensor(N, 1)
    c = np.float32(np.abs(x).max())
    assert c == np.float32(9.0)
    s, r = orc.uniform_scale(np.array([c], np.float32), k)
    xd = torch.from_numpy(x).cuda()
    d = A.make_desc(A.UNIFORM, k, 1, N)
    print("compress", flush=True)
    header, payload = A.accept_compress(d, xd)
    xh = A.accept_decompress(d, header, payload)
    torch.cuda.synchronize()
    assert dev_bytes(header) == s.astype("<f4").tobytes()
    assert payload.numel() == (N * k + 7) // 8
    g = sampled_groups(N, 2)
    idx = (g[:, None] * 8 + np.arange(8)[None, :]).reshape(-1)
    q = orc.uniform_quantize(x[idx], r, k, 1, idx.size)
    exp = orc.pack_stream(orc.uniform_codes(q, k), k).reshape(-1, k)
    byte_idx = torch.from_numpy((g[:, None] * k + np.arange(k)[None, :]).reshape(-1)).cuda()
    got = payload[byte_idx].cpu().numpy().reshape(-1, k)
    bad = np.nonzero((got != exp).any(axis=1))[0]
    assert bad.size == 0, "group %d differs" % g[bad[0]]
    out = xh[torch.from_numpy(idx).cuda()].cpu().numpy()
    assert out.tobytes() == (q.astype(np.float32) * s[0]).astype(np.float32).tobytes()
    # the ragged tail (last 5 elements and the last, partial byte) against the oracle
    tail0 = (N // 8) * 8
    qt = orc.uniform_quantize(x[tail0:], r, k, 1, N - tail0)
    expt = orc.pack_stream(orc.uniform_codes(qt, k), k)
    assert payload[(tail0 // 8) * k:].cpu().numpy().tobytes() == expt.tobytes()
    assert xh[tail0:].cpu().numpy().tobytes() == (qt.astype(np.float32) * s[0]).astype(np.float32).tobytes()


def test_mbq_beyond_2_31_elements(A):
    torch = torch_mod()
    n, m, k = 16, (1 << 27) + 1028, 2
    N = n * m
    assert N > (1 << 31)
    x = big_tensor(N, 3)
    alpha = np.array([1.0, 0.4], np.float32)
    xd = torch.from_numpy(x).cuda()
    d = A.make_desc(A.MBQ, k, n, m, t=7)
    header, payload = A.accept_compress(d, xd, alpha_prev=torch.from_numpy(alpha).cuda())
    xh = A.accept_decompress(d, header, payload)
    torch.cuda.synchronize()
    hb, pb = A.accept_packed_size(d)
    assert payload.numel() == pb == 2 * m * k
    rng = np.random.default_rng(4)
    cols = np.unique(np.concatenate([rng.integers(0, m, size=5000), np.arange(0, 8), np.arange(m - 8, m),
                                     np.arange(m // 2 - 8, m // 2 + 8)]))
    x2 = x.reshape(n, m)
    sub = np.ascontiguousarray(x2[:, cols])
    code = orc.mbq_assign(sub, alpha)
    exp = orc.mbq_pack(code, k, n, cols.size).reshape(2, cols.size, k)
    for grp in range(2):
        byte_idx = torch.from_numpy(((grp * m + cols)[:, None] * k + np.arange(k)[None, :]).reshape(-1)).cuda()
        got = payload[byte_idx].cpu().numpy().reshape(cols.size, k)
        assert got.tobytes() == exp[grp].tobytes()
    # decoded values of the sampled columns from the GPU's own header
    h = dev_bytes(header)
    ref = orc.mbq_decompress(h, exp.reshape(-1), k, n, cols.size).reshape(n, cols.size)
    out = xh.view(n, m)[:, torch.from_numpy(cols).cuda()].cpu().numpy()
    assert out.tobytes() == ref.tobytes()
    # header sanity at this size: alpha stays positive and near the least-squares scale
    hf = np.frombuffer(h, dtype="<f4")
    assert np.all(hf[:k] > 0) and np.all(np.isfinite(hf))

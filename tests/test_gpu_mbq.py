"""GPU parity, scheme M: bit planes bit-exact, header within 1e-6 * sum|alpha| (the sums
are reduced in a different order), decoded values within 1e-6 * sum|alpha| and bit-exact
when the decoder is fed the oracle's own header and payload."""
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


def run_case(A, x, k, n, m, t=1, alpha_prev=None, in_bf16=False, out_bf16=False, tag=""):
    torch = torch_mod()
    print("case", tag, "k", k, "n", n, "m", m, "t", t, "bf16", in_bf16, out_bf16, flush=True)
    xd, bits = to_dev(x, in_bf16)
    xin = orc.widen_bf16(bits) if in_bf16 else np.asarray(x, np.float32).reshape(-1)
    if alpha_prev is None:
        alpha_prev, _ = orc.mbq_residue_init(xin, k)
    ad = torch.from_numpy(np.asarray(alpha_prev, np.float32)).cuda()
    d = A.make_desc(A.MBQ, k, n, m, in_dtype=A.BF16 if in_bf16 else A.F32,
                    out_dtype=A.BF16 if out_bf16 else A.F32, t=t)
    header, payload = A.accept_compress(d, xd, alpha_prev=ad)
    xh = A.accept_decompress(d, header, payload)
    torch.cuda.synchronize()
    oh, op = orc.mbq_compress(bits if in_bf16 else x, k, n, m, alpha_prev, t, in_bf16)
    mm = first_mismatch(dev_bytes(payload), op.tobytes())
    assert mm is None, "payload differs: " + mm
    gh = np.frombuffer(dev_bytes(header), dtype="<f4")
    ohf = np.frombuffer(oh, dtype="<f4")
    scale = float(np.sum(np.abs(ohf[:k])))
    assert np.all(np.abs(gh.astype(np.float64) - ohf.astype(np.float64)) <= 1e-6 * scale), (gh, ohf)
    # decoder fed the oracle's header and payload: bit-exact
    xh2 = A.accept_decompress(d, bytes_to_dev(oh), bytes_to_dev(op.tobytes()))
    torch.cuda.synchronize()
    oxh = orc.mbq_decompress(oh, op, k, n, m, out_bf16)
    got2 = out_to_numpy(xh2)
    assert got2.tobytes() == oxh.tobytes()
    # decoder fed the GPU's own header: within tolerance of the oracle's output
    got = out_to_numpy(xh)
    if out_bf16:
        g32, o32 = orc.widen_bf16(got), orc.widen_bf16(oxh)
        assert np.all(np.abs(g32.astype(np.float64) - o32.astype(np.float64)) <= 2.0 ** -7 * np.abs(o32) + 1e-6 * scale)
    else:
        assert np.all(np.abs(got.astype(np.float64) - oxh.astype(np.float64)) <= 1e-6 * scale)
    return gh, ohf


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5, 6, 7, 8])
def test_small_shapes_every_k(A, k):
    for n, m in [(8, 1), (16, 5), (3, 7), (9, 4), (1, 1), (64, 36), (13, 260), (24, 1030)]:
        x = si.make_shape("relu_normal", (n, m), 1000 + 10 * k + n)
        run_case(A, x, k, n, m, t=3, tag="small")


@pytest.mark.parametrize("k", [2, 3, 4])
@pytest.mark.parametrize("t", [0, 1, 50, 100])
def test_multi_block_shapes(A, k, t):
    # several workgroups, row-group boundary inside a wavefront, n not a multiple of 8
    x = si.make_shape("relu_lognormal", (21, 4100), 2000 + k)
    run_case(A, x, k, 21, 4100, t=t, tag="21x4100")
    x = si.make_shape("relu_normal", (256, 1024), 2001 + k)
    run_case(A, x, k, 256, 1024, t=t, tag="256x1024")
    x = si.make_shape("student_t3", (12, 4099), 2002 + k)  # m not a multiple of 4: scalar path
    run_case(A, x, k, 12, 4099, t=t, tag="12x4099")


@pytest.mark.parametrize("k", [2, 3, 4])
def test_config1_activation_both_views(A, k):
    x = si.make("cfg1_act")
    run_case(A, x, k, 4, 65536, t=1, tag="cfg1 n=4 (padded to 8 rows)")
    run_case(A, x, k, 256, 1024, t=1, tag="cfg1 as 256x1024")


@pytest.mark.parametrize("k", [2, 4, 6])
@pytest.mark.parametrize("in_bf16,out_bf16", [(True, False), (False, True), (True, True)])
def test_bf16_io(A, k, in_bf16, out_bf16):
    x = si.make_shape("relu_lognormal", (16, 2056), 3000 + k)
    run_case(A, x, k, 16, 2056, in_bf16=in_bf16, out_bf16=out_bf16, tag="bf16 vec8")
    x = si.make_shape("relu_lognormal", (10, 1004), 3001 + k)  # 1004 % 8 != 0: scalar path
    run_case(A, x, k, 10, 1004, in_bf16=in_bf16, out_bf16=out_bf16, tag="bf16 scalar")


def test_alpha_carried_across_batches(A):
    """Feed header[0..k) back as alpha_prev for a few batches, oracle and GPU each on
    their own chain; the chains must stay within tolerance of each other."""
    torch = torch_mod()
    k, n, m = 3, 32, 2048
    a_gpu = a_orc = None
    for t in range(4):
        x = si.make_shape("relu_normal", (n, m), 4000 + t)
        if t == 0:
            a_orc, _ = orc.mbq_residue_init(x, k)
            a_gpu = a_orc.copy()
        xd, _ = to_dev(x)
        d = A.make_desc(A.MBQ, k, n, m, t=t)
        header, payload = A.accept_compress(d, xd, alpha_prev=torch.from_numpy(a_gpu).cuda())
        torch.cuda.synchronize()
        oh, op = orc.mbq_compress(x, k, n, m, a_orc, t)
        a_gpu = np.frombuffer(dev_bytes(header), dtype="<f4")[:k].copy()
        a_orc = np.frombuffer(oh, dtype="<f4")[:k].copy()
        assert np.all(np.abs(a_gpu - a_orc) <= 4e-6 * np.sum(np.abs(a_orc)))
        differing = np.count_nonzero(np.frombuffer(dev_bytes(payload), np.uint8) != op)
        assert differing <= 0.001 * op.size  # only elements within an ulp of a threshold may move


def test_singular_gram_and_special_values(A):
    # constant input: every element takes the same level, B^T B is singular -> alpha stays
    x = np.full((8, 64), 5.0, np.float32)
    gh, ohf = run_case(A, x, 2, 8, 64, alpha_prev=np.array([1.0, 0.5], np.float32), tag="singular")
    assert gh[:2].tolist() == [1.0, 0.5]
    # duplicate levels (alpha_0 == alpha_1) and a zero coefficient
    x = si.make_shape("relu_normal", (16, 260), 5000)
    run_case(A, x, 2, 16, 260, alpha_prev=np.array([0.5, 0.5], np.float32), tag="dup-levels")
    run_case(A, x, 3, 16, 260, alpha_prev=np.array([0.7, 0.0, 0.2], np.float32), tag="zero-alpha")
    # positive and negative denormals must fall on their own side of the zero threshold;
    # exact threshold values go to the lower level
    a = np.array([0.75, 0.25], np.float32)
    _, _, tau = orc.mbq_levels(a)
    vals = np.concatenate([tau, [1e-40, -1e-40, 0.0, -0.0, 1e-45, -1e-45]]).astype(np.float32)
    x = np.resize(vals, (8, 36)).astype(np.float32)
    run_case(A, x, 2, 8, 36, alpha_prev=a, tag="thresholds+denormals")


@pytest.mark.parametrize("k,alpha", [(3, [1.0, 0.03, 0.02]), (4, [1.0, 0.5, 0.03, 0.02]), (4, [0.6, 0.58, 0.3, 0.29])])
def test_two_thresholds_per_bucket(A, k, alpha):
    """Levels closer than the width of a bucket of the level search's float-prefix table: the
    encoder then compares against two thresholds per element.  The shapes give whole pipelined
    rounds, a last incomplete round and a ragged last row group; values sit on and next to the
    thresholds as well."""
    a = np.asarray(alpha, np.float32)
    _, _, tau = orc.mbq_levels(a)
    for n, m, bf in [(8, 8 * 1024 * 100 + 4 * 37, False), (19, 400004, False), (16, 800008, True), (5, 1003, False)]:
        x = si.make_shape("student_t3", (n, m), 7100 + n)
        x = (x * np.float32(0.8 / x.std())).astype(np.float32)
        edge = np.concatenate([tau, np.nextafter(tau, np.float32(np.inf)), np.nextafter(tau, np.float32(-np.inf))])
        x.reshape(-1)[: edge.size * 5 : 5] = edge.astype(np.float32)
        run_case(A, x, k, n, m, alpha_prev=a, in_bf16=bf, tag="two-per-bucket")


@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_residue_init(A, k):
    torch = torch_mod()
    for shape, bf in [((16, 1000), False), ((7, 333), False), ((16, 1000), True)]:
        x = si.make_shape("relu_lognormal", shape, 6000 + k)
        xd, bits = to_dev(x, bf)
        xin = orc.widen_bf16(bits) if bf else x
        d = A.make_desc(A.MBQ, k, shape[0], shape[1], in_dtype=A.BF16 if bf else A.F32)
        a0 = A.accept_mbq_init(d, xd)
        torch.cuda.synchronize()
        exp, _ = orc.mbq_residue_init(xin, k)
        got = a0.cpu().numpy()
        assert np.all(np.abs(got.astype(np.float64) - exp.astype(np.float64)) <= 1e-6 * float(np.sum(np.abs(exp)))), (got, exp)


@pytest.mark.parametrize("k", [1, 2, 3, 4, 6])
def test_batch0_compress(A, k):
    """accept_mbq_compress_first: header [alpha^0, m_q] within 1e-6 * sum|alpha| of the oracle's,
    bit planes of B^0 bit-exact for the GPU's own alpha^0 bits, and the decoder reads the pair
    like any other batch."""
    torch = torch_mod()
    for shape, bf in [((16, 1000), False), ((7, 333), False), ((21, 4100), False), ((24, 2056), True), ((10, 1004), True),
                      ((64, 8192 + 4), False)]:
        n, m = shape
        print("batch0 k", k, "shape", shape, "bf16", bf, flush=True)
        x = si.make_shape("relu_lognormal", shape, 6500 + k)
        x.reshape(-1)[::97] = 0.0
        xd, bits = to_dev(x, bf)
        xin = orc.widen_bf16(bits) if bf else x
        d = A.make_desc(A.MBQ, k, n, m, in_dtype=A.BF16 if bf else A.F32)
        header, payload = A.accept_mbq_compress_first(d, xd)
        xh = A.accept_decompress(d, header, payload)
        torch.cuda.synchronize()
        gh = np.frombuffer(dev_bytes(header), dtype="<f4")
        oh, _ = orc.mbq_compress_first(xin, k, n, m)
        ohf = np.frombuffer(oh, dtype="<f4")
        scale = float(np.sum(np.abs(ohf[:k])))
        assert np.all(np.abs(gh.astype(np.float64) - ohf.astype(np.float64)) <= 1e-6 * scale), (gh, ohf)
        op = orc.mbq_pack(orc.mbq_residue_signs(xin, gh[:k]), k, n, m)
        mm = first_mismatch(dev_bytes(payload), op.tobytes())
        assert mm is None, "B^0 planes differ: " + mm
        ref = orc.mbq_decompress(dev_bytes(header), op, k, n, m)
        assert out_to_numpy(xh).tobytes() == ref.tobytes()
        # the stand-alone initialisation gives the same alpha^0 bits
        a0 = A.accept_mbq_init(d, xd)
        torch.cuda.synchronize()
        assert a0.cpu().numpy().tobytes() == gh[:k].tobytes()

"""GPU parity, scheme U: the HIP path (through the C ABI) against the CPU oracle.

Payload and header must match bit for bit; decoded values must match within
1e-6 * scale (they are in fact produced by the same single float32 multiply)."""
import numpy as np
import pytest

import synthetic_inputs as si
from oracle import accept_oracle as orc

from gpu_util import bytes_to_dev, dev_bytes, first_mismatch, out_to_numpy, to_dev, torch_mod

pytestmark = pytest.mark.gpu

KS = [2, 3, 4, 5, 6, 7, 8]


@pytest.fixture(scope="module")
def A():
    torch = torch_mod()
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2311_05827_amd as pkg
    return pkg


def run_case(A, x, k, n, m, channels=0, in_bf16=False, out_bf16=False, rounding=0, seed=0, tag=""):
    torch = torch_mod()
    print("case", tag, "k", k, "n", n, "m", m, "C", channels, "bf16", in_bf16, out_bf16, "rnd", rounding, flush=True)
    xd, bits = to_dev(x, in_bf16)
    d = A.make_desc(A.UNIFORM, k, n, m, channels=channels, in_dtype=A.BF16 if in_bf16 else A.F32,
                    out_dtype=A.BF16 if out_bf16 else A.F32, rounding=rounding, seed=seed)
    header, payload = A.accept_compress(d, xd)
    xh = A.accept_decompress(d, header, payload)
    torch.cuda.synchronize()
    oh, op = orc.uniform_compress(bits if in_bf16 else x, k, n, m, channels, in_bf16, rounding, seed)
    assert dev_bytes(header) == oh, "header differs " + str(first_mismatch(dev_bytes(header), oh))
    mm = first_mismatch(dev_bytes(payload), op.tobytes())
    assert mm is None, "payload differs: " + mm
    oxh = orc.uniform_decompress(oh, op, k, n, m, channels, out_bf16)
    got = out_to_numpy(xh)
    if out_bf16:
        assert got.tolist() == oxh.tolist()
    else:
        scale = float(np.max(np.frombuffer(oh, dtype="<f4"))) * (2 ** (k - 1) - 1)
        assert np.all(np.abs(got.astype(np.float64) - oxh.astype(np.float64)) <= 1e-6 * scale)
        assert got.tobytes() == oxh.tobytes()
    return oh, op


@pytest.mark.parametrize("k", KS)
def test_multi_tile_with_ragged_tail(A, k):
    # three full 8192-element tiles plus a tail that is neither a multiple of 32 nor of 8
    N = 3 * 8192 + 777
    x = si.make_shape("grad_outliers", (1, N), 10 + k)
    run_case(A, x, k, 1, N, tag="ragged")
    x = si.make_shape("relu_normal", (3, 8455), 20 + k)
    run_case(A, x, k, 3, 8455, tag="relu")


@pytest.mark.parametrize("N", [1, 2, 3, 7, 8, 9, 31, 32, 33, 63, 64, 65, 255, 8191, 8192, 8193])
def test_tiny_and_boundary_sizes(A, N):
    for k in KS:
        x = si.make_shape("student_t3", (1, N), 100 + N)
        run_case(A, x, k, 1, N, tag="tiny")


@pytest.mark.parametrize("k", [3, 4, 8])
def test_odd_shapes(A, k):
    x = si.make_shape("student_t3", (3, 5, 7), 5)
    run_case(A, x, k, 3, 35, tag="3x5x7")
    x = si.make_shape("student_t3", (15, 127, 67), 6)
    run_case(A, x, k, 15, 127 * 67, tag="15x127x67")


@pytest.mark.parametrize("k", KS)
@pytest.mark.parametrize("in_bf16,out_bf16", [(True, False), (False, True), (True, True)])
def test_bf16_io(A, k, in_bf16, out_bf16):
    x = si.make_shape("relu_lognormal", (4, 5000), 30 + k)
    run_case(A, x, k, 4, 5000, in_bf16=in_bf16, out_bf16=out_bf16, tag="bf16")
    x = si.make_shape("grad", (2, 8192 + 13), 31 + k)
    run_case(A, x, k, 2, 8192 + 13, in_bf16=in_bf16, out_bf16=out_bf16, tag="bf16-tail")


def test_max_found_at_every_lane_and_block_position(A):
    """The range reduction must see every element: plant the maximum at many positions."""
    N = 5 * 4096 + 5
    base = (si.make_shape("grad", (1, N), 77) * np.float32(0.5)).astype(np.float32)
    for pos in list(range(0, 300, 7)) + [4095, 4096, 8191, 12345, N - 6, N - 5, N - 1]:
        x = base.copy()
        x[0, pos] = np.float32(-3.0)
        oh, _ = run_case(A, x, 8, 1, N, tag="maxpos%d" % pos)
        assert np.frombuffer(oh, dtype="<f4")[0] == np.float32(3.0) / np.float32(127)


def test_all_zero_tiny_and_denormal_tensors(A):
    for k in (2, 5, 8):
        run_case(A, np.zeros((2, 5000), np.float32), k, 2, 5000, tag="zeros")
        run_case(A, np.full((2, 5000), 1e-40, np.float32), k, 2, 5000, tag="denormal")
        run_case(A, np.full((1, 40), 2.0 ** -101, np.float32), k, 1, 40, tag="below-threshold")
        run_case(A, np.full((1, 40), 2.0 ** -100, np.float32), k, 1, 40, tag="at-threshold")
        x = np.zeros((1, 9000), np.float32)
        x[0, 4567] = -1.0
        run_case(A, x, k, 1, 9000, tag="single-spike")


def test_exact_ties_round_to_even(A):
    for k in KS:
        L = 2 ** (k - 1) - 1
        j = np.arange(-2 * L, 2 * L + 1)
        x = np.tile((j * 0.125 / 2).astype(np.float32), 70)[None, :]
        run_case(A, x, k, 1, x.size, tag="ties")


@pytest.mark.parametrize("k", [4, 6, 8])
@pytest.mark.parametrize("in_bf16", [False, True])
def test_per_channel_segmented(A, k, in_bf16):
    # segments of 1024 and 3136 elements (>= 512 and vector aligned): wave-per-segment range pass
    x = si.make_shape("relu_lognormal_chgain", (3, 5, 32, 32), 40 + k)
    run_case(A, x, k, 3, 5 * 1024, channels=5, in_bf16=in_bf16, out_bf16=in_bf16, tag="seg1024")
    x = si.make_shape("relu_lognormal_chgain", (5, 7, 56, 56), 41 + k)
    run_case(A, x, k, 5, 7 * 3136, channels=7, in_bf16=in_bf16, tag="seg3136")
    # a segment longer than one chunk (4096 vectors): 2 x 3 x 20000 floats
    x = si.make_shape("relu_lognormal_chgain", (2, 3, 20000), 42 + k)
    run_case(A, x, k, 2, 60000, channels=3, in_bf16=in_bf16, tag="seg20000")


@pytest.mark.parametrize("k", [2, 5, 8])
def test_per_channel_whole_tiles(A, k):
    """Tensors of whole 8192-element tiles with long segments: the quantize pass finishes the
    channels' ranges itself, tile by tile.  Tiles that touch more segments than there are
    channels, one segment over several tiles (two chunks per segment), many rows (several
    partial maxima per lane), float32 and bfloat16, and the same shapes one row short of whole
    tiles (separate U1b kernel) for comparison."""
    for n, C, seg in [(16, 3, 512), (4, 16, 512), (8, 40, 1024), (2, 5, 8192), (4, 2, 16384), (300, 4, 2048),
                      (64, 3, 1536), (1024, 1, 512)]:
        if C == 1:
            continue  # one channel is the per-tensor mode
        x = si.make_shape("relu_lognormal_chgain", (n, C, seg), 80 + k)
        gain = np.float32(10.0) ** np.linspace(-2, 2, C, dtype=np.float32)
        x = np.ascontiguousarray(x * gain[None, :, None], dtype=np.float32)
        assert (n * C * seg) % 8192 == 0
        run_case(A, x, k, n, C * seg, channels=C, tag="whole tiles seg%d C%d" % (seg, C))
        run_case(A, x, k, n, C * seg, channels=C, in_bf16=True, out_bf16=True, tag="whole tiles bf16")
        run_case(A, x[: n - 1], k, n - 1, C * seg, channels=C, tag="one row short") if (n - 1) * C * seg % 8192 else None
    x = si.make_shape("grad_outliers", (8, 4, 2048), 90 + k)
    run_case(A, x, k, 8, 8192, channels=4, rounding=1, seed=5, tag="whole tiles stochastic")


@pytest.mark.parametrize("k", [3, 8])
def test_more_tiles_than_workgroups(A, k):
    """Tensors of more than 2048 tiles: workgroups take several tiles each, last-read first, and
    step their channel position backwards; a few tiles after the last whole group of eight keep
    their plain places.  One range, one range per channel (with and without whole tiles) and
    one range per element."""
    T = 8192
    # one range: 2051 whole tiles (3 after the reversed part) and a ragged tail
    x = si.make_shape("grad_outliers", (1, 2051 * T + 77), 95 + k)
    run_case(A, x, k, 1, 2051 * T + 77, tag="2051 tiles + tail")
    # one range per channel, whole tiles (ranges finished tile by tile): 64 x 5 x 53248 = 2080 tiles
    x = si.make_shape("relu_lognormal_chgain", (64, 5, 53248), 96 + k)
    run_case(A, x, k, 64, 5 * 53248, channels=5, tag="2080 tiles per channel")
    run_case(A, x, k, 64, 5 * 53248, channels=5, in_bf16=True, out_bf16=True, tag="1040 tiles per channel bf16")
    # few rows, so few partial maxima per channel: the quantize pass finishes the ranges itself,
    # also for the workgroups that take two tiles (16 x 160 x 6656 = 2080 tiles of 2-3 segments)
    x = si.make_shape("relu_lognormal_chgain", (16, 160, 6656), 99 + k)
    run_case(A, x, k, 16, 160 * 6656, channels=160, tag="2080 tiles, ranges per tile")
    run_case(A, x, k, 16, 160 * 6656, channels=160, in_bf16=True, out_bf16=True, tag="1040 tiles bf16, ranges per tile")
    # the same one segment length off whole tiles (range table from the U1b kernel, ragged tail)
    x = si.make_shape("relu_lognormal_chgain", (64, 5, 53256), 97 + k)
    run_case(A, x, k, 64, 5 * 53256, channels=5, tag="2080 tiles + tail per channel")
    # channels-last: 266240 rows of 64 channels = 2080 tiles, and 5 rows more
    x = si.make_shape("grad", (266245, 64), 98 + k) * (np.arange(1, 65, dtype=np.float32)[None, :])
    x = np.ascontiguousarray(x, dtype=np.float32)
    run_case(A, x[:266240], k, 266240, 64, channels=64, tag="2080 tiles channels-last")
    run_case(A, x, k, 266245, 64, channels=64, tag="2080 tiles channels-last + tail")


@pytest.mark.parametrize("k", [3, 4, 8])
def test_per_channel_generic_geometries(A, k):
    # short aligned segments (vector quantize path, column range pass)
    x = si.make_shape("relu_lognormal_chgain", (6, 10, 12), 50 + k)
    run_case(A, x, k, 6, 120, channels=10, tag="seg12")
    x = si.make_shape("relu_lognormal_chgain", (40, 64, 8, 8), 51 + k)
    run_case(A, x, k, 40, 64 * 64, channels=64, tag="seg64")
    run_case(A, x, k, 40, 64 * 64, channels=64, in_bf16=True, out_bf16=True, tag="seg64-bf16")
    # segments that no 16-byte vector respects: element-wise path
    x = si.make_shape("relu_lognormal_chgain", (9, 11, 7), 52 + k)
    run_case(A, x, k, 9, 77, channels=11, tag="seg7")
    x = si.make_shape("relu_lognormal_chgain", (300, 33, 5), 53 + k)
    run_case(A, x, k, 300, 165, channels=33, in_bf16=True, tag="seg5-bf16")
    # one element per channel (channels-last 2-D tensor)
    x = si.make_shape("grad", (50, 96), 54 + k)
    run_case(A, x, k, 50, 96, channels=96, tag="seg1")
    # channels-last with many rows (several row blocks in the column pass), aligned and not
    x = si.make_shape("grad_outliers", (5000, 256), 55 + k)
    run_case(A, x, k, 5000, 256, channels=256, tag="channels-last 256")
    run_case(A, x, k, 5000, 256, channels=256, in_bf16=True, out_bf16=True, tag="channels-last 256 bf16")
    x = si.make_shape("relu_lognormal", (3001, 30, 11), 56 + k)
    run_case(A, x, k, 3001, 330, channels=30, tag="seg11 unaligned rows")
    x = si.make_shape("student_t3", (37, 1300, 3), 57 + k)
    run_case(A, x, k, 37, 3900, channels=1300, tag="seg3 wide")


@pytest.mark.parametrize("k", KS)
def test_channels_last_one_range_per_element(A, k):
    """Rows of C channels with one element each and a gain per channel spanning six decades: whole
    tiles (vector path, every element of a vector its own range) plus a ragged tail, float32 and
    bfloat16, nearest-even and stochastic; row lengths that no 16-byte vector divides take the plain path."""
    for rows, C in [(700, 64), (301, 136), (1237, 40), (530, 36), (2100, 8)]:
        x = si.make_shape("grad", (rows, C), 70 + k)
        gain = np.float32(10.0) ** np.linspace(-3, 3, C, dtype=np.float32)
        x = np.ascontiguousarray(x * gain[None, :], dtype=np.float32)
        run_case(A, x, k, rows, C, channels=C, tag="channels-last %d" % C)
        run_case(A, x, k, rows, C, channels=C, in_bf16=True, out_bf16=True, tag="channels-last %d bf16" % C)
    run_case(A, x, k, rows, C, channels=C, rounding=1, seed=77, tag="channels-last stochastic")


def test_channels_last_decoder_with_unaligned_header(A):
    """A header that is only 4-byte aligned (the contract's minimum) decodes to the same values."""
    torch = torch_mod()
    rows, C, k = 900, 64, 5
    x = si.make_shape("grad", (rows, C), 91) * (np.arange(1, C + 1, dtype=np.float32)[None, :])
    x = np.ascontiguousarray(x, dtype=np.float32)
    xd, _ = to_dev(x)
    d = A.make_desc(A.UNIFORM, k, rows, C, channels=C)
    header, payload = A.accept_compress(d, xd)
    ref = A.accept_decompress(d, header, payload)
    shifted = torch.empty(header.numel() + 4, dtype=torch.uint8, device=header.device)
    shifted[4:] = header
    got = A.accept_decompress(d, shifted[4:], payload)
    torch.cuda.synchronize()
    assert shifted[4:].data_ptr() % 16 == 4
    oh, op = orc.uniform_compress(x, k, rows, C, C)
    assert out_to_numpy(got).tobytes() == orc.uniform_decompress(oh, op, k, rows, C, C).tobytes()
    assert out_to_numpy(ref).tobytes() == out_to_numpy(got).tobytes()


@pytest.mark.parametrize("k", [2, 4, 7, 8])
def test_stochastic_rounding_bit_exact(A, k):
    x = si.make_shape("grad_outliers", (2, 8192 + 100), 60 + k)
    run_case(A, x, k, 2, 8292, rounding=1, seed=1234567, tag="stoch")
    run_case(A, x, k, 2, 8292, rounding=1, seed=(1 << 63) + 5, tag="stoch-bigseed")
    run_case(A, x, k, 4, 4146, channels=2, rounding=1, seed=9, in_bf16=True, tag="stoch-ch")


def test_decoder_on_oracle_stream(A):
    """Feed the oracle's own header and payload to the GPU decoder."""
    torch = torch_mod()
    for k in KS:
        for N in (5, 64, 8192 * 2 + 50):
            x = si.make_shape("student_t3", (1, N), 70 + k)
            oh, op = orc.uniform_compress(x, k, 1, N)
            d = A.make_desc(A.UNIFORM, k, 1, N)
            xh = A.accept_decompress(d, bytes_to_dev(oh), bytes_to_dev(op.tobytes() + b"\0" * 16)[: op.size])
            torch.cuda.synchronize()
            assert xh.cpu().numpy().tobytes() == orc.uniform_decompress(oh, op, k, 1, N).tobytes()


def test_payload_tail_is_not_overwritten(A):
    """Bytes after ceil(N k / 8) belong to the caller."""
    torch = torch_mod()
    for k, N in [(3, 8192 + 5), (5, 77), (7, 3), (2, 9)]:
        x = si.make_shape("grad", (1, N), 80 + k)
        xd, _ = to_dev(x)
        d = A.make_desc(A.UNIFORM, k, 1, N)
        hb, pb = A.accept_packed_size(d)
        buf = torch.full((pb + 64,), 0xAB, dtype=torch.uint8, device="cuda")
        A.accept_compress(d, xd, payload=buf[:pb])
        torch.cuda.synchronize()
        assert buf[pb:].cpu().numpy().tolist() == [0xAB] * 64
        assert buf[:pb].cpu().numpy().tobytes() == orc.uniform_compress(x, k, 1, N)[1].tobytes()

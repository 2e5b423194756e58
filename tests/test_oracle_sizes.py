"""Oracle pins that come straight from numbers and formulas the paper prints."""
import math

import pytest

from oracle import accept_oracle as orc


def _elems(original_kb):
    # "Original" rows carry the same transport framing as the others (weight version,
    # batch id); the tensor itself is the largest whole number of KB below the print.
    return int(math.floor(original_kb)) * 1024 // 4


def test_size_table_payload_column(golden_rows):
    """Section "Communication Overhead Comparison", size table: every printed size is the
    payload N*k/8 (or N*k, N bytes without the encoder) plus a constant of transport
    framing that does not depend on the tensor: ~1.1 KB forward, ~0.5 KB backward."""
    rows = golden_rows("size_table.txt")
    assert len(rows) == 32
    for tensor, orig, row, k, printed in rows:
        N, k, printed = _elems(float(orig)), int(k), float(printed)
        if row == "comp":
            hdr, pay = orc.packed_size(orc.SCHEME_MBQ, k, 128, N // 128)
            assert pay == N * k // 8
            assert hdr == 4 * (k + 1)
            assert 1.04 <= printed - pay / 1024 <= 1.16, (tensor, row, k)
        elif row == "ucomp":
            hdr, pay = orc.packed_size(orc.SCHEME_UNIFORM, k, 128, N // 128)
            assert pay == N * k // 8 and hdr == 4
            assert 0.44 <= printed - pay / 1024 <= 0.56, (tensor, row, k)
            # the paper's own count, n/(8/k) x w x h x c bytes, is the batch layout's size
            assert orc.packed_size(orc.SCHEME_UNIFORM, k, 128, N // 128, layout=orc.LAYOUT_BATCH)[1] == pay
        elif row == "noenc":
            # every binary base stored in a byte of its own
            _, pay = orc.packed_size(orc.SCHEME_MBQ, k, 128, N // 128, layout=orc.LAYOUT_UNENCODED)
            assert pay == N * k
            assert 0.9 <= printed - pay / 1024 <= 1.2, (tensor, row, k)
        else:
            # every quantized gradient in a byte of its own
            _, pay = orc.packed_size(orc.SCHEME_UNIFORM, k, 128, N // 128, layout=orc.LAYOUT_UNENCODED)
            assert pay == N
            assert 0.0 <= printed - pay / 1024 <= 0.6, (tensor, row, k)


@pytest.mark.parametrize("n,m,k", [(128, 8192, 2), (128, 8192, 4), (5, 33, 3), (8, 1, 4), (9, 7, 1), (1, 1, 8)])
def test_forward_size_formula(n, m, k):
    """Total bits = 32k + ceil(n/8)*m*k*8 + 32 (section "Transmission Data Comparison")."""
    hdr, pay = orc.packed_size(orc.SCHEME_MBQ, k, n, m)
    assert 8 * (hdr + pay) == 32 * k + math.ceil(n / 8) * m * k * 8 + 32
    cf = orc.compression_ratio_forward(n, m, k)
    assert cf == pytest.approx(n * m * 32 / (8 * (hdr + pay)))


@pytest.mark.parametrize("n,m,k", [(128, 8192, 4), (128, 8192, 8), (16, 390912, 3), (3, 35, 5), (1, 1, 2), (1, 7, 7)])
def test_backward_size_formula(n, m, k):
    """Total bits = n/(8/k)*w*h*c*8 + 32 for k in {4, 8}; ceil(N k / 8) bytes in general."""
    hdr, pay = orc.packed_size(orc.SCHEME_UNIFORM, k, n, m)
    assert hdr == 4
    assert pay == math.ceil(n * m * k / 8)
    if (n * m * k) % 8 == 0 and k in (4, 8):
        assert 8 * (hdr + pay) == (n * m) // (8 // k) * 8 + 32
    assert orc.packed_size(orc.SCHEME_UNIFORM, k, n, m * 6, channels=6)[0] == 24


def test_ratio_is_about_32_over_k():
    for k in (2, 3, 4):
        assert orc.compression_ratio_forward(128, 8192, k) == pytest.approx(32 / k, rel=1e-3)


def test_beta_printed_formula(golden_kv):
    kv = golden_kv("worked_examples.txt")
    assert orc.beta(0) == pytest.approx(0.1)
    assert orc.beta(1) == pytest.approx(2 / 11)
    assert orc.beta(79) == pytest.approx(80 / 89)
    assert orc.beta(80) == float(kv["beta_cap"])
    assert orc.beta(81) == float(kv["beta_cap"]) and orc.beta(10 ** 6) == 0.9
    assert all(orc.beta(t) <= orc.beta(t + 1) for t in range(100))


def _average(direction, changes, epochs):
    tot = 0
    for e in range(epochs):
        tot += orc.bits_schedule(direction, sum(1 for c in changes if e >= c))
    return tot / epochs


def test_bit_width_schedule_printed_averages(golden_kv):
    """Section "Model Performance Evaluation": average widths 2.48, 2.9, 7.2, 6.4."""
    kv = golden_kv("worked_examples.txt")
    E = int(kv["epochs"])
    for model in ("mobilenetv2", "simplecnn"):
        fc = [int(v) for v in kv[f"forward_changes_{model}"].split()]
        bc = [int(v) for v in kv[f"backward_changes_{model}"].split()]
        assert round(_average(0, fc, E), 2) == pytest.approx(float(kv[f"forward_average_{model}"]), abs=0.0051)
        assert _average(1, bc, E) == pytest.approx(float(kv[f"backward_average_{model}"]))
    assert [orc.bits_schedule(0, c) for c in range(5)] == [2, 3, 4, 4, 4]
    assert [orc.bits_schedule(1, c) for c in range(3)] == [8, 4, 4]

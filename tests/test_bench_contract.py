"""Host-side checks of bench.py: byte accounting against the oracle's sizes, and the one-GPU rule."""
import subprocess
import sys
import os

import pytest

import bench
from oracle import accept_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("k", [2, 3, 4, 5, 6, 7, 8])
def test_algorithmic_bytes_follow_the_packed_sizes(k):
    n, m = 64, 802816
    N = n * m
    hu, pu = orc.packed_size(orc.SCHEME_UNIFORM, k, n, m)
    assert bench.alg_bytes("range", N, n, m, k) == 4 * N
    assert bench.alg_bytes("quantize_pack", N, n, m, k) == 4 * N + pu + hu
    assert bench.alg_bytes("unpack_dequant", N, n, m, k) == pu + hu + 4 * N
    assert bench.alg_bytes("unpack_dequant", N, n, m, k, 2, 2) == pu + hu + 2 * N
    hm, pm = orc.packed_size(orc.SCHEME_MBQ, k, n, m)
    assert bench.alg_bytes("mbq_encode", N, n, m, k) == 4 * N + pm
    assert bench.alg_bytes("mbq_decode", N, n, m, k) == pm + hm + 4 * N


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       cwd=ROOT, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""

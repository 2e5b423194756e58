"""The library only enqueues kernels on the caller's stream (no allocation, no memset, no
synchronisation), so a round trip can be captured in a HIP graph.  Every replay, with eager
work and synchronisations in between, must reproduce the eager result bit for bit."""
import numpy as np
import pytest

import synthetic_inputs as si
from oracle import accept_oracle as orc

from gpu_util import dev_bytes, torch_mod

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def A():
    torch = torch_mod()
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2311_05827_amd as pkg
    return pkg


@pytest.mark.parametrize("scheme", ["uniform", "uniform_per_channel", "mbq"])
def test_round_trip_under_graph_replay(A, scheme):
    torch = torch_mod()
    n, C, inner = 16, 8, 1024
    m = C * inner
    xs = [si.make_shape("relu_lognormal_chgain", (n, C, inner), 900 + i) for i in range(3)]
    k = 3 if scheme == "mbq" else 5
    if scheme == "mbq":
        d = A.make_desc(A.MBQ, k, n, m, t=2)
        alpha_np, _ = orc.mbq_residue_init(xs[0], k)
        alpha = torch.from_numpy(alpha_np).cuda()
    else:
        d = A.make_desc(A.UNIFORM, k, n, m, channels=C if scheme == "uniform_per_channel" else 0)
        alpha = None
    x = torch.empty(n * m, dtype=torch.float32, device="cuda")
    header, payload, ws = A.alloc_outputs(d, x.device)
    out = torch.empty(n * m, dtype=torch.float32, device="cuda")

    def round_trip():
        A.accept_compress(d, x, alpha_prev=alpha, header=header, payload=payload, workspace=ws)
        A.accept_decompress(d, header, payload, out=out)

    # eager references for three different inputs
    eager = []
    for xi in xs:
        x.copy_(torch.from_numpy(xi.reshape(-1)))
        round_trip()
        torch.cuda.synchronize()
        eager.append((dev_bytes(header), dev_bytes(payload), dev_bytes(out)))
    # capture on a side stream (the binding launches on the current stream)
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        round_trip()  # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            round_trip()
    torch.cuda.synchronize()
    for rep in range(2):
        for i, xi in enumerate(xs):
            x.copy_(torch.from_numpy(xi.reshape(-1)))
            header.zero_(); payload.zero_(); out.zero_()      # eager work between replays
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            got = (dev_bytes(header), dev_bytes(payload), dev_bytes(out))
            assert got[1] == eager[i][1], "payload differs on replay %d input %d" % (rep, i)
            assert got[0] == eager[i][0] and got[2] == eager[i][2]
    # and the eager result itself is the oracle's
    if scheme != "mbq":
        oh, op = orc.uniform_compress(xs[2], k, n, m, C if scheme == "uniform_per_channel" else 0)
        assert eager[2][0] == oh and eager[2][1] == op.tobytes()

"""The training-loop glue: alpha / t carried across batches, bit-width controllers, and the
straight-through estimator with a compressed backward pass, each checked against the oracle."""
import numpy as np
import pytest

import synthetic_inputs as si
from oracle import accept_oracle as orc

from gpu_util import dev_bytes, first_mismatch, torch_mod

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mods():
    torch = torch_mod()
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2311_05827_amd as A
    from paper_2311_05827_amd import boundary as Bd
    return A, Bd


def test_forward_chain_with_width_changes(mods):
    A, Bd = mods
    torch = torch_mod()
    n, m = 16, 2052
    fwd = Bd.ForwardCompressor(n, m)
    widths = []
    alpha_prev = None
    for step in range(6):
        if step == 2 or step == 4:
            fwd.controller.on_lr_change()      # 2 -> 3 -> 4
        k = fwd.controller.bits
        widths.append(k)
        x = si.make_shape("relu_normal", (n, m), 700 + step)
        xd = torch.from_numpy(x.reshape(-1)).cuda()
        fresh = fwd.alpha is None or fwd._k != k
        t = fwd.t
        d, header, payload = fwd.compress(xd)
        torch.cuda.synchronize()
        gh = np.frombuffer(dev_bytes(header), dtype="<f4")
        if fresh:
            # batch 0 (and the first batch after a width change): the residue method's own B^0, alpha^0
            oh, _ = orc.mbq_compress_first(x, k, n, m)
            op = orc.mbq_pack(orc.mbq_residue_signs(x, gh[:k]), k, n, m)  # B^0 for the GPU's alpha^0 bits
        else:
            oh, op = orc.mbq_compress(x, k, n, m, alpha_prev, t)
        assert first_mismatch(dev_bytes(payload), op.tobytes()) is None
        ohf = np.frombuffer(oh, dtype="<f4")
        assert np.all(np.abs(gh - ohf) <= 1e-6 * np.abs(ohf[:k]).sum())
        assert fwd.alpha.cpu().numpy().tobytes() == gh[:k].tobytes()
        alpha_prev = gh[:k].copy()              # the next batch starts from the GPU's alpha
        assert fwd.transmitted_bytes() == 4 * (k + 1) + ((n + 7) // 8) * m * k
    assert widths == [2, 2, 3, 3, 4, 4]
    fwd.start_epoch()
    assert fwd.t == 0 and fwd.alpha is None


def test_backward_controller_and_sizes(mods):
    A, Bd = mods
    bwd = Bd.BackwardCompressor(8, 1024)
    assert bwd.controller.bits == 8 and bwd.transmitted_bytes() == 4 + 8 * 1024
    bwd.controller.on_lr_change()
    assert bwd.controller.bits == 4 and bwd.transmitted_bytes() == 4 + 8 * 1024 // 2
    bwd.controller.on_lr_change()
    assert bwd.controller.bits == 4


@pytest.mark.parametrize("compressed_backward", [False, True])
def test_straight_through_estimator(mods, compressed_backward):
    A, Bd = mods
    torch = torch_mod()
    n, m = 8, 4100
    x_np = si.make_shape("relu_lognormal", (n, m), 810)
    w_np = si.make_shape("grad", (n, m), 811)
    x = torch.from_numpy(x_np).cuda().requires_grad_(True)
    w = torch.from_numpy(w_np).cuda()
    fwd = Bd.ForwardCompressor(n, m)
    bwd = Bd.BackwardCompressor(n, m, stochastic=True, seed=77) if compressed_backward else None
    y = Bd.boundary(x, fwd, bwd)
    (y * w).sum().backward()
    torch.cuda.synchronize()
    # forward value: batch 0, i.e. the oracle's decompress(compress_first(x))
    k = 2
    oh, op = orc.mbq_compress_first(x_np, k, n, m)
    ref = orc.mbq_decompress(oh, op, k, n, m).reshape(n, m)
    scale = float(np.abs(np.frombuffer(oh, dtype="<f4")[:k]).sum())
    assert np.all(np.abs(y.detach().cpu().numpy() - ref) <= 1e-6 * scale)
    # gradient: identity through the quantizer; then the link's own round trip if compressed
    g = x.grad.cpu().numpy()
    if not compressed_backward:
        assert g.tobytes() == w_np.tobytes()
    else:
        gh, gp = orc.uniform_compress(w_np, 8, n, m, rounding=1, seed=77)
        assert g.reshape(-1).tobytes() == orc.uniform_decompress(gh, gp, 8, n, m).tobytes()
        assert bwd.calls == 1

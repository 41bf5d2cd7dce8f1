"""Tensors of 2 GiB and more: the kernels that address a tensor through 32-bit byte
offsets (Winograd, the pointwise streaming kernels) must step aside for the general
kernels, which index elements.  One 3x3 layer and one 1x1 layer whose input is just
above 2^31 bytes, checked on sampled outputs against the oracle's element-by-element
functions."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_1606_04884_amd import binding as B          # noqa: E402
import oracle                                          # noqa: E402
from gpu_util import TOL_IGEMM                         # noqa: E402

CASES = [
    (2, 64, 2050, 2050, 8, 3, 3, 1, 1, 1, 1),      # x: 2.15e9 bytes
    (2, 66, 2048, 2048, 8, 1, 1, 1, 1, 0, 0),      # x: 2.21e9 bytes
]


@pytest.mark.parametrize("geom", CASES, ids=["x".join(map(str, g[:7])) for g in CASES])
def test_tensors_beyond_2gib(geom):
    N, C, H, W, K, R, S = geom[:7]
    assert N * C * H * W * 4 >= 2 ** 31
    print("geom", geom, flush=True)
    for op in (B.OP_FWD, B.OP_BWD_DATA, B.OP_BWD_WEIGHT):
        assert B.conv2d_pick_algo(geom, op) == B.ALGO_IGEMM
    assert B.conv2d_workspace_bytes(geom, B.OP_FWD, B.ALGO_WINOGRAD) == 0
    P, Q = B.conv2d_output_dims(geom)
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(31000 + R)
    x = torch.randn((N, C, H, W), device=dev, generator=gen)
    w = torch.randn((K, C, R, S), device=dev, generator=gen) * (2.0 / (C * R * S)) ** 0.5
    b = (torch.rand((K,), device=dev, generator=gen) - 0.5) * 0.2
    dy = torch.randn((N, K, P, Q), device=dev, generator=gen)
    y = torch.full_like(dy, float("nan"))
    dx = torch.full_like(x, float("nan"))
    dw = torch.full_like(w, float("nan"))
    db = torch.full_like(b, float("nan"))
    B.conv2d_fwd(geom, x, w, b, y)
    B.conv2d_bwd_data(geom, dy, w, dx)
    B.conv2d_bwd_weight(geom, x, dy, dw, db)
    torch.cuda.synchronize()
    assert not torch.isnan(y).any() and not torch.isnan(dx).any()
    hx, hw, hb, hdy = (t.cpu().numpy() for t in (x, w, b, dy))
    rng = np.random.default_rng(31)

    def check(name, got_t, n_samples, fn, first_and_last=True):
        idx = rng.integers(0, got_t.numel(), size=n_samples)
        if first_and_last:                    # both ends of the index range
            idx[0], idx[1] = 0, got_t.numel() - 1
        ref = fn(idx)
        got = got_t.reshape(-1)[torch.from_numpy(idx).to(dev)].cpu().numpy().astype(np.float64)
        scale = float(np.abs(ref).max())
        err = float(np.abs(got - ref).max())
        assert err <= TOL_IGEMM * scale, "%s: err %.3e vs %.3e*%.3e" % (name, err, TOL_IGEMM, scale)

    check("y", y, 20000, lambda i: oracle.fwd_at(geom, hx, hw, hb, i))
    check("dx", dx, 20000, lambda i: oracle.bwd_data_at(geom, hdy, hw, i))
    check("dw", dw, 96, lambda i: oracle.bwd_weight_at(geom, hx, hdy, i))
    ref_db = hdy.astype(np.float64).sum(axis=(0, 2, 3))
    assert np.abs(db.cpu().numpy().astype(np.float64) - ref_db).max() <= TOL_IGEMM * np.abs(ref_db).max()

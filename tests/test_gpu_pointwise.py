"""Parity of the pointwise (1x1, stride 1, unpadded) kernels with the CPU oracle.

The shapes walk through the cases the streaming kernels distinguish: the number of
32-row tiles of the small operand (1, 2, 3, 4, 6, 8), depths that are not a multiple
of the 8-channel load group or of the ring of groups in flight, maps whose pixel count
is not a multiple of anything, pixel tiles that straddle images, filters that cannot be
fetched as 16-byte vectors, and for backward-weight every accumulator-block shape, the
pixel phases, ragged last steps and the fall-backs (H*W not a multiple of 4, unaligned
tensors, too many filters or channels).
"""
import numpy as np
import pytest

import oracle
from paper_1606_04884_amd import binding as B
from paper_1606_04884_amd import synth
from gpu_util import TOL_IGEMM, gpu_layer, max_err_ratio, oracle_layer, random_layer

pytestmark = pytest.mark.gpu


def PW(N, C, H, W, K):
    return (N, C, H, W, K, 1, 1, 1, 1, 0, 0)


POINTWISE_SHAPES = [
    PW(3, 16, 6, 6, 8),          # one row tile both ways, two depth groups
    PW(2, 40, 7, 9, 50),         # odd number of depth groups (5 / 7), 63 pixels per image
    PW(2, 72, 8, 8, 96),         # 3 row tiles, 9 depth groups: ring wraps with a remainder
    PW(2, 100, 4, 8, 128),       # 4 row tiles forward and backward, 13 / 16 groups
    PW(2, 136, 5, 4, 190),       # 6 and 5->6 row tiles, depth not a multiple of 4 (scalar filter fetch)
    PW(2, 60, 6, 6, 250),        # 8 row tiles forward, last depth group half full
    PW(5, 21, 3, 5, 33),         # everything ragged, tiles straddle images (15 pixels each)
    PW(2, 64, 8, 8, 300),        # forward too tall for the streaming kernel (gather kernel's 1x1 path)
    PW(2, 300, 8, 8, 24),        # backward-data too tall; backward-weight beyond 256 channels
    PW(7, 24, 56, 56, 20),       # enough pixels for 32+ splits (wide split reduction), phases
    PW(4, 192, 28, 28, 64),      # inception 3a 1x1 at a small batch
    PW(3, 48, 4, 4, 16),         # H*W = 16: a single pixel phase
    PW(2, 32, 2, 6, 144),        # H*W = 12 < 16 and 144 filters: backward-weight falls back
    PW(3, 96, 5, 5, 40),         # H*W = 25, not a multiple of 4: backward-weight falls back
    PW(2, 256, 4, 8, 128),       # widest streamed backward-weight: 8 x 2 tiles in 8 column groups
    PW(3, 130, 4, 6, 100),       # 9 channel tiles in 4 groups of 3 (ragged), 7 filter tiles -> 8
    PW(2, 80, 6, 6, 20),         # 5 channel tiles in 2 groups of 3, 2 filter tiles
    # more 32-pixel tiles (2352) than waves of a full grid (2048): waves take a second tile,
    # with 12 depth groups (ring of 8 + 4) one way and a single group the other way
    PW(24, 96, 56, 56, 8),
    PW(24, 8, 56, 56, 96),
    # a single channel / a single filter: both strides of the small operand are 1, so its
    # contiguous axis cannot be told from them
    PW(2, 1, 17, 21, 96),
    PW(4, 1, 4, 12, 1),
    PW(3, 40, 5, 8, 1),
]


@pytest.mark.parametrize("geom", POINTWISE_SHAPES, ids=["x".join(map(str, g[:5])) for g in POINTWISE_SHAPES])
def test_pointwise_parity(geom):
    x, w, b, dy = random_layer(geom, 7000 + sum(geom))
    print("geom", geom, flush=True)
    got = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_AUTO)
    ref = oracle_layer(geom, x, w, b, dy)
    for name in ("y", "dx", "dw", "db"):
        assert np.isfinite(got[name]).all(), name
        r = max_err_ratio(got[name], ref[name])
        assert r <= TOL_IGEMM, "%s: max err ratio %.3e" % (name, r)


def test_pointwise_scale_accumulate_and_no_bias():
    geom = PW(3, 64, 8, 8, 48)
    x, w, b, dy = random_layer(geom, 7101)
    dw0 = synth.normal((48, 64, 1, 1), 7102)
    db0 = synth.normal((48,), 7103)
    got = gpu_layer(geom, x, w, None, dy, scale=0.25, dw0=dw0, db0=db0)
    ref_y = oracle.fwd(geom, x, w, None)
    ref_dw, ref_db = oracle.bwd_weight(geom, x, dy, 0.25)
    assert max_err_ratio(got["y"], ref_y) <= TOL_IGEMM
    assert max_err_ratio(got["dw"], ref_dw + dw0.astype(np.float64)) <= TOL_IGEMM
    assert max_err_ratio(got["db"], ref_db + db0.astype(np.float64)) <= TOL_IGEMM


def test_pointwise_unaligned_tensors():
    """Views that start 4 bytes into an allocation: the filters are fetched element by
    element and backward-weight takes the general kernel; results are unchanged."""
    import torch
    geom = PW(2, 32, 4, 8, 24)
    N, C, H, W, K = geom[:5]
    x, w, b, dy = random_layer(geom, 7201)
    dev = torch.device("cuda:0")

    def shifted(a):
        buf = torch.empty(a.size + 1, device=dev)
        v = buf[1:].view(*a.shape)
        v.copy_(torch.from_numpy(a))
        return v

    tx, tw, tdy = shifted(x), shifted(w), shifted(dy)
    assert tx.data_ptr() % 16 != 0 and tw.data_ptr() % 16 != 0
    tb = torch.from_numpy(b).to(dev)
    y = shifted(np.full((N, K, H, W), np.nan, np.float32))
    dx = shifted(np.full((N, C, H, W), np.nan, np.float32))
    dw = torch.full((K, C, 1, 1), float("nan"), device=dev)
    db = torch.full((K,), float("nan"), device=dev)
    B.conv2d_fwd(geom, tx, tw, tb, y)
    B.conv2d_bwd_data(geom, tdy, tw, dx)
    B.conv2d_bwd_weight(geom, tx, tdy, dw, db)
    torch.cuda.synchronize()
    ref = oracle_layer(geom, x, w, b, dy)
    assert max_err_ratio(y.cpu().numpy(), ref["y"]) <= TOL_IGEMM
    assert max_err_ratio(dx.cpu().numpy(), ref["dx"]) <= TOL_IGEMM
    assert max_err_ratio(dw.cpu().numpy(), ref["dw"]) <= TOL_IGEMM
    assert max_err_ratio(db.cpu().numpy(), ref["db"]) <= TOL_IGEMM


def test_pointwise_identity_is_exact():
    """w = identity: y = x + bias with a single rounding, dx = dy exactly."""
    geom = PW(2, 40, 5, 7, 40)
    x, _, b, dy = random_layer(geom, 7301)
    w = np.eye(40, dtype=np.float32).reshape(40, 40, 1, 1)
    got = gpu_layer(geom, x, w, b, dy, passes=("fwd", "bwd_data"))
    assert np.array_equal(got["y"], x + b.reshape(1, -1, 1, 1))
    assert np.array_equal(got["dx"], dy)


def test_pointwise_deterministic():
    geom = PW(6, 48, 12, 12, 36)
    x, w, b, dy = random_layer(geom, 7401)
    a = gpu_layer(geom, x, w, b, dy)
    c = gpu_layer(geom, x, w, b, dy)
    for name in ("y", "dx", "dw", "db"):
        assert np.array_equal(a[name], c[name]), name


def test_pointwise_full_batch_is_stable_over_launches():
    """The inception 1x1 layer at its full batch, many launches: every launch gives the same
    bits and the oracle's values on sampled elements.  (16-byte stores whose data registers
    are reused right after the store once wrote stale first elements in a few tiles per launch,
    a different few each time.)"""
    import torch
    geom = PW(128, 192, 28, 28, 64)
    N, C, H, W, K = geom[:5]
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(7501)
    x = torch.randn((N, C, H, W), device=dev, generator=gen)
    w = torch.randn((K, C, 1, 1), device=dev, generator=gen) * (2.0 / C) ** 0.5
    b = torch.rand((K,), device=dev, generator=gen) - 0.5
    y0 = torch.full((N, K, H, W), float("nan"), device=dev)
    B.conv2d_fwd(geom, x, w, b, y0)
    idx = np.random.default_rng(7502).integers(0, y0.numel(), size=20000)
    ref = oracle.fwd_at(geom, x.cpu().numpy(), w.cpu().numpy(), b.cpu().numpy(), idx)
    got = y0.reshape(-1)[torch.from_numpy(idx).to(dev)].cpu().numpy().astype(np.float64)
    assert np.abs(got - ref).max() <= TOL_IGEMM * np.abs(ref).max()
    y = torch.empty_like(y0)
    for _ in range(30):
        y.fill_(float("nan"))
        B.conv2d_fwd(geom, x, w, b, y)
        assert torch.equal(y, y0)

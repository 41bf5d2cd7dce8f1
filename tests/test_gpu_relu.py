"""conv2d_fwd_relu against the oracle on every forward route: the gather kernel, the
streaming kernels (pointwise with 16-byte and with dword stores, taps form with both ring
sizes), the Winograd kernels (tile pairs, ragged chunk, general kernel, sub-filters of a
5x5, tiles cut by the persistent schedule and finished by the fix-up kernel) and the
strided layer taken through the rearrangement.  Also: where the plain forward result is
positive the two entry points agree bit for bit, elsewhere the fused one stores 0."""
import numpy as np
import pytest

import oracle
from paper_1606_04884_amd import binding as B
from gpu_util import TOL_IGEMM, TOL_WINOGRAD, max_err_ratio, random_layer

pytestmark = pytest.mark.gpu

RELU_SHAPES = [
    # (geom, algo)
    ((2, 3, 16, 16, 8, 3, 3, 1, 1, 1, 1), B.ALGO_AUTO),          # taps, ring of 4
    ((2, 3, 35, 35, 96, 11, 11, 4, 4, 2, 2), B.ALGO_AUTO),       # taps, ring of 8, dword stores
    ((3, 16, 12, 12, 32, 5, 5, 1, 1, 2, 2), B.ALGO_IGEMM),       # taps, 16-byte stores
    ((2, 40, 7, 9, 50, 1, 1, 1, 1, 0, 0), B.ALGO_AUTO),          # pointwise, dword stores
    ((4, 192, 28, 28, 64, 1, 1, 1, 1, 0, 0), B.ALGO_AUTO),       # pointwise, 16-byte stores
    ((2, 64, 8, 8, 300, 1, 1, 1, 1, 0, 0), B.ALGO_AUTO),         # 1x1 through the gather kernel
    ((2, 20, 9, 11, 24, 3, 3, 2, 2, 1, 1), B.ALGO_AUTO),         # gather kernel, strided
    ((2, 24, 13, 10, 40, 4, 2, 1, 1, 1, 0), B.ALGO_IGEMM),       # gather kernel, odd filter
    ((2, 64, 28, 28, 64, 3, 3, 1, 1, 1, 1), B.ALGO_WINOGRAD),    # tile-pair kernel
    ((2, 6, 24, 24, 32, 3, 3, 1, 1, 1, 1), B.ALGO_WINOGRAD),     # tile pairs, ragged chunk
    ((3, 32, 13, 13, 48, 3, 3, 1, 1, 1, 1), B.ALGO_WINOGRAD),    # general Winograd kernel
    ((2, 32, 27, 27, 40, 5, 5, 1, 1, 2, 2), B.ALGO_WINOGRAD),    # four 3x3 sub-filters
    ((9, 128, 28, 28, 128, 3, 3, 1, 1, 1, 1), B.ALGO_WINOGRAD),  # more tile blocks than fit a round: cut tiles
    ((2, 3, 35, 35, 64, 11, 11, 4, 4, 2, 2), B.ALGO_WINOGRAD),   # strided layer through the rearrangement
]


@pytest.mark.parametrize("geom,algo", RELU_SHAPES, ids=["x".join(map(str, g)) + "a%d" % a for g, a in RELU_SHAPES])
def test_fwd_relu_parity(geom, algo):
    import torch
    x, w, b, _ = random_layer(geom, 15000 + sum(geom))
    print("geom", geom, "algo", algo, flush=True)
    dev = torch.device("cuda:0")
    N, C, H, W, K = geom[:5]
    P, Q = B.conv2d_output_dims(geom)
    tx, tw, tb = (torch.from_numpy(a).to(dev) for a in (x, w, b))
    y = torch.full((N, K, P, Q), float("nan"), device=dev)
    yr = torch.full((N, K, P, Q), float("nan"), device=dev)
    B.conv2d_fwd(geom, tx, tw, tb, y, algo=algo)
    B.conv2d_fwd_relu(geom, tx, tw, tb, yr, algo=algo)
    torch.cuda.synchronize()
    got, plain = yr.cpu().numpy(), y.cpu().numpy()
    ref = oracle.fwd_relu(geom, x, w, b)
    used = B.conv2d_pick_algo(geom, B.OP_FWD) if algo == B.ALGO_AUTO else algo
    tol = TOL_WINOGRAD if used == B.ALGO_WINOGRAD else TOL_IGEMM
    assert np.isfinite(got).all()
    # the bar is relative to max|ref| of the unrectified tensor's scale as well: same sums
    assert max_err_ratio(got, ref) <= tol
    assert np.array_equal(got, np.maximum(plain, 0.0))
    assert (got == 0).any() and (got > 0).any()


def test_fwd_relu_without_bias_and_argument_checks():
    import torch
    geom = (2, 16, 10, 10, 24, 3, 3, 1, 1, 1, 1)
    x, w, _, _ = random_layer(geom, 15101)
    dev = torch.device("cuda:0")
    y = torch.full((2, 24, 10, 10), float("nan"), device=dev)
    B.conv2d_fwd_relu(geom, torch.from_numpy(x).to(dev), torch.from_numpy(w).to(dev), None, y)
    torch.cuda.synchronize()
    assert max_err_ratio(y.cpu().numpy(), oracle.fwd_relu(geom, x, w, None)) <= TOL_IGEMM
    with pytest.raises(B.Conv2dError):
        B.conv2d_fwd_relu((2, 16, 9, 9, 24, 9, 9, 1, 1, 0, 0), torch.zeros((2, 16, 9, 9), device=dev),
                          torch.zeros((24, 16, 9, 9), device=dev), None, torch.zeros((2, 24, 1, 1), device=dev),
                          algo=B.ALGO_WINOGRAD)


POOL_SHAPES = [
    (2, 64, 28, 28, 64, 3, 3, 1, 1, 1, 1),       # tile-pair kernel
    (2, 3, 24, 24, 32, 3, 3, 1, 1, 1, 1),        # tile pairs, ragged chunk (first layer)
    (3, 32, 14, 14, 48, 3, 3, 1, 1, 1, 1),       # general Winograd kernel (7 tiles per row)
    (2, 32, 26, 26, 40, 5, 5, 1, 1, 2, 2),       # four 3x3 sub-filters
    (2, 16, 10, 12, 20, 3, 3, 1, 1, 0, 0),       # unpadded: 8 x 10 output
    (9, 128, 28, 28, 128, 3, 3, 1, 1, 1, 1),     # tiles cut by the persistent schedule: fix-up kernel pools too
]


@pytest.mark.parametrize("geom", POOL_SHAPES, ids=["x".join(map(str, g)) for g in POOL_SHAPES])
def test_fwd_relu_pool2_parity(geom):
    import torch
    x, w, b, _ = random_layer(geom, 15200 + sum(geom))
    print("geom", geom, flush=True)
    dev = torch.device("cuda:0")
    N, C, H, W, K = geom[:5]
    P, Q = B.conv2d_output_dims(geom)
    tx, tw, tb = (torch.from_numpy(a).to(dev) for a in (x, w, b))
    yp = torch.full((N, K, P // 2, Q // 2), float("nan"), device=dev)
    yr = torch.full((N, K, P, Q), float("nan"), device=dev)
    B.conv2d_fwd_relu_pool2(geom, tx, tw, tb, yp)
    B.conv2d_fwd_relu(geom, tx, tw, tb, yr, algo=B.ALGO_WINOGRAD)
    torch.cuda.synchronize()
    got = yp.cpu().numpy()
    assert np.isfinite(got).all()
    assert max_err_ratio(got, oracle.fwd_relu_pool2(geom, x, w, b)) <= TOL_WINOGRAD
    # the same sums as the unpooled entry point: pooling its output gives the same bits
    full = yr.cpu().numpy()
    assert np.array_equal(got, full.reshape(N, K, P // 2, 2, Q // 2, 2).max(axis=(3, 5)))


def test_fwd_relu_pool2_refusals():
    import torch
    dev = torch.device("cuda:0")
    z = lambda *s: torch.zeros(s, device=dev)
    with pytest.raises(B.Conv2dError):      # odd map
        B.conv2d_fwd_relu_pool2((1, 8, 13, 13, 8, 3, 3, 1, 1, 1, 1), z(1, 8, 13, 13), z(8, 8, 3, 3), None, z(1, 8, 6, 6))
    with pytest.raises(B.Conv2dError):      # not a layer the Winograd path takes
        B.conv2d_fwd_relu_pool2((1, 8, 12, 12, 8, 1, 1, 1, 1, 0, 0), z(1, 8, 12, 12), z(8, 8, 1, 1), None, z(1, 8, 6, 6))

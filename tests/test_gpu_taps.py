"""Parity of the taps form of the streaming kernel (forward pass, and stride-1 backward-data
pass, of layers whose whole filter bank fits in LDS: first layers, small 5x5 layers) with the
CPU oracle.

The shapes cover every row-tile count (1..4), strides that differ by axis, padding wider
than one tap (whole window rows and columns outside the image), images smaller than the
filter, 15-tap-wide filters (the last bit of the row / column sets), depths that are not a
multiple of the 8-entry load group, more pixel tiles than waves in a full grid, and tiles
that straddle rows and images."""
import numpy as np
import pytest

import oracle
from paper_1606_04884_amd import binding as B
from gpu_util import TOL_IGEMM, gpu_layer, max_err_ratio, random_layer

pytestmark = pytest.mark.gpu

TAP_SHAPES = [
    (2, 3, 20, 20, 64, 3, 3, 1, 1, 1, 1),        # VGG-like first layer, 27 taps
    (2, 3, 35, 35, 96, 11, 11, 4, 4, 2, 2),      # AlexNet-like first layer, 363 taps, 3 row tiles
    (2, 3, 39, 39, 96, 11, 11, 4, 4, 0, 0),      # Overfeat-like first layer, no padding
    (3, 16, 12, 12, 32, 5, 5, 1, 1, 2, 2),       # inception 5x5: 400 taps, one row tile
    (3, 5, 9, 11, 20, 3, 5, 2, 1, 1, 3),         # strides and pads differ by axis
    (2, 4, 7, 7, 128, 4, 4, 1, 1, 0, 0),         # 4 row tiles, even filter, unpadded
    (1, 1, 6, 6, 3, 15, 15, 1, 1, 7, 7),         # 15 x 15 taps: every bit of the sets
    (1, 1, 6, 6, 3, 16, 16, 1, 1, 8, 8),         # one more: the gather kernel takes over
    (2, 2, 3, 3, 4, 5, 5, 1, 1, 2, 2),           # image smaller than the filter
    (2, 3, 8, 8, 8, 3, 3, 1, 1, 2, 2),           # padding 2 under a 3x3: windows with one valid row
    (24, 3, 56, 56, 8, 3, 3, 1, 1, 1, 1),        # 2352 pixel tiles: waves take a second tile
    (5, 7, 5, 3, 33, 2, 3, 1, 2, 1, 0),          # everything ragged
]


@pytest.mark.parametrize("geom", TAP_SHAPES, ids=["x".join(map(str, g)) for g in TAP_SHAPES])
def test_tap_stream_forward_parity(geom):
    x, w, b, dy = random_layer(geom, 9100 + sum(geom))
    print("geom", geom, flush=True)
    got = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_IGEMM, passes=("fwd",))
    ref = oracle.fwd(geom, x, w, b)
    assert np.isfinite(got["y"]).all()
    r = max_err_ratio(got["y"], ref)
    assert r <= TOL_IGEMM, "y: max err ratio %.3e" % r


def test_tap_stream_no_bias_and_single_tap_filter():
    """No bias; a filter that is zero except one tap shifts the image: exact."""
    geom = (2, 3, 10, 12, 3, 3, 3, 1, 1, 1, 1)
    x, _, _, dy = random_layer(geom, 9201)
    w = np.zeros((3, 3, 3, 3), np.float32)
    for k in range(3):
        w[k, k, 0, 2] = 1.0            # y[n,k,p,q] = x[n,k,p-1,q+1]
    got = gpu_layer(geom, x, w, None, dy, algo=B.ALGO_IGEMM, passes=("fwd",))
    want = np.zeros_like(x)
    want[:, :, 1:, :-1] = x[:, :, :-1, 1:]
    assert np.array_equal(got["y"], want)


# backward-data in the taps form: stride 1, at least 12 channels (rows), K*R*S taps over dy
TAP_BWD_SHAPES = [
    (3, 16, 12, 12, 32, 5, 5, 1, 1, 2, 2),       # inception 5x5: 800 taps, one row tile
    (2, 12, 9, 11, 7, 3, 5, 1, 1, 1, 0),         # pads differ by axis, window partly left of dy
    (2, 40, 8, 8, 5, 4, 4, 1, 1, 0, 0),          # unpadded: dx border pixels see one tap
    (2, 33, 6, 7, 6, 3, 3, 1, 1, 2, 2),          # padding 2: P, Q larger than H, W; 2 row tiles, ragged
    (2, 128, 5, 5, 3, 2, 2, 1, 1, 1, 1),         # 4 row tiles
    (9, 16, 56, 56, 4, 5, 5, 1, 1, 2, 2),        # 882 pixel tiles of full-size rows
    (40, 16, 56, 56, 2, 3, 3, 1, 1, 1, 1),       # 3920 pixel tiles: waves take a second tile
]


@pytest.mark.parametrize("geom", TAP_BWD_SHAPES, ids=["x".join(map(str, g)) for g in TAP_BWD_SHAPES])
def test_tap_stream_backward_data_parity(geom):
    x, w, b, dy = random_layer(geom, 9300 + sum(geom))
    print("geom", geom, flush=True)
    got = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_IGEMM, passes=("bwd_data",))
    ref = oracle.bwd_data(geom, dy, w)
    assert np.isfinite(got["dx"]).all()
    r = max_err_ratio(got["dx"], ref)
    assert r <= TOL_IGEMM, "dx: max err ratio %.3e" % r


def test_tap_stream_backward_data_is_the_default_for_small_5x5():
    assert B.conv2d_pick_algo((128, 16, 28, 28, 32, 5, 5, 1, 1, 2, 2), B.OP_BWD_DATA) == B.ALGO_IGEMM
    # a single-tap filter: dx is dy shifted the other way, exactly
    geom = (2, 12, 6, 8, 12, 3, 3, 1, 1, 1, 1)
    x, _, _, dy = random_layer(geom, 9401)
    w = np.zeros((12, 12, 3, 3), np.float32)
    for k in range(12):
        w[k, k, 0, 2] = 1.0            # y[n,k,p,q] = x[n,k,p-1,q+1]  =>  dx[n,c,h,u] = dy[n,c,h+1,u-1]
    got = gpu_layer(geom, x, w, None, dy, algo=B.ALGO_IGEMM, passes=("bwd_data",))
    want = np.zeros_like(dy)
    want[:, :, :-1, 1:] = dy[:, :, 1:, :-1]
    assert np.array_equal(got["dx"], want)

"""Seeded random geometries through every entry point and both algorithm choices.

The fixed shapes of the other files are aimed at the cases each kernel distinguishes; this
sweep draws small layers at random (filters 1..7, strides 1..4, padding up to the filter,
channel and filter counts around the tile sizes, odd and even maps) so that the routes
between the kernels (first-layer forms, pointwise, taps, Winograd sub-filters, strided
rearrangement, the general kernels) are crossed in combinations nobody wrote down.  Every
tensor is compared with the oracle at the bar of the algorithm that produced it."""
import numpy as np
import pytest

import oracle
from paper_1606_04884_amd import binding as B
from gpu_util import TOL_IGEMM, TOL_WINOGRAD, gpu_layer, max_err_ratio, oracle_layer, random_layer

pytestmark = pytest.mark.gpu


def draw(rng):
    while True:
        R = int(rng.choice([1, 1, 2, 3, 3, 3, 4, 5, 5, 7]))
        S = R if rng.random() < 0.7 else int(rng.integers(1, 8))
        sh = int(rng.choice([1, 1, 1, 2, 3, 4]))
        sw = sh if rng.random() < 0.8 else int(rng.integers(1, 4))
        ph = int(rng.integers(0, R))
        pw = ph if rng.random() < 0.7 and ph < S else int(rng.integers(0, S))
        C = int(rng.choice([1, 3, 4, 8, 12, 16, 24, 33, 64, 96]))
        K = int(rng.choice([1, 5, 8, 16, 32, 40, 64, 96, 130]))
        H = int(rng.integers(max(1, R - 2 * ph), 30))
        W = int(rng.integers(max(1, S - 2 * pw), 30))
        N = int(rng.integers(1, 5))
        if (H + 2 * ph - R) < 0 or (W + 2 * pw - S) < 0:
            continue
        P = (H + 2 * ph - R) // sh + 1
        Q = (W + 2 * pw - S) // sw + 1
        # keep the oracle's work per case small
        if N * K * P * Q * C * R * S > 6e7:
            continue
        return (N, C, H, W, K, R, S, sh, sw, ph, pw)


def cases(seed, count):
    rng = np.random.default_rng(seed)
    return [draw(rng) for _ in range(count)]


RANDOM_GEOMS = cases(20260611, 48)


@pytest.mark.parametrize("geom", RANDOM_GEOMS, ids=["x".join(map(str, g)) for g in RANDOM_GEOMS])
def test_random_geometry(geom):
    x, w, b, dy = random_layer(geom, 11000 + sum(geom))
    print("geom", geom, flush=True)
    ref = oracle_layer(geom, x, w, b, dy)
    ops = {"y": B.OP_FWD, "dx": B.OP_BWD_DATA, "dw": B.OP_BWD_WEIGHT, "db": B.OP_BWD_WEIGHT}
    for algo in (B.ALGO_AUTO, B.ALGO_IGEMM):
        got = gpu_layer(geom, x, w, b, dy, algo=algo)
        for name in ("y", "dx", "dw", "db"):
            assert np.isfinite(got[name]).all(), (algo, name)
            used = B.conv2d_pick_algo(geom, ops[name]) if algo == B.ALGO_AUTO else B.ALGO_IGEMM
            tol = TOL_WINOGRAD if used == B.ALGO_WINOGRAD else TOL_IGEMM
            r = max_err_ratio(got[name], ref[name])
            assert r <= tol, "algo %d %s: max err ratio %.3e" % (algo, name, r)

"""GPU parity of the unfused Winograd F(4x4,3x3) path (CONV2D_ALGO_WINOGRAD4: filter,
input and output transform kernels around 36 batched GEMMs) against the CPU oracle,
element by element at the Winograd tolerance: forward and backward-data on shapes that
span several GEMM tiles and ragged tails (odd maps, tile grids cut by the map edge,
channel counts off the 8-channel chunk, filter counts off the 64-row wave tile, every
padding the path takes)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_1606_04884_amd import binding as B          # noqa: E402
from gpu_util import TOL_WINOGRAD, gpu_layer, max_err_ratio, oracle_layer, random_layer  # noqa: E402

SHAPES = [
    # N, C, H, W, K, R, S, sh, sw, ph, pw
    (2, 32, 16, 16, 64, 3, 3, 1, 1, 1, 1),
    (3, 64, 28, 28, 128, 3, 3, 1, 1, 1, 1),       # several column tiles
    (2, 20, 13, 13, 40, 3, 3, 1, 1, 1, 1),        # odd map, ragged chunk, ragged filter tile
    (5, 8, 14, 14, 200, 3, 3, 1, 1, 1, 1),        # two row tiles of the 128-row form
    (2, 16, 9, 11, 24, 3, 3, 1, 1, 0, 0),         # unpadded
    (2, 24, 7, 10, 72, 3, 3, 1, 1, 2, 2),         # full padding
    (1, 3, 12, 12, 8, 3, 3, 1, 1, 1, 0),          # very few channels, unequal pads
    (40, 16, 12, 12, 300, 3, 3, 1, 1, 1, 1),      # 360 tiles: two column tiles, three row tiles
    (1, 136, 6, 5, 64, 3, 3, 1, 1, 1, 1),         # map smaller than two tiles
    (32, 64, 32, 32, 256, 3, 3, 1, 1, 1, 1),      # 576 GEMM tiles for 512 resident workgroups: the last 64 in 8 depth shares
    (36, 40, 30, 30, 200, 3, 3, 1, 1, 1, 1),      # 648 tiles, the last 136 in 3 unequal shares of 5 chunks
    (32, 16, 32, 32, 192, 3, 3, 1, 1, 1, 1),      # 192 filters: the 64-row x 512-column workgroup tile
    # filters beyond 3x3 as sums of 3x3 sub-filters of shifted inputs
    (2, 16, 12, 12, 24, 5, 5, 1, 1, 2, 2),
    (3, 8, 9, 11, 16, 5, 5, 1, 1, 0, 0),
    (2, 24, 13, 10, 40, 5, 5, 1, 1, 4, 1),
    (2, 8, 9, 9, 8, 4, 4, 1, 1, 1, 2),
    (2, 12, 10, 12, 16, 6, 6, 1, 1, 3, 2),
    (2, 16, 8, 9, 8, 3, 5, 1, 1, 1, 2),
    (4, 64, 27, 27, 192, 5, 5, 1, 1, 2, 2),       # AlexNet conv2 at a small batch
]


@pytest.mark.parametrize("geom", SHAPES, ids=[str(i) for i in range(len(SHAPES))])
def test_wino4_parity(geom):
    print("case", geom, flush=True)
    x, w, b, dy = random_layer(geom, seed=4400 + sum(geom))
    got = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_WINOGRAD4, passes=("fwd", "bwd_data"))
    ref = oracle_layer(geom, x, w, b, dy)
    for name in ("y", "dx"):
        assert np.isfinite(got[name]).all(), name
        r = max_err_ratio(got[name], ref[name])
        assert r <= TOL_WINOGRAD, "%s: %.3e" % (name, r)


WG_SHAPES = [
    (2, 32, 16, 16, 64, 3, 3, 1, 1, 1, 1),
    (3, 64, 28, 28, 128, 3, 3, 1, 1, 1, 1),
    (2, 20, 13, 13, 40, 3, 3, 1, 1, 1, 1),        # odd map: gradient tiles cut by the edge; ragged rows
    (5, 300, 14, 14, 200, 3, 3, 1, 1, 1, 1),      # several row and column tiles
    (4, 16, 9, 11, 24, 3, 3, 1, 1, 0, 0),
    (2, 24, 7, 10, 72, 3, 3, 1, 1, 2, 2),
    (2, 3, 12, 12, 8, 3, 3, 1, 1, 1, 0),
    (37, 48, 12, 12, 136, 3, 3, 1, 1, 1, 1),      # 333 tiles: last chunk ragged, unequal depth shares
    (4, 512, 12, 12, 192, 3, 3, 1, 1, 1, 1),      # 192 filters x 512 channels: the 64 x 512 workgroup tile
    (2, 16, 12, 12, 24, 5, 5, 1, 1, 2, 2),        # sub-filter gradients scattered into the 5x5 gradient
    (5, 8, 9, 11, 16, 5, 5, 1, 1, 0, 0),
    (2, 24, 13, 10, 40, 5, 4, 1, 1, 4, 1),
    (2, 12, 10, 12, 16, 6, 6, 1, 1, 3, 2),
    (4, 64, 27, 27, 192, 5, 5, 1, 1, 2, 2),
]


@pytest.mark.parametrize("geom", WG_SHAPES, ids=[str(i) for i in range(len(WG_SHAPES))])
def test_wino4_wgrad_parity(geom):
    print("case", geom, flush=True)
    x, w, b, dy = random_layer(geom, seed=4600 + sum(geom))
    got = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_WINOGRAD4, passes=("bwd_weight",))
    ref = oracle_layer(geom, x, w, b, dy)
    for name in ("dw", "db"):
        assert np.isfinite(got[name]).all(), name
        r = max_err_ratio(got[name], ref[name])
        assert r <= TOL_WINOGRAD, "%s: %.3e" % (name, r)


def test_wino4_wgrad_scale_accumulate_and_no_dbias():
    import oracle
    geom = (3, 32, 14, 14, 64, 3, 3, 1, 1, 1, 1)
    x, w, b, dy = random_layer(geom, seed=4699)
    rng = np.random.default_rng(5)
    dw0 = rng.standard_normal(w.shape).astype(np.float32)
    db0 = rng.standard_normal(b.shape).astype(np.float32)
    got = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_WINOGRAD4, passes=("bwd_weight",), scale=0.5, dw0=dw0, db0=db0)
    rdw, rdb = oracle.bwd_weight(geom, x, dy, 0.5)
    assert max_err_ratio(got["dw"], rdw + dw0) <= TOL_WINOGRAD
    assert max_err_ratio(got["db"], rdb + db0) <= TOL_WINOGRAD
    import torch
    dev = torch.device("cuda:0")
    dw = torch.full(w.shape, float("nan"), device=dev)
    B.conv2d_bwd_weight(geom, torch.from_numpy(x).to(dev), torch.from_numpy(dy).to(dev), dw, None, algo=B.ALGO_WINOGRAD4)
    assert max_err_ratio(dw.cpu().numpy(), oracle.bwd_weight(geom, x, dy, 1.0)[0]) <= TOL_WINOGRAD


def test_wino4_relu_and_no_bias():
    import torch
    geom = (2, 32, 14, 14, 64, 3, 3, 1, 1, 1, 1)
    x, w, b, dy = random_layer(geom, seed=4499)
    dev = torch.device("cuda:0")
    tx, tw, tb = (torch.from_numpy(t).to(dev) for t in (x, w, b))
    P, Q = B.conv2d_output_dims(geom)
    y = torch.full((2, 64, P, Q), float("nan"), device=dev)
    B.conv2d_fwd_relu(geom, tx, tw, tb, y, algo=B.ALGO_WINOGRAD4)
    import oracle
    ref = oracle.fwd_relu(geom, x, w, b)
    assert max_err_ratio(y.cpu().numpy(), ref) <= TOL_WINOGRAD
    y2 = torch.full((2, 64, P, Q), float("nan"), device=dev)
    B.conv2d_fwd(geom, tx, tw, None, y2, algo=B.ALGO_WINOGRAD4)
    assert max_err_ratio(y2.cpu().numpy(), oracle.fwd(geom, x, w, None)) <= TOL_WINOGRAD


def test_wino4_refuses_what_it_cannot_do():
    for geom, op in (((2, 8, 16, 16, 8, 7, 7, 1, 1, 3, 3), B.OP_FWD),
                     ((2, 8, 16, 16, 8, 3, 3, 2, 2, 1, 1), B.OP_FWD),
                     ((1, 8, 8, 8, 8, 3, 3, 1, 1, 1, 1), B.OP_BWD_WEIGHT)):        # 4 tiles: too few to split
        assert B.conv2d_workspace_bytes(geom, op, B.ALGO_WINOGRAD4) == 0

"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element
by element, on seeded inputs.  Bar: max|gpu - ref| <= 1e-4 * max|ref| per output
tensor for the implicit-GEMM path (ref = the oracle's fp64 value)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from paper_1606_04884_amd import binding as B          # noqa: E402
from paper_1606_04884_amd import synth                 # noqa: E402
import oracle                                          # noqa: E402
from gpu_util import (TOL_IGEMM, gpu_layer, max_err_ratio, oracle_layer,   # noqa: E402
                      random_layer)


def G(N, C, H, W, K, R, S, s, p):
    return (N, C, H, W, K, R, S, s, s, p, p)


# shapes chosen to span several tiles in every GEMM dimension and leave ragged
# tails: filters not a multiple of 32/64/128, depth not a multiple of 16, pixel
# counts not a multiple of 128/256, odd maps, every stride/pad of the configs.
SHAPES = [
    G(2, 3, 16, 16, 8, 3, 3, 1, 1),          # the single-layer benchmark configuration
    G(3, 17, 19, 23, 40, 3, 3, 1, 1),
    G(2, 64, 14, 14, 96, 3, 3, 1, 1),
    G(2, 3, 67, 67, 64, 11, 11, 4, 2),       # AlexNet conv1 geometry, small map
    G(2, 3, 59, 59, 96, 11, 11, 4, 0),       # Overfeat conv1 geometry
    G(2, 16, 27, 27, 48, 5, 5, 1, 2),
    G(3, 24, 24, 24, 72, 5, 5, 1, 0),
    G(4, 48, 13, 13, 160, 1, 1, 1, 0),       # 1x1
    G(2, 192, 28, 28, 16, 1, 1, 1, 0),       # inception 1x1 reduce (vector-load 1x1 path)
    G(3, 20, 12, 12, 96, 1, 1, 1, 0),        # 1x1 path, depth and pixel count ragged
    G(5, 72, 8, 10, 200, 1, 1, 1, 0),        # 1x1 path, several filter tiles
    G(2, 8, 20, 21, 130, 3, 2, 2, 1),
    G(1, 5, 9, 9, 3, 3, 3, 3, 0),
    G(2, 20, 12, 12, 33, 5, 5, 1, 0),
    G(1, 1, 5, 5, 1, 3, 3, 1, 1),
    G(1, 130, 12, 12, 300, 3, 3, 1, 1),
    G(5, 7, 13, 13, 20, 3, 3, 1, 2),         # pad > (R-1)/2
    G(2, 6, 15, 11, 10, 1, 1, 2, 0),         # 1x1 stride 2: phases without taps
    (2, 4, 17, 14, 9, 3, 5, 2, 3, 1, 2),     # stride_h != stride_w, pad_h != pad_w
    (1, 3, 30, 9, 5, 7, 1, 5, 1, 3, 0),      # stride 5 in h: 5 phases
    G(2, 40, 15, 16, 24, 3, 3, 2, 1),        # strided with many channels: per-phase backward-data
    G(2, 3, 23, 23, 16, 5, 5, 2, 2),         # strided with few channels: depth-to-space backward-data
]


@pytest.mark.parametrize("geom", SHAPES, ids=[("x".join(map(str, g))) for g in SHAPES])
def test_layer_parity(geom):
    x, w, b, dy = random_layer(geom, 1000 + sum(geom))
    print("geom", geom, flush=True)
    got = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_IGEMM)
    ref = oracle_layer(geom, x, w, b, dy)
    for name in ("y", "dx", "dw", "db"):
        assert np.isfinite(got[name]).all(), name
        r = max_err_ratio(got[name], ref[name])
        assert r <= TOL_IGEMM, "%s: max err ratio %.3e" % (name, r)


def test_config1_distribution():
    """The single-layer benchmark configuration with its own value distributions (U(-1,1), dy ~ N(0,1))."""
    L = synth.config_layers(0)[0]
    geom = L.desc()
    t = synth.layer_tensors(0, 0, L, oracle.output_dims(geom))
    got = gpu_layer(geom, t["x"], t["w"], t["b"], t["dy"])
    ref = oracle_layer(geom, t["x"], t["w"], t["b"], t["dy"])
    for name in ("y", "dx", "dw", "db"):
        assert max_err_ratio(got[name], ref[name]) <= TOL_IGEMM, name


def test_no_bias_and_no_dbias():
    geom = G(2, 9, 11, 12, 21, 3, 3, 1, 1)
    x, w, b, dy = random_layer(geom, 77)
    dev = torch.device("cuda:0")
    P, Q = B.conv2d_output_dims(geom)
    y = torch.empty((2, 21, P, Q), device=dev)
    B.conv2d_fwd(geom, torch.from_numpy(x).to(dev), torch.from_numpy(w).to(dev), None, y)
    assert max_err_ratio(y.cpu().numpy(), oracle.fwd(geom, x, w, None)) <= TOL_IGEMM
    dw = torch.empty((21, 9, 3, 3), device=dev)
    B.conv2d_bwd_weight(geom, torch.from_numpy(x).to(dev), torch.from_numpy(dy).to(dev), dw, None)
    assert max_err_ratio(dw.cpu().numpy(), oracle.bwd_weight(geom, x, dy)[0]) <= TOL_IGEMM


def test_scale_and_accumulate():
    geom = G(3, 10, 14, 14, 24, 3, 3, 1, 1)
    x, w, b, dy = random_layer(geom, 88)
    dw0 = synth.normal((24, 10, 3, 3), 5, std=30.0)
    db0 = synth.normal((24,), 6, std=30.0)
    got = gpu_layer(geom, x, w, b, dy, scale=0.25, dw0=dw0.copy(), db0=db0.copy(),
                    passes=("bwd_weight",))
    dw, db = oracle.bwd_weight(geom, x, dy, 0.25)
    assert max_err_ratio(got["dw"], dw + dw0) <= TOL_IGEMM
    assert max_err_ratio(got["db"], db + db0) <= TOL_IGEMM
    got = gpu_layer(geom, x, w, b, dy, scale=-2.0, passes=("bwd_weight",))
    dw, db = oracle.bwd_weight(geom, x, dy, -2.0)
    assert max_err_ratio(got["dw"], dw) <= TOL_IGEMM
    assert max_err_ratio(got["db"], db) <= TOL_IGEMM


def test_identity_filter_is_bit_exact():
    N, C, H, W = 2, 5, 9, 10
    geom = G(N, C, H, W, C, 3, 3, 1, 1)
    x = synth.normal((N, C, H, W), 3)
    w = np.zeros((C, C, 3, 3), np.float32)
    for c in range(C):
        w[c, c, 1, 1] = 1.0
    got = gpu_layer(geom, x, w, None, x, passes=("fwd", "bwd_data"))
    np.testing.assert_array_equal(got["y"], x)
    np.testing.assert_array_equal(got["dx"], x)


def test_run_to_run_deterministic():
    geom = G(4, 32, 28, 28, 64, 3, 3, 1, 1)
    x, w, b, dy = random_layer(geom, 99)
    a = gpu_layer(geom, x, w, b, dy)
    c = gpu_layer(geom, x, w, b, dy)
    for name in ("y", "dx", "dw", "db"):
        np.testing.assert_array_equal(a[name], c[name])


def test_large_split_reduction_depth():
    """Long reduction axis for the weight gradient (many splits), small output."""
    geom = G(8, 3, 96, 96, 16, 3, 3, 1, 1)
    x, w, b, dy = random_layer(geom, 123)
    got = gpu_layer(geom, x, w, b, dy, passes=("bwd_weight",))
    dw, db = oracle.bwd_weight(geom, x, dy)
    assert max_err_ratio(got["dw"], dw) <= TOL_IGEMM
    assert max_err_ratio(got["db"], db) <= TOL_IGEMM


# ---------------------------------------------------------------------------
# Winograd F(2x2,3x3) path (3x3, stride 1): bar 1e-3 * max|ref|
# ---------------------------------------------------------------------------
WINO_SHAPES = [
    G(2, 8, 16, 16, 8, 3, 3, 1, 1),
    G(3, 16, 19, 23, 40, 3, 3, 1, 1),        # odd map: half-filled edge tiles
    G(2, 64, 14, 14, 96, 3, 3, 1, 1),
    G(4, 24, 13, 13, 72, 3, 3, 1, 1),        # AlexNet-sized odd map
    G(1, 136, 12, 12, 296, 3, 3, 1, 1),      # K and tiles not multiples of 64
    G(2, 32, 9, 9, 64, 3, 3, 1, 0),          # no padding
    G(2, 16, 10, 7, 16, 3, 3, 1, 2),         # full padding
    (2, 8, 11, 12, 24, 3, 3, 1, 1, 0, 2),    # pad_h != pad_w
    G(5, 40, 28, 28, 136, 3, 3, 1, 1),
    # more output tiles than compute units: unit ranges cut tiles (fixup path), with
    # ragged filter and tile counts; second shape cuts tiles in backward-data
    G(40, 16, 28, 28, 136, 3, 3, 1, 1),
    G(36, 136, 26, 26, 24, 3, 3, 1, 1),
    # tile-pair kernel (pad_w 1, even width) with other pad_h, narrow maps, rows ending
    # inside a tile block
    (2, 16, 7, 10, 24, 3, 3, 1, 1, 0, 1),
    (3, 8, 9, 6, 16, 3, 3, 1, 1, 2, 1),
    G(3, 24, 20, 36, 40, 3, 3, 1, 1),
    # tile-pair kernel with a ragged last channel chunk: first-layer forward (3 channels in
    # one chunk), 12 channels (a full chunk and half a chunk), and backward-data over 20 filters
    G(2, 3, 16, 16, 64, 3, 3, 1, 1),
    G(3, 12, 20, 24, 40, 3, 3, 1, 1),
    G(2, 8, 12, 12, 20, 3, 3, 1, 1),
    G(40, 3, 32, 32, 64, 3, 3, 1, 1),        # more tile blocks than compute units, 3 channels
]


@pytest.mark.parametrize("geom", WINO_SHAPES, ids=[("x".join(map(str, g))) for g in WINO_SHAPES])
def test_winograd_parity(geom):
    from gpu_util import TOL_WINOGRAD
    x, w, b, dy = random_layer(geom, 2000 + sum(geom))
    print("geom", geom, flush=True)
    got = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_WINOGRAD, passes=("fwd", "bwd_data"))
    ref = {"y": oracle.fwd(geom, x, w, b), "dx": oracle.bwd_data(geom, dy, w)}
    for name in ("y", "dx"):
        assert np.isfinite(got[name]).all(), name
        r = max_err_ratio(got[name], ref[name])
        assert r <= TOL_WINOGRAD, "%s: max err ratio %.3e" % (name, r)


def test_winograd_refused_where_it_does_not_apply():
    dev = torch.device("cuda:0")
    # C not a multiple of the channel chunk on an odd-width map (the tile-pair kernel, which
    # takes a ragged chunk, needs an even width)
    geom = G(1, 4, 9, 9, 8, 3, 3, 1, 1)
    x = torch.zeros((1, 4, 9, 9), device=dev)
    w = torch.zeros((8, 4, 3, 3), device=dev)
    y = torch.zeros((1, 8, 9, 9), device=dev)
    with pytest.raises(B.Conv2dError) as e:
        B.conv2d_fwd(geom, x, w, None, y, algo=B.ALGO_WINOGRAD, ws=B.alloc_workspace(1 << 20))
    assert e.value.status == -3


WINO_WGRAD_SHAPES = [
    G(2, 32, 16, 16, 32, 3, 3, 1, 1),
    G(3, 64, 19, 23, 96, 3, 3, 1, 1),        # odd map, K = 64 + 32
    G(2, 96, 14, 14, 64, 3, 3, 1, 1),        # C = 64 + 32
    G(4, 160, 13, 13, 224, 3, 3, 1, 1),
    G(2, 32, 9, 9, 64, 3, 3, 1, 0),
    G(2, 32, 10, 7, 32, 3, 3, 1, 2),
    (2, 32, 11, 12, 32, 3, 3, 1, 1, 0, 2),
    G(7, 64, 28, 28, 128, 3, 3, 1, 1),
    # vector-load variants (pad_w 1, even width): even and odd tile-row widths,
    # rows that end inside a step, other pad_h
    G(3, 64, 12, 12, 64, 3, 3, 1, 1),
    G(5, 96, 20, 36, 160, 3, 3, 1, 1),
    (2, 32, 7, 10, 32, 3, 3, 1, 1, 0, 1),
    (2, 64, 9, 6, 32, 3, 3, 1, 1, 2, 1),
    G(3, 32, 15, 22, 96, 3, 3, 1, 1),
]


@pytest.mark.parametrize("geom", WINO_WGRAD_SHAPES, ids=[("x".join(map(str, g))) for g in WINO_WGRAD_SHAPES])
def test_winograd_wgrad_parity(geom):
    from gpu_util import TOL_WINOGRAD
    x, w, b, dy = random_layer(geom, 3000 + sum(geom))
    print("geom", geom, flush=True)
    got = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_WINOGRAD, passes=("bwd_weight",))
    dw, db = oracle.bwd_weight(geom, x, dy)
    assert np.isfinite(got["dw"]).all()
    r = max_err_ratio(got["dw"], dw)
    assert r <= TOL_WINOGRAD, "dw: max err ratio %.3e" % r
    assert max_err_ratio(got["db"], db) <= TOL_IGEMM
    # scale / accumulate go through the same split reduction
    dw0 = synth.normal(dw.shape, 8, std=5.0)
    db0 = synth.normal(db.shape, 9, std=5.0)
    got = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_WINOGRAD, scale=0.5, dw0=dw0.copy(), db0=db0.copy(),
                    passes=("bwd_weight",))
    assert max_err_ratio(got["dw"], 0.5 * dw + dw0) <= TOL_WINOGRAD


@pytest.mark.parametrize("geom", [G(2, 3, 16, 16, 8, 3, 3, 1, 1), G(3, 3, 19, 24, 20, 3, 3, 1, 1),
                                  G(2, 1, 9, 8, 5, 3, 3, 1, 1), G(2, 4, 12, 12, 7, 3, 3, 1, 1),
                                  (2, 2, 10, 12, 6, 3, 3, 1, 1, 2, 1), (1, 3, 7, 4, 3, 3, 3, 1, 1, 0, 1)],
                         ids=lambda g: "x".join(map(str, g)))
def test_first_layer_backward_data_direct(geom):
    """AUTO routes 3x3 stride-1 backward-data into <= 4 channels to the direct kernel."""
    x, w, b, dy = random_layer(geom, 4000 + sum(geom))
    got = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_AUTO, passes=("bwd_data",))
    ref = oracle.bwd_data(geom, dy, w)
    assert max_err_ratio(got["dx"], ref) <= TOL_IGEMM


GROUP_CASES = [
    # (N, C, H, W, [K_g...])
    (3, 24, 10, 10, [16, 8, 40]),          # pointwise vector path (H*W % 4 == 0)
    (2, 13, 7, 9, [5, 70]),                # gather path, ragged everything
    (4, 192, 28, 28, [64, 96, 16]),        # the inception module's same-input 1x1 group
    (2, 40, 6, 6, [33]),                   # a single group
    (2, 16, 8, 8, [8, 8, 8, 8]),           # four groups
]


@pytest.mark.parametrize("case", GROUP_CASES, ids=[str(c[:4]) + str(c[4]) for c in GROUP_CASES])
def test_grouped_1x1_forward(case):
    """Several 1x1 convolutions of one input in one call: every group's output
    against the oracle, and bit-identical to the single-layer call."""
    import torch
    N, Cc, H, W, Ks = case
    dev = torch.device("cuda:0")
    seed = 7000 + N + Cc + H + sum(Ks)
    x = synth.normal((N, Cc, H, W), seed)
    ws_np = [synth.normal((k, Cc, 1, 1), seed + 10 + i, std=float(np.sqrt(2.0 / Cc))) for i, k in enumerate(Ks)]
    bs_np = [synth.uniform((k,), seed + 20 + i, -0.1, 0.1) if i != 1 else None for i, k in enumerate(Ks)]
    tx = torch.from_numpy(x).to(dev)
    tws = [torch.from_numpy(w).to(dev) for w in ws_np]
    tbs = [torch.from_numpy(b).to(dev) if b is not None else None for b in bs_np]
    ys = [torch.full((N, k, H, W), float("nan"), device=dev) for k in Ks]
    geom = (N, Cc, H, W, sum(Ks), 1, 1, 1, 1, 0, 0)
    print("case", case, flush=True)
    B.conv2d_fwd_1x1_group(geom, tx, tws, tbs, ys)
    torch.cuda.synchronize()
    for i, k in enumerate(Ks):
        g1 = (N, Cc, H, W, k, 1, 1, 1, 1, 0, 0)
        ref = oracle.fwd(g1, x, ws_np[i], bs_np[i])
        got = ys[i].cpu().numpy()
        assert np.isfinite(got).all()
        assert max_err_ratio(got, ref) <= TOL_IGEMM, "group %d" % i
        # the header's claim: the same summation order as the group's own conv2d_fwd call
        y1 = torch.full((N, k, H, W), float("nan"), device=dev)
        B.conv2d_fwd(g1, tx, tws[i], tbs[i], y1, algo=B.ALGO_IGEMM)
        torch.cuda.synchronize()
        assert torch.equal(ys[i], y1), "group %d differs from the single-layer call" % i


WINO_LARGE_FILTER_SHAPES = [
    G(2, 16, 12, 12, 24, 5, 5, 1, 2),
    (3, 8, 9, 11, 16, 5, 5, 1, 1, 0, 0),
    (2, 24, 13, 10, 40, 5, 5, 1, 1, 4, 1),
    (2, 8, 9, 9, 8, 4, 4, 1, 1, 1, 2),
    (2, 8, 10, 12, 16, 6, 6, 1, 1, 3, 2),
    (2, 16, 8, 9, 8, 3, 5, 1, 1, 1, 2),
    (2, 16, 9, 8, 8, 5, 3, 1, 1, 0, 1),
    G(4, 64, 27, 27, 192, 5, 5, 1, 2),          # AlexNet conv2 at a small batch
    # C and K multiples of 32: backward-weight too
    G(2, 32, 12, 12, 64, 5, 5, 1, 2),
    (3, 64, 9, 11, 32, 5, 5, 1, 1, 0, 0),
    (2, 32, 10, 12, 32, 6, 6, 1, 1, 3, 2),
    (2, 32, 8, 9, 32, 3, 5, 1, 1, 1, 2),
    (2, 96, 13, 10, 32, 5, 4, 1, 1, 4, 1),
]


@pytest.mark.parametrize("geom", WINO_LARGE_FILTER_SHAPES,
                         ids=[("x".join(map(str, g))) for g in WINO_LARGE_FILTER_SHAPES])
def test_winograd_large_filters(geom):
    """Filters up to 6x6 through the Winograd path (sums of 3x3 sub-filters of shifted
    inputs): forward and backward-data against the oracle."""
    from gpu_util import TOL_WINOGRAD
    x, w, b, dy = random_layer(geom, 8000 + sum(geom))
    print("geom", geom, flush=True)
    got = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_WINOGRAD, passes=("fwd", "bwd_data"))
    assert np.isfinite(got["y"]).all() and np.isfinite(got["dx"]).all()
    assert max_err_ratio(got["y"], oracle.fwd(geom, x, w, b)) <= TOL_WINOGRAD
    assert max_err_ratio(got["dx"], oracle.bwd_data(geom, dy, w)) <= TOL_WINOGRAD
    if geom[1] % 32 == 0 and geom[4] % 32 == 0:
        got = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_WINOGRAD, passes=("bwd_weight",))
        dw, db = oracle.bwd_weight(geom, x, dy)
        assert np.isfinite(got["dw"]).all()
        assert max_err_ratio(got["dw"], dw) <= TOL_WINOGRAD
        assert max_err_ratio(got["db"], db) <= TOL_IGEMM
        # scale / accumulate through the sub-filter reduction
        dw0 = synth.normal(dw.shape, 18, std=2.0)
        got = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_WINOGRAD, scale=-0.5, dw0=dw0.copy(),
                        db0=np.zeros_like(db, dtype=np.float32), passes=("bwd_weight",))
        assert max_err_ratio(got["dw"], -0.5 * dw + dw0) <= TOL_WINOGRAD


# strided layers whose filter spans 3 x 3 strides, computed as stride-1 3x3 Winograd
# layers over the space-to-depth rearrangement of the input
STRIDED_WINO_SHAPES = [
    G(2, 3, 67, 67, 64, 11, 11, 4, 2),       # AlexNet conv1 geometry, small map
    G(2, 3, 59, 59, 96, 11, 11, 4, 0),       # Overfeat conv1 geometry
    (3, 4, 21, 23, 32, 5, 5, 2, 2, 2, 2),    # 5x5 stride 2, odd non-square map
    (2, 8, 20, 20, 32, 6, 6, 2, 2, 1, 1),    # filter exactly 3 strides wide
    (2, 3, 40, 37, 64, 9, 9, 3, 3, 4, 4),    # stride 3
    (2, 3, 50, 47, 32, 11, 10, 4, 4, 3, 1),  # 11x10 filter, pads differ, map not a multiple of the stride
    (2, 5, 26, 26, 40, 5, 5, 2, 2, 0, 0),    # K % 32 != 0: backward-weight stays with the general kernel
    (1, 20, 17, 17, 64, 5, 5, 2, 2, 2, 2),   # 80 rearranged channels (not chosen by default)
]


@pytest.mark.parametrize("geom", STRIDED_WINO_SHAPES, ids=[("x".join(map(str, g))) for g in STRIDED_WINO_SHAPES])
def test_strided_layers_through_winograd(geom):
    from gpu_util import TOL_WINOGRAD
    x, w, b, dy = random_layer(geom, 9000 + sum(geom))
    print("geom", geom, flush=True)
    ref = oracle_layer(geom, x, w, b, dy)
    got = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_WINOGRAD, passes=("fwd", "bwd_data"))
    for name in ("y", "dx"):
        assert np.isfinite(got[name]).all(), name
        r = max_err_ratio(got[name], ref[name])
        assert r <= TOL_WINOGRAD, "%s: max err ratio %.3e" % (name, r)
    if geom[4] % 32 != 0:
        assert B.conv2d_pick_algo(geom, B.OP_BWD_WEIGHT) == B.ALGO_IGEMM
        return
    got = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_WINOGRAD, passes=("bwd_weight",))
    assert max_err_ratio(got["dw"], ref["dw"]) <= TOL_WINOGRAD
    assert max_err_ratio(got["db"], ref["db"]) <= TOL_IGEMM
    dw0 = synth.normal(ref["dw"].shape, 18, std=3.0)
    db0 = synth.normal(ref["db"].shape, 19, std=3.0)
    got = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_WINOGRAD, scale=0.5, dw0=dw0.copy(), db0=db0.copy(),
                    passes=("bwd_weight",))
    assert max_err_ratio(got["dw"], 0.5 * ref["dw"] + dw0) <= TOL_WINOGRAD
    assert max_err_ratio(got["db"], 0.5 * ref["db"] + db0) <= TOL_IGEMM


def test_strided_first_layer_backward_takes_winograd_by_default():
    """AUTO on the AlexNet conv1 geometry: the backward passes are the rearranged Winograd
    path (same result as asking for it), the forward pass the gather kernel."""
    geom = G(2, 3, 67, 67, 64, 11, 11, 4, 2)
    assert B.conv2d_pick_algo(geom, B.OP_FWD) == B.ALGO_IGEMM
    for op in (B.OP_BWD_DATA, B.OP_BWD_WEIGHT):
        assert B.conv2d_pick_algo(geom, op) == B.ALGO_WINOGRAD
    x, w, b, dy = random_layer(geom, 9100)
    a = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_AUTO)
    c = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_WINOGRAD)
    d = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_IGEMM, passes=("fwd",))
    for name in ("dx", "dw", "db"):
        assert np.array_equal(a[name], c[name]), name
    assert np.array_equal(a["y"], d["y"])


# backward-weight of small stride-1 filters over very few channels (C*R*S <= 32 taps, Q % 4
# == 0): the taps form of the streaming backward-weight kernel.  Filter-tile counts 1, 2, 3,
# 4, 6, 8; 3x3 and 5x5 and 2x3 filters; paddings 0, 1, 2; rows shorter than a 16-pixel step.
TAP_WGRAD_SHAPES = [
    G(2, 3, 16, 16, 8, 3, 3, 1, 1),
    (3, 3, 12, 20, 64, 3, 3, 1, 1, 1, 1),
    (2, 2, 9, 8, 40, 3, 3, 1, 1, 1, 1),
    (2, 1, 8, 12, 24, 5, 5, 1, 1, 2, 2),
    G(4, 3, 32, 32, 96, 3, 3, 1, 1),
    (2, 3, 10, 14, 128, 3, 3, 1, 1, 0, 0),
    (3, 2, 6, 6, 16, 3, 3, 1, 1, 2, 2),
    (2, 4, 7, 9, 20, 2, 3, 1, 1, 0, 1),
    G(9, 3, 40, 40, 64, 3, 3, 1, 1),         # enough pixels for several splits and all 8 phases
]


@pytest.mark.parametrize("geom", TAP_WGRAD_SHAPES, ids=[("x".join(map(str, g))) for g in TAP_WGRAD_SHAPES])
def test_first_layer_backward_weight_taps(geom):
    x, w, b, dy = random_layer(geom, 9500 + sum(geom))
    print("geom", geom, flush=True)
    assert B.conv2d_pick_algo(geom, B.OP_BWD_WEIGHT) == B.ALGO_IGEMM
    got = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_AUTO, passes=("bwd_weight",))
    dw, db = oracle.bwd_weight(geom, x, dy)
    assert np.isfinite(got["dw"]).all()
    assert max_err_ratio(got["dw"], dw) <= TOL_IGEMM
    assert max_err_ratio(got["db"], db) <= TOL_IGEMM
    dw0 = synth.normal(dw.shape, 28, std=2.0)
    db0 = synth.normal(db.shape, 29, std=2.0)
    got = gpu_layer(geom, x, w, b, dy, scale=0.125, dw0=dw0.copy(), db0=db0.copy(), passes=("bwd_weight",))
    assert max_err_ratio(got["dw"], 0.125 * dw + dw0) <= TOL_IGEMM
    assert max_err_ratio(got["db"], 0.125 * db + db0) <= TOL_IGEMM

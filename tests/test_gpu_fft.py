"""GPU parity of the frequency-domain path (CONV2D_ALGO_FFT: one 32 x 32 tile per image,
image / filter spectra, 544 complex products as real GEMMs, inverse transform) against the
CPU oracle, element by element, all three passes: the 5x5 layer shapes of the paper's
configurations at reduced channel counts, image counts off the 16-image group and the 4-image
depth chunk, channel and filter counts off every tile, rectangular maps and filters, padded
input filling the tile exactly, more images than one column tile."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from paper_1606_04884_amd import binding as B          # noqa: E402
from gpu_util import TOL_IGEMM, gpu_layer, max_err_ratio, oracle_layer, random_layer  # noqa: E402

# every output is a sum over channels of 32-term fp32 dot products with rounded sines and cosines,
# no large transform constants: the bar of the direct path holds (measured 2e-7 .. 4e-7, printed)
TOL_FFT = TOL_IGEMM

SHAPES = [
    # N, C, H, W, K, R, S, sh, sw, ph, pw
    (8, 16, 27, 27, 24, 5, 5, 1, 1, 2, 2),        # AlexNet's 5x5 layer shape (31 padded)
    (5, 12, 28, 28, 20, 5, 5, 1, 1, 0, 0),        # Overfeat's: unpadded
    (4, 16, 28, 28, 32, 5, 5, 1, 1, 2, 2),        # the inception module's: the padded input fills the tile
    (3, 8, 14, 14, 16, 3, 3, 1, 1, 1, 1),         # a 3x3 layer
    (6, 6, 9, 14, 5, 7, 4, 1, 1, 3, 1),           # rectangular map and filter, channels off the chunk, odd filter count
    (2, 3, 32, 32, 8, 11, 11, 1, 1, 0, 0),        # 11x11 at stride 1 on a full tile
    (21, 5, 12, 12, 7, 5, 5, 1, 1, 2, 2),         # image count off 16 and off 4
    (130, 4, 12, 12, 6, 5, 5, 1, 1, 2, 2),        # more images than one 128-column tile
    (3, 70, 10, 10, 140, 5, 5, 1, 1, 2, 2),       # 280 product rows: several row tiles; 18 depth chunks
    (1, 1, 5, 5, 1, 5, 5, 1, 1, 0, 0),            # a single output pixel
    (2, 4, 8, 8, 4, 1, 1, 1, 1, 0, 0),            # 1x1 filter
    (4, 64, 27, 27, 192, 5, 5, 1, 1, 2, 2),       # AlexNet conv2 at a small batch
    (40, 8, 12, 12, 200, 5, 5, 1, 1, 2, 2),       # 40 rows x 400 columns: the 64-row x 512-column workgroup tile
    (2, 4, 10, 10, 4, 3, 3, 1, 1, 3, 3),          # padding beyond the filter's reach: output rows that see only zeros
    (3, 5, 6, 20, 6, 1, 7, 1, 1, 0, 3),           # one-row filter
    (2, 36, 16, 16, 36, 5, 5, 1, 1, 2, 2),        # 72 product columns, 9 depth chunks: the 128 x 128 workgroup tile
]


@pytest.mark.parametrize("geom", SHAPES, ids=[str(i) for i in range(len(SHAPES))])
def test_fft_parity(geom):
    print("case", geom, flush=True)
    x, w, b, dy = random_layer(geom, seed=5400 + sum(geom))
    got = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_FFT)
    ref = oracle_layer(geom, x, w, b, dy)
    for name in ("y", "dx", "dw", "db"):
        assert np.isfinite(got[name]).all(), name
        r = max_err_ratio(got[name], ref[name])
        print("  %s max|gpu-ref|/max|ref| %.2e" % (name, r), flush=True)
        assert r <= TOL_FFT, "%s: %.3e" % (name, r)


def test_fft_wgrad_scale_accumulate_and_no_dbias():
    import oracle
    geom = (6, 12, 13, 13, 20, 5, 5, 1, 1, 2, 2)
    x, w, b, dy = random_layer(geom, seed=5699)
    rng = np.random.default_rng(5)
    dw0 = rng.standard_normal(w.shape).astype(np.float32)
    db0 = rng.standard_normal(b.shape).astype(np.float32)
    got = gpu_layer(geom, x, w, b, dy, algo=B.ALGO_FFT, passes=("bwd_weight",), scale=0.5, dw0=dw0, db0=db0)
    rdw, rdb = oracle.bwd_weight(geom, x, dy, 0.5)
    assert max_err_ratio(got["dw"], rdw + dw0) <= TOL_FFT
    assert max_err_ratio(got["db"], rdb + db0) <= TOL_FFT
    import torch
    dev = torch.device("cuda:0")
    dw = torch.full(w.shape, float("nan"), device=dev)
    B.conv2d_bwd_weight(geom, torch.from_numpy(x).to(dev), torch.from_numpy(dy).to(dev), dw, None, algo=B.ALGO_FFT)
    assert max_err_ratio(dw.cpu().numpy(), oracle.bwd_weight(geom, x, dy, 1.0)[0]) <= TOL_FFT


def test_fft_relu_and_no_bias():
    import torch
    import oracle
    geom = (5, 12, 13, 13, 20, 5, 5, 1, 1, 2, 2)
    x, w, b, dy = random_layer(geom, seed=5499)
    dev = torch.device("cuda:0")
    tx, tw, tb = (torch.from_numpy(t).to(dev) for t in (x, w, b))
    P, Q = B.conv2d_output_dims(geom)
    y = torch.full((5, 20, P, Q), float("nan"), device=dev)
    B.conv2d_fwd_relu(geom, tx, tw, tb, y, algo=B.ALGO_FFT)
    assert max_err_ratio(y.cpu().numpy(), oracle.fwd_relu(geom, x, w, b)) <= TOL_FFT
    y2 = torch.full((5, 20, P, Q), float("nan"), device=dev)
    B.conv2d_fwd(geom, tx, tw, None, y2, algo=B.ALGO_FFT)
    assert max_err_ratio(y2.cpu().numpy(), oracle.fwd(geom, x, w, None)) <= TOL_FFT


def test_fft_refuses_what_it_cannot_do():
    for geom in ((2, 8, 30, 30, 8, 5, 5, 1, 1, 2, 2),          # 34 padded: more than one tile
                 (2, 8, 33, 8, 8, 3, 3, 1, 1, 0, 0),
                 (2, 8, 16, 16, 8, 3, 3, 2, 2, 1, 1)):         # strided
        for op in (B.OP_FWD, B.OP_BWD_DATA, B.OP_BWD_WEIGHT):
            assert B.conv2d_workspace_bytes(geom, op, B.ALGO_FFT) == 0

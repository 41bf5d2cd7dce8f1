"""Chained forward of the VGG-16 conv stack (all 13 layers, 2x2/stride-2 max pooling
between blocks) through the C-ABI: shows that the per-layer calls compose.  Every
layer's GPU output is judged against the oracle applied to that layer's ACTUAL
device input (copied back), so an error in one layer cannot hide in the next.
The pooling between blocks is support code (a plain tensor reduction), not part
of the path under test.  Run twice: without an activation function between the layers,
and with the rectifier fused into every convolution (conv2d_fwd_relu), which is how the
stack is used: from the second layer on the inputs are then non-negative and sparse."""
import numpy as np
import pytest

import oracle
from paper_1606_04884_amd import binding as B
from paper_1606_04884_amd import synth
from gpu_util import max_err_ratio, TOL_IGEMM, TOL_WINOGRAD

pytestmark = pytest.mark.gpu

POOL_AFTER = {"conv1_2", "conv2_2", "conv3_3", "conv4_3"}


@pytest.mark.parametrize("relu", [False, True], ids=["linear", "relu"])
def test_vgg16_chained_forward_batch2(relu):
    import torch
    dev = torch.device("cuda:0")
    layers = synth.config_layers(2, batch=2)
    H0 = layers[0].H
    x = torch.from_numpy(synth.normal((2, 3, H0, H0), synth.layer_seed(2, 0, 0))).to(dev)
    for li, L in enumerate(layers):
        geom = L.desc()
        assert tuple(x.shape) == (L.N, L.C, L.H, L.W), (L.name, tuple(x.shape))
        P, Q = B.conv2d_output_dims(geom)
        std = float(np.sqrt(2.0 / (L.C * L.R * L.S)))
        w = synth.normal((L.K, L.C, L.R, L.S), synth.layer_seed(2, li, 1), std=std)
        b = synth.uniform((L.K,), synth.layer_seed(2, li, 2), -0.1, 0.1)
        y = torch.full((L.N, L.K, P, Q), float("nan"), device=dev)
        print("layer", L.name, geom, flush=True)
        (B.conv2d_fwd_relu if relu else B.conv2d_fwd)(geom, x, torch.from_numpy(w).to(dev),
                                                      torch.from_numpy(b).to(dev), y)
        torch.cuda.synchronize()
        ref = (oracle.fwd_relu if relu else oracle.fwd)(geom, x.cpu().numpy(), w, b)
        got = y.cpu().numpy()
        assert np.isfinite(got).all(), L.name
        tol = TOL_WINOGRAD if B.conv2d_pick_algo(geom, B.OP_FWD) == B.ALGO_WINOGRAD else TOL_IGEMM
        r = max_err_ratio(got, ref)
        assert r <= tol, "%s: max err ratio %.3e" % (L.name, r)
        x = y
        if L.name in POOL_AFTER:
            x = x.view(L.N, L.K, P // 2, 2, Q // 2, 2).amax(dim=(3, 5)).contiguous()
    assert tuple(x.shape) == (2, 512, 14, 14)

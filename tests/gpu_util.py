"""Helpers for the GPU parity tests: run one layer through the C-ABI binding and
compare with the CPU oracle.  The HIP path and the oracle only meet here."""
from __future__ import annotations

import numpy as np

import oracle
from paper_1606_04884_amd import binding as B
from paper_1606_04884_amd import synth

TOL_IGEMM = 1e-4      # max|gpu - ref| <= tol * max|ref|, per output tensor
TOL_WINOGRAD = 1e-3


def max_err_ratio(got: np.ndarray, ref64: np.ndarray) -> float:
    denom = float(np.abs(ref64).max())
    err = float(np.abs(got.astype(np.float64) - ref64).max())
    if denom == 0.0:
        return 0.0 if err == 0.0 else float("inf")
    return err / denom


def gpu_layer(geom, x, w, b, dy, algo=B.ALGO_AUTO, scale=1.0, dw0=None, db0=None,
              passes=("fwd", "bwd_data", "bwd_weight")):
    """Runs the requested passes on the GPU; numpy in, numpy (fp32) out."""
    import torch
    dev = torch.device("cuda:0")
    N, C, H, W, K, R, S = geom[:7]
    P, Q = B.conv2d_output_dims(geom)
    tx = torch.from_numpy(x).to(dev)
    tw = torch.from_numpy(w).to(dev)
    tb = torch.from_numpy(b).to(dev) if b is not None else None
    tdy = torch.from_numpy(dy).to(dev) if dy is not None else None
    out = {}
    if "fwd" in passes:
        y = torch.full((N, K, P, Q), float("nan"), device=dev)
        B.conv2d_fwd(geom, tx, tw, tb, y, algo=algo)
        out["y"] = y.cpu().numpy()
    if "bwd_data" in passes:
        dx = torch.full((N, C, H, W), float("nan"), device=dev)
        B.conv2d_bwd_data(geom, tdy, tw, dx, algo=algo)
        out["dx"] = dx.cpu().numpy()
    if "bwd_weight" in passes:
        acc = dw0 is not None
        dw = torch.from_numpy(dw0).to(dev) if acc else torch.full((K, C, R, S), float("nan"), device=dev)
        db = torch.from_numpy(db0).to(dev) if acc else torch.full((K,), float("nan"), device=dev)
        B.conv2d_bwd_weight(geom, tx, tdy, dw, db, scale=scale, accumulate=acc, algo=algo)
        out["dw"] = dw.cpu().numpy()
        out["db"] = db.cpu().numpy()
    torch.cuda.synchronize()
    return out


def oracle_layer(geom, x, w, b, dy, scale=1.0):
    ref = {"y": oracle.fwd(geom, x, w, b), "dx": oracle.bwd_data(geom, dy, w)}
    ref["dw"], ref["db"] = oracle.bwd_weight(geom, x, dy, scale)
    return ref


def random_layer(geom, seed, he=True):
    N, C, H, W, K, R, S = geom[:7]
    P, Q = oracle.output_dims(geom)
    x = synth.normal((N, C, H, W), seed)
    std = float(np.sqrt(2.0 / (C * R * S))) if he else 1.0
    w = synth.normal((K, C, R, S), seed + 1, std=std)
    b = synth.uniform((K,), seed + 2, -0.1, 0.1)
    dy = synth.normal((N, K, P, Q), seed + 3)
    return x, w, b, dy

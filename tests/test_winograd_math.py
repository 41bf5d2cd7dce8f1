"""The Winograd F(2x2,3x3) transform matrices the HIP path uses, checked on the
CPU against direct correlation.  The paper (Sec. 4.2 "Winograd") names the
algorithm but prints no matrices; these are the standard ones for the points
{0, 1, -1, inf}.  Exact rational arithmetic: the identity must hold exactly."""
import os
from fractions import Fraction as F

import numpy as np

import oracle
from paper_1606_04884_amd import synth

BT = [[1, 0, -1, 0], [0, 1, 1, 0], [0, -1, 1, 0], [0, 1, 0, -1]]
G = [[1, 0, 0], [F(1, 2), F(1, 2), F(1, 2)], [F(1, 2), F(-1, 2), F(1, 2)], [0, 0, 1]]
AT = [[1, 1, 1, 0], [0, 1, -1, -1]]


def mm(a, b):
    return [[sum(F(a[i][k]) * F(b[k][j]) for k in range(len(b))) for j in range(len(b[0]))]
            for i in range(len(a))]


def tr(a):
    return [list(r) for r in zip(*a)]


def parse(path):
    out = {}
    for line in open(path):
        line = line.strip()
        if line and not line.startswith("#"):
            k, *v = line.split()
            out[k] = [F(x) for x in v]
    return out


def test_golden_1d(golden_dir):
    g = parse(os.path.join(golden_dir, "winograd_f2x3_1d.txt"))
    Gg = [sum(F(G[i][k]) * g["g"][k] for k in range(3)) for i in range(4)]
    Btd = [sum(F(BT[i][k]) * g["d"][k] for k in range(4)) for i in range(4)]
    prod = [x * y for x, y in zip(Gg, Btd)]
    y = [sum(F(AT[i][k]) * prod[k] for k in range(4)) for i in range(2)]
    assert Gg == g["Gg"] and Btd == g["Btd"] and prod == g["prod"] and y == g["y"]
    direct = [sum(g["d"][i + k] * g["g"][k] for k in range(3)) for i in range(2)]
    assert y == direct


def test_2d_identity_exact():
    rng = np.random.default_rng(3)
    for _ in range(20):
        C = 3
        d = rng.integers(-9, 10, size=(C, 4, 4))
        g = rng.integers(-9, 10, size=(C, 3, 3))
        M = [[F(0)] * 4 for _ in range(4)]
        for c in range(C):
            U = mm(mm(G, g[c].tolist()), tr(G))
            V = mm(mm(BT, d[c].tolist()), tr(BT))
            for i in range(4):
                for j in range(4):
                    M[i][j] += U[i][j] * V[i][j]
        Y = mm(mm(AT, M), tr(AT))
        for p in range(2):
            for q in range(2):
                direct = sum(int(d[c, p + r, q + s]) * int(g[c, r, s])
                             for c in range(C) for r in range(3) for s in range(3))
                assert Y[p][q] == direct


def test_backward_data_is_forward_with_rotated_filter():
    """dx = correlation of dy (zero-extended by 2-pad) with the 180-degree rotated,
    k<->c swapped filter: the identity the Winograd backward-data call relies on."""
    import oracle
    from paper_1606_04884_amd import synth
    for pad in (0, 1, 2):
        N, C, H, W, K = 1, 2, 6, 7, 3
        geom = (N, C, H, W, K, 3, 3, 1, 1, pad, pad)
        P, Q = oracle.output_dims(geom)
        dy = synth.dyadic((N, K, P, Q), 5 + pad)
        w = synth.dyadic((K, C, 3, 3), 9)
        dx = oracle.bwd_data(geom, dy, w)
        wr = np.ascontiguousarray(w[:, :, ::-1, ::-1].transpose(1, 0, 2, 3))
        g2 = (N, K, P, Q, C, 3, 3, 1, 1, 2 - pad, 2 - pad)
        np.testing.assert_array_equal(oracle.fwd(g2, dy, wr), dx)


def test_weight_gradient_identity_exact():
    """dg = G^T [(A dy A^T) .* (B^T d B)] G equals sum_{p,q} dy[p][q] d[p+r][q+s]."""
    A = tr(AT)
    rng = np.random.default_rng(4)
    for _ in range(20):
        d = rng.integers(-9, 10, size=(4, 4)).tolist()
        dy = rng.integers(-9, 10, size=(2, 2)).tolist()
        Dp = mm(mm(A, dy), AT)
        V = mm(mm(BT, d), tr(BT))
        M = [[Dp[i][j] * V[i][j] for j in range(4)] for i in range(4)]
        dg = mm(mm(tr(G), M), G)
        for r in range(3):
            for s in range(3):
                direct = sum(dy[p][q] * d[p + r][q + s] for p in range(2) for q in range(2))
                assert dg[r][s] == direct


def test_large_filter_is_a_sum_of_shifted_3x3_filters():
    """A stride-1 R x S correlation (R, S <= 6) equals the sum over 3x3 sub-filters
    (taps 3a.., 3b.., zero where the filter ends) of 3x3 correlations of the input
    shifted by (3a, 3b): the decomposition the Winograd path uses for 5x5 layers.
    Exact on dyadic data; the sub-correlations are evaluated by the oracle with the
    shift expressed through asymmetric zero padding of the input."""
    for (R, S, ph, pw, H, W) in [(5, 5, 2, 2, 9, 8), (5, 5, 0, 0, 8, 9), (4, 6, 1, 3, 7, 9), (3, 5, 1, 2, 6, 7)]:
        N, C, K = 2, 3, 4
        x = synth.dyadic((N, C, H, W), 31 + R)
        w = synth.dyadic((K, C, R, S), 32 + S)
        full = oracle.fwd((N, C, H, W, K, R, S, 1, 1, ph, pw), x, w, None)
        P, Q = full.shape[2:]
        acc = np.zeros_like(full)
        # zero-extend the input once, by the padding plus room for the sub-filter overhang
        xe = np.zeros((N, C, H + 2 * ph + 3, W + 2 * pw + 3), dtype=np.float32)
        xe[:, :, ph:ph + H, pw:pw + W] = x
        for a in range((R + 2) // 3):
            for b in range((S + 2) // 3):
                g = np.zeros((K, C, 3, 3), dtype=np.float32)
                rr, ss = min(3, R - 3 * a), min(3, S - 3 * b)
                g[:, :, :rr, :ss] = w[:, :, 3 * a:3 * a + rr, 3 * b:3 * b + ss]
                xs = np.ascontiguousarray(xe[:, :, 3 * a:3 * a + P + 2, 3 * b:3 * b + Q + 2])
                acc += oracle.fwd((N, C, P + 2, Q + 2, K, 3, 3, 1, 1, 0, 0), xs, g, None)
        assert np.array_equal(acc, full), (R, S)


# ---- F(4x4,3x3): the larger tile of the unfused Winograd path -----------------
# Standard minimal-filtering matrices for the points {0, 1, -1, 2, -2, inf} (the paper's
# Sec. 4.2 "Winograd" cites the algorithm and prints none).
BT4 = [[4, 0, -5, 0, 1, 0], [0, -4, -4, 1, 1, 0], [0, 4, -4, -1, 1, 0],
       [0, -2, -1, 2, 1, 0], [0, 2, -1, -2, 1, 0], [0, 4, 0, -5, 0, 1]]
G4 = [[F(1, 4), 0, 0], [F(-1, 6), F(-1, 6), F(-1, 6)], [F(-1, 6), F(1, 6), F(-1, 6)],
      [F(1, 24), F(1, 12), F(1, 6)], [F(1, 24), F(-1, 12), F(1, 6)], [0, 0, 1]]
AT4 = [[1, 1, 1, 1, 1, 0], [0, 1, -1, 2, -2, 0], [0, 1, 1, 4, 4, 0], [0, 1, -1, 8, -8, 1]]


def test_f4x4_1d_identity_exact():
    rng = np.random.default_rng(11)
    for _ in range(20):
        d = [F(int(v)) for v in rng.integers(-9, 10, size=6)]
        g = [F(int(v)) for v in rng.integers(-9, 10, size=3)]
        Gg = [sum(F(G4[i][k]) * g[k] for k in range(3)) for i in range(6)]
        Btd = [sum(F(BT4[i][k]) * d[k] for k in range(6)) for i in range(6)]
        y = [sum(F(AT4[i][k]) * Gg[k] * Btd[k] for k in range(6)) for i in range(4)]
        assert y == [sum(d[i + k] * g[k] for k in range(3)) for i in range(4)]


def test_f4x4_2d_identity_exact():
    rng = np.random.default_rng(12)
    for _ in range(10):
        C = 3
        d = rng.integers(-9, 10, size=(C, 6, 6))
        g = rng.integers(-9, 10, size=(C, 3, 3))
        M = [[F(0)] * 6 for _ in range(6)]
        for c in range(C):
            U = mm(mm(G4, g[c].tolist()), tr(G4))
            V = mm(mm(BT4, d[c].tolist()), tr(BT4))
            for i in range(6):
                for j in range(6):
                    M[i][j] += U[i][j] * V[i][j]
        Y = mm(mm(AT4, M), tr(AT4))
        for p in range(4):
            for q in range(4):
                direct = sum(int(d[c, p + r, q + s]) * int(g[c, r, s])
                             for c in range(C) for r in range(3) for s in range(3))
                assert Y[p][q] == direct


def test_f4x4_weight_gradient_identity_exact():
    """dg = G^T [(A dy A^T) .* (B^T d B)] G with the F(4x4,3x3) matrices equals
    sum_{p,q<4} dy[p][q] d[p+r][q+s] (the transpose of the bilinear tile relation)."""
    A = tr(AT4)
    rng = np.random.default_rng(13)
    for _ in range(10):
        d = rng.integers(-9, 10, size=(6, 6)).tolist()
        dy = rng.integers(-9, 10, size=(4, 4)).tolist()
        Dp = mm(mm(A, dy), AT4)
        V = mm(mm(BT4, d), tr(BT4))
        M = [[Dp[i][j] * V[i][j] for j in range(6)] for i in range(6)]
        dg = mm(mm(tr(G4), M), G4)
        for r in range(3):
            for s in range(3):
                direct = sum(dy[p][q] * d[p + r][q + s] for p in range(4) for q in range(4))
                assert dg[r][s] == direct

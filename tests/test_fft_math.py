"""The identities the frequency-domain path (Sec. 4.2 "fft": convolution as a product of
spectra, the choice for large filters) is built on, checked on the CPU in fp64 against the
oracle's direct correlation.  The path uses one 32 x 32 tile per image (the padded input must
fit), the half spectrum u = 0..16 of a real signal, dense DFT matrices instead of butterflies,
and the complex products as real matrix products with 2 x 2 blocks.  Each step is written here
from the DFT's definition in plain numpy, in the order the kernels take them; numpy's own FFT is
used only as a second opinion on the spectra."""
import numpy as np
import pytest

import oracle
from paper_1606_04884_amd import synth

L = 32            # tile edge
UH = 17           # kept rows of the spectrum of a real tile

# (N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w): padded input <= 32 in both directions
GEOMS = [
    (2, 3, 27, 27, 4, 5, 5, 1, 1, 2, 2),        # the 5x5 layer shape of AlexNet (31 padded)
    (2, 2, 28, 28, 3, 5, 5, 1, 1, 0, 0),        # Overfeat's: no padding
    (1, 2, 28, 28, 2, 5, 5, 1, 1, 2, 2),        # the inception module's: 32 padded, no slack at all
    (2, 3, 9, 14, 2, 7, 4, 1, 1, 3, 1),         # rectangular everything
    (1, 1, 5, 5, 1, 5, 5, 1, 1, 0, 0),          # single output pixel
    (2, 4, 10, 10, 4, 3, 3, 1, 1, 3, 3),        # padding beyond the filter's reach
    (3, 5, 6, 20, 6, 1, 7, 1, 1, 0, 3),         # one-row filter
]


def dft_mats():
    j = np.arange(L)
    ang = 2.0 * np.pi * np.outer(j, j) / L
    return np.cos(ang), np.sin(ang)               # C[a][b], S[a][b]; forward kernel: C - iS


def tile_spectrum(img, off_h, off_w):
    """Half spectrum Y[u][v], u < 17, of the image placed at (off_h, off_w) of a zero tile:
    rows first (sum over h), then columns (sum over w), as two real matrix products each."""
    Cm, Sm = dft_mats()
    X = np.zeros((L, L))
    X[off_h:off_h + img.shape[0], off_w:off_w + img.shape[1]] = img
    Zr = Cm[:UH] @ X                               # Z[u][w] = sum_h X[h][w] exp(-2 pi i h u / 32)
    Zi = -Sm[:UH] @ X
    Yr = Zr @ Cm + Zi @ Sm                         # Y[u][v] = sum_w Z[u][w] exp(-2 pi i w v / 32)
    Yi = Zi @ Cm - Zr @ Sm
    return Yr, Yi


def tile_inverse(Yr, Yi):
    """Real 32 x 32 tile from its half spectrum: the full axis v first, then the halved axis
    u with weights 1, 2, ..., 2, 1 (the rows 17..31 are the conjugates of rows 15..1)."""
    Cm, Sm = dft_mats()
    Tr = Yr @ Cm - Yi @ Sm                         # T[u][q] = sum_v Y[u][v] exp(+2 pi i v q / 32)
    Ti = Yr @ Sm + Yi @ Cm
    wu = np.full(UH, 2.0)
    wu[0] = wu[16] = 1.0
    Gc = (Cm[:, :UH] * wu) / (L * L)               # [p][u]
    Gs = (-Sm[:, :UH] * wu) / (L * L)
    return Gc @ Tr + Gs @ Ti


def test_half_spectrum_is_numpys_rfft2_transposed_roles():
    x = synth.normal((L, L), 5).astype(np.float64)
    Yr, Yi = tile_spectrum(x, 0, 0)
    ref = np.fft.fft2(x)[:UH, :]
    assert np.allclose(Yr, ref.real, atol=1e-10) and np.allclose(Yi, ref.imag, atol=1e-10)
    assert np.allclose(tile_inverse(Yr, Yi), x, atol=1e-12)


def block_matrix(Ar, Ai):
    """Real form of a complex matrix A[m][d] acting on stacked (re, im) pairs: rows 2m + po,
    columns 2d + pi."""
    M, D = Ar.shape
    out = np.zeros((2 * M, 2 * D))
    out[0::2, 0::2] = Ar
    out[0::2, 1::2] = -Ai
    out[1::2, 0::2] = Ai
    out[1::2, 1::2] = Ar
    return out


def stack(Br, Bi):
    D, N = Br.shape
    out = np.zeros((2 * D, N))
    out[0::2] = Br
    out[1::2] = Bi
    return out


def filter_spectrum(w):
    """W[u][v] = sum_{r,s} w[r][s] exp(-2 pi i (u r + v s) / 32), u < 17, by the definition."""
    R, S = w.shape
    u = np.arange(UH)[:, None, None, None]
    v = np.arange(L)[None, :, None, None]
    r = np.arange(R)[None, None, :, None]
    s = np.arange(S)[None, None, None, :]
    th = 2.0 * np.pi * (u * r + v * s) / L
    return (w * np.cos(th)).sum((2, 3)), -(w * np.sin(th)).sum((2, 3))


def tensors(geom, seed):
    N, C, H, W, K, R, S = geom[:7]
    P, Q = oracle.output_dims(geom)
    x = synth.normal((N, C, H, W), seed)
    w = synth.normal((K, C, R, S), seed + 1, std=0.3)
    b = synth.uniform((K,), seed + 2, -0.5, 0.5)
    dy = synth.normal((N, K, P, Q), seed + 3)
    return x, w, b, dy, P, Q


@pytest.mark.parametrize("geom", GEOMS)
def test_forward_as_products_of_spectra(geom):
    N, C, H, W, K, R, S, _, _, ph, pw = geom
    x, w, b, _, P, Q = tensors(geom, 11)
    X = [[tile_spectrum(x[n, c].astype(np.float64), ph, pw) for n in range(N)] for c in range(C)]
    Wf = [[filter_spectrum(w[k, c].astype(np.float64)) for c in range(C)] for k in range(K)]
    y = np.zeros((N, K, P, Q))
    Mr = np.zeros((K, N, UH, L))
    Mi = np.zeros((K, N, UH, L))
    for u in range(UH):
        for v in range(L):
            # correlation: the conjugate of the filter's spectrum
            Ar = np.array([[Wf[k][c][0][u, v] for c in range(C)] for k in range(K)])
            Ai = np.array([[-Wf[k][c][1][u, v] for c in range(C)] for k in range(K)])
            Br = np.array([[X[c][n][0][u, v] for n in range(N)] for c in range(C)])
            Bi = np.array([[X[c][n][1][u, v] for n in range(N)] for c in range(C)])
            prod = block_matrix(Ar, Ai) @ stack(Br, Bi)          # rows 2k + po, columns n
            Mr[:, :, u, v] = prod[0::2]
            Mi[:, :, u, v] = prod[1::2]
    for n in range(N):
        for k in range(K):
            y[n, k] = tile_inverse(Mr[k, n], Mi[k, n])[:P, :Q] + b[k]
    ref = oracle.fwd(geom, x, w, b)
    assert np.abs(y - ref).max() <= 1e-5 * np.abs(ref).max()      # the oracle's tensors are fp32


@pytest.mark.parametrize("geom", GEOMS)
def test_backward_data_as_products_of_spectra(geom):
    N, C, H, W, K, R, S, _, _, ph, pw = geom
    _, w, _, dy, P, Q = tensors(geom, 21)
    DY = [[tile_spectrum(dy[n, k].astype(np.float64), 0, 0) for n in range(N)] for k in range(K)]
    Wf = [[filter_spectrum(w[k, c].astype(np.float64)) for c in range(C)] for k in range(K)]
    dx = np.zeros((N, C, H, W))
    for n in range(N):
        for c in range(C):
            # plain convolution: the spectra multiply without a conjugate
            Mr = sum(Wf[k][c][0] * DY[k][n][0] - Wf[k][c][1] * DY[k][n][1] for k in range(K))
            Mi = sum(Wf[k][c][0] * DY[k][n][1] + Wf[k][c][1] * DY[k][n][0] for k in range(K))
            dx[n, c] = tile_inverse(Mr, Mi)[ph:ph + H, pw:pw + W]  # gradient of the padded input, cropped
    ref = oracle.bwd_data(geom, dy, w)
    assert np.abs(dx - ref).max() <= 1e-5 * np.abs(ref).max()


@pytest.mark.parametrize("geom", GEOMS)
def test_backward_weight_as_products_of_spectra(geom):
    N, C, H, W, K, R, S, _, _, ph, pw = geom
    x, _, _, dy, P, Q = tensors(geom, 31)
    X = [[tile_spectrum(x[n, c].astype(np.float64), ph, pw) for n in range(N)] for c in range(C)]
    DY = [[tile_spectrum(dy[n, k].astype(np.float64), 0, 0) for n in range(N)] for k in range(K)]
    dw = np.zeros((K, C, R, S))
    db = np.zeros(K)
    for k in range(K):
        for c in range(C):
            # D = sum_n conj(dY) X, through the block form with the images as the depth
            Dr = np.zeros((UH, L))
            Di = np.zeros((UH, L))
            for u in range(UH):
                for v in range(L):
                    Ar = np.array([[DY[k][n][0][u, v] for n in range(N)]])
                    Ai = np.array([[-DY[k][n][1][u, v] for n in range(N)]])
                    Br = np.array([[X[c][n][0][u, v]] for n in range(N)])
                    Bi = np.array([[X[c][n][1][u, v]] for n in range(N)])
                    prod = block_matrix(Ar, Ai) @ stack(Br, Bi)
                    Dr[u, v], Di[u, v] = prod[0, 0], prod[1, 0]
            dw[k, c] = tile_inverse(Dr, Di)[:R, :S]
        db[k] = sum(DY[k][n][0][0, 0] for n in range(N))          # the zero frequency is the tile's sum
    ref_dw, ref_db = oracle.bwd_weight(geom, x, dy)
    assert np.abs(dw - ref_dw).max() <= 1e-5 * np.abs(ref_dw).max()
    assert np.abs(db - ref_db).max() <= 1e-5 * np.abs(ref_db).max()


def test_filter_gradient_taps_by_the_definition_of_the_inverse():
    """The filter gradient needs only R x S values of the inverse: summed tap by tap over the
    half spectrum with the weights 1, 2, ..., 2, 1 it equals the full inverse's corner."""
    x = synth.normal((L, L), 4).astype(np.float64)
    Yr, Yi = tile_spectrum(x, 0, 0)
    wu = np.full(UH, 2.0)
    wu[0] = wu[16] = 1.0
    u = np.arange(UH)[:, None]
    v = np.arange(L)[None, :]
    for r, s in ((0, 0), (1, 3), (4, 4), (6, 2)):
        th = 2.0 * np.pi * (u * r + v * s) / L
        val = (wu[:, None] * (Yr * np.cos(th) - Yi * np.sin(th))).sum() / (L * L)
        assert abs(val - x[r, s]) < 1e-11

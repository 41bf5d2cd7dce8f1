"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol,
and its host-side logic (shape maths, workspace sizing, argument validation)
behaves as include/mi355conv.h states.  No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

from paper_1606_04884_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "mi355conv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b((?:conv2d|apply)_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.load()
    names = declared_symbols()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_binding_has_same_names():
    for n in declared_symbols():
        assert callable(getattr(B, n))


@pytest.mark.parametrize("geom,pq", [
    ((128, 3, 224, 224, 64, 11, 11, 4, 4, 2, 2), (55, 55)),
    ((128, 3, 231, 231, 96, 11, 11, 4, 4, 0, 0), (56, 56)),
    ((128, 96, 24, 24, 256, 5, 5, 1, 1, 0, 0), (20, 20)),
    ((64, 512, 14, 14, 512, 3, 3, 1, 1, 1, 1), (14, 14)),
    ((1, 1, 7, 9, 1, 3, 2, 2, 3, 1, 0), (4, 3)),
])
def test_output_dims(geom, pq):
    assert B.conv2d_output_dims(geom) == pq


@pytest.mark.parametrize("geom", [
    (0, 3, 8, 8, 4, 3, 3, 1, 1, 1, 1), (1, 3, 8, 8, 4, 3, 3, 0, 1, 1, 1),
    (1, 3, 8, 8, 4, 3, 3, 1, 1, -1, 1), (1, 3, 2, 2, 4, 5, 5, 1, 1, 0, 0),
    (1, 3, 8, 8, 0, 3, 3, 1, 1, 1, 1), (1, 3, 20000, 8, 4, 3, 3, 1, 1, 1, 1),
    (4096, 1024, 64, 64, 4, 3, 3, 1, 1, 1, 1),      # x has 2^34 elements
])
def test_bad_geometry_is_refused(geom):
    with pytest.raises(B.Conv2dError) as e:
        B.conv2d_output_dims(geom)
    assert e.value.status == -2
    for op in (B.OP_FWD, B.OP_BWD_DATA, B.OP_BWD_WEIGHT):
        assert B.conv2d_workspace_bytes(geom, op) == 0


def test_null_and_workspace_errors_enqueue_nothing():
    lib = B.load()
    d = B.make_desc((2, 3, 16, 16, 8, 3, 3, 1, 1, 1, 1))
    assert lib.conv2d_fwd(None, 1, 1, None, 1, 1, 1 << 20, 0, None) == -1
    assert lib.conv2d_fwd(C.byref(d), None, 1, None, 1, 1, 1 << 20, 0, None) == -1
    assert lib.conv2d_bwd_data(C.byref(d), 1, None, 1, 1, 1 << 20, 0, None) == -1
    assert lib.conv2d_bwd_weight(C.byref(d), 1, 1, None, None, 1.0, 0, 1, 1 << 20, 0, None) == -1
    # workspace: missing, or one byte short
    for op, call in ((B.OP_FWD, lambda ws, n: lib.conv2d_fwd(C.byref(d), 1, 1, None, 1, ws, n, 0, None)),
                     (B.OP_BWD_DATA, lambda ws, n: lib.conv2d_bwd_data(C.byref(d), 1, 1, 1, ws, n, 0, None)),
                     (B.OP_BWD_WEIGHT, lambda ws, n: lib.conv2d_bwd_weight(C.byref(d), 1, 1, 1, None, 1.0, 0, ws, n, 0, None))):
        need = B.conv2d_workspace_bytes(d, op)
        assert need > 0
        assert call(None, need) == -4
        assert call(1, need - 1) == -4
    # unknown algorithm / Winograd on a geometry it cannot do
    assert lib.conv2d_fwd(C.byref(d), 1, 1, None, 1, 1, 1 << 20, 7, None) == -3
    d5 = B.make_desc((2, 3, 16, 16, 8, 5, 5, 1, 1, 2, 2))
    assert lib.conv2d_fwd(C.byref(d5), 1, 1, None, 1, 1, 1 << 30, B.ALGO_WINOGRAD, None) == -3
    d2 = B.make_desc((2, 3, 16, 16, 8, 3, 3, 2, 2, 1, 1))
    assert lib.conv2d_bwd_data(C.byref(d2), 1, 1, 1, 1, 1 << 30, B.ALGO_WINOGRAD, None) == -3
    assert B.conv2d_workspace_bytes(d5, B.OP_FWD, B.ALGO_WINOGRAD) == 0


def test_status_strings_and_version():
    seen = set()
    for s in (0, -1, -2, -3, -4, -5, -99):
        t = B.conv2d_status_string(s)
        assert t
        seen.add(t)
    assert len(seen) == 7
    assert "gfx950" in B.conv2d_version()


def test_pick_algo_is_consistent_with_workspace():
    for geom in ((64, 64, 56, 56, 64, 3, 3, 1, 1, 1, 1), (8, 3, 32, 32, 16, 5, 5, 2, 2, 2, 2)):
        for op in (B.OP_FWD, B.OP_BWD_DATA, B.OP_BWD_WEIGHT):
            algo = B.conv2d_pick_algo(geom, op)
            assert algo in (B.ALGO_IGEMM, B.ALGO_WINOGRAD)
            assert B.conv2d_workspace_bytes(geom, op, algo) == B.conv2d_workspace_bytes(geom, op, B.ALGO_AUTO)


def test_grouped_1x1_argument_checks():
    lib = B.load()
    vp = C.c_void_p
    d = B.make_desc((2, 8, 6, 6, 12, 1, 1, 1, 1, 0, 0))
    K = (C.c_int32 * 2)(4, 8)
    one = (vp * 2)(1, 1)
    need = B.conv2d_workspace_bytes(d, B.OP_FWD, B.ALGO_IGEMM)
    # null lists, bad group count, filter counts that do not add up, workspace too small
    assert lib.conv2d_fwd_1x1_group(C.byref(d), 1, 2, None, one, None, one, 1, need, None) == -1
    assert lib.conv2d_fwd_1x1_group(C.byref(d), 1, 0, K, one, None, one, 1, need, None) == -2
    assert lib.conv2d_fwd_1x1_group(C.byref(d), 1, 5, K, one, None, one, 1, need, None) == -2
    Kbad = (C.c_int32 * 2)(4, 4)
    assert lib.conv2d_fwd_1x1_group(C.byref(d), 1, 2, Kbad, one, None, one, 1, need, None) == -2
    assert lib.conv2d_fwd_1x1_group(C.byref(d), 1, 2, K, one, None, one, 1, need - 1, None) == -4
    nul = (vp * 2)(1, None)
    assert lib.conv2d_fwd_1x1_group(C.byref(d), 1, 2, K, nul, None, one, 1, need, None) == -1
    # not a 1x1 stride-1 unpadded layer
    d3 = B.make_desc((2, 8, 6, 6, 12, 3, 3, 1, 1, 1, 1))
    assert lib.conv2d_fwd_1x1_group(C.byref(d3), 1, 2, K, one, None, one, 1, 1 << 20, None) == -3


def test_apply_argument_checks():
    lib = B.load()
    assert lib.apply_mul_add(1, 1, -1, 1.0, 0.0, None) == -2
    assert lib.apply_mul_add(None, None, 0, 1.0, 0.0, None) == 0
    assert lib.apply_mul_add(None, 1, 8, 1.0, 0.0, None) == -1


def test_algo_choice_rules():
    """AUTO policy as the header states it: Winograd for 3x3 stride-1 layers with enough
    reduction channels whose gathered tensor fits 32-bit byte offsets, else implicit GEMM."""
    pick = B.conv2d_pick_algo
    vgg = (64, 128, 112, 112, 128, 3, 3, 1, 1, 1, 1)            # large map, few channels: fused F(2x2,3x3)
    assert pick(vgg, B.OP_FWD) == B.ALGO_WINOGRAD
    assert pick(vgg, B.OP_BWD_DATA) == B.ALGO_WINOGRAD
    assert pick(vgg, B.OP_BWD_WEIGHT) == B.ALGO_WINOGRAD
    deep = (64, 512, 28, 28, 512, 3, 3, 1, 1, 1, 1)             # many channels, small map: unfused F(4x4,3x3)
    assert pick(deep, B.OP_FWD) == B.ALGO_WINOGRAD4
    assert pick(deep, B.OP_BWD_DATA) == B.ALGO_WINOGRAD4
    # its workspace holds the transformed input and the products: 2.25 x input + 2.25 x output at least
    assert B.conv2d_workspace_bytes(deep, B.OP_FWD) > 2.25 * 4 * 2 * 64 * 512 * 28 * 28
    assert B.conv2d_workspace_bytes(deep, B.OP_FWD, B.ALGO_WINOGRAD) < 64 << 20
    first = (64, 3, 224, 224, 64, 3, 3, 1, 1, 1, 1)              # 3 input channels
    assert pick(first, B.OP_FWD) == B.ALGO_IGEMM                # taps kernel: the filter bank in LDS
    assert pick((64, 6, 224, 224, 64, 3, 3, 1, 1, 1, 1), B.OP_FWD) == B.ALGO_WINOGRAD   # tile-pair kernel, one ragged chunk
    assert pick((64, 3, 224, 224, 160, 3, 3, 1, 1, 1, 1), B.OP_FWD) == B.ALGO_WINOGRAD  # too many filters for the taps kernel
    assert pick(first, B.OP_BWD_DATA) == B.ALGO_IGEMM
    assert pick(first, B.OP_BWD_WEIGHT) == B.ALGO_IGEMM
    assert pick((64, 3, 225, 225, 64, 3, 3, 1, 1, 1, 1), B.OP_FWD) == B.ALGO_IGEMM      # odd width: no pairs
    assert pick((64, 3, 224, 224, 16, 3, 3, 1, 1, 1, 1), B.OP_FWD) == B.ALGO_IGEMM      # few filters
    assert B.conv2d_workspace_bytes((64, 3, 225, 225, 64, 3, 3, 1, 1, 1, 1), B.OP_FWD, B.ALGO_WINOGRAD) == 0
    five = (128, 64, 27, 27, 192, 5, 5, 1, 1, 2, 2)            # 5x5 on a map that fits one 32x32 tile: four 3x3
    for op in (B.OP_FWD, B.OP_BWD_DATA, B.OP_BWD_WEIGHT):      # sub-filters, fused or unfused, or the product of spectra
        assert pick(five, op) in (B.ALGO_WINOGRAD, B.ALGO_WINOGRAD4, B.ALGO_FFT)
        assert B.conv2d_workspace_bytes(five, op, B.ALGO_WINOGRAD) > 0
        assert B.conv2d_workspace_bytes(five, op, B.ALGO_WINOGRAD4) > 0
        assert B.conv2d_workspace_bytes(five, op, B.ALGO_FFT) > 0
    big5 = (16, 64, 56, 56, 64, 5, 5, 1, 1, 2, 2)              # the same filter on a larger map: never the spectra
    for op in (B.OP_FWD, B.OP_BWD_DATA, B.OP_BWD_WEIGHT):
        assert pick(big5, op) in (B.ALGO_WINOGRAD, B.ALGO_WINOGRAD4)
        assert B.conv2d_workspace_bytes(big5, op, B.ALGO_FFT) == 0
    assert pick((128, 16, 28, 28, 32, 5, 5, 1, 1, 2, 2), B.OP_FWD) != B.ALGO_FFT          # a handful of channels
    small5 = (128, 32, 27, 27, 64, 5, 5, 1, 1, 2, 2)           # few channels: the fused kernels
    assert pick(small5, B.OP_FWD) == B.ALGO_WINOGRAD
    assert pick((8, 64, 20, 20, 64, 4, 4, 1, 1, 1, 1), B.OP_FWD) == B.ALGO_IGEMM          # 4x4: no saving
    assert pick((8, 64, 20, 20, 64, 7, 7, 1, 1, 3, 3), B.OP_FWD) == B.ALGO_IGEMM          # above 6x6
    assert pick((8, 64, 56, 56, 64, 3, 3, 2, 2, 1, 1), B.OP_FWD) == B.ALGO_IGEMM          # stride 2
    # strided first layers whose filter spans 3 x 3 strides: the backward passes go through a
    # rearrangement into a stride-1 3x3 layer over stride^2 * C channels (Winograd), which
    # needs K % 8 (backward-data) / K % 32 (backward-weight) like every Winograd layer; the
    # forward pass takes that route only on request
    alex1 = (128, 3, 224, 224, 64, 11, 11, 4, 4, 2, 2)
    assert pick(alex1, B.OP_FWD) == B.ALGO_IGEMM
    assert B.conv2d_workspace_bytes(alex1, B.OP_FWD, B.ALGO_WINOGRAD) > 128 * 48 * 57 * 57 * 4
    for op in (B.OP_BWD_DATA, B.OP_BWD_WEIGHT):
        assert pick(alex1, op) == B.ALGO_WINOGRAD
        # room for the rearranged tensor (128 x 48.. x 57 x 57 floats) on top of the inner workspace
        assert B.conv2d_workspace_bytes(alex1, op, B.ALGO_AUTO) > 128 * 48 * 57 * 57 * 4
    odd_k = (4, 3, 67, 67, 20, 11, 11, 4, 4, 2, 2)
    assert B.conv2d_workspace_bytes(odd_k, B.OP_FWD, B.ALGO_WINOGRAD) > 0
    assert pick(odd_k, B.OP_BWD_DATA) == B.ALGO_IGEMM
    assert pick(odd_k, B.OP_BWD_WEIGHT) == B.ALGO_IGEMM
    assert B.conv2d_workspace_bytes(odd_k, B.OP_BWD_DATA, B.ALGO_WINOGRAD) == 0
    assert pick((4, 3, 40, 40, 32, 5, 5, 2, 2, 2, 2), B.OP_BWD_DATA) == B.ALGO_WINOGRAD    # 5x5 stride 2
    assert pick((4, 3, 40, 40, 32, 7, 7, 2, 2, 3, 3), B.OP_BWD_DATA) == B.ALGO_IGEMM       # 4 x 4 strides
    assert pick((4, 64, 40, 40, 32, 5, 5, 2, 2, 2, 2), B.OP_BWD_DATA) == B.ALGO_IGEMM      # many channels: not by default
    assert B.conv2d_workspace_bytes((4, 64, 40, 40, 32, 5, 5, 2, 2, 2, 2), B.OP_BWD_DATA, B.ALGO_WINOGRAD) > 0
    assert pick((4, 3, 40, 40, 32, 5, 5, 2, 1, 2, 2), B.OP_BWD_DATA) == B.ALGO_IGEMM       # unequal strides
    big = (256, 64, 224, 224, 64, 3, 3, 1, 1, 1, 1)             # x and y are 3.3 GB each
    for op in (B.OP_FWD, B.OP_BWD_DATA, B.OP_BWD_WEIGHT):
        assert pick(big, op) == B.ALGO_IGEMM
        assert B.conv2d_workspace_bytes(big, op, B.ALGO_WINOGRAD) == 0

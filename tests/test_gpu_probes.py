"""The measurement helpers of the library, through the binding: the copy / fill probe moves
exactly the bytes it is given (whole 1024-vector spans, the ragged rest, sizes below one
span) and nothing beside them; the MFMA probe reports the flops of its launch shape; the
per-launch profile names the kernel a call ran and gives it a duration."""
import pytest

from paper_1606_04884_amd import binding as B
from paper_1606_04884_amd import synth

pytestmark = pytest.mark.gpu

GUARD = 64          # floats on either side of the probed range that must stay as they were

# floats (multiples of 4): below one span, exactly one span, spans + ragged rest, many spans per
# workgroup slot of the largest grid + rest
SIZES = [4, 1000, 4096, 4096 * 3 + 2800, 4096 * 70000 + 12]


@pytest.mark.parametrize("n", SIZES)
def test_probe_copy_moves_exactly_its_range(n):
    import torch
    dev = torch.device("cuda:0")
    # any distinct values do: the probe is not part of the method (exact in fp32 below 2^24, merely
    # deterministic above)
    src = torch.arange(n, device=dev, dtype=torch.float32)
    buf = torch.full((n + 2 * GUARD,), -3.0, device=dev)
    dst = buf[GUARD:GUARD + n]
    assert dst.data_ptr() % 16 == 0
    B.conv2d_probe_copy(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    assert bool((buf[:GUARD] == -3.0).all()) and bool((buf[GUARD + n:] == -3.0).all())


@pytest.mark.parametrize("n", SIZES)
def test_probe_fill_writes_exactly_its_range(n):
    import torch
    dev = torch.device("cuda:0")
    buf = torch.full((n + 2 * GUARD,), -3.0, device=dev)
    dst = buf[GUARD:GUARD + n]
    B.conv2d_probe_copy(None, dst)
    torch.cuda.synchronize()
    assert bool((dst == 1.0).all())
    assert bool((buf[:GUARD] == -3.0).all()) and bool((buf[GUARD + n:] == -3.0).all())


def test_probe_copy_rejects_ragged_and_misaligned():
    import torch
    dev = torch.device("cuda:0")
    a = torch.zeros(64, device=dev)
    b = torch.zeros(64, device=dev)
    with pytest.raises(B.Conv2dError):
        B.conv2d_probe_copy(a[:6], b[:6])           # not a multiple of 4 floats
    with pytest.raises(B.Conv2dError):
        B.conv2d_probe_copy(a[1:9], b[0:8])         # source not 16-byte aligned


def test_probe_mfma_reports_its_flops():
    import torch
    dev = torch.device("cuda:0")
    sink = torch.zeros(1, device=dev)
    iters = 10
    flops = B.conv2d_probe_mfma_f32(sink, iters)
    torch.cuda.synchronize()
    # 512 workgroups x 4 waves x iters x 32 instructions of 32x32x2 (2 flops per multiply-add)
    assert flops == 512 * 4 * iters * 32 * (2 * 32 * 32 * 2)
    assert float(sink[0]) == 0.0                      # the sink is never written


def test_profile_records_the_kernel_of_a_call():
    import torch
    dev = torch.device("cuda:0")
    geom = (4, 64, 28, 28, 64, 3, 3, 1, 1, 1, 1)
    N, Cc, H, W, K, R, S = geom[:7]
    P, Q = B.conv2d_output_dims(geom)
    x = torch.from_numpy(synth.normal((N, Cc, H, W), 5)).to(dev)
    w = torch.from_numpy(synth.normal((K, Cc, R, S), 6, std=0.05)).to(dev)
    y = torch.empty((N, K, P, Q), device=dev)
    d = B.make_desc(geom)
    ws = torch.empty(max(256, B.conv2d_workspace_bytes(d, B.OP_FWD, B.ALGO_WINOGRAD)), dtype=torch.uint8, device=dev)
    B.conv2d_fwd(d, x, w, None, y, ws, B.ALGO_WINOGRAD)          # unprofiled reference run
    torch.cuda.synchronize()
    y_ref = y.clone()
    y.zero_()
    B.conv2d_profile_begin(16)
    B.conv2d_fwd(d, x, w, None, y, ws, B.ALGO_WINOGRAD)
    torch.cuda.synchronize()
    n = B.conv2d_profile_end()
    assert n >= 1
    names = []
    for i in range(n):
        kid, flops, nbytes, ms = B.conv2d_profile_record(i)
        names.append(B.conv2d_profile_kernel_name(kid))
        assert ms > 0.0 and (flops > 0.0 or nbytes > 0.0)
    assert any(nm.startswith("wino_") for nm in names), names
    assert torch.equal(y, y_ref)                      # profiling changes no result

"""Per-element kernel (Sec. 3.3 experiment) against its oracle: bit-exact, for sizes
around the vector width and the launch geometry, unaligned views and in place."""
import numpy as np
import pytest

import oracle
from paper_1606_04884_amd import binding as B
from paper_1606_04884_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n", [0, 1, 3, 4, 5, 255, 256, 1023, 1024, 4099, 65536 + 7, 1 << 20, 3 * (1 << 20) + 1,
                               (1 << 24) + 13])
def test_apply_mul_add_bit_exact(n):
    import torch
    dev = torch.device("cuda:0")
    x = synth.normal((n,), 900 + (n % 1000)) if n else np.zeros((0,), dtype=np.float32)
    a, b = 1.7320508, -0.3333333
    tx = torch.from_numpy(x).to(dev)
    ty = torch.full((n,), float("nan"), device=dev)
    print("n", n, flush=True)
    B.apply_mul_add(tx, ty, a, b)
    torch.cuda.synchronize()
    assert np.array_equal(ty.cpu().numpy(), oracle.apply_mul_add(x, a, b))


def test_apply_unaligned_and_in_place():
    import torch
    dev = torch.device("cuda:0")
    n = 10007
    x = synth.normal((n + 3,), 77)
    base = torch.from_numpy(x).to(dev)
    out = torch.full((n + 5,), float("nan"), device=dev)
    # views starting 4 and 12 bytes into their allocations: the scalar path
    B.apply_mul_add(base[1:n + 1], out[3:n + 3], 4097.0, -16785408.0)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.array_equal(got[3:n + 3], oracle.apply_mul_add(x[1:n + 1], 4097.0, -16785408.0))
    assert np.isnan(got[:3]).all() and np.isnan(got[n + 3:]).all()
    # in place
    t = torch.from_numpy(x).to(dev)
    B.apply_mul_add(t, t, -2.5, 0.125)
    torch.cuda.synchronize()
    assert np.array_equal(t.cpu().numpy(), oracle.apply_mul_add(x, -2.5, 0.125))


def test_apply_two_roundings_not_fused():
    import torch
    dev = torch.device("cuda:0")
    x = np.full((1024,), 4097.0, dtype=np.float32)
    t = torch.from_numpy(x).to(dev)
    y = torch.empty_like(t)
    B.apply_mul_add(t, y, 4097.0, -16785408.0)
    torch.cuda.synchronize()
    assert (y.cpu().numpy() == 0.0).all()       # a fused multiply-add would give 1

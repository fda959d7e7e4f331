"""GPU parity of tg_saxpy (axpy of Sec. 5.2: z = alpha.x + y) against the CPU oracle.

The kernel computes one fused multiply-add per element, i.e. the exact alpha*x+y rounded once
to fp32; the oracle value is exact to 2^-53.  The bar is therefore half an fp32 ulp of the
result, |z - z_ref| <= 2^-24 |z_ref| (plus the fp64 slack), and bit-exactness on
integer-valued inputs.
"""
import numpy as np
import pytest

import paper_1904_03383_amd as tg
from paper_1904_03383_amd import inputgen as ig

from gpu_common import say, to_dev

pytestmark = pytest.mark.gpu

HALF_ULP = 2.0 ** -24


def _check(alpha, x, y, z, exact=False):
    from oracle import oracle
    ref = oracle.saxpy_f64(alpha, x, y)
    assert z.shape == ref.shape and z.dtype == np.float32
    if z.size == 0:
        return
    if exact:
        assert np.array_equal(z, ref.astype(np.float32))
    err = np.abs(z.astype(np.float64) - ref)
    bound = HALF_ULP * np.abs(ref) * (1 + 1e-9) + 2.0 ** -149
    worst = int(np.argmax(err - bound))
    assert np.all(err <= bound), (worst, z[worst], ref[worst])


@pytest.mark.parametrize("n", [0, 1, 3, 4, 5, 255, 256, 1023, 4099, 1 << 20, (1 << 22) + 7])
def test_saxpy_sizes(n):
    import torch
    say(f"saxpy n={n}")
    x, y = ig.normal(501, (n,)), ig.uniform(502, (n,))
    out = torch.full((n,), float("nan"), device="cuda")
    tg.saxpy(1.7, to_dev(x), to_dev(y), out=out)
    torch.cuda.synchronize()
    _check(1.7, x, y, out.cpu().numpy())
    xi, yi = ig.small_int(503, (n,), -50, 50), ig.small_int(504, (n,), -999, 999)
    zi = tg.saxpy(-3.0, to_dev(xi), to_dev(yi))
    torch.cuda.synchronize()
    _check(-3.0, xi, yi, zi.cpu().numpy(), exact=True)


def test_saxpy_paper_size_2_pow_26():
    """n = 2^26, the size of the paper's axpy experiment (Table 1)."""
    import torch
    n = 1 << 26
    say(f"saxpy n=2^26")
    x, y = ig.uniform(505, (n,)), ig.normal(506, (n,))
    z = tg.saxpy(0.37, to_dev(x), to_dev(y))
    torch.cuda.synchronize()
    _check(0.37, x, y, z.cpu().numpy())


def test_saxpy_in_place_and_unaligned():
    import torch
    n = 100003
    say("saxpy in place / unaligned")
    x, y = ig.normal(507, (n,)), ig.normal(508, (n,))
    dy = to_dev(y)
    tg.saxpy(2.5, to_dev(x), dy, out=dy)          # z aliases y
    torch.cuda.synchronize()
    _check(2.5, x, y, dy.cpu().numpy())
    dx = to_dev(x)
    tg.saxpy(-0.75, dx, to_dev(y), out=dx)        # z aliases x
    torch.cuda.synchronize()
    _check(-0.75, x, y, dx.cpu().numpy())
    # vectors that start 4 bytes off a 16-byte boundary take the scalar path
    bx, by, bz = to_dev(np.concatenate([[0], x]).astype(np.float32)), to_dev(np.concatenate([[0], y]).astype(np.float32)), torch.zeros(n + 1, device="cuda")
    tg.saxpy(1.25, bx[1:], by[1:], out=bz[1:])
    torch.cuda.synchronize()
    assert bz[0].item() == 0.0
    _check(1.25, x, y, bz[1:].cpu().numpy())


def test_saxpy_special_alphas():
    import torch
    n = 5000
    say("saxpy alpha = 0, 1, -1")
    x, y = ig.normal(509, (n,)), ig.normal(510, (n,))
    dx, dy = to_dev(x), to_dev(y)
    assert torch.equal(tg.saxpy(0.0, dx, dy), dy)
    assert torch.equal(tg.saxpy(1.0, dx, torch.zeros_like(dx)), dx)
    assert torch.all(tg.saxpy(-1.0, dx, dx) == 0)

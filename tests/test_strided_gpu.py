"""GPU parity of tg_sgemm_strided against the CPU oracle: the paper's strided matmul (Sec. 5.2:
1024^3 with consecutive elements of A 32 apart), transposed / column-major operands, odd strides
and ragged sizes.  Same bar as the plain product: per element 1e-5 * sum|a||b|, relative
Frobenius 1e-6, integer-valued inputs bit exact."""
import numpy as np
import pytest

import paper_1904_03383_amd as tg
from paper_1904_03383_amd import inputgen as ig

from gpu_common import check_against_oracle, say, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _clean_library_state():
    tg.force_config(None)
    tg.set_workspace(None)
    yield
    tg.force_config(None)
    tg.set_workspace(None)


def _run(da, db, m, n):
    import torch
    out = torch.full((m, n), float("nan"), device="cuda")
    tg.sgemm_strided(da, db, out=out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def test_paper_strided_matmul_1024_stride_32():
    """matmul 1024x1024x1024 with A's consecutive elements stored with a stride of 32 (Sec. 5.2)."""
    say("strided matmul 1024^3, A element stride 32")
    m = n = k = 1024
    for dist in ("uniform", "int"):
        gen = ig.uniform if dist == "uniform" else ig.small_int
        a_store = gen(601, (m, k * 32))
        b = gen(602, (k, n))
        a = a_store[:, ::32]
        c = _run(to_dev(a_store)[:, ::32], to_dev(b), m, n)
        assert "_edge" in tg.last_config()
        check_against_oracle(c, np.ascontiguousarray(a), b, exact=(dist == "int"), what="strided 1024^3 " + dist)


LAYOUTS = ["A^T", "B^T", "A^T B^T", "csa3", "csb5", "csa2 csb7", "rsa wide"]


@pytest.mark.parametrize("layout", LAYOUTS)
@pytest.mark.parametrize("shape", [(256, 192, 160), (131, 77, 53), (1, 9, 300), (70, 1, 5)], ids=str)
def test_strided_and_transposed_layouts(layout, shape):
    m, n, k = shape
    say(f"layout {layout} shape {shape}")
    for dist in ("normal", "int"):
        gen = ig.normal if dist == "normal" else ig.small_int
        if "A^T" in layout:                       # A stored column-major: a = store.T
            a_store = gen(611, (k, m + 3))
            a_np, da = a_store[:, :m].T, to_dev(a_store)[:, :m].T
        elif "csa" in layout:
            cs = int(layout.split("csa")[1].split()[0])
            a_store = gen(611, (m, k * cs + 1))
            a_np, da = a_store[:, :k * cs:cs], to_dev(a_store)[:, :k * cs:cs]
        elif layout == "rsa wide":
            a_store = gen(611, (m, 2 * k + 5))
            a_np, da = a_store[:, :k], to_dev(a_store)[:, :k]
        else:
            a_store = gen(611, (m, k))
            a_np, da = a_store, to_dev(a_store)
        if "B^T" in layout:                       # B stored column-major
            b_store = gen(612, (n, k + 2))
            b_np, db = b_store[:, :k].T, to_dev(b_store)[:, :k].T
        elif "csb" in layout:
            cs = int(layout.split("csb")[1].split()[0])
            b_store = gen(612, (k, n * cs))
            b_np, db = b_store[:, ::cs], to_dev(b_store)[:, ::cs]
        else:
            b_store = gen(612, (k, n))
            b_np, db = b_store, to_dev(b_store)
        assert da.shape == (m, k) and db.shape == (k, n)
        c = _run(da, db, m, n)
        check_against_oracle(c, np.ascontiguousarray(a_np), np.ascontiguousarray(b_np), exact=(dist == "int"),
                             what=f"{layout} {shape} {dist}")


def test_column_major_output_via_swapped_operands():
    """A column-major C = A.B is C^T = B^T.A^T in row-major terms: swap operands, exchange strides."""
    import torch
    say("column-major C through swapped operands")
    m, n, k = 96, 80, 64
    a = ig.small_int(621, (m, k))
    b = ig.small_int(622, (k, n))
    da, db = to_dev(a), to_dev(b)
    ct = torch.full((n, m), float("nan"), device="cuda")            # row-major n x m  ==  column-major m x n
    tg.sgemm_strided(db.T, da.T, out=ct)
    torch.cuda.synchronize()
    check_against_oracle(ct.cpu().numpy().T.copy(), a, b, exact=True, what="column-major C")


def test_unit_strides_take_the_plain_path():
    import torch
    say("strided entry point with unit strides")
    a, b = ig.make_operands(1, 256, 256, 128, "int", 631, 632)
    da, db = to_dev(a[0]), to_dev(b[0])
    c1 = tg.sgemm_strided(da, db)
    cfg = tg.last_config()
    c2 = tg.sgemm(da, db)
    torch.cuda.synchronize()
    assert cfg == tg.last_config() and "_edge" not in cfg
    assert torch.equal(c1, c2)


@pytest.mark.parametrize("forced", ["t128x128x16_w64x64_edge", "t64x64x16_w32x32_edge", "t128x128x16_w64x64_acc2_edge"])
def test_strided_through_each_predicated_kernel(forced):
    say(f"strided forced {forced}")
    m, n, k = 200, 150, 1100 if "acc2" in forced else 90
    a_store = ig.small_int(641, (m, k * 4))
    b_store = ig.small_int(642, (n, k))
    tg.force_config(forced)
    c = _run(to_dev(a_store)[:, ::4], to_dev(b_store).T, m, n)
    check_against_oracle(c, np.ascontiguousarray(a_store[:, ::4]), np.ascontiguousarray(b_store.T), exact=True, what=forced)

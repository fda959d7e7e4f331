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
        assert "_ga" in tg.last_config() and "+pack" not in tg.last_config()      # gathered inside the product kernel
        check_against_oracle(c, np.ascontiguousarray(a), b, exact=(dist == "int"), what="strided 1024^3 " + dist)
        tg.force_config("t64x64x16_w32x32_edge")                                   # and through the predicated kernel
        c = _run(to_dev(a_store)[:, ::32], to_dev(b), m, n)
        assert "_edge" in tg.last_config()
        tg.force_config(None)
        check_against_oracle(c, np.ascontiguousarray(a), b, exact=(dist == "int"), what="strided 1024^3 predicated " + dist)


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


# ---- packed path: with a workspace, strided operands are gathered once and the unit-stride kernels run ----

def _with_workspace(m, n, k, csa, csb, extra=0):
    import torch
    nbytes = tg.strided_workspace_bytes(m, n, k, csa, csb) + extra
    ws = torch.full((max(nbytes // 4, 4),), float("nan"), device="cuda")
    tg.set_workspace(ws)
    return ws


def test_paper_strided_matmul_1024_packed():
    """Sec. 5.2 strided matmul through the packing pass (a forced plain kernel cannot read the strided A itself):
    A is gathered once into the workspace (+packA), then that kernel runs on the copy."""
    say("strided matmul 1024^3, A element stride 32, packed")
    m = n = k = 1024
    ws = _with_workspace(m, n, k, 32, 1)
    tg.force_config("d64x64x32_w32x32")
    for dist in ("uniform", "int"):
        gen = ig.uniform if dist == "uniform" else ig.small_int
        a_store = gen(651, (m, k * 32))
        b = gen(652, (k, n))
        c = _run(to_dev(a_store)[:, ::32], to_dev(b), m, n)
        cfg = tg.last_config()
        assert cfg.endswith("+packA") and "_edge" not in cfg, cfg
        check_against_oracle(c, np.ascontiguousarray(a_store[:, ::32]), b, exact=(dist == "int"), what="packed strided 1024^3 " + dist)
    del ws


PACK_CASES = [
    # (m, n, k, layout of A, layout of B, expected suffix)
    (512, 384, 256, "T", "N", "+packA"),
    (512, 384, 256, "N", "T", "+packB"),
    (512, 384, 256, "T", "T", "+packAB"),
    (300, 257, 131, "T", "T", "+packAB"),        # ragged: partial 64 x 64 pack tiles, k padded to 132
    (200, 1000, 70, "s3", "N", "+packA"),
    (1000, 200, 70, "N", "s5", "+packB"),
    (1000, 100, 70, "s3", "s5", "+packB"),        # n <= 128: A is fetched by one tile column only, stays strided
    (100, 100, 70, "s3", "s5", ""),               # nothing is re-fetched: no packing at all
]


def _operand(gen, seed, rows, cols, layout):
    if layout == "T":
        store = gen(seed, (cols, rows + 3))
        return store[:, :rows].T, to_dev(store)[:, :rows].T
    if layout.startswith("s"):
        cs = int(layout[1:])
        store = gen(seed, (rows, cols * cs + 1))
        return store[:, :cols * cs:cs], to_dev(store)[:, :cols * cs:cs]
    store = gen(seed, (rows, cols))
    return store, to_dev(store)


@pytest.mark.parametrize("case", PACK_CASES, ids=str)
def test_packed_operands(case):
    m, n, k, la, lb, suffix = case
    say(f"packed {case}")
    csa = 1 if la == "N" else 7
    csb = 1 if lb == "N" else 7
    ws = _with_workspace(m, n, k, csa, csb)
    for dist in ("normal", "int"):
        gen = ig.normal if dist == "normal" else ig.small_int
        a_np, da = _operand(gen, 661, m, k, la)
        b_np, db = _operand(gen, 662, k, n, lb)
        c = _run(da, db, m, n)
        cfg = tg.last_config()
        if suffix:
            assert cfg.endswith(suffix), cfg
        else:
            assert "+pack" not in cfg, cfg
        check_against_oracle(c, np.ascontiguousarray(a_np), np.ascontiguousarray(b_np), exact=(dist == "int"), what=f"{case} {dist}")
    del ws


def test_packed_path_with_split_k_shares_the_workspace():
    """Packed copies sit in front of the split-K partials; a forced split must still fit and be right."""
    say("packed + split-K")
    m, n, k = 256, 256, 1024
    ws = _with_workspace(m, n, k, 1, 1, extra=4 * (m * k + 4 * m * n))
    a_np, da = _operand(ig.small_int, 671, m, k, "T")
    b = ig.small_int(672, (k, n))
    tg.force_config("t128x128x16_w64x64:s4")
    c = _run(da, to_dev(b), m, n)
    assert tg.last_config().endswith("+packA") and ":s4" in tg.last_config()
    check_against_oracle(c, np.ascontiguousarray(a_np), b, exact=True, what="packed + split-K")
    del ws


def test_workspace_too_small_for_packing_falls_back_to_gather():
    import torch
    say("strided with a workspace too small to pack")
    m, n, k = 256, 256, 128
    ws = torch.empty((1024,), device="cuda")
    tg.set_workspace(ws)
    a_np, da = _operand(ig.small_int, 681, m, k, "T")
    b = ig.small_int(682, (k, n))
    c = _run(da, to_dev(b), m, n)
    assert "+pack" not in tg.last_config()
    check_against_oracle(c, np.ascontiguousarray(a_np), b, exact=True, what="no room to pack")
    del ws


def test_with_room_to_pack_the_cost_model_picks_between_gathering_and_packing():
    """A gather asks for each strided element once per tile that uses it, the packing pass once in all.  With a
    workspace the cost model compares the two: a strided A stays fused (the paper's 1024^3, and 2048x2048x512 where
    a row panel asks for every element once or twice: 52 us against 64 us packed), a strided B, which no variant
    gathers that sparingly, is packed first (1024^3 at stride 32: 48 us against 78 us).  All must match the oracle
    on sampled rows."""
    import torch
    for (m, n, k, sa, sb, want) in ((1024, 1024, 1024, 32, 1, "_ga"), (2048, 2048, 512, 32, 1, "_ga"), (1024, 1024, 1024, 1, 32, "+packB")):
        say(f"strided {m}x{n}x{k}, element strides {sa} / {sb}, workspace set: expecting {want}")
        ws = _with_workspace(m, n, k, sa, sb, extra=tg.workspace_bytes(1, m, n, k))
        a_store = ig.small_int(691, (m, k * sa))
        b_store = ig.small_int(692, (k, n * sb))
        c = _run(to_dev(a_store)[:, ::sa], to_dev(b_store)[:, ::sb], m, n)
        cfg = tg.last_config()
        assert want in cfg and "_edge" not in cfg and ("+pack" in cfg) == want.startswith("+pack"), cfg
        rows = np.arange(0, m, 37)
        a = np.ascontiguousarray(a_store[:, ::sa])
        check_against_oracle(c[rows], a[rows], np.ascontiguousarray(b_store[:, ::sb]), exact=True,
                             what=f"strided {m}x{n}x{k} ({sa}, {sb}) with workspace")
        tg.set_workspace(None)
        del ws

"""GPU parity of the kernel variants that read transposed or element-strided operands as they lie (no
workspace, no separate gather / transpose pass): the paper's strided matmul (Sec. 5.2: 1024^3 with
consecutive elements of A 32 apart) and its transposed layouts, through tg_sgemm_strided.  Every variant
is forced by name on shapes that span several tiles with ragged last tiles, and on a long K (second
accumulation level); the automatic choice is checked to take them.  Same bar as the plain product: per
element 1e-5 * sum|a||b|, relative Frobenius 1e-6, integer-valued inputs bit exact."""
import re

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


def _mode_variants():
    return [n for n in tg.kernel_names() if re.search(r"_(ta|tb|ga|gb)(_|$)", n)]


def _tile(name):
    bm, bn, bk = (int(x) for x in re.match(r"[a-z](\d+)x(\d+)x(\d+)_", name).groups())
    return bm, bn, bk


def _operand(gen, seed, rows, cols, layout, stride=3):
    """(host view, device view) of a rows x cols operand: 'N' row-major, 'T' stored transposed with 16-byte
    aligned columns, 'S' element stride `stride` along its rows (and a row stride that is no multiple of it)."""
    if layout == "T":
        ld = (rows + 3) // 4 * 4 + 4
        store = gen(seed, (cols, ld))
        return store[:, :rows].T, to_dev(store)[:, :rows].T
    if layout == "S":
        store = gen(seed, (rows, cols * stride + 5))
        return store[:, :cols * stride:stride], to_dev(store)[:, :cols * stride:stride]
    store = gen(seed, (rows, cols))
    return store, to_dev(store)


def _layouts_of(name):
    la = "T" if "_ta" in name else ("S" if "_ga" in name else "N")
    lb = "T" if "_tb" in name else ("S" if "_gb" in name else "N")
    return la, lb


def _run(da, db, m, n):
    import torch
    out = torch.full((m, n), float("nan"), device="cuda")
    tg.sgemm_strided(da, db, out=out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def test_variant_list_is_not_empty():
    names = _mode_variants()
    assert len(names) >= 12 and any("_ga" in n for n in names) and any("_ta_tb" in n for n in names)


@pytest.mark.parametrize("name", [pytest.param(n, id=n) for n in (
    # listed literally so that collection does not need the library; checked against the table below
    "d64x64x32_w32x32_acc2_st4_ga", "d32x128x32_w32x32_acc2_st4_ga", "d128x128x32_w64x64_acc2_st3_ga",
    "d128x256x32_w64x128_acc2_st3_ga", "d64x64x32_w32x32_acc2_ta", "d128x128x32_w64x64_acc2_ta",
    "d128x256x32_w64x128_acc2_ta", "d64x64x32_w32x32_acc2_tb", "d128x128x32_w64x64_acc2_tb",
    "d128x256x32_w64x128_acc2_tb", "d64x64x32_w32x32_acc2_ta_tb", "d128x128x32_w64x64_acc2_ta_tb",
    "d128x256x32_w64x128_acc2_ta_tb", "d64x64x32_w32x32_acc2_st4_gb", "d128x128x32_w64x64_acc2_st3_gb",
    "d64x64x32_w32x32_acc2_st4_ga_gb", "d128x128x32_w64x64_acc2_st3_ga_gb", "d64x64x32_w32x32_acc2_st4_ga_tb",
    "d128x128x32_w64x64_acc2_st3_ga_tb", "d64x64x32_w32x32_acc2_st4_ta_gb", "d128x128x32_w64x64_acc2_st3_ta_gb",
    "d16x256x32_w16x64_acc2_st4_ga", "d16x256x32_w16x64_acc2_st3_ga",
    "g16x1024x64_w16x128_acc2_ga", "g16x512x64_w16x128_acc2_ga", "g32x512x64_w32x128_acc2_ga", "g32x1024x64_w32x128_ga",
    "g32x512x64_w32x64_acc2_ga", "g16x512x64_w16x64_acc2_ga", "g16x256x64_w16x64_acc2_ga",
    "g32x512x64_w32x64_acc2_b3_ga", "g16x512x64_w16x64_acc2_b3_ga", "g16x256x64_w16x64_acc2_b3_ga",
    "g32x512x128_w32x64_acc2_b3_ga", "g16x256x128_w16x64_acc2_b3_ga", "g32x512x256_w32x64_acc2_b3_ga",
    "d64x64x32_w32x32_acc2_tf_ta", "d64x64x32_w32x32_acc2_tf_tb", "d64x64x32_w32x32_acc2_tf_ta_tb",
    "d64x64x32_w32x32_acc2_tf_ga", "d64x64x32_w32x32_acc2_tf_gb")])
def test_every_variant_forced(name):
    assert name in _mode_variants()
    bm, bn, bk = _tile(name)
    la, lb = _layouts_of(name)
    # several tiles with ragged last ones (a transposed A needs m % 4 == 0, a plain B n % 4 == 0; the others take
    # anything), K of a few tiles (fewer than the LDS ring is deep for one of them), and one long K
    m_odd = 0 if la == "T" else 1
    n_odd = 0 if lb == "N" else 1
    shapes = [(2 * bm + 40 + m_odd, bn + 36 + n_odd, 5 * bk), (bm + 4, 2 * bn, bk)]
    if "_acc2" in name:     # (one accumulation level: K ranges up to 1024 only)
        shapes.append((bm, bn, 65 * bk))
    for (m, n, k) in shapes:
        for dist in ("normal", "int"):
            say(f"forced {name} {m}x{n}x{k} A:{la} B:{lb} {dist}")
            gen = ig.normal if dist == "normal" else ig.small_int
            a_np, da = _operand(gen, 701, m, k, la)
            b_np, db = _operand(gen, 702, k, n, lb, stride=5)
            tg.force_config(name)
            c = _run(da, db, m, n)
            assert tg.last_config().startswith(name) and "+pack" not in tg.last_config()
            check_against_oracle(c, np.ascontiguousarray(a_np), np.ascontiguousarray(b_np), exact=(dist == "int"),
                                 what=f"{name} {m}x{n}x{k} {dist}")


def test_paper_strided_matmul_1024_is_fused_without_a_workspace():
    """matmul 1024x1024x1024 with A's consecutive elements 32 apart (Sec. 5.2): gathered inside the product kernel."""
    m = n = k = 1024
    for dist in ("uniform", "int"):
        say(f"fused strided matmul 1024^3, A element stride 32, {dist}")
        gen = ig.uniform if dist == "uniform" else ig.small_int
        a_store = gen(711, (m, k * 32))
        b = gen(712, (k, n))
        c = _run(to_dev(a_store)[:, ::32], to_dev(b), m, n)
        cfg = tg.last_config()
        assert "_ga" in cfg and "_edge" not in cfg and "+pack" not in cfg, cfg
        check_against_oracle(c, np.ascontiguousarray(a_store[:, ::32]), b, exact=(dist == "int"), what="fused strided 1024^3 " + dist)


@pytest.mark.parametrize("layout", ["A^T", "B^T", "A^T B^T"])
@pytest.mark.parametrize("shape", [(1024, 1024, 1024), (512, 768, 2048), (260, 132, 96)], ids=str)
def test_transposed_layouts_are_read_as_they_lie(layout, shape):
    m, n, k = shape
    la = "T" if "A^T" in layout else "N"
    lb = "T" if "B^T" in layout else "N"
    for dist in ("normal", "int"):
        say(f"fused transposed {layout} {shape} {dist}")
        gen = ig.normal if dist == "normal" else ig.small_int
        a_np, da = _operand(gen, 721, m, k, la)
        b_np, db = _operand(gen, 722, k, n, lb)
        c = _run(da, db, m, n)
        cfg = tg.last_config()
        want = ("_ta" if la == "T" else "") + ("_tb" if lb == "T" else "")
        assert want in cfg and "_edge" not in cfg and "+pack" not in cfg, cfg
        check_against_oracle(c, np.ascontiguousarray(a_np), np.ascontiguousarray(b_np), exact=(dist == "int"),
                             what=f"{layout} {shape} {dist}")


def test_fused_variant_is_preferred_to_packing_when_a_workspace_is_set():
    import torch
    say("fused A^T with a workspace set")
    m, n, k = 512, 512, 256
    ws = torch.full((tg.strided_workspace_bytes(m, n, k, 7, 1) // 4,), float("nan"), device="cuda")
    tg.set_workspace(ws)
    a_np, da = _operand(ig.small_int, 731, m, k, "T")
    b = ig.small_int(732, (k, n))
    c = _run(da, to_dev(b), m, n)
    assert "_ta" in tg.last_config() and "+pack" not in tg.last_config(), tg.last_config()
    check_against_oracle(c, np.ascontiguousarray(a_np), b, exact=True, what="fused with workspace")
    del ws


PANELS = ["g16x1024x64_w16x128_acc2_ga", "g16x512x64_w16x128_acc2_ga", "g32x512x64_w32x128_acc2_ga", "g32x1024x64_w32x128_ga",
          "g32x512x64_w32x64_acc2_ga", "g16x512x64_w16x64_acc2_ga", "g16x256x64_w16x64_acc2_ga",
          "g32x512x64_w32x64_acc2_b3_ga", "g16x256x64_w16x64_acc2_b3_ga", "g32x512x128_w32x64_acc2_b3_ga",
          "g32x512x256_w32x64_acc2_b3_ga"]


@pytest.mark.parametrize("name", PANELS)
@pytest.mark.parametrize("splits", [2, 3, 4])
def test_row_panel_variants_with_a_k_split(name, splits):
    """The row-panel kernels fill the chip through a K split when the panels alone are too few: partial products in
    the workspace, added by the reduction in a fixed order.  Ragged rows, a partly used last column tile, K ranges
    of unequal length (13 chunks over 2, 3 or 4 ranges)."""
    import torch
    bk = _tile(name)[2]
    for (m, n, k, stride) in [(1000, 1024, max(1024, 8 * bk), 32), (73, 1060, 13 * bk, 3)]:
        ws = torch.full((4 * m * n + 64,), float("nan"), device="cuda")
        tg.set_workspace(ws)
        for dist in ("normal", "int"):
            say(f"forced {name}:s{splits} {m}x{n}x{k} A element stride {stride} {dist}")
            gen = ig.normal if dist == "normal" else ig.small_int
            a_np, da = _operand(gen, 741, m, k, "S", stride=stride)
            b = gen(742, (k, n))
            tg.force_config(f"{name}:s{splits}:g1")
            c = _run(da, to_dev(b), m, n)
            assert tg.last_config().startswith(f"{name}:s{splits}"), tg.last_config()
            check_against_oracle(c, np.ascontiguousarray(a_np), b, exact=(dist == "int"),
                                 what=f"{name}:s{splits} {m}x{n}x{k} {dist}")
        tg.set_workspace(None)
        del ws


@pytest.mark.parametrize("name", PANELS)
def test_row_panel_variants_on_a_batch_of_plain_operands(name):
    """A gather reads plain rows too: forced on a batch through tg_sgemm_batched (problem strides, padded leading
    dimensions, rows of C off the 16-byte grid)."""
    import torch
    batch, m, n, k = 3, 50, 1028, 3 * _tile(name)[2]
    say(f"forced {name} on a batch {batch} x {m}x{n}x{k}")
    a = ig.small_int(751, (batch, m, k + 4))
    b = ig.small_int(752, (batch, k, n + 8))
    out = torch.full((batch, m, n + 1), float("nan"), device="cuda")
    tg.force_config(name)
    tg.sgemm_batched(to_dev(a)[:, :, :k], to_dev(b)[:, :, :n], out=out[:, :, :n])
    torch.cuda.synchronize()
    assert tg.last_config().startswith(name), tg.last_config()
    c = out.cpu().numpy()
    assert np.isnan(c[:, :, n]).all()                     # the padding column of C is not written
    for i in range(batch):
        check_against_oracle(c[i, :, :n], np.ascontiguousarray(a[i, :, :k]), np.ascontiguousarray(b[i, :, :n]), exact=True,
                             what=f"{name} batch problem {i}")


@pytest.mark.parametrize("name", ["g16x256x64_w16x64_acc2_b3_ga", "g32x512x128_w32x64_acc2_b3_ga", "g32x1024x64_w32x128_ga"])
def test_row_panel_variants_behind_a_padded_copy_of_b(name):
    """n not a multiple of 4 with a workspace set: B is fetched from a copy padded to the next multiple of 4 columns,
    and the last, partial group of four columns of C must leave element by element (a 16-byte store there wrote the
    first element of the next row: the tuner's result check caught it on 1023 x 1023 x 1023).  Rows of C are packed, so
    a write past the end of a row would land in the result."""
    import torch
    m, n, k = 530, 1023, 1024
    say(f"forced {name} on {m}x{n}x{k} behind a padded copy of B")
    a = ig.small_int(781, (m, k))
    b = ig.small_int(782, (k, n))
    ws = torch.empty(16 << 20, dtype=torch.uint8, device="cuda")
    out = torch.full((m + 1, n), float("nan"), device="cuda")
    try:
        tg.set_workspace(ws)
        tg.force_config(name)
        tg.sgemm(to_dev(a), to_dev(b), out=out[:m])
        torch.cuda.synchronize()
        cfg = tg.last_config()
    finally:
        tg.set_workspace(None)
    assert cfg.startswith(name) and "+align" in cfg, cfg
    c = out.cpu().numpy()
    assert np.isnan(c[m]).all()                           # nothing written behind the last row
    check_against_oracle(c[:m], a, b, exact=True, what=f"{name} behind a padded B")


def test_tall_strided_product_takes_a_row_panel_without_a_workspace():
    """4096 x 1024 x 1024 with A at element stride 32: row panels of 16 or 32 rows fill the chip by themselves, every
    element of A is requested once or twice, nothing is packed and no workspace is needed."""
    m, n, k = 4096, 1024, 1024
    say("automatic choice, 4096x1024x1024 with A at element stride 32, no workspace")
    a_store = ig.uniform(761, (m, k * 32))
    b = ig.uniform(762, (k, n))
    c = _run(to_dev(a_store)[:, ::32], to_dev(b), m, n)
    cfg = tg.last_config()
    assert re.match(r"g(16|32)x", cfg) and "+pack" not in cfg, cfg
    rows = np.arange(0, m, 37)
    check_against_oracle(c[rows], np.ascontiguousarray(a_store[rows, ::32]), b, what="tall strided product, sampled rows")


WALKS = [("g32x512x64_w32x64_rw_ga", 1, (4096, 4096, 128)), ("g32x512x64_w32x64_rw_ga", 2, (4096, 4096, 128)),
         ("g32x512x64_w32x64_acc2_rw_ga", 1, (8192, 2048, 192)), ("g16x512x64_w16x64_acc2_rw_ga", 1, (4096, 4096, 64)),
         ("g16x256x64_w16x64_acc2_rw_ga", 2, (4096, 1024, 1088)), ("g32x512x64_w32x64_b3_rw_ga", 1, (4096, 2048, 256)),
         ("g16x512x64_w16x64_b3_rw_ga", 1, (4096, 2048, 128)), ("g32x512x64_w32x64_acc2_b3_rw_ga", 1, (4096, 4096, 128)),
         ("g32x512x128_w32x64_acc2_b3_rw_ga", 2, (4096, 4096, 256)),
         # A resident in LDS over the whole K range: one barrier per workgroup, the waves on their own from there
         ("g32x512x64_w32x64_res_ga", 1, (4096, 4096, 128)), ("g32x512x64_w32x64_res_ga", 2, (4096, 4096, 128)),
         ("g32x512x64_w32x64_res_ga", 4, (4096, 4096, 64)), ("g32x1024x64_w32x64_res_ga", 1, (4096, 4096, 128)),
         ("g32x1024x64_w32x64_res_ga", 2, (8192, 2048, 192)), ("g32x512x64_w32x64_b3_res_ga", 1, (2048, 8192, 448)),
         ("g32x512x64_w32x64_b3_res_ga", 2, (4096, 2048, 64)), ("g32x1024x64_w32x64_res_ga", 1, (4096, 2048, 320))]


@pytest.mark.parametrize("name,per_cu,shape", WALKS, ids=lambda v: v if isinstance(v, str) else str(v))
def test_row_panel_variants_that_walk_along_their_panel(name, per_cu, shape):
    """Persistent forms for short K: a workgroup takes several neighbouring column tiles of one row panel, with the chunk
    pipeline running on across the tile boundaries, or with its rows of A resident in LDS and every wave on its own
    behind a single barrier.  Plain operands (the tuned 4096x4096x128 configuration is one of these) and a strided
    A; sampled rows against the oracle, and no element of C left unwritten."""
    m, n, k = shape
    for layout, dist in (("N", "normal"), ("N", "int"), ("S", "int")):
        say(f"forced {name}:p{per_cu} {m}x{n}x{k} A:{layout} {dist}")
        gen = ig.normal if dist == "normal" else ig.small_int
        a_np, da = _operand(gen, 771, m, k, layout, stride=5)
        b = gen(772, (k, n))
        tg.force_config(f"{name}:s1:g1:p{per_cu}")
        c = _run(da, to_dev(b), m, n)
        assert tg.last_config().startswith(name), tg.last_config()
        rows = np.arange(0, m, 7)
        check_against_oracle(c[rows], np.ascontiguousarray(a_np[rows]), b, exact=(dist == "int"), what=f"{name}:p{per_cu} {shape} {layout} {dist}")
        assert np.isfinite(c).all()


def test_walking_variants_refuse_what_they_cannot_divide():
    import torch
    a = torch.zeros((4096, 128), device="cuda")
    b = torch.zeros((128, 1536), device="cuda")      # 128 x 3 tiles of 32 x 512: 384 tiles do not divide over 256 workgroups
    tg.force_config("g32x512x64_w32x64_rw_ga:s1:g1:p1")
    with pytest.raises(Exception, match="divide evenly"):
        tg.sgemm(a, b)
    # the variants that keep their rows of A in LDS take no K range that does not fit there
    a = torch.zeros((4096, 512), device="cuda")
    b = torch.zeros((512, 4096), device="cuda")
    tg.force_config("g32x512x64_w32x64_res_ga:s1:g1:p1")
    with pytest.raises(Exception, match="do not fit its LDS"):
        tg.sgemm(a, b)
    tg.force_config(None)
    # ... and a batch or a K split goes to the other variants
    tg.force_config("g32x512x64_w32x64_res_ga:s2:g1:p1")
    with pytest.raises(Exception, match="one problem and one K range"):
        tg.sgemm(torch.zeros((4096, 256), device="cuda"), torch.zeros((256, 4096), device="cuda"))

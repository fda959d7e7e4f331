"""GPU parity: the HIP path (through the C-ABI) against the CPU oracle, element by element.

Cases: the five benchmark workloads at full size with their distributions, the integer
variant of every workload (bit exact), every compiled kernel variant forced in turn on a
shape spanning several tiles, ragged sizes, padded leading dimensions, split-K, batch
strides, k = 0, and run-to-run bit identity.
"""
import numpy as np
import pytest

import paper_1904_03383_amd as tg
from paper_1904_03383_amd import inputgen as ig

from gpu_common import check_against_oracle, run_hip, say, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _clean_library_state():
    tg.force_config(None)
    tg.set_workspace(None)
    yield
    tg.force_config(None)
    tg.set_workspace(None)


def _squeeze(a, b):
    return (a[0], b[0]) if a.shape[0] == 1 else (a, b)


# ---- the five workloads, at full size, in the configuration the library picks itself ----

@pytest.mark.parametrize("name", list(ig.CONFIGS))
def test_workload_matches_oracle(name):
    say(f"workload {name} ({ig.CONFIGS[name]})")
    a, b = _squeeze(*ig.make_config(name))
    c = run_hip(a, b)
    m = check_against_oracle(c, a, b, what=name)
    say(f"  config {tg.last_config()}  max_ratio {m['max_ratio']:.2e}  rel_fro {m['rel_fro']:.2e}"
        f"  (worst single problem {m['rel_fro_max_problem']:.2e})")


@pytest.mark.parametrize("name", list(ig.CONFIGS))
def test_workload_integer_variant_is_bit_exact(name):
    """Entries in {-4..4}: every partial sum is an integer below 2^24, so any summation order is exact."""
    say(f"integer variant of {name}")
    a, b = _squeeze(*ig.make_config(name, dist="int"))
    c = run_hip(a, b)
    check_against_oracle(c, a, b, exact=True, what=name + "/int")


@pytest.mark.parametrize("name", list(ig.CONFIGS))
def test_workload_in_the_tuned_configuration_matches_oracle(name):
    """Every workload in the launch configuration the benchmark times: after tg_tune, with the benchmark's
    split-K workspace set; all elements against the oracle, and the integer variant bit for bit."""
    import torch
    say(f"{name} after tune")
    ws_bytes = max(tg.workspace_bytes(*ig.CONFIGS[w][:4]) for w in ig.CONFIGS)
    ws = torch.empty(max(ws_bytes // 4, 4), dtype=torch.float32, device="cuda")
    tg.set_workspace(ws)
    a, b = _squeeze(*ig.make_config(name))
    da, db = to_dev(a), to_dev(b)
    call = tg.sgemm if a.ndim == 2 else tg.sgemm_batched
    tg.clear_tune_cache()
    try:
        c = tg.tune(da, db, reps=2)
        torch.cuda.synchronize()
        tuned = tg.last_config()
        c2 = call(da, db)
        torch.cuda.synchronize()
        assert tg.last_config() == tuned
        assert torch.equal(c, c2)
        m = check_against_oracle(c2.cpu().numpy(), a, b, what=f"{name} tuned {tuned}")
        say(f"  tuned {tuned}  rel_fro {m['rel_fro']:.2e}")
        ai, bi = _squeeze(*ig.make_config(name, dist="int"))
        ci = call(to_dev(ai), to_dev(bi))
        torch.cuda.synchronize()
        assert tg.last_config() == tuned
        check_against_oracle(ci.cpu().numpy(), ai, bi, exact=True, what=f"{name}/int tuned {tuned}")
    finally:
        tg.clear_tune_cache()
        del ws


# ---- every kernel variant, forced -----------------------------------------------------------

def _shape_for(name: str):
    """A shape valid for the named variant that spans several tiles (ragged for predicated ones)."""
    if name.startswith("wave16x"):          # aligned operands, n a multiple of 4; ragged tiles and a partial k step
        return 1, 70, 44, 76
    if name.startswith("wave"):
        return 1, 70, 45, 61
    body = name.split("_")[0][1:]
    bm, bn, bk = (int(x) for x in body.split("x"))
    k = 1536 if "acc2" in name else 320      # acc2 variants need a K range above 1024
    if name.endswith("_edge"):
        return 1, 2 * bm + 37, bn + 21, k + 13
    return 1, 2 * bm, 3 * bn, k


@pytest.mark.parametrize("dist", ["uniform", "int"])
def test_each_kernel_variant(dist):
    import torch
    ws = torch.empty(1 << 24, dtype=torch.float32, device="cuda")   # 64 MiB: the piece images of the "c" variants
    for name in tg.kernel_names():
        if "_ta" in name or "_tb" in name or "_rw_" in name or "_res_" in name:
            continue    # variants for transposed operands cannot read plain ones: forced in test_fused_layouts_gpu.py
                        # (the gathering "_ga" / "_gb" variants can, and do so here); the row-panel variants that walk
                        # along their panel (or keep it in LDS) need 256 workgroups' worth of tiles: forced there too
        tg.set_workspace(ws if name.startswith("c") else None)
        batch, m, n, k = _shape_for(name)
        say(f"forced {name} on {m}x{n}x{k} ({dist})")
        a, b = ig.make_operands(batch, m, n, k, dist, 301, 302)
        spec = name + ":s1:g2" + (":p1" if name.startswith("p") else "")
        tg.force_config(spec)
        c = run_hip(a[0], b[0])
        assert tg.last_config() == spec
        check_against_oracle(c, a[0], b[0], exact=(dist == "int"), what=name)


@pytest.mark.parametrize("spec", ["p128x128x16_w64x64:p1", "p128x128x32_w64x64:p2:o2", "p128x128x32_w64x64:p3:g3",
                                  "p128x128x16_w64x64:s2:p1",
                                  # deferred stores: every workgroup has several items, so tiles are stored during
                                  # the next item's first K tile (and the last one at the end)
                                  "p128x128x16_w64x64_ds:p1", "p128x128x16_w64x64_ds:p2:o2", "p128x128x16_w64x64_ds:p3:g3"])
def test_persistent_launch(spec):
    """Fewer workgroups than tiles: every workgroup loops over several tiles."""
    import torch
    say(f"persistent {spec}")
    m, n, k = 40 * 128, 26 * 128, 192        # 1040 tiles of 128x128 on 256 x p workgroups
    ws = torch.empty(2 * m * n, dtype=torch.float32, device="cuda")
    tg.set_workspace(ws)
    a, b = ig.make_operands(1, m, n, k, "int", 313, 314)
    tg.force_config(spec)
    check_against_oracle(run_hip(a[0], b[0]), a[0], b[0], exact=True, what=spec)


def test_deferred_store_variant_says_what_it_cannot_take():
    import torch
    m, n, k = 256, 256, 64
    a, b = ig.make_operands(1, m, n, k, "int", 315, 316)
    da, db = to_dev(a[0]), to_dev(b[0])
    ws = torch.empty(4 * m * n, dtype=torch.float32, device="cuda")
    tg.set_workspace(ws)
    tg.force_config("p128x128x16_w64x64_ds:s2:p1")
    with pytest.raises(tg.TgemmError, match="no split-K"):
        tg.sgemm(da, db)
    buf = torch.empty(m * n + 1, device="cuda")
    tg.force_config("p128x128x16_w64x64_ds:p1")
    with pytest.raises(tg.TgemmError, match="rows of C are not aligned"):
        tg.sgemm(da, db, out=buf[1:].view(m, n))
    out = tg.sgemm(da, db)   # a fresh, aligned C: accepted
    torch.cuda.synchronize()
    check_against_oracle(out.cpu().numpy(), a[0], b[0], exact=True, what="deferred stores, aligned C")


@pytest.mark.parametrize("group", [1, 3, 8, 64])
def test_tile_order_groups(group):
    say(f"tile order group {group}")
    a, b = ig.make_operands(1, 5 * 128, 3 * 128, 64, "int", 311, 312)
    tg.force_config(f"t128x128x16_w64x64:s1:g{group}")
    check_against_oracle(run_hip(a[0], b[0]), a[0], b[0], exact=True, what=f"group {group}")


# ---- ragged shapes, padded leading dimensions, batches ---------------------------------------

RAGGED = [(1, 1, 1), (1, 7, 3), (7, 1, 5), (31, 33, 65), (33, 31, 7), (65, 100, 257), (100, 257, 31),
          (257, 65, 100), (129, 127, 1030), (300, 200, 2100), (2, 3000, 9), (3000, 2, 40)]


@pytest.mark.parametrize("shape", RAGGED, ids=lambda s: "x".join(map(str, s)))
def test_ragged_shapes(shape):
    m, n, k = shape
    say(f"ragged {m}x{n}x{k}")
    for dist in ("normal", "int"):
        a, b = ig.make_operands(1, m, n, k, dist, 321, 322)
        c = run_hip(a[0], b[0])
        check_against_oracle(c, a[0], b[0], exact=(dist == "int"), what=f"ragged {shape} {dist}")


@pytest.mark.parametrize("forced", [None, "t128x128x16_w64x64_edge", "t64x64x16_w32x32_edge", "wave32", "wave16", "wave16k4"])
def test_ragged_through_each_predicated_kernel(forced):
    m, n, k = 150, 139, 77
    say(f"ragged {m}x{n}x{k} forced={forced}")
    a, b = ig.make_operands(1, m, n, k, "int", 331, 332)
    if forced:
        tg.force_config(forced)
    check_against_oracle(run_hip(a[0], b[0]), a[0], b[0], exact=True, what=str(forced))


# Ragged m and n on the exact-fit kernels (k a multiple of the K tile, n of 4): the last tile row / column
# re-reads the last row / vector of the operand and masks its stores.
RAGGED_FAST = [
    ("t128x128x16_w64x64", (1000, 1000, 1024)), ("t128x128x16_w64x64", (129, 4, 48)), ("t128x128x16_w64x64", (1, 260, 64)),
    ("t128x128x32_w64x64_acc2", (130, 132, 2080)), ("t256x128x32_w128x64", (257, 136, 96)), ("t128x256x16_w64x128", (100, 516, 64)),
    ("t64x64x32_w32x32", (65, 68, 96)), ("t128x64x32_w64x32", (200, 100, 64)), ("t64x128x32_w32x64", (70, 200, 64)),
    ("d128x128x32_w64x64", (1000, 1000, 1024)), ("d128x256x32_w64x128_acc2", (300, 260, 2112)), ("d256x128x32_w128x64", (258, 132, 64)),
    ("d128x256x32_w64x128_acc2_st3", (129, 257 * 4, 1056)), ("d64x64x32_w32x32", (1, 4, 32)), ("d64x64x32_w32x32_st4", (67, 72, 160)),
    ("d64x64x32_w32x32_k2", (130, 68, 96)), ("d64x64x32_w32x32_k2_st4", (63, 60, 256)),
    ("t128x128x16_w64x64:s3", (200, 136, 1024)), ("d128x128x32_w64x64:s2", (130, 260, 512)),
    # 32-row tiles for skinny products (m <= 32, wide n)
    ("t32x256x32_w32x64", (7, 260, 96)), ("d32x256x32_w32x64", (32, 516, 64)), ("t32x256x32_w32x64_acc2", (20, 256, 2080)),
    ("d32x256x32_w32x64:s4", (9, 520, 1024)), ("t32x256x32_w32x64", (70, 300, 64)),
    # ... and 32-column tiles for tall ones (n <= 32)
    ("t256x32x32_w64x32", (300, 8, 96)), ("d256x32x32_w64x32", (520, 32, 64)), ("t256x32x32_w64x32_acc2", (260, 20, 2080)),
    ("d256x32x32_w64x32:s4", (515, 12, 1024)), ("t256x32x32_w64x32", (300, 72, 64)),
]


@pytest.mark.parametrize("spec,shape", RAGGED_FAST, ids=lambda v: v if isinstance(v, str) else "x".join(map(str, v)))
def test_ragged_m_n_on_exact_fit_kernels(spec, shape):
    import torch
    m, n, k = shape
    say(f"ragged fast {spec} {m}x{n}x{k}")
    if ":s" in spec:
        ws = torch.empty(4 * m * n + 4, device="cuda")
        tg.set_workspace(ws)
    tg.force_config(spec)
    for dist in ("normal", "int"):
        a, b = ig.make_operands(1, m, n, k, dist, 341, 342)
        c = run_hip(a[0], b[0])
        assert tg.last_config().startswith(spec)
        check_against_oracle(c, a[0], b[0], exact=(dist == "int"), what=f"{spec} {shape} {dist}")


# k not a multiple of the K tile on the register-staged exact-fit kernels (k % 4 == 0, k >= BK): the
# remainder is multiplied first, as a zero-padded K tile.
K_TAIL = [
    ("t128x128x16_w64x64", (256, 256, 20)), ("t128x128x16_w64x64", (1000, 1000, 1000)), ("t128x128x32_w64x64", (128, 128, 36)),
    ("t128x128x32_w64x64_acc2", (130, 132, 2076)), ("t256x128x32_w128x64", (256, 128, 60)), ("t128x256x16_w64x128_acc2", (100, 516, 1044)),
    ("t64x64x32_w32x32", (65, 68, 100)), ("t128x64x32_w64x32", (200, 100, 92)), ("t64x128x32_w32x64", (70, 200, 68)),
    ("t128x128x16_w64x64:s3", (200, 136, 1000)), ("t128x128x32_w64x64:s2", (128, 128, 2020)), ("t64x64x32_w32x32:s4", (64, 64, 1028)),
    ("t32x256x32_w32x64", (30, 256, 100)), ("t32x256x32_w32x64:s2", (5, 512, 1000)),
    ("t256x32x32_w64x32", (256, 28, 100)), ("t256x32x32_w64x32:s2", (512, 4, 1000)),
]


@pytest.mark.parametrize("spec,shape", K_TAIL, ids=lambda v: v if isinstance(v, str) else "x".join(map(str, v)))
def test_k_remainder_on_exact_fit_kernels(spec, shape):
    import torch
    m, n, k = shape
    say(f"k tail {spec} {m}x{n}x{k}")
    if ":s" in spec:
        ws = torch.empty(4 * m * n + 4, device="cuda")
        tg.set_workspace(ws)
    tg.force_config(spec)
    for dist in ("normal", "int"):
        a, b = ig.make_operands(1, m, n, k, dist, 371, 372)
        c = run_hip(a[0], b[0])
        assert tg.last_config().startswith(spec)
        check_against_oracle(c, a[0], b[0], exact=(dist == "int"), what=f"{spec} {shape} {dist}")


def test_k_remainder_reads_nothing_past_the_operands():
    """A and B sit at the very end of their allocations and are followed by NaN-poisoned memory inside the same
    buffer; with lda > k the columns between k and lda hold NaN too.  Nothing of that may reach C."""
    import torch
    say("k tail: poisoned surroundings")
    m, n, k, lda = 130, 132, 1000, 1004
    a, b = ig.make_operands(1, m, n, k, "int", 381, 382)
    abuf = torch.full((m + 2, lda), float("nan"), device="cuda")
    abuf[:m, :k] = to_dev(a[0])
    bbuf = torch.full((k + 2, n + 4), float("nan"), device="cuda")
    bbuf[:k, :n] = to_dev(b[0])
    for spec in ("t128x128x16_w64x64", "t64x64x32_w32x32", "t128x128x32_w64x64", None):
        tg.force_config(spec)
        out = torch.full((m, n), float("nan"), device="cuda")
        tg.sgemm(abuf[:m, :k], bbuf[:k, :n], out=out)
        torch.cuda.synchronize()
        check_against_oracle(out.cpu().numpy(), a[0], b[0], exact=True, what=f"poisoned surroundings {spec}")


def test_ragged_fast_path_leaves_padding_and_neighbours_alone():
    """Output rows past m and columns past n (inside ldc, and the memory after the last row) stay untouched."""
    import torch
    say("ragged fast path: no stray stores")
    m, n, k, ldc = 130, 132, 64, 140
    a, b = ig.make_operands(1, m, n, k, "int", 351, 352)
    buf = torch.full((m + 3, ldc), 7.0, device="cuda")
    for spec in ("t128x128x16_w64x64", "d128x128x32_w64x64", "d64x64x32_w32x32_k2", None):
        tg.force_config(spec)
        buf.fill_(7.0)
        tg.sgemm(to_dev(a[0]), to_dev(b[0]), out=buf[:m, :n])
        torch.cuda.synchronize()
        host = buf.cpu().numpy()
        assert np.all(host[:m, n:] == 7.0) and np.all(host[m:, :] == 7.0), spec
        check_against_oracle(np.ascontiguousarray(host[:m, :n]), a[0], b[0], exact=True, what=f"no stray stores {spec}")


def test_ragged_batched_on_exact_fit_kernels():
    say("ragged batched fast path")
    a, b = ig.make_operands(5, 70, 36, 64, "int", 361, 362)
    for spec in ("t64x64x32_w32x32", "d64x64x32_w32x32", None):
        tg.force_config(spec)
        check_against_oracle(run_hip(a, b), a, b, exact=True, what=f"batched ragged {spec}")


@pytest.mark.parametrize("pads", [(0, 0, 0), (4, 8, 12), (1, 3, 5)], ids=str)
@pytest.mark.parametrize("shape", [(256, 256, 64), (130, 70, 50)], ids=str)
def test_leading_dimensions_and_untouched_padding(shape, pads):
    """lda > k, ldb > n, ldc > n; elements of C beyond column n must keep their sentinel."""
    import torch
    m, n, k = shape
    pa, pb, pc = pads
    say(f"leading dimensions {shape} pads {pads}")
    a_full = ig.small_int(341, (m, k + pa))
    b_full = ig.small_int(342, (k, n + pb))
    da, db = to_dev(a_full)[:, :k], to_dev(b_full)[:, :n]
    c_full = torch.full((m, n + pc), -777.0, device="cuda")
    out = c_full[:, :n]
    tg.sgemm(da, db, out=out)
    torch.cuda.synchronize()
    host = c_full.cpu().numpy()
    assert np.all(host[:, n:] == -777.0)
    check_against_oracle(host[:, :n], np.ascontiguousarray(a_full[:, :k]), np.ascontiguousarray(b_full[:, :n]),
                         exact=True, what=f"ld {shape} {pads}")


def test_unaligned_base_pointers():
    """Operands that start 4 bytes off a 16-byte boundary take the predicated path."""
    import torch
    say("unaligned base pointers")
    m, n, k = 128, 128, 64
    a = ig.small_int(351, (m * k + 1,))
    b = ig.small_int(352, (k * n + 1,))
    da = to_dev(a)[1:].view(m, k)
    db = to_dev(b)[1:].view(k, n)
    buf = torch.empty(m * n + 1, device="cuda")
    out = buf[1:].view(m, n)
    assert da.data_ptr() % 16 == 4
    tg.sgemm(da, db, out=out)
    torch.cuda.synchronize()
    assert "_edge" in tg.last_config() or tg.last_config().startswith("wave")
    check_against_oracle(out.cpu().numpy(), a[1:].reshape(m, k), b[1:].reshape(k, n), exact=True, what="unaligned")


@pytest.mark.parametrize("name", ["wave16x32", "wave16x64"])
@pytest.mark.parametrize("batch", [1, 3])
def test_wide_wave_tiles(name, batch):
    """16x32 and 16x64 tiles per wave: aligned A and B, ragged m and n, a partial last k step, and a C whose rows
    are not 16-byte aligned (element stores) with a sentinel behind every row."""
    import torch
    m, n, k, ldc = 50, 36, 44, 39
    say(f"{name} batch {batch} {m}x{n}x{k} ldc {ldc}")
    a, b = ig.make_operands(batch, m, n, k, "int", 361, 362)
    da, db = to_dev(a), to_dev(b)
    buf = torch.full((batch * m * ldc + 1,), -777.0, device="cuda")
    out = buf[1:].view(batch, m, ldc)[:, :, :n]
    assert out.data_ptr() % 16 == 4
    tg.force_config(name)
    if batch == 1:
        tg.sgemm(da[0], db[0], out=out[0])
    else:
        tg.sgemm_batched(da, db, out=out)
    torch.cuda.synchronize()
    assert tg.last_config().startswith(name)
    host = buf[1:].view(batch, m, ldc).cpu().numpy()
    assert np.all(host[:, :, n:] == -777.0)
    for i in range(batch):
        check_against_oracle(host[i, :, :n], a[i], b[i], exact=True, what=f"{name} problem {i}")
    # aligned C: vector stores
    tg.force_config(name)
    c = run_hip(a, b) if batch > 1 else run_hip(a[0], b[0])[None]
    for i in range(batch):
        check_against_oracle(c[i], a[i], b[i], exact=True, what=f"{name} aligned problem {i}")


@pytest.mark.parametrize("name,kmax", [("wave32", 2048), ("wave16", 2048), ("wave16x32", 2048), ("wave16x64", 2048),
                                       ("wave16k4", 8192)])
def test_wave_kernels_at_their_longest_k(name, kmax):
    """One accumulator chain per wave: the longest K a wave kernel accepts must still meet the Frobenius bar on
    normal(0,1) operands (the case that forces the second accumulation level on the tile kernels), and one more
    k is refused."""
    m, n = 96, 64
    say(f"{name} at k = {kmax}")
    a, b = ig.make_operands(1, m, n, kmax, "normal", 371, 372)
    tg.force_config(name)
    c = run_hip(a[0], b[0])
    assert tg.last_config().startswith(name)
    met = check_against_oracle(c, a[0], b[0], what=f"{name} k {kmax}")
    say(f"  rel_fro {met['rel_fro']:.2e}")
    a2, b2 = ig.make_operands(1, 16, 16, kmax + 4, "int", 373, 374)
    with pytest.raises(tg.TgemmError, match="k too long"):
        run_hip(a2[0], b2[0])


@pytest.mark.parametrize("case", [(3, 32, 32, 64), (5, 70, 33, 20), (2, 256, 128, 96), (1, 64, 64, 64), (130, 16, 16, 16)], ids=str)
def test_batched_shapes(case):
    batch, m, n, k = case
    say(f"batched {case}")
    a, b = ig.make_operands(batch, m, n, k, "int", 361, 362)
    check_against_oracle(run_hip(a, b), a, b, exact=True, what=f"batched {case}")
    a, b = ig.make_operands(batch, m, n, k, "uniform", 363, 364)
    check_against_oracle(run_hip(a, b), a, b, what=f"batched {case}")


def test_batched_strides_and_broadcast():
    """Batch strides larger than a matrix, and strideB = 0 (one B shared by all problems)."""
    import torch
    say("batched strides / broadcast")
    batch, m, n, k = 4, 64, 64, 32
    a_big = ig.small_int(371, (batch, m + 3, k))
    da = to_dev(a_big)[:, :m, :]                      # strideA = (m+3)*k
    b_one = ig.small_int(372, (1, k, n))
    db = to_dev(b_one).expand(batch, k, n)            # strideB = 0
    out = tg.sgemm_batched(da, db)
    torch.cuda.synchronize()
    a = np.ascontiguousarray(a_big[:, :m, :])
    b = np.ascontiguousarray(np.broadcast_to(b_one, (batch, k, n)))
    check_against_oracle(out.cpu().numpy(), a, b, exact=True, what="batched strides")


# ---- split-K ----------------------------------------------------------------------------

@pytest.mark.parametrize("spec,shape", [
    ("t128x128x16_w64x64:s4", (256, 384, 1024)),
    ("t128x128x16_w64x64:s3", (256, 128, 1008)),
    ("t128x128x16_w64x64_acc2:s2", (256, 256, 4096)),
    ("t64x64x32_w32x32:s8", (128, 192, 2048)),
    ("t64x64x16_w32x32_edge:s5", (100, 77, 1000)),
    ("t128x128x16_w64x64_edge:s2", (130, 250, 333)),
], ids=str)
def test_split_k(spec, shape):
    import torch
    m, n, k = shape
    say(f"split-K {spec} on {shape}")
    ws = torch.empty(16 * m * n, dtype=torch.float32, device="cuda")
    tg.set_workspace(ws)
    tg.force_config(spec)
    for dist in ("int", "uniform"):
        a, b = ig.make_operands(1, m, n, k, dist, 381, 382)
        c = run_hip(a[0], b[0])
        assert tg.last_config().startswith(spec)
        check_against_oracle(c, a[0], b[0], exact=(dist == "int"), what=spec)


def test_split_k_batched_and_workspace_too_small():
    import torch
    say("split-K batched / workspace checks")
    batch, m, n, k = 3, 128, 128, 512
    a, b = ig.make_operands(batch, m, n, k, "int", 391, 392)
    tg.force_config("t128x128x16_w64x64:s4")
    with pytest.raises(tg.TgemmError) as ei:
        run_hip(a, b)
    assert ei.value.status_name == "TG_ERR_WORKSPACE"
    ws = torch.empty(batch * 4 * m * n - 4, dtype=torch.float32, device="cuda")
    tg.set_workspace(ws)
    with pytest.raises(tg.TgemmError):
        run_hip(a, b)
    ws = torch.empty(batch * 4 * m * n, dtype=torch.float32, device="cuda")
    tg.set_workspace(ws)
    check_against_oracle(run_hip(a, b), a, b, exact=True, what="split-K batched")


# ---- degenerate sizes -------------------------------------------------------------------------

def test_k_zero_gives_zeros_and_empty_outputs_are_noops():
    import torch
    say("k == 0 and empty outputs")
    a = torch.empty((5, 0), device="cuda")
    b = torch.empty((0, 7), device="cuda")
    out = torch.full((5, 9), 3.0, device="cuda")
    tg.sgemm(a, b, out=out[:, :7])
    torch.cuda.synchronize()
    host = out.cpu().numpy()
    assert np.all(host[:, :7] == 0.0) and np.all(host[:, 7:] == 3.0)
    assert tg.sgemm(torch.empty((0, 4), device="cuda"), torch.empty((4, 6), device="cuda")).shape == (0, 6)
    assert tg.sgemm(torch.empty((3, 4), device="cuda"), torch.empty((4, 0), device="cuda")).shape == (3, 0)
    assert tg.sgemm_batched(torch.empty((0, 3, 4), device="cuda"), torch.empty((0, 4, 5), device="cuda")).shape == (0, 3, 5)
    ab = torch.empty((2, 3, 0), device="cuda")
    bb = torch.empty((2, 0, 4), device="cuda")
    assert torch.all(tg.sgemm_batched(ab, bb) == 0)


def test_output_may_start_as_nan():
    """C is overwritten, never read: NaNs already in the output buffer do not leak."""
    import torch
    say("NaN-initialised output")
    a, b = ig.make_operands(1, 256, 256, 128, "int", 401, 402)
    out = torch.full((256, 256), float("nan"), device="cuda")
    tg.sgemm(to_dev(a[0]), to_dev(b[0]), out=out)
    torch.cuda.synchronize()
    check_against_oracle(out.cpu().numpy(), a[0], b[0], exact=True, what="nan out")


# ---- determinism --------------------------------------------------------------------------------

@pytest.mark.parametrize("spec,shape", [("t128x128x16_w64x64", (512, 512, 512)),
                                        ("t128x128x16_w64x64:s4", (256, 256, 2048)),
                                        ("wave32", (96, 96, 200)), ("wave16", (96, 96, 200)), ("wave16k4", (96, 96, 200)), ("wave16x32", (96, 96, 200)),
                                        ("wave16x64", (96, 96, 200))], ids=str)
def test_repeated_launches_are_bit_identical(spec, shape):
    """No atomics and a barrier between LDS stages: 50 launches must agree bit for bit."""
    import torch
    m, n, k = shape
    say(f"determinism {spec} {shape}")
    ws = torch.empty(4 * m * n, dtype=torch.float32, device="cuda")
    tg.set_workspace(ws)
    tg.force_config(spec)
    a, b = ig.make_operands(1, m, n, k, "normal", 411, 412)
    da, db = to_dev(a[0]), to_dev(b[0])
    first = tg.sgemm(da, db).clone()
    for _ in range(50):
        again = tg.sgemm(da, db)
        assert torch.equal(first, again)
    torch.cuda.synchronize()


# ---- tuner ------------------------------------------------------------------------------------------

def test_tune_picks_a_valid_configuration_and_is_used_afterwards():
    import torch
    say("tuner on 1024^3 with workspace")
    a, b = _squeeze(*ig.make_config("c2_1024"))
    da, db = to_dev(a), to_dev(b)
    ws = torch.empty(tg.workspace_bytes(1, 1024, 1024, 1024) // 4, dtype=torch.float32, device="cuda")
    tg.set_workspace(ws)
    tg.clear_tune_cache()
    try:
        c = tg.tune(da, db, reps=3)
        tuned = tg.last_config()
        assert tuned.split(":")[0] in tg.kernel_names()
        assert tg.get_config(1, 1024, 1024, 1024) == tuned
        check_against_oracle(c.cpu().numpy(), a, b, what="tuned c2 " + tuned)
        c2 = tg.sgemm(da, db)
        torch.cuda.synchronize()
        assert tg.last_config() == tuned and torch.equal(c, c2)
        # the tuned split-K entry is not used once the workspace is gone; the call still succeeds
        tg.set_workspace(None)
        c3 = tg.sgemm(da, db)
        torch.cuda.synchronize()
        assert ":s1:" in tg.last_config()
        check_against_oracle(c3.cpu().numpy(), a, b, what="c2 without workspace")
    finally:
        tg.clear_tune_cache()


@pytest.mark.parametrize("shape", [(1, 256, 256, 32), (1, 1024, 1024, 1024), (512, 32, 32, 64), (1, 4096, 4096, 128),
                                   (1, 1000, 1000, 1000)], ids=lambda s: "x".join(map(str, s)))
def test_lower_bound_of_every_candidate_holds_on_the_device(shape):
    """The cut of the search (Sec. 5.1) is only safe if no configuration ever runs faster than its bound:
    time every candidate the tuner would consider, forced, and compare.  Times come from events around 20
    back-to-back launches, so they include launch gaps and can only be above the kernel's own time."""
    import torch
    batch, m, n, k = shape
    say(f"lower bounds vs device times at {shape}")
    g = torch.Generator(device="cpu").manual_seed(11)
    a = torch.rand((batch, m, k), generator=g, dtype=torch.float32).cuda()
    b = torch.rand((batch, k, n), generator=g, dtype=torch.float32).cuda()
    out = torch.empty((batch, m, n), dtype=torch.float32, device="cuda")
    ws = torch.empty(max(tg.workspace_bytes(batch, m, n, k) // 4, 1), dtype=torch.float32, device="cuda")
    tg.set_workspace(ws)
    cands = tg.candidates(batch, m, n, k)
    assert cands
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    worst = (10.0, "")
    for spec, bound_us, _ in cands:
        tg.force_config(spec)
        tg.sgemm_batched(a, b, out=out)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(20):
            tg.sgemm_batched(a, b, out=out)
        e1.record()
        e1.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / 20
        worst = min(worst, (us / bound_us, spec))
        assert us >= bound_us, f"{spec}: {us:.2f} us measured is below its lower bound {bound_us:.2f} us"
    say(f"  {len(cands)} candidates; tightest: {worst[1]} at {worst[0]:.2f}x its bound")


# ---- tail split: the last tile rows as a second launch with split-K -----------------------------

TAIL_SPLITS = [("t128x128x16_w64x64:t1x2", (1, 700, 520, 256)), ("t128x256x32_w64x128_acc2:t2x3", (1, 640, 516, 2112)),
               ("d128x128x32_w64x64:t1x4", (1, 300, 260, 512)), ("t64x64x32_w32x32:t3x2", (1, 500, 200, 192)),
               ("t128x128x32_w64x64_acc2:t1x2", (3, 390, 132, 2080)), ("t128x128x16_w64x64_edge:t2x2", (1, 517, 203, 301))]


@pytest.mark.parametrize("spec,shape", TAIL_SPLITS, ids=lambda v: v if isinstance(v, str) else "x".join(map(str, v)))
def test_tail_split_matches_oracle(spec, shape):
    import torch
    batch, m, n, k = shape
    say(f"tail split {spec} on {shape}")
    ws = torch.empty(8 * batch * 256 * n + 64, device="cuda")
    tg.set_workspace(ws)
    tg.force_config(spec)
    for dist in ("normal", "int"):
        a, b = ig.make_operands(batch, m, n, k, dist, 351, 352)
        c = run_hip(a[0], b[0]) if batch == 1 else run_hip(a, b)
        assert tg.last_config().endswith(spec.split(":", 1)[1]) and tg.last_config().startswith(spec.split(":")[0])
        for i in range(batch):
            check_against_oracle(c if batch == 1 else c[i], a[i], b[i], exact=(dist == "int"), what=f"{spec} {shape} {dist}")


def test_tuner_offers_and_times_tail_splits():
    """3072^3 on 128x256 tiles is 288 tiles for 256 CUs: the tuner must at least consider a tail split, and
    whatever it picks must match the oracle on sampled rows and not be slower than the best single launch."""
    import torch
    say("tuner at 3072^3 with workspace")
    m = n = k = 3072
    a, b = ig.make_operands(1, m, n, k, "normal", 361, 362)
    da, db = to_dev(a[0]), to_dev(b[0])
    ws = torch.empty(tg.workspace_bytes(1, m, n, k) // 4 + 64, device="cuda")
    tg.set_workspace(ws)
    assert any(":t" in s for s, _, _ in tg.candidates(1, m, n, k))
    tg.clear_tune_cache()
    try:
        c = tg.tune(da, db, reps=2)
        tuned = tg.last_config()
        say(f"  tuned {tuned}")
        rows = np.linspace(0, m - 1, 48).astype(int)
        check_against_oracle(c.cpu().numpy()[rows], a[0][rows], b[0], what="tuned 3072^3 " + tuned)
    finally:
        tg.clear_tune_cache()


def test_tail_split_is_offered_for_batches_too():
    """Four 1536^3 problems on 128x256 tiles are 288 tiles: the candidates (no tuning) include tail splits of that
    tiling; every problem is cut at the same tile row."""
    import torch
    say("batched tail split, first such candidate of the cost model")
    batch, m, n, k = 4, 1536, 1536, 1536
    ws = torch.empty(tg.workspace_bytes(batch, m, n, k) // 4 + 64, device="cuda")
    tg.set_workspace(ws)
    offered = [spec for (spec, _, _) in tg.candidates(batch, m, n, k) if ":t" in spec and "x256x" in spec]
    assert offered, tg.candidates(batch, m, n, k)[:5]
    chosen = offered[0]
    tg.force_config(chosen)
    a, b = ig.make_operands(batch, m, n, k, "int", 371, 372)
    c = run_hip(a, b)
    assert tg.last_config() == chosen
    rows = np.linspace(0, m - 1, 24).astype(int)
    for i in range(batch):
        check_against_oracle(c[i][rows], a[i][rows], b[i], exact=True, what=f"batched tail split {i}")


# ---- operands off the 16-byte grid: aligned copies in the workspace, element stores for C ------

def test_unaligned_and_odd_operands_are_copied_when_the_workspace_has_room():
    import torch
    from test_random_shapes_gpu import _place
    say("aligned copies of A and B, element stores for C")
    ws = torch.empty(1 << 22, device="cuda")
    cases = [  # (m, n, k, pads (lda-k, ldb-n, ldc-n), offsets (A, B, C), expected suffix)
        (1030, 771, 777, (0, 0, 0), (0, 0, 0), "+alignAB"),     # k and n odd
        (900, 1028, 512, (0, 0, 0), (1, 0, 0), "+alignA"),      # A one float off the grid
        (900, 1030, 512, (0, 0, 0), (0, 0, 0), "+alignB"),      # n not a multiple of 4
        (896, 1024, 512, (4, 3, 0), (0, 0, 0), "+alignB"),      # odd leading dimension of B
        (896, 1024, 512, (0, 0, 1), (0, 0, 3), ""),             # only C off the grid: no copy, element stores
        (517, 771, 333, (0, 0, 0), (0, 0, 0), ""),              # too small for copies to pay: the wave kernels take it
    ]
    for m, n, k, pads, offs, suffix in cases:
        a = ig.small_int(381, (1, m, k))
        b = ig.small_int(382, (1, k, n))
        _, da = _place(a, pads[0], offs[0], 0, float("nan"))
        _, db = _place(b, pads[1], offs[1], 0, float("nan"))
        for with_ws in (True, False):
            tg.set_workspace(ws if with_ws else None)
            cflat, dc = _place(np.zeros((1, m, n), np.float32), pads[2], offs[2], 0, 7.0)
            cflat.fill_(7.0)
            tg.sgemm(da[0], db[0], out=dc[0])
            torch.cuda.synchronize()
            cfg = tg.last_config()
            say(f"  {m}x{n}x{k} pads {pads} offsets {offs} workspace {with_ws}: {cfg}")
            if with_ws:
                assert cfg.endswith(suffix) and "_edge" not in cfg and ("+align" in cfg) == bool(suffix), cfg
            else:
                # (no room for copies: the predicated kernels, the wave kernels, or - k being a multiple of 32 - a
                # variant that gathers the operand that is off the grid with 4-byte loads)
                assert "+align" not in cfg and (suffix == "" or "_edge" in cfg or cfg.startswith("wave") or
                                                "_ga" in cfg or "_gb" in cfg), cfg
            check_against_oracle(dc[0].cpu().numpy(), a[0], b[0], exact=True, what=f"{m}x{n}x{k} {cfg}")
            mask = torch.ones_like(cflat, dtype=torch.bool)
            torch.as_strided(mask, (1, m, n), dc.stride(), offs[2]).fill_(False)
            assert bool((cflat[mask] == 7.0).all()), f"{cfg}: stores outside the output"


# ---- lane offsets beyond 2^31 bytes: the exact-fit kernels keep them as unsigned 32-bit byte offsets ----------------

@pytest.mark.parametrize("spec", ["t128x128x16_w64x64", "t128x256x32_w64x128_acc2", "p128x128x16_w64x64_ds:p1",
                                  "d64x64x32_w32x32_tf", "d128x128x32_w64x64", "d128x256x32_w64x128_acc2"])
def test_leading_dimensions_that_put_a_tile_row_beyond_2_gib(spec):
    """A with 2^22 floats per row: the last rows of a 128-row tile start 2.1 GB after its origin, beyond the range of
    a signed 32-bit byte offset and still within the 2^30 elements that the host admits for these kernels; C with a
    leading dimension of 2^21 likewise stretches the byte offsets of the stores.  (A is a view of a 4 GiB buffer.)"""
    import torch
    m, n, k = 256, 256, 64
    lda, ldc = 1 << 22, 1 << 21
    say(f"forced {spec} on {m}x{n}x{k} with lda = 2^22, ldc = 2^21")
    a, b = ig.make_operands(1, m, n, k, "int", 391, 392)
    a, b = a[0], b[0]
    big_a = torch.empty(m * lda, dtype=torch.float32, device="cuda")
    da = big_a.view(m, lda)[:, :k]
    da.copy_(to_dev(a))
    big_c = torch.empty(m * ldc, dtype=torch.float32, device="cuda")
    dc = big_c.view(m, ldc)[:, :n]
    dc.fill_(float("nan"))
    tg.force_config(spec)
    tg.sgemm(da, to_dev(b), out=dc)
    torch.cuda.synchronize()
    assert tg.last_config().startswith(spec.split(":")[0]), tg.last_config()
    check_against_oracle(dc.cpu().numpy(), a, b, exact=True, what=f"{spec} with rows 16 MB apart")
    del big_a, big_c

"""Host-only checks of the C-ABI: the library loads, exports every declared symbol, and
rejects bad arguments before touching a GPU.  No compute call with valid arguments is
made here (fake pointers are only ever passed together with arguments that must be
rejected, or with empty extents that launch nothing)."""
import ctypes
import pathlib
import re

import pytest

import paper_1904_03383_amd as tg
from paper_1904_03383_amd import binding

ROOT = pathlib.Path(__file__).resolve().parents[1]
FAKE = 0x1000  # 16-byte aligned, never dereferenced


@pytest.fixture(scope="module")
def lib():
    return tg.load_library()


def test_library_is_in_tree_and_exports_every_declared_symbol(lib):
    assert tg.library_path().exists() and ROOT in tg.library_path().parents
    header = (ROOT / "include" / "tgemm.h").read_text()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(tg_[a-z0-9_]+)\s*\(", header))
    assert declared == set(binding.SIGNATURES), declared ^ set(binding.SIGNATURES)
    for name in declared:
        assert hasattr(lib, name), name


def test_version_status_strings_and_kernel_table(lib):
    assert tg.version() >= 100
    assert lib.tg_status_string(0) == b"TG_OK" and lib.tg_status_string(1) == b"TG_ERR_INVALID_ARG"
    assert lib.tg_status_string(77) == b"TG_ERR_UNKNOWN"
    names = tg.kernel_names()
    assert len(names) == len(set(names)) >= 8 and "wave32" in names
    buf = ctypes.create_string_buffer(4)
    assert lib.tg_kernel_name(0, ctypes.cast(buf, ctypes.c_void_p), 4) == 1      # buffer too small
    assert lib.tg_kernel_name(-1, ctypes.cast(buf, ctypes.c_void_p), 4) == 1
    assert lib.tg_kernel_name(len(names), ctypes.cast(buf, ctypes.c_void_p), 4) == 1


BAD_SGEMM = [
    # (m, n, k, A, lda, B, ldb, C, ldc, fragment of the message)
    (-1, 4, 4, FAKE, 4, FAKE, 4, FAKE, 4, "negative"),
    (4, -1, 4, FAKE, 4, FAKE, 4, FAKE, 4, "negative"),
    (4, 4, -1, FAKE, 4, FAKE, 4, FAKE, 4, "negative"),
    (4, 4, 8, FAKE, 7, FAKE, 4, FAKE, 4, "leading dimension"),
    (4, 4, 8, FAKE, 8, FAKE, 3, FAKE, 4, "leading dimension"),
    (4, 4, 8, FAKE, 8, FAKE, 4, FAKE, 3, "leading dimension"),
    (4, 4, 8, None, 8, FAKE, 4, FAKE, 4, "null"),
    (4, 4, 8, FAKE, 8, None, 4, FAKE, 4, "null"),
    (4, 4, 8, FAKE, 8, FAKE, 4, None, 4, "null"),
    (4, 4, 0, None, 1, None, 4, None, 4, "null"),            # k == 0 still writes C
    (1 << 40, 4, 4, FAKE, 1 << 61, FAKE, 4, FAKE, 4, "overflow"),
]


@pytest.mark.parametrize("args", BAD_SGEMM, ids=lambda a: f"{a[-1]}-{a[0]}x{a[1]}x{a[2]}")
def test_sgemm_rejects_bad_arguments_before_any_gpu_call(lib, args):
    *call, frag = args
    st = lib.tg_sgemm(*call, None)
    assert st == 1, (st, lib.tg_last_error())
    assert frag in lib.tg_last_error().decode()


def test_dimension_beyond_int32_is_unsupported(lib):
    big = (1 << 31)
    st = lib.tg_sgemm(big, 1, 1, FAKE, 1, FAKE, 1, FAKE, 1, None)
    assert st == 2 and b"2^31" in lib.tg_last_error()


def test_batched_rejects_bad_strides(lib):
    ok = dict(batch=3, m=4, n=4, k=4)
    st = lib.tg_sgemm_batched(3, 4, 4, 4, FAKE, 4, 16, FAKE, 4, 16, FAKE, 4, 15, None)   # outputs overlap
    assert st == 1 and b"strideC" in lib.tg_last_error()
    st = lib.tg_sgemm_batched(3, 4, 4, 4, FAKE, 4, -1, FAKE, 4, 16, FAKE, 4, 16, None)
    assert st == 1 and b"stride" in lib.tg_last_error()
    st = lib.tg_sgemm_batched(-3, 4, 4, 4, FAKE, 4, 16, FAKE, 4, 16, FAKE, 4, 16, None)
    assert st == 1
    st = lib.tg_sgemm_batched(1 << 20, 1 << 20, 1 << 20, 4, FAKE, 4, 1 << 42, FAKE, 1 << 20, 16,
                              FAKE, 1 << 20, 1 << 42, None)
    assert st == 1 and b"overflow" in lib.tg_last_error()
    assert ok  # (kept for readability of the valid shape the cases above perturb)


def test_empty_problems_return_ok_without_a_launch(lib):
    assert lib.tg_sgemm(0, 5, 3, None, 3, None, 5, None, 5, None) == 0
    assert lib.tg_sgemm(5, 0, 3, None, 3, None, 1, None, 1, None) == 0
    assert lib.tg_sgemm_batched(0, 5, 5, 5, None, 5, 25, None, 5, 25, None, 5, 25, None) == 0
    assert lib.tg_tune(0, 5, 5, 5, None, 5, 25, None, 5, 25, None, 5, 25, None, 3) == 0


def test_strided_argument_checks(lib):
    ok = lib.tg_sgemm_strided
    assert ok(4, 4, 4, FAKE, 4, 0, FAKE, 4, 1, FAKE, 4, None) == 1 and b"positive" in lib.tg_last_error()
    assert ok(4, 4, 4, FAKE, 4, 2, FAKE, 4, -1, FAKE, 4, None) == 1
    assert ok(4, 4, 4, FAKE, 0, 2, FAKE, 4, 1, FAKE, 4, None) == 1
    assert ok(4, 4, 4, FAKE, 8, 2, FAKE, 4, 1, FAKE, 3, None) == 1 and b"leading dimension" in lib.tg_last_error()
    assert ok(4, 4, 4, None, 8, 2, FAKE, 4, 1, FAKE, 4, None) == 1 and b"null" in lib.tg_last_error()
    assert ok(1 << 30, 4, 1 << 30, FAKE, 1 << 40, 1 << 40, FAKE, 4, 1, FAKE, 4, None) == 1 and b"overflow" in lib.tg_last_error()
    assert ok(4, 4, 4, FAKE, 3, 1, FAKE, 4, 1, FAKE, 4, None) == 1          # unit strides: lda >= k as in tg_sgemm
    assert ok(0, 4, 4, None, 1, 7, None, 1, 9, None, 4, None) == 0          # empty: no launch


def test_saxpy_argument_checks(lib):
    assert lib.tg_saxpy(-1, 1.0, FAKE, FAKE, FAKE, None) == 1 and b"negative" in lib.tg_last_error()
    assert lib.tg_saxpy(8, 1.0, None, FAKE, FAKE, None) == 1 and b"null" in lib.tg_last_error()
    assert lib.tg_saxpy(8, 1.0, FAKE, None, FAKE, None) == 1
    assert lib.tg_saxpy(8, 1.0, FAKE, FAKE, None, None) == 1
    assert lib.tg_saxpy(0, 1.0, None, None, None, None) == 0          # empty: no launch


def test_tune_validates_like_sgemm(lib):
    st = lib.tg_tune(1, 4, 4, 8, FAKE, 7, 0, FAKE, 4, 0, FAKE, 4, 0, None, 3)
    assert st == 1 and b"leading dimension" in lib.tg_last_error()


def test_workspace_arguments(lib):
    assert lib.tg_set_workspace(FAKE, 0) == 1
    assert lib.tg_set_workspace(None, 64) == 1
    assert lib.tg_set_workspace(FAKE + 4, 64) == 1 and b"aligned" in lib.tg_last_error()
    assert lib.tg_set_workspace(None, 0) == 0
    assert tg.workspace_bytes(1, 1024, 1024, 1024) >= 2 * 1024 * 1024 * 4
    assert tg.workspace_bytes(1, 0, 8, 8) == 0 and tg.workspace_bytes(1, -1, 8, 8) == 0
    assert tg.workspace_bytes(1, 4096, 4096, 4096) == 0      # enough tiles: no split-K candidate
    # packed copies of the strided operands (rows padded to 4 floats) on top of the split-K need
    assert tg.strided_workspace_bytes(4096, 4096, 4096, 2, 1) == 4096 * 4096 * 4
    assert tg.strided_workspace_bytes(4096, 4096, 4096, 2, 3) == 2 * 4096 * 4096 * 4
    assert tg.strided_workspace_bytes(10, 4096, 7, 5, 1) == tg.workspace_bytes(1, 10, 4096, 7) + 10 * 8 * 4
    assert tg.strided_workspace_bytes(8, 8, 8, 0, 1) == 0 and tg.strided_workspace_bytes(8, 0, 8, 1, 1) == 0


def test_force_config_grammar_and_get_config(lib):
    names = tg.kernel_names()
    try:
        with pytest.raises(tg.TgemmError, match="unknown kernel"):
            tg.force_config("t1x1x1_w1x1")
        with pytest.raises(tg.TgemmError, match="bad"):
            tg.force_config(names[0] + ":x3")
        with pytest.raises(tg.TgemmError, match="bad"):
            tg.force_config(names[0] + ":s0")
        tg.force_config("t128x128x16_w64x64:s1:g4")
        assert tg.get_config(1, 1024, 1024, 1024) == "t128x128x16_w64x64:s1:g4"
        # forced but not valid for the shape: reported, not silently replaced
        with pytest.raises(tg.TgemmError, match="not valid here"):
            tg.get_config(1, 1024, 1024, 1001)           # a K remainder must be a multiple of 4 ...
        with pytest.raises(tg.TgemmError, match="not valid here"):
            tg.get_config(1, 1024, 1024, 12)             # ... and k at least one K tile
        assert tg.get_config(1, 1024, 1024, 1000) == "t128x128x16_w64x64:s1:g4"   # remainder tile goes first
        tg.force_config("d128x128x32_w64x64")
        with pytest.raises(tg.TgemmError, match="not valid here"):
            tg.get_config(1, 1024, 1024, 1000)           # the direct-to-LDS variants need whole K tiles
        tg.force_config("t128x128x16_w64x64:s1:g4")
        with pytest.raises(tg.TgemmError, match="not valid here"):
            tg.get_config(1, 1024, 1022, 1024)           # n must be a multiple of 4
        assert tg.get_config(1, 1000, 1000, 1024) == "t128x128x16_w64x64:s1:g4"   # ragged m and n are fine
        with pytest.raises(tg.TgemmError, match="single accumulator"):
            tg.get_config(1, 4096, 4096, 4096)
        tg.force_config("t128x128x16_w64x64:s4")
        with pytest.raises(tg.TgemmError) as ei:
            tg.get_config(1, 1024, 1024, 1024)           # split-K without workspace
        assert ei.value.status_name == "TG_ERR_WORKSPACE"
    finally:
        tg.force_config(None)
    # heuristic choices (nothing tuned, nothing forced)
    assert "_acc2" in tg.get_config(1, 4096, 4096, 4096).split(":")[0]              # long K: two levels
    assert "acc2" not in tg.get_config(1, 4096, 4096, 128)
    assert tg.get_config(512, 32, 32, 64).startswith("wave")
    assert "_edge" in tg.get_config(1, 1000, 1000, 1001) or tg.get_config(1, 1000, 1000, 1001).startswith("wave")
    assert "_edge" not in tg.get_config(1, 1000, 1000, 1024)      # ragged m, n with k % 32 == 0: exact-fit kernels
    assert tg.get_config(1, 1000, 1000, 1000).startswith("t")     # k % 4 == 0: register-staged exact-fit kernels
    assert "_edge" not in tg.get_config(1, 1000, 1000, 1000)
    tg.force_config("p128x128x16_w64x64:p2")
    try:
        with pytest.raises(tg.TgemmError, match="not valid here"):
            tg.get_config(1, 1000, 1024, 1024)           # the persistent variants walk whole tiles only
        tg.force_config("p128x128x16_w64x64_ds:p2")
        assert tg.get_config(1, 4096, 4096, 128) == "p128x128x16_w64x64_ds:s1:g8:p2"
        tg.force_config("p128x128x16_w64x64_ds:s2:p2")
        with pytest.raises(tg.TgemmError, match="no split-K"):
            tg.get_config(1, 1024, 1024, 1024)           # the deferred-store variant writes C only
    finally:
        tg.force_config(None)
    buf = ctypes.create_string_buffer(4)
    assert lib.tg_get_config(1, 64, 64, 64, ctypes.cast(buf, ctypes.c_void_p), 4) == 1
    assert lib.tg_get_config(1, 0, 64, 64, ctypes.cast(buf, ctypes.c_void_p), 4) == 1


def test_tune_cache_file_round_trip(tmp_path, lib):
    path = tmp_path / "cache.txt"
    path.write_text("tgemm-tune-cache 3 gfx950\n"
                    "1 1024 1024 1024 1 t128x128x16_w64x64 1 4 0 0 20.5\n"
                    "1 512 512 512 1 p128x128x32_w64x64 1 2 2 3 7.5\n"
                    "1 2048 2048 2048 1 some_kernel_of_another_build 1 4 0 0 99.0\n")
    try:
        tg.clear_tune_cache()
        tg.load_tune_cache(path)
        assert tg.get_config(1, 1024, 1024, 1024) == "t128x128x16_w64x64:s1:g4"
        out = tmp_path / "saved.txt"
        tg.save_tune_cache(out)
        text = out.read_text().splitlines()
        assert tg.get_config(1, 512, 512, 512) == "p128x128x32_w64x64:s1:g2:o2:p3"
        # written in the current format (version 5: two tail-split fields before the time, 16 x math mode in the
        # layout class); version 3 and 4 files load
        assert text[0] == "tgemm-tune-cache 5 gfx950" and len(text) == 3
        assert text[1].startswith("1 512 512 512 1 p128x128x32_w64x64 1 2 2 3 0 1 ")
        assert text[2].startswith("1 1024 1024 1024 1 t128x128x16_w64x64 1 4 0 0 0 1 ")
        v4 = tmp_path / "v4.txt"
        v4.write_text("tgemm-tune-cache 4 gfx950\n"
                      "1 3072 3072 3072 1 t128x256x32_w64x128_acc2 1 8 0 0 3 6 440.0\n"
                      "this line is damaged\n"
                      "1 640 512 256 1 t128x128x16_w64x64 1 2 0 0 0 1 9.0\n")
        tg.clear_tune_cache()
        tg.load_tune_cache(v4)
        assert tg.get_config(1, 640, 512, 256) == "t128x128x16_w64x64:s1:g2"
        # (the tail-split entry needs a workspace to be used; without one the heuristic answers)
        assert ":t" not in tg.get_config(1, 3072, 3072, 3072)
        lib.tg_set_workspace(ctypes.c_void_p(0x10000), 1 << 30)
        assert tg.get_config(1, 3072, 3072, 3072) == "t128x256x32_w64x128_acc2:s1:g8:t3x6"
        lib.tg_set_workspace(None, 0)
        bad = tmp_path / "bad.txt"
        bad.write_text("something else\n")
        with pytest.raises(tg.TgemmError):
            tg.load_tune_cache(bad)
        with pytest.raises(tg.TgemmError):
            tg.load_tune_cache(tmp_path / "missing.txt")
    finally:
        tg.clear_tune_cache()
    assert tg.get_config(1, 1024, 1024, 1024) != "t128x128x16_w64x64:s1:g4"


def test_binding_refuses_non_device_tensors():
    import torch
    a = torch.zeros(4, 4)
    with pytest.raises(ValueError, match="device memory"):
        tg.sgemm(a, a)
    with pytest.raises(ValueError, match="device memory"):
        tg.sgemm_batched(a[None], a[None])


def test_strided_binding_refuses_views_without_positive_strides():
    """An expanded view (stride 0) has no element-stride form; turning the 0 into 1 would read past its storage."""
    import torch
    from paper_1904_03383_amd import binding
    v = torch.zeros(8)
    with pytest.raises(ValueError, match="positive strides"):
        binding._elem_strides(v.expand(5, 8))          # strides (0, 1)
    with pytest.raises(ValueError, match="positive strides"):
        binding._elem_strides(v[:, None].expand(8, 5))  # strides (1, 0)
    assert binding._elem_strides(torch.zeros(6, 64)[:, ::32]) == (64, 32)
    assert binding._elem_strides(torch.zeros(6, 4).T) == (1, 4)
    assert binding._elem_strides(v.expand(1, 8)) == (1, 1)   # extent 1: its stride is never used


def test_header_is_plain_c_and_every_entry_point_links(tmp_path, may_spawn):
    """gcc -std=c99 program that includes only tgemm.h, links libtgemm.so and calls each entry point's error path."""
    import os
    import subprocess
    exe = tmp_path / "abi_check"
    libdir = tg.library_path().parent
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", str(ROOT / "include"),
                    str(ROOT / "tests" / "c_abi" / "abi_check.c"), "-o", str(exe),
                    "-L", str(libdir), "-ltgemm", f"-Wl,-rpath,{libdir}"], check=True)
    env = dict(os.environ)
    r = subprocess.run([str(exe)], capture_output=True, text=True, env=env)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "abi_check: ok" in r.stdout


def test_product_package_does_not_import_the_oracle():
    pkg = ROOT / "paper_1904_03383_amd"
    for f in list(pkg.rglob("*.py")) + list(pkg.rglob("*.hip")) + list(pkg.rglob("*.cpp")) + list(pkg.rglob("*.h*")):
        if any(part.startswith("_build") for part in f.parts):
            continue
        text = f.read_text()
        assert "oracle" not in text.lower().replace("oracle's tests", ""), f
    for f in (ROOT / "oracle").glob("*"):
        if f.suffix in (".py", ".c"):
            assert "paper_1904_03383_amd" not in f.read_text() and "tgemm" not in f.read_text(), f


def test_tune_cli_shape_parser():
    from paper_1904_03383_amd.tune import parse_shape
    assert parse_shape("4096x4096x128") == (1, 4096, 4096, 128)
    assert parse_shape("512:32x32X64") == (512, 32, 32, 64)
    for bad in ("0x4x4", "4x4", "2:4x4x0", "axbxc"):
        with pytest.raises(ValueError):
            parse_shape(bad)


def test_host_logic_survives_random_sizes_specs_and_cache_files(tmp_path, may_spawn):
    """tests/c_abi/host_fuzz.c: 40000 random shapes through the chooser, 20000 random specs, 300 random cache files."""
    import subprocess
    exe = tmp_path / "host_fuzz"
    pkg = ROOT / "paper_1904_03383_amd"
    subprocess.run(["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-I", str(ROOT / "include"), str(ROOT / "tests" / "c_abi" / "host_fuzz.c"),
                    "-L", str(pkg), "-ltgemm", f"-Wl,-rpath,{pkg}", "-o", str(exe)], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True, cwd=tmp_path)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "fuzz: ok" in r.stdout


# --- the tuner's search space: cost-model order and the lower-bound cut (Sec. 5.1) ---------------

PEAK_FLOPS = 157.3e12   # published fp32 MFMA rate of the chip
PEAK_HBM = 8e12
SEARCH_SHAPES = [(1, 256, 256, 32), (1, 1024, 1024, 1024), (512, 32, 32, 64), (1, 4096, 4096, 128),
                 (1, 4096, 4096, 4096), (1, 1000, 1000, 1000), (1, 32, 8192, 8192), (7, 130, 68, 36),
                 (1, 33, 65, 17)]


@pytest.mark.parametrize("shape", SEARCH_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_candidates_are_valid_ordered_and_bounded(lib, shape):
    batch, m, n, k = shape
    cands = tg.candidates(batch, m, n, k)
    assert cands and len({c[0] for c in cands}) == len(cands)
    names = set(tg.kernel_names())
    flops = 2.0 * batch * m * n * k
    data = 4.0 * batch * (m * k + k * n + m * n)
    floor_us = 1e6 * max(flops / PEAK_FLOPS, data / PEAK_HBM)
    models = [c[2] for c in cands]
    assert models == sorted(models)                    # timed cheapest-first, so the cut bites early
    for spec, bound_us, model_us in cands:
        assert spec.split(":")[0] in names
        # no configuration can beat the chip: every bound includes the whole-chip floor ...
        assert bound_us >= floor_us * (1 - 1e-12)
        # ... and the cost model (which adds launch cost and an efficiency below 1) never undercuts it
        assert model_us >= bound_us, (spec, bound_us, model_us)
        # the spec is usable as it stands
        tg.force_config(spec)
        assert tg.get_config(batch, m, n, k) == spec
    tg.force_config(None)
    # what an untuned call runs is the head of the list
    assert tg.get_config(batch, m, n, k) == cands[0][0]


@pytest.mark.parametrize("shape,expect", [
    # short K, plain operands, tiles that divide over 256 workgroups: the row panels with A resident in LDS
    ((4096, 4096, 128), r"g32x(512|1024)x64_w32x64(_b3)?_res_ga:.*:p1$"),
    ((2048, 8192, 256), r"g32x(512|1024)x64_w32x64(_b3)?_res_ga:"),
    # ... but not below 512 rows (B's lines are then first touched by the wave that needs them) nor from k = 512 on
    ((256, 16384, 256), r"[tdw]"),
    ((4096, 4096, 512), r"[td]"),
    # a single long-K product whose 32 x 512 panels fill every CU the same number of times: deep-chunk row panels
    ((8192, 8192, 8192), r"g32x512x(128|256)_w32x64_acc2_b3_ga:s1"),
    ((2048, 2048, 2048), r"g32x512x(128|256)_w32x64_acc2_b3_ga:s1"),
    # ... with a partly empty last round the tile kernels keep the product (576 panels over 256 CUs)
    ((3072, 3072, 3072), r"[td]"),
    ((2048, 1024, 4096), r"[td]"),
], ids=str)
def test_untuned_choice_on_shapes_the_row_panels_were_measured_on(lib, shape, expect):
    """The cost model's first choice for a few shapes on either side of the rules that hand plain products to the
    row-panel kernels (each rule stands on same-process measurements quoted beside it in the cost model)."""
    import re
    m, n, k = shape
    first = tg.candidates(1, m, n, k)[0][0]
    assert re.match(expect, first), first
    batch = tg.candidates(4, m, n, k)[0][0] if m * n * k <= 2048 ** 3 else None
    if batch is not None and k >= 2048:
        assert not batch.startswith("g"), batch          # on batches the tile kernels are level or ahead


def test_lower_bound_reflects_tile_quantisation_and_wave_share(lib):
    by = {spec: (lb, model) for spec, lb, model in tg.candidates(1, 4096, 4096, 4096)}
    simd_flops = 64 * 2.4e9            # one SIMD: 64 flop per clock at 2.4 GHz; 1024 of them make the chip
    chip_us = 1e6 * 2.0 * 4096 ** 3 / (1024 * simd_flops)
    # 128x128 tiles: 1024 workgroups of 4 waves = exactly 4 full rounds over 256 CUs x 4 SIMDs: the chip floor
    assert by["t128x128x32_w64x64_acc2:s1:g8"][0] == pytest.approx(chip_us, rel=1e-9)
    # 256x256 tiles at 1024^3: 16 workgroups on 16 CUs, each wave owns 128x128x1024 -> 16x the chip floor
    mid = {spec: lb for spec, lb, _ in tg.candidates(1, 1024, 1024, 1024)}
    assert mid["d256x256x32_w128x128:s1:g8"] == pytest.approx(1e6 * 2.0 * 128 * 128 * 1024 / simd_flops, rel=1e-9)
    assert mid["d64x64x32_w32x32:s1:g8"] == pytest.approx(1e6 * 2.0 * 1024 ** 3 / (1024 * simd_flops), rel=1e-9)
    # a small problem: one 64x64 tile per CU at most -> a wave's own 32x32xK share on its SIMD binds,
    # which is far above the whole-chip floor
    small = {spec: lb for spec, lb, _ in tg.candidates(1, 256, 256, 32)}
    assert small["t64x64x32_w32x32:s1:g8"] == pytest.approx(1e6 * 2.0 * 32 * 32 * 32 / simd_flops, rel=1e-9)
    # 1000^3 on 128x128 tiles: 64 workgroups -> one round of 64x64x1000(+tail) per wave
    rag = {spec: lb for spec, lb, _ in tg.candidates(1, 1000, 1000, 1000)}
    assert rag["t128x128x16_w64x64:s1:g8"] == pytest.approx(1e6 * 2.0 * 64 * 64 * 1000 / simd_flops, rel=1e-9)


def test_lower_bound_cut_never_drops_a_config_that_could_win(lib):
    """Replay of the sweep on the host: candidates are taken in order, one is skipped when its bound is
    not below the best time so far.  With any timings that respect the bounds (time >= bound), the
    configuration with the smallest time is never among the skipped ones."""
    import random
    rng = random.Random(5)
    for shape in SEARCH_SHAPES:
        cands = tg.candidates(*shape)
        for _ in range(20):
            times = [lb * (1.0 + rng.random() * rng.choice([0.05, 0.5, 3.0])) for _, lb, _ in cands]
            best, skipped = float("inf"), []
            for i, (_, lb, _) in enumerate(cands):
                if lb >= best:
                    skipped.append(i)
                    continue
                best = min(best, times[i])
            assert best == min(times)
            assert all(times[i] >= best for i in skipped)
    # and the cut does bite: at 1024^3 the big tiles leave most of the chip idle, and their bounds say so
    mid = tg.candidates(1, 1024, 1024, 1024)
    assert max(lb for _, lb, _ in mid) > 10 * min(lb for _, lb, _ in mid)


def test_candidate_argument_checks(lib):
    buf = ctypes.create_string_buffer(64)
    p = ctypes.cast(buf, ctypes.c_void_p)
    assert lib.tg_num_candidates(1, 0, 64, 64) == -1 and b"positive" in lib.tg_last_error()
    assert lib.tg_candidate(1, 64, 64, 64, 0, None, 0, None, None) == 1
    assert lib.tg_candidate(1, 64, 64, 64, 0, p, 2, None, None) == 1          # buffer too small
    count = lib.tg_num_candidates(1, 64, 64, 64)
    assert count > 0
    assert lib.tg_candidate(1, 64, 64, 64, count, p, 64, None, None) == 1      # index out of range
    assert lib.tg_candidate(1, 64, 64, 64, -1, p, 64, None, None) == 1
    assert lib.tg_candidate(1, 64, 64, 64, 0, p, 64, None, None) == 0 and buf.value
    assert lib.tg_candidate(1, 2 ** 31, 64, 64, 0, p, 64, None, None) == 2


# --- math mode ------------------------------------------------------------------------------------

def test_math_mode_gates_the_piece_kernels(lib):
    assert tg.get_math() == tg.MATH_FP32_MFMA
    assert lib.tg_set_math(7) == 1 and b"math mode" in lib.tg_last_error()
    shape = (1, 4096, 4096, 4096)
    try:
        fp32 = tg.candidates(*shape)
        assert not any(s.startswith("e") for s, _, _ in fp32)
        tg.set_math(tg.MATH_BF16_PIECES)
        assert tg.get_math() == tg.MATH_BF16_PIECES
        both = tg.candidates(*shape)
        pieces = {s: (lb, model) for s, lb, model in both if s.startswith("e")}
        assert set(pieces) == {"e128x256x32_w64x128_x6:s1:g8", "e128x256x32_w64x128_x9:s1:g8",
                               "e128x128x32_w64x64_x6:s1:g8", "e64x64x32_w32x32_x6:s1:g8"}
        assert {s for s, _, _ in fp32} == {s for s, _, _ in both} - set(pieces)
        # bounds: 16/6 and 16/9 of the fp32 pipe's rate
        chip_us = 1e6 * 2.0 * 4096 ** 3 / (1024 * 64 * 2.4e9)
        assert pieces["e128x256x32_w64x128_x6:s1:g8"][0] == pytest.approx(chip_us * 6 / 16, rel=1e-9)
        assert pieces["e128x256x32_w64x128_x9:s1:g8"][0] == pytest.approx(chip_us * 9 / 16, rel=1e-9)
        # the cost model ranks the six-product kernel first for this size
        assert tg.get_config(*shape).startswith("e128x256x32_w64x128_x6")
        # not offered where they cannot run: k not a multiple of 32, or a K range beyond 8192 without a split
        assert not any(s.startswith("e") for s, _, _ in tg.candidates(1, 4096, 4096, 4080))
        assert not any(s.startswith("e") for s, _, _ in tg.candidates(1, 512, 512, 16384))
    finally:
        tg.set_math(tg.MATH_FP32_MFMA)
    assert not tg.get_config(*shape).startswith("e")
    # a forced piece kernel is accepted in either mode
    tg.force_config("e128x256x32_w64x128_x9")
    assert tg.get_config(*shape) == "e128x256x32_w64x128_x9:s1:g8"
    tg.force_config(None)


def test_tail_split_grammar_validity_and_candidates(lib):
    """t<rows>x<splits>: the last tile rows go out as a second launch with split-K (Sec. 5.1's space grows by
    one decision; here it is offered when the tile count is a little above a multiple of the chip's slots)."""
    for bad in ("t128x256x32_w64x128_acc2:t3", "t128x256x32_w64x128_acc2:t0x4", "t128x256x32_w64x128_acc2:t3x1", "t128x256x32_w64x128_acc2:tx4"):
        assert lib.tg_force_config(bad.encode()) == 1, bad
    try:
        lib.tg_set_workspace(ctypes.c_void_p(0x10000), 1 << 30)
        tg.force_config("t128x256x32_w64x128_acc2:t3x6")
        assert tg.get_config(1, 3072, 3072, 3072) == "t128x256x32_w64x128_acc2:s1:g8:t3x6"
        buf = ctypes.create_string_buffer(256)
        p = ctypes.cast(buf, ctypes.c_void_p)
        tg.force_config("t128x256x32_w64x128_acc2:t24x2")          # 3072 rows are 24 tile rows: none left for the first launch
        assert lib.tg_get_config(1, 3072, 3072, 3072, p, 256) == 1 and b"at least one tile row" in lib.tg_last_error()
        tg.force_config("p128x128x16_w64x64:p1:t1x2")
        assert lib.tg_get_config(1, 1024, 1024, 64, p, 256) == 1 and b"no tail split" in lib.tg_last_error()
        tg.force_config("t128x256x32_w64x128_acc2:s2:t3x6")
        assert lib.tg_get_config(1, 3072, 3072, 3072, p, 256) == 1 and b"goes with s1" in lib.tg_last_error()
        tg.force_config(None)
        # 3072^3 on 128x256 tiles: 288 tiles = 256 + 32 -> the last 3 tile rows (36 tiles), split 6 ways
        specs = {s: (lb, model) for s, lb, model in tg.candidates(1, 3072, 3072, 3072)}
        assert "t128x256x32_w64x128_acc2:s1:g8:t3x6" in specs and "d128x256x32_w64x128_acc2:s1:g8:t3x6" in specs
        plain, tail = specs["t128x256x32_w64x128_acc2:s1:g8"], specs["t128x256x32_w64x128_acc2:s1:g8:t3x6"]
        assert tail[1] < 0.75 * plain[1]              # the cost model sees one round and a bit instead of two
        assert tail[0] <= tail[1]
        # 4096^3 fills its two rounds exactly: nothing to split off
        assert not any(":t" in s for s, _, _ in tg.candidates(1, 4096, 4096, 4096))
        # and without a workspace no tail split is offered
        lib.tg_set_workspace(None, 0)
        assert not any(":t" in s for s, _, _ in tg.candidates(1, 3072, 3072, 3072))
    finally:
        tg.force_config(None)
        lib.tg_set_workspace(None, 0)


def test_tuned_entries_are_kept_per_math_mode(tmp_path, lib):
    """A cache file holds the math mode in the shape class (16 x mode + layout class; 4 x mode in files of
    versions 3 and 4, converted on loading): an entry tuned in the piece mode is used only there."""
    f = tmp_path / "cache.txt"
    f.write_text("tgemm-tune-cache 3 gfx950\n"
                 "1 4096 4096 4096 1 t128x256x32_w64x128_acc2 1 4 0 0 975.0\n"
                 "1 4096 4096 4096 5 e128x256x32_w64x128_x9 1 2 0 0 830.0\n")
    try:
        tg.load_tune_cache(f)
        assert tg.get_config(1, 4096, 4096, 4096) == "t128x256x32_w64x128_acc2:s1:g4"
        tg.set_math(tg.MATH_BF16_PIECES)
        assert tg.get_config(1, 4096, 4096, 4096) == "e128x256x32_w64x128_x9:s1:g2"
        out = tmp_path / "again.txt"
        tg.save_tune_cache(out)
        lines = sorted(out.read_text().splitlines()[1:])
        assert [l.split()[4:6] for l in lines] == [["1", "t128x256x32_w64x128_acc2"], ["17", "e128x256x32_w64x128_x9"]]
    finally:
        tg.set_math(tg.MATH_FP32_MFMA)
        tg.clear_tune_cache()
    # nothing tuned any more: the heuristic answers, with a kernel that has the second accumulation level K = 4096 needs
    assert "_acc2" in tg.get_config(1, 4096, 4096, 4096).split(":")[0]


def test_launch_bound_classification_comes_from_the_cost_model(lib):
    """tg_tune times launch-bound problems as graph replays.  Which problems those are is a function of the sizes
    alone (the cost model's device time of the first candidate, under 12 us), so no measured per-call time, however
    inflated by a slow host or a profiler, can switch the device-time measurement off."""
    assert tg.tune_is_launch_bound(1, 256, 256, 32)            # c1
    assert tg.tune_is_launch_bound(512, 32, 32, 64)            # c3
    assert not tg.tune_is_launch_bound(1, 1024, 1024, 1024)    # c2: 20 us of device time
    assert not tg.tune_is_launch_bound(1, 4096, 4096, 128)
    assert not tg.tune_is_launch_bound(1, 4096, 4096, 4096)
    # the answer agrees with the model's own figure for the first candidate
    for shape in [(1, 256, 256, 32), (512, 32, 32, 64), (1, 512, 512, 256), (1, 1024, 1024, 1024), (1, 2048, 2048, 64)]:
        first = tg.candidates(*shape)[0]
        assert tg.tune_is_launch_bound(*shape) == (first[2] - 4.0 < 12.0), (shape, first)
    with pytest.raises(tg.TgemmError):
        tg.tune_is_launch_bound(1, 0, 8, 8)


def test_tune_cache_named_by_the_environment_is_loaded_at_first_use(tmp_path, may_spawn):
    """TG_TUNE_CACHE is read once, at the first call that chooses a configuration: checked in a fresh process."""
    import os
    import subprocess
    import sys
    cache = tmp_path / "env_cache.txt"
    cache.write_text("tgemm-tune-cache 5 gfx950\n1 1024 1024 1024 1 t128x128x16_w64x64 1 4 0 0 0 1 20.5\n")
    code = ("import paper_1904_03383_amd as tg; print(tg.get_config(1, 1024, 1024, 1024)); "
            "print(tg.get_config(1, 512, 512, 512))")
    env = dict(os.environ, TG_TUNE_CACHE=str(cache), PYTHONPATH=str(ROOT))
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=env)
    assert r.returncode == 0, r.stderr
    lines = r.stdout.split()
    assert lines[0] == "t128x128x16_w64x64:s1:g4" and not lines[1].startswith("t128x128x16_w64x64:s1:g4")
    # a file that does not exist (yet) is not an error; a damaged one is reported and ignored
    env["TG_TUNE_CACHE"] = str(tmp_path / "not_there.txt")
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=env)
    assert r.returncode == 0 and "ignoring" not in r.stderr
    bad = tmp_path / "bad.txt"
    bad.write_text("garbage\n")
    env["TG_TUNE_CACHE"] = str(bad)
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, env=env)
    assert r.returncode == 0 and "ignoring TG_TUNE_CACHE" in r.stderr


def test_the_poison_flavour_really_writes_into_lds(tmp_path, may_spawn):
    """The direct-to-LDS kernels fill LDS by loads only: the release build of one of them holds no LDS write at all,
    the TG_POISON_LDS build must (the NaN it puts into every stage before the stage is refilled)."""
    import subprocess
    from paper_1904_03383_amd import build as lib_build
    src = ROOT / "paper_1904_03383_amd" / "csrc" / "tile_inst_deep.hip"
    counts = {}
    for flavour, defs in (("release", []), ("poison", ["-DTG_POISON_LDS"])):
        out = tmp_path / f"{flavour}.s"
        cmd = [lib_build._hipcc()] + lib_build.HIP_FLAGS + defs + ["--cuda-device-only", "-S", str(src), "-o", str(out)]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
        counts[flavour] = len(re.findall(r"^\s*ds_write", out.read_text(), flags=re.M))
    assert counts["release"] == 0 and counts["poison"] >= 8, counts

"""The debug flavour of the library (libtgemm_poison.so, compiled with TG_POISON_LDS): every LDS-staged kernel
overwrites a stage with NaN once it has given it up and before it is refilled.  A kernel that read staging memory
too late (after the barrier that releases it) or too early (before its loads had landed) would return NaN here
where the release flavour returns stale but plausible numbers; every kernel family must still match the oracle, to
the same bar as the release library, on K ranges of several tiles (so that every stage of a ring is reused)."""
import re

import numpy as np
import pytest

import paper_1904_03383_amd as tg
from paper_1904_03383_amd import inputgen as ig

from gpu_common import check_against_oracle, say, to_dev

pytestmark = pytest.mark.gpu

_lib = None


def _poison():
    global _lib
    if _lib is None:
        _lib = tg.open_library(tg.poison_library_path())
    return _lib


def _sgemm(lib, spec, a, b, ws=None):
    import torch
    m, k = a.shape
    n = b.shape[1]
    da, db = to_dev(a), to_dev(b)
    out = torch.full((m, n), float("nan"), device="cuda")
    assert lib.tg_set_workspace(ws.data_ptr() if ws is not None else None, ws.numel() * 4 if ws is not None else 0) == 0
    assert lib.tg_force_config(spec.encode()) == 0, lib.tg_last_error().decode()
    try:
        st = lib.tg_sgemm(m, n, k, da.data_ptr(), k, db.data_ptr(), n, out.data_ptr(), n, torch.cuda.current_stream().cuda_stream)
        assert st == 0, lib.tg_last_error().decode()
        torch.cuda.synchronize()
        assert lib.tg_last_config().decode().startswith(spec.split(":")[0])
    finally:
        lib.tg_force_config(None)
        lib.tg_set_workspace(None, 0)
    return out.cpu().numpy()


def test_the_flavour_says_what_it_is():
    assert _poison().tg_version() == tg.version() + 1000000
    assert _poison().tg_num_kernels() == len(tg.kernel_names())


# one or two variants of every kernel family that stages operands through LDS: register-staged (t), predicated
# (edge), persistent stream with and without deferred stores (p), direct-to-LDS rings of two to four stages (d),
# the whole-tile fragment prefetch (tf), gathering and transposed-operand loaders (on plain operands where they
# can read them), row panels with producer waves (g)
SPECS = ["t128x128x16_w64x64", "t128x256x32_w64x128_acc2", "t64x64x32_w32x32", "t64x64x16_w32x32_edge",
         "p128x128x16_w64x64:p1", "p128x128x16_w64x64_ds:p2", "p128x128x32_w64x64:p2",
         "d128x128x32_w64x64", "d128x256x32_w64x128_acc2_st3", "d64x64x32_w32x32_st4", "d64x64x32_w32x32_k2",
         "d64x64x32_w32x32_tf", "d64x64x64_w32x32_acc2_tf", "d256x256x32_w128x128",
         "d64x64x32_w32x32_acc2_st4_ga", "d16x256x32_w16x64_acc2_st3_ga", "d64x64x32_w32x32_acc2_tf_gb",
         "g16x1024x64_w16x128_acc2_ga", "g32x512x64_w32x128_acc2_ga", "g32x1024x64_w32x128_ga",
         "g32x512x64_w32x64_acc2_ga", "g16x256x64_w16x64_acc2_b3_ga", "g32x512x64_w32x64_acc2_b3_ga",
         "g32x512x128_w32x64_acc2_b3_ga", "g32x512x64_w32x64_rw_ga:p1", "g32x512x64_w32x64_res_ga:p1",
         "g32x1024x64_w32x64_res_ga:p1"]


@pytest.mark.parametrize("spec", SPECS)
def test_no_kernel_reads_a_stage_it_has_given_up(spec):
    lib = _poison()
    persistent = spec.startswith("p")
    # (a second accumulation level is needed, and tested, beyond k = 1024)
    shapes = [(512, 512, 448)] if persistent else [(300, 260, 448)] + ([(256, 512, 2112)] if "acc2" in spec else [])
    if "_edge" in spec:
        shapes = [(301, 259, 413)]
    if "_rw_" in spec or "_res_" in spec:         # workgroups that walk two column tiles each (one of 1024 columns)
        shapes = [(4096, 2048, 192)]
    if re.match(r"[a-z]\d+x\d+x128_", spec):      # K tiles of 128
        shapes = [(300, 260, 384), (256, 512, 2176)]
    for (m, n, k) in shapes:
        for dist in ("normal", "int"):
            say(f"poison flavour, forced {spec} on {m}x{n}x{k} ({dist})")
            (a, b) = ig.make_operands(1, m, n, k, dist, 801, 802)
            c = _sgemm(lib, spec, a[0], b[0])
            check_against_oracle(c, a[0], b[0], exact=(dist == "int"), what=f"poison {spec} {m}x{n}x{k} {dist}")


def test_the_automatic_choice_on_the_benchmark_shapes():
    lib = _poison()
    import torch
    for name in ("c1_256x256x32", "c2_1024", "c4_4096x4096x128"):
        a, b = ig.make_config(name)
        a, b = a[0], b[0]
        m, k = a.shape
        n = b.shape[1]
        say(f"poison flavour, automatic choice on {name}")
        da, db = to_dev(a), to_dev(b)
        out = torch.full((m, n), float("nan"), device="cuda")
        assert lib.tg_sgemm(m, n, k, da.data_ptr(), k, db.data_ptr(), n, out.data_ptr(), n, torch.cuda.current_stream().cuda_stream) == 0
        torch.cuda.synchronize()
        rows = np.arange(0, m, max(1, m // 64))
        check_against_oracle(out.cpu().numpy()[rows], a[rows], b, what=f"poison auto {name}")

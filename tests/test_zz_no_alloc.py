"""GPU test of tg_sgemm_splitk_static, the entry point for callers that cannot allocate: its split-K
partials live in the library's own fixed device array.  Two calls in a row, the second with a smaller
input (the array keeps the first call's contents), each compared with the same split configuration run
through tg_sgemm on a caller workspace (must be bit-identical: same kernels, same summation order) and
with the CPU oracle to the bar of the benchmark definition; plus what the entry point refuses."""
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


def _static_then_workspace(a, b, exact):
    """Runs the static-scratch entry point, then tg_sgemm forced to the configuration it chose with a
    workspace of the scratch's size; returns both results."""
    import torch
    m, n = a.shape[0], b.shape[1]
    da, db = to_dev(a), to_dev(b)
    out = torch.full((m, n), float("nan"), device="cuda")
    tg.sgemm_splitk_static(da, db, out=out)
    torch.cuda.synchronize()
    cfg = tg.last_config()
    assert ":s1:" not in cfg + ":" and ":s" in cfg, cfg          # a real split
    c_static = out.cpu().numpy()
    check_against_oracle(c_static, a, b, exact=exact, what=f"static scratch {a.shape}x{b.shape} {cfg}")
    return da, db, cfg, c_static


def test_two_calls_in_a_row_second_smaller_match_the_workspace_path():
    import torch
    first = (256, 256, 4096)
    second = (192, 160, 2048)       # smaller, and ragged against every tile shape
    results = []
    for (m, n, k), seed in ((first, 901), (second, 903)):
        for dist in ("normal", "int"):
            say(f"static scratch {m}x{n}x{k} {dist}")
            gen = ig.normal if dist == "normal" else ig.small_int
            a, b = gen(seed, (m, k)), gen(seed + 1, (k, n))
            results.append((a, b, dist) + _static_then_workspace(a, b, dist == "int"))
    # the same configurations through the existing entry point, on a caller workspace (allocated only now,
    # after every static call has run)
    ws = torch.full((tg.binding.STATIC_SCRATCH_BYTES // 4,), float("nan"), device="cuda")
    tg.set_workspace(ws)
    for a, b, dist, da, db, cfg, c_static in results:
        say(f"workspace path {a.shape}x{b.shape} {dist} forced {cfg}")
        tg.force_config(cfg)
        out = torch.full(c_static.shape, float("nan"), device="cuda")
        tg.sgemm(da, db, out=out)
        torch.cuda.synchronize()
        assert tg.last_config() == cfg
        assert np.array_equal(out.cpu().numpy(), c_static), f"{cfg}: static scratch and workspace results differ"
    tg.force_config(None)
    tg.set_workspace(None)
    del ws


def test_forced_split_and_leading_dimensions():
    import torch
    say("static scratch, forced t128x128x32_w64x64:s4, padded rows")
    m, n, k = 200, 136, 1024
    a_store, b_store = ig.small_int(911, (m, k + 8)), ig.small_int(912, (k, n + 12))
    da, db = to_dev(a_store)[:, :k], to_dev(b_store)[:, :n]
    c_store = torch.full((m, n + 4), -7.0, device="cuda")
    tg.force_config("t128x128x32_w64x64:s4")
    tg.sgemm_splitk_static(da, db, out=c_store[:, :n])
    torch.cuda.synchronize()
    assert tg.last_config().startswith("t128x128x32_w64x64:s4")
    host = c_store.cpu().numpy()
    assert (host[:, n:] == -7.0).all()                              # padding of C untouched
    check_against_oracle(host[:, :n].copy(), a_store[:, :k].copy(), b_store[:, :n].copy(), exact=True, what="forced split")


def test_what_the_entry_point_refuses():
    import torch
    say("static scratch refusals (no launch)")
    # beyond the scratch: 2 * m * n * 4 bytes > 32 MiB
    m = n = 2304
    a = torch.zeros((m, 64), device="cuda")
    b = torch.zeros((64, n), device="cuda")
    with pytest.raises(tg.TgemmError) as e:
        tg.sgemm_splitk_static(a, b)
    assert e.value.status_name == "TG_ERR_WORKSPACE" and "static scratch" in str(e.value)
    # K too short to split
    a = torch.zeros((64, 32), device="cuda")
    b = torch.zeros((32, 64), device="cuda")
    with pytest.raises(tg.TgemmError) as e:
        tg.sgemm_splitk_static(a, b)
    assert e.value.status_name == "TG_ERR_UNSUPPORTED"
    # a forced configuration that is no split
    tg.force_config("t64x64x32_w32x32")
    a = torch.zeros((64, 1024), device="cuda")
    b = torch.zeros((1024, 64), device="cuda")
    with pytest.raises(tg.TgemmError) as e:
        tg.sgemm_splitk_static(a, b)
    assert e.value.status_name == "TG_ERR_INVALID_ARG"
    tg.force_config(None)
    # degenerate sizes: nothing to do, and k == 0 zero-fills
    out = torch.full((8, 8), float("nan"), device="cuda")
    tg.sgemm_splitk_static(torch.zeros((8, 0), device="cuda"), torch.zeros((0, 8), device="cuda"), out=out)
    torch.cuda.synchronize()
    assert (out.cpu().numpy() == 0).all()

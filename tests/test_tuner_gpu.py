"""GPU tests of the timing tuner (tg_tune): launch-bound problems are timed by their device time whatever the
host's per-call cost, every candidate's product is checked against the first candidate's before it may lead,
and a tune cache named by the environment is rewritten after a tuning."""
import os

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
    tg.clear_tune_cache()
    yield
    for var in ("TG_TUNE_TEST_HOST_DELAY_US", "TG_TUNE_TEST_SPOIL_REFERENCE", "TG_TUNE_CACHE"):
        os.environ.pop(var, None)
    tg.force_config(None)
    tg.set_workspace(None)
    tg.clear_tune_cache()


@pytest.mark.parametrize("name", ["c1_256x256x32", "c3_batched_512x32x32x64"])
def test_launch_bound_workloads_get_a_wave_kernel_even_on_a_slow_host(name):
    """With 40 us of host time after every launch all per-call times look alike; the choice must still be made by
    device time (graph replays), and for these two workloads that is one of the one-wave-per-tile kernels."""
    import torch
    say(f"tune {name} with a slow host")
    a, b = ig.make_config(name)
    if a.shape[0] == 1:
        a, b = a[0], b[0]
    da, db = to_dev(a), to_dev(b)
    os.environ["TG_TUNE_TEST_HOST_DELAY_US"] = "40"
    out = tg.tune(da, db, reps=3)
    torch.cuda.synchronize()
    cfg = tg.last_config()
    assert cfg.startswith("wave"), cfg
    check_against_oracle(out.cpu().numpy(), a, b, what=f"tuned {name} {cfg}")


def test_every_candidate_is_checked_against_the_first_one():
    """A normal tuning passes the check; with the kept reference spoilt on purpose every other candidate fails it,
    nothing is cached and the call reports the disagreement."""
    import torch
    say("tuner result check")
    m, n, k = 512, 384, 256
    a, b = ig.normal(801, (m, k)), ig.normal(802, (k, n))
    da, db = to_dev(a), to_dev(b)
    ws = torch.empty(tg.workspace_bytes(1, m, n, k) // 4 + 4, device="cuda")
    tg.set_workspace(ws)
    before = tg.get_config(1, m, n, k)
    os.environ["TG_TUNE_TEST_SPOIL_REFERENCE"] = "1"
    with pytest.raises(tg.TgemmError) as e:
        tg.tune(da, db, reps=2)
    assert e.value.status_name == "TG_ERR_INTERNAL" and "result check" in str(e.value) and "differs" in str(e.value)
    assert tg.get_config(1, m, n, k) == before                     # nothing was cached
    del os.environ["TG_TUNE_TEST_SPOIL_REFERENCE"]
    out = tg.tune(da, db, reps=2)
    torch.cuda.synchronize()
    check_against_oracle(out.cpu().numpy(), a, b, what=f"tuned {tg.last_config()}")
    assert tg.get_config(1, m, n, k) == tg.last_config()
    del ws


@pytest.mark.parametrize("shape,workspace", [((1023, 1023, 1023), True), ((530, 1023, 1024), True), ((2047, 1025, 515), True),
                                             ((777, 2222, 333), False), ((1025, 520, 1025), True), ((2048, 2048, 192), False)],
                         ids=str)
def test_every_candidate_agrees_on_ragged_shapes(shape, workspace):
    """The tuner runs every valid variant on the problem and compares each product with the first one's: a tuning that
    succeeds says that all of them agree.  Ragged sizes, with a workspace (the exact-fit kernels then run on aligned,
    zero-padded copies: n not a multiple of 4 behind such a copy is how a 16-byte store past the end of a row was
    found) and without (predicated kernels).  The tuned choice against the oracle."""
    import torch
    m, n, k = shape
    say(f"tune {m}x{n}x{k} {'with' if workspace else 'without'} a workspace: all candidates must agree")
    a, b = ig.normal(821, (m, k)), ig.normal(822, (k, n))
    da, db = to_dev(a), to_dev(b)
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda") if workspace else None
    tg.set_workspace(ws)
    out = torch.full((m + 1, n), float("nan"), device="cuda")
    tg.tune(da, db, out=out[:m], reps=1)
    torch.cuda.synchronize()
    c = out.cpu().numpy()
    assert np.isnan(c[m]).all()                                    # nothing written behind the last row
    rows = np.arange(0, m, 5)
    check_against_oracle(c[rows], a[rows], b, what=f"tuned {tg.last_config()} on {shape}")
    tg.set_workspace(None)
    del ws


def test_result_check_samples_rows_of_a_large_product():
    """4096 x 4096 x 64: C is 64 MiB, twice the room for the reference, so every other row is compared."""
    import torch
    say("tuner result check on a large C")
    m, n, k = 4096, 4096, 64
    a, b = ig.small_int(811, (m, k)), ig.small_int(812, (k, n))
    da, db = to_dev(a), to_dev(b)
    out = tg.tune(da, db, reps=1)
    torch.cuda.synchronize()
    rows = list(range(0, m, 37))
    from oracle import oracle
    c_ref, _ = oracle.sgemm_f64(a, b, rows=rows, want_abs=True)
    assert np.array_equal(out.cpu().numpy()[rows].astype(np.float64), c_ref)


def test_tune_cache_named_by_the_environment_is_rewritten(tmp_path):
    import torch
    say("TG_TUNE_CACHE written after tuning")
    path = tmp_path / "cache.txt"
    os.environ["TG_TUNE_CACHE"] = str(path)
    a, b = ig.small_int(821, (192, 128)), ig.small_int(822, (128, 160))
    tg.tune(to_dev(a), to_dev(b), reps=1)
    torch.cuda.synchronize()
    text = path.read_text().splitlines()
    assert text[0] == "tgemm-tune-cache 5 gfx950"
    assert any(line.startswith("1 192 160 128 ") for line in text[1:]), text

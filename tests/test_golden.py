"""The stored integer facts under tests/golden/ (written by tests/golden/make_int_golden.py from the CPU oracle).

CPU: the fixture still follows from today's generator and oracle, and agrees with two identities that do not
go through the oracle's loop (total sum from column and row sums; sum of squares from the Gram matrices, formed
with the library's fp64 product, every entry of which is an exactly representable integer here).
GPU: the HIP path reproduces the stored integers on all five shapes.
"""
import pathlib

import numpy as np
import pytest

from paper_1904_03383_amd import inputgen as ig

GOLDEN = pathlib.Path(__file__).parent / "golden" / "int_variant.txt"


def load_golden():
    out = {}
    for line in GOLDEN.read_text().splitlines():
        if not line or line.startswith("#"):
            continue
        f = line.split()
        samples = []
        for tok in f[7:]:
            pos, val = tok.split("=")
            p, i, j = (int(x) for x in pos.split(":"))
            samples.append((p, i, j, int(val)))
        out[f[0]] = {"shape": tuple(int(x) for x in f[1:5]), "sum": int(f[5]), "sumsq": int(f[6]), "samples": samples}
    return out


def check_integer_result(c, gold, what):
    ci = np.rint(c).astype(np.int64)
    assert np.array_equal(ci.astype(c.dtype), c), f"{what}: result is not integral"
    assert int(ci.sum()) == gold["sum"], what
    assert int((ci * ci).sum()) == gold["sumsq"], what
    for (p, i, j, v) in gold["samples"]:
        assert int(ci[p, i, j]) == v, f"{what}: entry {p}:{i}:{j}"


def test_fixture_covers_the_five_workloads():
    gold = load_golden()
    assert list(gold) == list(ig.CONFIGS)
    for name, g in gold.items():
        assert g["shape"] == ig.CONFIGS[name][:4] and len(g["samples"]) == 6


@pytest.mark.parametrize("name", list(ig.CONFIGS))
def test_oracle_reproduces_the_fixture_and_the_identities_hold(name):
    from oracle import oracle
    gold = load_golden()[name]
    a, b = ig.make_config(name, "int")
    check_integer_result(oracle.sgemm_f64(a, b), gold, name)
    ai, bi = a.astype(np.int64), b.astype(np.int64)
    assert int((ai.sum(axis=1) * bi.sum(axis=2)).sum()) == gold["sum"]
    # ||A B||_F^2 = sum_pq (A^T A)_pq (B B^T)_pq; Gram entries are integers of at most 16 * max(m, n) <= 2^16
    a64, b64 = a.astype(np.float64), b.astype(np.float64)
    ga = np.rint(np.matmul(a64.transpose(0, 2, 1), a64)).astype(np.int64)
    gb = np.rint(np.matmul(b64, b64.transpose(0, 2, 1))).astype(np.int64)
    assert int((ga * gb).sum()) == gold["sumsq"]


@pytest.mark.gpu
@pytest.mark.parametrize("name", list(ig.CONFIGS))
def test_hip_path_reproduces_the_fixture(name):
    from gpu_common import run_hip, say
    import paper_1904_03383_amd as tg
    gold = load_golden()[name]
    a, b = ig.make_config(name, "int")
    say(f"golden integers {name}")
    tg.force_config(None)
    c = run_hip(a, b) if a.shape[0] > 1 else run_hip(a[0], b[0])[None]
    check_integer_result(c, gold, f"{name} ({tg.last_config()})")

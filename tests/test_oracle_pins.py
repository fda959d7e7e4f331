"""The CPU oracle against what the paper's definition and mathematics fix (no GPU).

The paper prints no numeric worked example of a matrix product (Table 1 of Sec. 5.2
holds timings only), so there is no printed value to pin against; the pins are closed
forms, exact rational brute force, invariants, Freivalds' check and a library dgemm.
The second half plants plausible mistakes in a numpy re-implementation and checks the
same pin set rejects each of them, i.e. that the pins have teeth.
"""
import numpy as np
import pytest

from oracle import oracle
from paper_1904_03383_amd import inputgen as ig

from oracle_pins import ALL_PINS, pin_freivalds, pin_library_dgemm


def oracle_gemm(a, b):
    return oracle.sgemm_f64(a, b)


@pytest.mark.parametrize("pin", ALL_PINS, ids=lambda p: p.__name__)
def test_oracle_passes_pin(pin):
    pin(oracle_gemm)


def test_all_ones_k_2_pow_24():
    k = 1 << 24
    c = oracle.sgemm_f64(np.ones((1, k), np.float32), np.ones((k, 1), np.float32))
    assert c[0, 0] == float(k)


def test_oracle_large_freivalds_and_dgemm():
    """1024^3 (paper shape, Table 1): pins the oracle at a size spanning all thread shares."""
    pin_freivalds(oracle_gemm, 1024, 1024, 1024, reps=2)
    pin_library_dgemm(oracle_gemm, (512, 384, 2048))


def test_thread_count_does_not_change_bits():
    a = ig.normal(71, (67, 130))
    b = ig.normal(72, (130, 45))
    c1 = oracle.sgemm_f64(a, b, threads=1)
    for t in (2, 3, 8, 64, 1000):
        assert np.array_equal(c1, oracle.sgemm_f64(a, b, threads=t))


def test_batched_is_independent_problems():
    a = ig.uniform(73, (6, 5, 9))
    b = ig.uniform(74, (6, 9, 4))
    c = oracle.sgemm_f64(a, b)
    assert c.shape == (6, 5, 4)
    for i in range(6):
        assert np.array_equal(c[i], oracle.sgemm_f64(a[i], b[i]))
    assert oracle.sgemm_f64(a[:0], b[:0]).shape == (0, 5, 4)


def test_leading_dimensions_and_row_subset():
    big_a = ig.uniform(75, (10, 40))
    big_b = ig.uniform(76, (40, 50))
    a = big_a[:7, :33]          # lda = 40 > k = 33
    b = big_b[:33, :21]         # ldb = 50 > n = 21
    c = oracle.sgemm_f64(a, b)
    assert np.array_equal(c, oracle.sgemm_f64(np.ascontiguousarray(a), np.ascontiguousarray(b)))
    rows = [6, 0, 3, 3]
    assert np.array_equal(oracle.sgemm_f64(a, b, rows=rows), c[rows])
    with pytest.raises(RuntimeError):
        oracle.sgemm_f64(a, b, rows=[7])


def test_abs_sum_is_product_of_absolute_values():
    a = ig.normal(77, (12, 31))
    b = ig.normal(78, (31, 9))
    c, s = oracle.sgemm_f64(a, b, want_abs=True)
    assert np.array_equal(c, oracle.sgemm_f64(a, b))
    assert np.array_equal(s, oracle.sgemm_f64(np.abs(a), np.abs(b)))
    assert np.all(s >= np.abs(c))


def test_parity_metrics_definitions():
    c_ref = np.array([[1.0, -2.0], [0.0, 4.0]])
    s = np.array([[1.0, 2.0], [0.0, 8.0]])
    good = c_ref.astype(np.float32)
    m = oracle.parity_metrics(good, c_ref, s)
    assert m["bit_exact"] and m["zero_ok"] and m["max_ratio"] == 0 and m["rel_fro"] == 0
    bad = good.copy()
    bad[1, 1] += 0.5
    m = oracle.parity_metrics(bad, c_ref, s)
    assert not m["bit_exact"] and m["max_ratio"] == 0.5 / 8 and abs(m["rel_fro"] - 0.5 / np.sqrt(21)) < 1e-15
    bad = good.copy()
    bad[1, 0] = 1e-30
    assert not oracle.parity_metrics(bad, c_ref, s)["zero_ok"]
    neg0 = good.copy()
    neg0[1, 0] = -0.0
    assert oracle.parity_metrics(neg0, c_ref, s)["bit_exact"]
    # a batch: the whole-batch figure pools all entries, the per-problem figure is the worst single problem
    c3 = np.stack([c_ref, 10.0 * c_ref])
    s3 = np.stack([s, 10.0 * s])
    t3 = c3.astype(np.float32)
    t3[0, 1, 1] += 0.5                      # problem 0: error 0.5 against a norm of sqrt(21)
    m = oracle.parity_metrics(t3, c3, s3)
    assert abs(m["rel_fro"] - 0.5 / np.sqrt(21 + 2100)) < 1e-15
    assert abs(m["rel_fro_max_problem"] - 0.5 / np.sqrt(21)) < 1e-15
    assert oracle.parity_metrics(bad, c_ref, s)["rel_fro_max_problem"] == oracle.parity_metrics(bad, c_ref, s)["rel_fro"]


# ---- planted mistakes: each must be caught by at least one pin -------------------------

def _mut_drop_last_term(a, b):
    a, b = a.astype(np.float64), b.astype(np.float64)
    return a[:, :-1] @ b[:-1] if a.shape[1] > 1 else a @ b


def _mut_skip_first_term(a, b):
    a, b = a.astype(np.float64), b.astype(np.float64)
    return a[:, 1:] @ b[1:]


def _mut_transposed_a(a, b):
    a, b = a.astype(np.float64), b.astype(np.float64)
    return (a.T @ b) if a.shape[0] == a.shape[1] else a @ b


def _mut_transposed_b(a, b):
    a, b = a.astype(np.float64), b.astype(np.float64)
    return (a @ b.T) if b.shape[0] == b.shape[1] else a @ b


def _mut_transposed_out(a, b):
    c = a.astype(np.float64) @ b.astype(np.float64)
    return c.T.copy() if c.shape[0] == c.shape[1] else c


def _mut_sign(a, b):
    return -(a.astype(np.float64) @ b.astype(np.float64))


def _mut_abs(a, b):
    return np.abs(a).astype(np.float64) @ b.astype(np.float64)


def _mut_fp32_accumulate(a, b):
    acc = np.zeros((a.shape[0], b.shape[1]), np.float32)
    for p in range(a.shape[1]):
        acc = acc + a[:, p:p + 1] * b[p:p + 1]
    return acc.astype(np.float64)


def _mut_row_shift(a, b):
    c = a.astype(np.float64) @ b.astype(np.float64)
    return np.roll(c, 1, axis=0)


def _mut_elementwise(a, b):
    c = a.astype(np.float64) @ b.astype(np.float64)
    if a.shape == b.shape:
        return (a * b).astype(np.float64)
    return c


MUTANTS = [_mut_drop_last_term, _mut_skip_first_term, _mut_transposed_a, _mut_transposed_b,
           _mut_transposed_out, _mut_sign, _mut_abs, _mut_fp32_accumulate, _mut_row_shift,
           _mut_elementwise]


@pytest.mark.parametrize("mutant", MUTANTS, ids=lambda f: f.__name__)
def test_pins_reject_planted_mistake(mutant):
    caught = []
    for pin in ALL_PINS:
        try:
            pin(mutant)
        except (AssertionError, ValueError, IndexError):
            caught.append(pin.__name__)
    assert caught, f"no pin noticed {mutant.__name__}"


# ---- axpy ---------------------------------------------------------------------------------------

from oracle_pins import AXPY_PINS  # noqa: E402


@pytest.mark.parametrize("pin", AXPY_PINS, ids=lambda p: p.__name__)
def test_axpy_oracle_passes_pin(pin):
    pin(oracle.saxpy_f64)


AXPY_MUTANTS = [
    lambda al, x, y: al * x.astype(np.float64),                                  # y dropped
    lambda al, x, y: al * x.astype(np.float64) - y,                              # wrong sign
    lambda al, x, y: x + al * y.astype(np.float64),                              # alpha on the wrong vector
    lambda al, x, y: al * (x.astype(np.float64) + y),                            # alpha on both
    lambda al, x, y: (np.float32(al) * x + y).astype(np.float64) + 1e-7,         # off by a constant
    lambda al, x, y: np.roll(al * x.astype(np.float64) + y, 1),                  # shifted by one element
]


@pytest.mark.parametrize("idx", range(len(AXPY_MUTANTS)))
def test_axpy_pins_reject_planted_mistake(idx):
    caught = []
    for pin in AXPY_PINS:
        try:
            pin(AXPY_MUTANTS[idx])
        except (AssertionError, ValueError, IndexError):
            caught.append(pin.__name__)
    assert caught, f"no axpy pin noticed mutant {idx}"


# ---- sanitizer build ------------------------------------------------------------------------------

def test_oracle_c_under_address_and_ub_sanitizers(tmp_path, may_spawn):
    """oracle.c compiled with -fsanitize=address,undefined and run on closed-form cases (threads, strides, row subsets)."""
    import pathlib
    import subprocess
    root = pathlib.Path(__file__).resolve().parents[1]
    exe = tmp_path / "oracle_selftest"
    subprocess.run(["gcc", "-std=c11", "-O1", "-g", "-Wall", "-Wextra", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-pthread", str(root / "oracle" / "oracle.c"),
                    str(root / "tests" / "c_abi" / "oracle_selftest.c"), "-o", str(exe), "-lm"], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "oracle_selftest: ok" in r.stdout

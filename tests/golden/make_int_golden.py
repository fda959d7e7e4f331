"""Writes tests/golden/int_variant.txt: exact integer facts about C = A.B for the integer-valued variant of the
five benchmark workloads (entries of A and B uniform in {-4..4} from the seeded generator).

    python tests/golden/make_int_golden.py

The values come from the CPU oracle (oracle/) alone, which evaluates the definition of matmul in Sec. 5.2 of the
paper; with integer inputs of this size every partial sum is an integer below 2^24, so the result is the same
integer matrix in any precision and any summation order.  Before a line is written it is checked against two
facts that do not go through the oracle's loop: the total sum against sum_p (column sum of A)_p (row sum of B)_p
in int64, and the sampled entries against exact rational arithmetic in pure Python.
"""
from __future__ import annotations

import pathlib
import sys

import numpy as np

ROOT = pathlib.Path(__file__).resolve().parents[2]
sys.path.insert(0, str(ROOT))

from oracle import oracle, py_exact              # noqa: E402
from paper_1904_03383_amd import inputgen as ig   # noqa: E402  (seeded inputs only: no GEMM arithmetic there)

OUT = pathlib.Path(__file__).with_name("int_variant.txt")
N_SAMPLES = 6


def sample_positions(name: str, batch: int, m: int, n: int):
    """Six (problem, row, column) positions from the workload's own counter-based generator (stream 7)."""
    bits = ig.raw_bits(ig.config_seeds(name)[0], 3 * N_SAMPLES, stream=7)
    pos = [(int(bits[3 * i] % np.uint64(batch)), int(bits[3 * i + 1] % np.uint64(m)), int(bits[3 * i + 2] % np.uint64(n)))
           for i in range(N_SAMPLES - 2)]
    return pos + [(0, 0, 0), (batch - 1, m - 1, n - 1)]


def facts(name: str):
    batch, m, n, k, _ = ig.CONFIGS[name]
    a, b = ig.make_config(name, "int")
    c = oracle.sgemm_f64(a, b)
    ci = np.rint(c).astype(np.int64)
    assert np.array_equal(ci.astype(np.float64), c), "oracle result is not integral"
    total, sumsq = int(ci.sum()), int((ci * ci).sum())
    ai, bi = a.astype(np.int64), b.astype(np.int64)
    assert total == int((ai.sum(axis=1) * bi.sum(axis=2)).sum()), "total differs from the column-sum/row-sum identity"
    samples = []
    for (p, i, j) in sample_positions(name, batch, m, n):
        exact = py_exact.matmul_exact([[int(x) for x in ai[p, i]]], [[int(bi[p, q, j])] for q in range(k)])[0][0]
        assert exact.denominator == 1 and exact == int(ci[p, i, j]), "sampled entry differs from exact arithmetic"
        exact = int(exact)
        samples.append((p, i, j, exact))
    return batch, m, n, k, total, sumsq, samples


def main() -> int:
    lines = ["# Integer-valued variant of the five workloads (A, B uniform in {-4..4}, seeds 1000+i / 2000+i):",
             "# exact facts about C = A.B (matmul, Sec. 5.2 of the paper; shapes of c1 and c2 from its Table 1).",
             "# Written by tests/golden/make_int_golden.py from the CPU oracle; see that file for the cross-checks.",
             "# name batch m n k sum(C) sum(C^2) then six samples problem:row:column=value"]
    for name in ig.CONFIGS:
        batch, m, n, k, total, sumsq, samples = facts(name)
        lines.append(" ".join([name, str(batch), str(m), str(n), str(k), str(total), str(sumsq)] +
                              [f"{p}:{i}:{j}={v}" for (p, i, j, v) in samples]))
        print(lines[-1], flush=True)
    OUT.write_text("\n".join(lines) + "\n")
    return 0


if __name__ == "__main__":
    sys.exit(main())

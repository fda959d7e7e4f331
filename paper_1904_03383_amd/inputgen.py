"""Seeded synthetic operands for the GEMM workloads.

This module only produces input matrices; it contains none of the matrix
multiplication arithmetic.  It is the single piece of code shared by the CPU
oracle's tests and the HIP path's tests/bench, so both sides see bit-identical
operands.  numpy only (no torch, no HIP library).

The workloads stand in for the matmul shapes of Table 1 in Sec. 5.2 of the paper
(256x256x32 and 1024^3) plus the batched / rectangular / 4096^3 shapes of the
benchmark definition; the paper uses no dataset, only dense matrices of these
shapes.

Generator: counter based.  Element with linear row-major index ``idx`` of a
tensor created from ``seed`` takes its bits from
``splitmix64(seed * 0x9E3779B97F4A7C15 + idx)``.  Any sub-range can therefore be
generated independently of the rest.
"""
from __future__ import annotations

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _splitmix64(x: np.ndarray) -> np.ndarray:
    """Finaliser of the splitmix64 generator applied to every counter in x."""
    with np.errstate(over="ignore"):
        z = x + _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def raw_bits(seed: int, count: int, start: int = 0, stream: int = 0) -> np.ndarray:
    """64 random bits for the counters start..start+count-1 of (seed, stream)."""
    with np.errstate(over="ignore"):
        base = np.uint64(seed) * _GOLDEN + np.uint64(stream) * np.uint64(0xD1B54A32D192ED03)
        ctr = np.arange(start, start + count, dtype=np.uint64) + base
    return _splitmix64(ctr)


def uniform(seed: int, shape, start: int = 0) -> np.ndarray:
    """i.i.d. uniform on the half-open interval [-1, 1), on a 2^-23 grid.

    Every value is (r - 2^23) * 2^-23 with r the top 24 bits of the counter's
    hash, hence exactly representable in fp32.
    """
    count = int(np.prod(shape, dtype=np.int64))
    r = (raw_bits(seed, count, start) >> np.uint64(40)).astype(np.int64)
    v = (r - (1 << 23)).astype(np.float32) * np.float32(2.0 ** -23)
    return v.reshape(shape)


def small_int(seed: int, shape, lo: int = -4, hi: int = 4, start: int = 0) -> np.ndarray:
    """i.i.d. integers uniform in {lo..hi}, stored as fp32 (for bit-exact checks)."""
    count = int(np.prod(shape, dtype=np.int64))
    r = (raw_bits(seed, count, start) >> np.uint64(40)).astype(np.int64)
    v = (r % (hi - lo + 1)) + lo
    return v.astype(np.float32).reshape(shape)


def normal(seed: int, shape, start: int = 0) -> np.ndarray:
    """i.i.d. standard normal: Box-Muller in fp64 on two 53-bit uniforms, rounded to fp32."""
    count = int(np.prod(shape, dtype=np.int64))
    u1 = ((raw_bits(seed, count, start, stream=1) >> np.uint64(11)).astype(np.float64) + 1.0) * 2.0 ** -53
    u2 = (raw_bits(seed, count, start, stream=2) >> np.uint64(11)).astype(np.float64) * 2.0 ** -53
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return z.astype(np.float32).reshape(shape)


_DISTS = {"uniform": uniform, "int": small_int, "normal": normal}

# The five benchmark workloads: name -> (batch, m, n, k, distribution).
CONFIGS = {
    "c1_256x256x32": (1, 256, 256, 32, "uniform"),
    "c2_1024": (1, 1024, 1024, 1024, "uniform"),
    "c3_batched_512x32x32x64": (512, 32, 32, 64, "uniform"),
    "c4_4096x4096x128": (1, 4096, 4096, 128, "uniform"),
    "c5_4096": (1, 4096, 4096, 4096, "normal"),
}


def config_seeds(name: str):
    """(seed_A, seed_B) of a named workload: 1000+i and 2000+i for the i-th config."""
    i = list(CONFIGS).index(name) + 1
    return 1000 + i, 2000 + i


def make_operands(batch: int, m: int, n: int, k: int, dist: str, seed_a: int, seed_b: int):
    """A (batch, m, k) and B (batch, k, n), row-major, packed contiguously per problem."""
    gen = _DISTS[dist]
    a = gen(seed_a, (batch, m, k))
    b = gen(seed_b, (batch, k, n))
    return a, b


def make_config(name: str, dist: str | None = None):
    """Operands of a named workload; ``dist`` overrides its distribution (e.g. "int")."""
    batch, m, n, k, d = CONFIGS[name]
    sa, sb = config_seeds(name)
    return make_operands(batch, m, n, k, dist or d, sa, sb)

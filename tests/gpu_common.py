"""Helpers shared by the GPU parity tests: run the HIP path through the C-ABI binding and
compare with the CPU oracle, element by element, to the bar of the benchmark definition:
every element within 1e-5 * sum_p |a_ip||b_pj| and relative Frobenius error <= 1e-6;
integer-valued inputs bit-exact."""
from __future__ import annotations

import sys

import numpy as np

ELEM_TOL = 1e-5   # per element, times S = sum_p |a_ip| |b_pj|
FRO_TOL = 1e-6    # relative Frobenius error


def say(msg: str):
    """Name the case before each GPU step, flushed, so a lost box still tells what ran."""
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def to_dev(x: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda")


def run_hip(a: np.ndarray, b: np.ndarray, fn=None):
    """a, b: 2-D or 3-D fp32 host arrays -> fp32 host result via tg_sgemm / tg_sgemm_batched."""
    import torch
    import paper_1904_03383_amd as tg
    da, db = to_dev(a), to_dev(b)
    if fn is None:
        fn = tg.sgemm if a.ndim == 2 else tg.sgemm_batched
    # NaN-filled output: a tile the kernel fails to write cannot pass as stale data
    shape = (a.shape[0], b.shape[1]) if a.ndim == 2 else (a.shape[0], a.shape[1], b.shape[2])
    out = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    c = fn(da, db, out=out)
    torch.cuda.synchronize()
    return c.cpu().numpy()


def check_against_oracle(c_hip: np.ndarray, a: np.ndarray, b: np.ndarray, exact: bool = False, what: str = ""):
    from oracle import oracle
    c_ref, s_abs = oracle.sgemm_f64(a, b, want_abs=True)
    assert c_hip.shape == c_ref.shape, (c_hip.shape, c_ref.shape)
    m = oracle.parity_metrics(c_hip, c_ref, s_abs)
    assert m["finite"], what
    if exact:
        assert m["bit_exact"], f"{what}: integer-valued case is not bit exact ({m})"
    assert m["zero_ok"], what
    assert m["max_ratio"] <= ELEM_TOL, f"{what}: per-element ratio {m['max_ratio']:.3e} > {ELEM_TOL}"
    assert m["rel_fro"] <= FRO_TOL, f"{what}: relative Frobenius error {m['rel_fro']:.3e} > {FRO_TOL}"
    return m

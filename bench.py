#!/usr/bin/env python3
"""Benchmark of the fp32 GEMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-others]

A step is one call of the whole hot path (tg_sgemm / tg_sgemm_batched: configuration
lookup, grid mapping, tile loads, LDS staging, MFMA loop, epilogue) on one synthetic
problem whose operands already sit in device memory.  The headline workload is the
4096^3 product, the shape the roofline target of the benchmark definition is quoted on;
the other four workloads are timed the same way and reported under "workloads".
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import pathlib
import sys
import time

import numpy as np

ROOT = pathlib.Path(__file__).resolve().parent
sys.path.insert(0, str(ROOT))

PEAK_MFMA_F32_TFLOPS = 157.3     # MI355X dense fp32 matrix peak
PEAK_MFMA_BF16_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak (the opt-in piece kernels run on it)
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E peak
ELEM_TOL, FRO_TOL = 1e-5, 1e-6


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def algorithmic_flops(batch, m, n, k):
    return 2.0 * batch * m * n * k


def algorithmic_bytes(batch, m, n, k):
    """A and B read once, C written once."""
    return 4.0 * batch * (m * k + k * n + m * n)


def time_workload(tg, torch, name, steps, warmup, reps_tune, vendor=False, min_warm_ms=0.0):
    """Tune, warm up, then time `steps` back-to-back calls.  Returns a dict of measurements."""
    from paper_1904_03383_amd import inputgen as ig
    batch, m, n, k, dist = ig.CONFIGS[name]
    a, b = ig.make_config(name)
    if batch == 1:
        a, b = a[0], b[0]
    da = torch.from_numpy(a).to("cuda")
    db = torch.from_numpy(b).to("cuda")
    call = tg.sgemm if batch == 1 else tg.sgemm_batched
    if reps_tune > 0:
        out = tg.tune(da, db, reps=reps_tune)
    else:                        # configuration comes from a loaded tune cache (or the heuristic)
        out = call(da, db)
    cfg = tg.last_config()
    stream = torch.cuda.current_stream()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    for _ in range(warmup):
        call(da, db, out=out)
    # The GPU has idled while the operands were generated and uploaded, and its clocks take some milliseconds of
    # work to come back: W calls of a 20 us product are over before they have (the first 200 timed calls of 1024^3
    # then read 22.8 us where every later block reads 20.3 us).  Short workloads therefore warm up for at least
    # `min_warm_ms` of device work; the headline's W calls of 1 ms each already do.
    ev0.record(stream)
    call(da, db, out=out)
    ev1.record(stream)
    torch.cuda.synchronize()
    extra_warm = int(min(min_warm_ms / max(ev0.elapsed_time(ev1), 1e-3), 20000)) - warmup
    for _ in range(max(extra_warm, 0)):
        call(da, db, out=out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(steps):
        call(da, db, out=out)          # launched on torch's current stream, where the events sit
    ev1.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall_ms = (t1 - t0) * 1e3 / steps
    dev_ms = ev0.elapsed_time(ev1) / steps
    flops, nbytes = algorithmic_flops(batch, m, n, k), algorithmic_bytes(batch, m, n, k)
    res = {
        "workload": name, "batch": batch, "m": m, "n": n, "k": k, "dist": dist, "tile_config": cfg,
        "ms_per_step": wall_ms, "device_ms_per_step": dev_ms,
        "tflops": flops / (wall_ms * 1e-3) / 1e12,
        "device_tflops": flops / (dev_ms * 1e-3) / 1e12,
        "frac_mfma_peak": flops / (dev_ms * 1e-3) / 1e12 / PEAK_MFMA_F32_TFLOPS,
        "algorithmic_gbs": nbytes / (dev_ms * 1e-3) / 1e9,
        "frac_hbm_peak": nbytes / (dev_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "flops": flops, "bytes": nbytes,
    }
    # Ten more timed blocks of R back-to-back calls each (R such that a block lasts >= 5 ms, at least 20 calls):
    # their median and minimum show how steady the figure above is.
    reps = max(20, int(5.0 / max(dev_ms, 1e-3)) + 1)
    blocks_ms = []
    for _ in range(10):
        ev0.record(stream)
        for _ in range(reps):
            call(da, db, out=out)
        ev1.record(stream)
        torch.cuda.synchronize()
        blocks_ms.append(ev0.elapsed_time(ev1) / reps)
    res["repeat_stats"] = {"blocks": 10, "calls_per_block": reps, "median_ms": float(np.median(blocks_ms)),
                           "min_ms": float(min(blocks_ms)), "max_ms": float(max(blocks_ms))}
    if dev_ms < 0.02:
        # The same calls made straight through the C ABI with the arguments marshalled once (what a C caller
        # pays per call: the library's host path plus the HIP launch, without the Python binding's checks).
        lib = tg.load_library()
        sh = int(stream.cuda_stream)
        if batch == 1:
            fn, args = lib.tg_sgemm, (m, n, k, da.data_ptr(), k, db.data_ptr(), n, out.data_ptr(), n, sh)
        else:
            fn, args = lib.tg_sgemm_batched, (batch, m, n, k, da.data_ptr(), k, m * k, db.data_ptr(), n, k * n,
                                              out.data_ptr(), n, m * n, sh)
        assert out.is_contiguous() and da.is_contiguous() and db.is_contiguous()
        ok = all(fn(*args) == 0 for _ in range(max(warmup, 1)))
        ev0.record(stream)
        for _ in range(steps):
            fn(*args)
        ev1.record(stream)
        torch.cuda.synchronize()
        if ok:
            res["abi_call_ms_per_step"] = ev0.elapsed_time(ev1) / steps
    if dev_ms < 0.1:
        # Launch-bound workload: per-call time is dominated by the host launch path.  Replay the
        # same calls from a HIP graph to show the device-side rate (reported separately).
        try:
            per_graph = 50
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for _ in range(per_graph):
                    call(da, db, out=out)
            g.replay()
            torch.cuda.synchronize()
            reps = max(1, steps // per_graph)
            ev0.record(torch.cuda.current_stream())
            for _ in range(reps):
                g.replay()
            ev1.record(torch.cuda.current_stream())
            torch.cuda.synchronize()
            res["graph_device_ms_per_step"] = ev0.elapsed_time(ev1) / (reps * per_graph)
            res["graph_tflops"] = flops / (res["graph_device_ms_per_step"] * 1e-3) / 1e12
        except Exception as ex:  # noqa: BLE001 - the graph figure is optional
            res["graph_error"] = str(ex)[:200]
    if batch == 1 and 32e6 <= nbytes <= 100e6:
        # HBM-relevant shape (c4): also time it "cold", rotating through enough operand/result sets
        # (> 512 MB in total) that nothing of a set is left in the 256 MB Infinity Cache when it comes round.
        sets = int(600e6 // nbytes) + 1
        das = [da] + [da.clone() for _ in range(sets - 1)]
        dbs = [db] + [db.clone() for _ in range(sets - 1)]
        outs = [out] + [torch.empty_like(out) for _ in range(sets - 1)]
        for i in range(sets):
            call(das[i], dbs[i], out=outs[i])
        torch.cuda.synchronize()
        ev0.record(stream)
        for i in range(steps):
            call(das[i % sets], dbs[i % sets], out=outs[i % sets])
        ev1.record(stream)
        torch.cuda.synchronize()
        res["cold_device_ms_per_step"] = ev0.elapsed_time(ev1) / steps
        res["cold_sets"] = sets
        res["cold_algorithmic_gbs"] = nbytes / (res["cold_device_ms_per_step"] * 1e-3) / 1e9
        del das, dbs, outs
    if vendor:
        # Context only (--vendor-context): the same product through torch.matmul, i.e. the vendor BLAS
        # behind PyTorch-ROCm, same buffers, same timing loop.  Not a target and not part of `value`.
        ref = torch.empty_like(out)
        for _ in range(max(warmup, 3)):
            torch.matmul(da, db, out=ref)
        torch.cuda.synchronize()
        ev0.record(stream)
        for _ in range(steps):
            torch.matmul(da, db, out=ref)
        ev1.record(stream)
        torch.cuda.synchronize()
        res["torch_matmul_device_ms_per_step"] = ev0.elapsed_time(ev1) / steps
        if batch == 1:
            # its error against the oracle on the same sampled rows (the vendor kernels keep one accumulation level)
            rows_v = sorted(set(int(r) for r in np.linspace(0, m - 1, num=min(m, 64))))
            pv = parity_on_rows(a, b, ref, rows_v)
            res["torch_matmul_rel_fro"] = pv["rel_fro"]
            res["torch_matmul_max_ratio"] = pv["max_ratio"]
        del ref
    ideal_compute = flops / (PEAK_MFMA_F32_TFLOPS * 1e12)
    ideal_hbm = nbytes / (PEAK_HBM_GBS * 1e9)
    res["bound"] = "mfma" if ideal_compute >= ideal_hbm else "hbm"
    return res, (a, b, out)


def time_axpy(tg, torch, steps, warmup):
    """axpy of Sec. 5.2 (z = alpha.x + y, n = 2^26): the paper's bandwidth-bound kernel.  HBM roofline."""
    from paper_1904_03383_amd import inputgen as ig
    from oracle import oracle
    n, alpha = 1 << 26, 0.37
    x, y = ig.uniform(3001, (n,)), ig.normal(3002, (n,))
    dx, dy = torch.from_numpy(x).to("cuda"), torch.from_numpy(y).to("cuda")
    dz = torch.empty_like(dx)
    for _ in range(max(warmup, 400)):          # about 50 ms of device work (see time_workload)
        tg.saxpy(alpha, dx, dy, out=dz)
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    ev0.record(torch.cuda.current_stream())
    for _ in range(steps):
        tg.saxpy(alpha, dx, dy, out=dz)
    ev1.record(torch.cuda.current_stream())
    torch.cuda.synchronize()
    dev_ms = ev0.elapsed_time(ev1) / steps
    nbytes = 12.0 * n
    # parity on a sample (every 1024th element plus the tail)
    idx = np.unique(np.concatenate([np.arange(0, n, 1024), np.arange(n - 64, n)]))
    ref = oracle.saxpy_f64(alpha, x[idx], y[idx])
    got = dz.cpu().numpy()[idx].astype(np.float64)
    ok = bool(np.all(np.abs(got - ref) <= 2.0 ** -24 * np.abs(ref) * (1 + 1e-9) + 2.0 ** -149))
    t0 = time.perf_counter()
    oracle.saxpy_f64(alpha, x, y)
    cpu_s = time.perf_counter() - t0
    return {"workload": "axpy_2p26", "n": n, "alpha": alpha, "device_ms_per_step": dev_ms, "bytes": nbytes, "flops": 2.0 * n,
            "algorithmic_gbs": nbytes / (dev_ms * 1e-3) / 1e9, "frac_hbm_peak": nbytes / (dev_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
            "bound": "hbm", "parity_ok": ok, "cpu_oracle_seconds": cpu_s, "cpu_oracle_gbs": nbytes / cpu_s / 1e9, "cpu_cores": 1}


def time_layout(tg, torch, name, m, n, k, layout_a, layout_b, steps, warmup, restore_ws, packed_kernel=None):
    """One product through tg_sgemm_strided with operands that are not plain row-major: layout 'N' plain, 'T' stored
    transposed (column-major), 'S32' element stride 32 along the rows (the strided matmul of Sec. 5.2).

    The figure reported is without a workspace: the operands are read as they lie by the kernel variants with fused
    gather / transposing loaders.  With `packed_kernel`, the packing path is timed too, for comparison: a workspace is
    set and that plain kernel forced, so every non-plain operand is first copied by the packing pass."""
    from paper_1904_03383_amd import inputgen as ig
    from oracle import oracle

    def operand(seed, rows, cols, layout):
        if layout == "T":
            store = ig.uniform(seed, (cols, rows))
            return np.ascontiguousarray(store.T), torch.from_numpy(store).to("cuda").T
        if layout.startswith("S"):
            cs = int(layout[1:])
            store = ig.uniform(seed, (rows, cols * cs))
            return np.ascontiguousarray(store[:, ::cs]), torch.from_numpy(store).to("cuda")[:, ::cs]
        store = ig.uniform(seed, (rows, cols))
        return store, torch.from_numpy(store).to("cuda")

    a, da = operand(3003, m, k, layout_a)
    b, db = operand(3004, k, n, layout_b)
    out = torch.empty((m, n), device="cuda")
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    rows = sorted(set(int(r) for r in np.linspace(0, m - 1, num=64)))
    c_ref, s_abs = oracle.sgemm_f64(a, b, rows=rows, want_abs=True)

    def timed(reps):
        out.fill_(float("nan"))
        for _ in range(warmup):
            tg.sgemm_strided(da, db, out=out)
        cfg = tg.last_config()
        # (at least 50 ms of device work before the timed calls: see time_workload)
        ev0.record(torch.cuda.current_stream())
        tg.sgemm_strided(da, db, out=out)
        ev1.record(torch.cuda.current_stream())
        torch.cuda.synchronize()
        for _ in range(max(int(min(50.0 / max(ev0.elapsed_time(ev1), 1e-3), 20000)) - warmup, 0)):
            tg.sgemm_strided(da, db, out=out)
        torch.cuda.synchronize()
        ev0.record(torch.cuda.current_stream())
        for _ in range(reps):
            tg.sgemm_strided(da, db, out=out)
        ev1.record(torch.cuda.current_stream())
        torch.cuda.synchronize()
        par = oracle.parity_metrics(out.cpu().numpy()[rows], c_ref, s_abs)
        ok = bool(par["max_ratio"] <= ELEM_TOL and par["rel_fro"] <= FRO_TOL and par["finite"])
        return ev0.elapsed_time(ev1) / reps, cfg, ok

    flops = 2.0 * m * n * k
    reps = max(5, min(max(steps, 200), int(50.0 / (flops / 100e12 * 1e3)) + 1))     # about 50 ms of work, 200 calls at most
    tg.set_workspace(None)
    dev_ms, cfg, ok = timed(reps)
    res = {"workload": name, "m": m, "n": n, "k": k, "layout_a": layout_a, "layout_b": layout_b, "workspace": False,
           "tile_config": cfg, "device_ms_per_step": dev_ms, "flops": flops, "device_tflops": flops / (dev_ms * 1e-3) / 1e12,
           "frac_mfma_peak": flops / (dev_ms * 1e-3) / 1e12 / PEAK_MFMA_F32_TFLOPS, "bound": "mfma", "parity_ok": ok}
    if packed_kernel:
        csa = 1 if layout_a == "N" else 32
        csb = 1 if layout_b == "N" else 32
        ws = torch.empty(max(tg.strided_workspace_bytes(m, n, k, csa, csb) // 4, 4), dtype=torch.float32, device="cuda")
        tg.set_workspace(ws)
        tg.force_config(packed_kernel)
        try:
            p_ms, p_cfg, p_ok = timed(reps)
        finally:
            tg.force_config(None)
        res["packed_with_workspace"] = {"tile_config": p_cfg, "device_ms_per_step": p_ms,
                                        "device_tflops": flops / (p_ms * 1e-3) / 1e12}
        res["parity_ok"] = ok and p_ok
        del ws
        if layout_a.startswith("S") or layout_b.startswith("S"):
            # the library's own choice with room for packed copies and for split-K partial products (a gathered A:
            # row panels with a K split)
            ws = torch.empty(max((tg.strided_workspace_bytes(m, n, k, csa, csb) + tg.workspace_bytes(1, m, n, k)) // 4, 4),
                             dtype=torch.float32, device="cuda")
            tg.set_workspace(ws)
            a_ms, a_cfg, a_ok = timed(reps)
            res["auto_with_workspace"] = {"tile_config": a_cfg, "device_ms_per_step": a_ms,
                                          "device_tflops": flops / (a_ms * 1e-3) / 1e12}
            res["parity_ok"] = res["parity_ok"] and a_ok
            del ws
    tg.set_workspace(restore_ws)
    return res


def time_pieces(tg, torch, steps, warmup, reps_tune, restore_ws):
    """The headline product in the opt-in math mode that forms fp32 products from bf16 pieces on the bf16
    matrix instructions (fp32 in, fp32 out, same accuracy bar).  Reported beside the headline, never as it:
    `device_tflops` counts 2mnk (fp32-equivalent work), `bf16_mfma_tflops` the piece products actually issued."""
    from paper_1904_03383_amd import inputgen as ig
    name = "c5_4096"
    batch, m, n, k, dist = ig.CONFIGS[name]
    a, b = ig.make_config(name)
    a, b = a[0], b[0]
    da, db = torch.from_numpy(a).to("cuda"), torch.from_numpy(b).to("cuda")
    tg.set_math(tg.MATH_BF16_PIECES)
    try:
        # room for the variants that cut the operands ahead into the workspace, so that the tuner times them too
        ws = torch.empty(max(tg.workspace_bytes(batch, m, n, k) // 4, 4), dtype=torch.float32, device="cuda")
        tg.set_workspace(ws)
        out = tg.tune(da, db, reps=reps_tune) if reps_tune > 0 else tg.sgemm(da, db)
        cfg = tg.last_config()
        stream = torch.cuda.current_stream()
        for _ in range(warmup):
            tg.sgemm(da, db, out=out)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        ev0.record(stream)
        for _ in range(steps):
            tg.sgemm(da, db, out=out)
        ev1.record(stream)
        torch.cuda.synchronize()
        assert tg.last_config() == cfg
    finally:
        tg.set_math(tg.MATH_FP32_MFMA)
        tg.set_workspace(restore_ws)
    dev_ms = ev0.elapsed_time(ev1) / steps
    flops = algorithmic_flops(batch, m, n, k)
    pieces = 9 if "_x9" in cfg else 6 if "_x6" in cfg else 0
    rows = sorted(set(int(r) for r in np.linspace(0, m - 1, num=64)))
    par = parity_on_rows(a, b, out, rows)
    res = {"workload": name + " in math mode BF16_PIECES (opt-in)", "batch": batch, "m": m, "n": n, "k": k, "dist": dist,
           "tile_config": cfg, "device_ms_per_step": dev_ms, "device_tflops": flops / (dev_ms * 1e-3) / 1e12,
           "piece_products_per_product": pieces,
           "parity": {"rows_checked": len(rows), "max_ratio": par["max_ratio"], "rel_fro": par["rel_fro"],
                      "ok": bool(par["finite"] and par["zero_ok"] and par["max_ratio"] <= ELEM_TOL and par["rel_fro"] <= FRO_TOL)}}
    if pieces:
        res["bf16_mfma_tflops"] = pieces * flops / (dev_ms * 1e-3) / 1e12
        res["frac_bf16_mfma_peak"] = res["bf16_mfma_tflops"] / PEAK_MFMA_BF16_TFLOPS
    return res


def device_info(torch):
    """Name, CU count and current shader clock of the GPU.  The clock comes from sysfs (the active line of
    pp_dpm_sclk), read as a plain file right after the timed region: no child process is started, a process
    that has initialised the GPU must not exec."""
    import glob
    import re
    prop = torch.cuda.get_device_properties(0)
    info = {"name": prop.name, "arch": getattr(prop, "gcnArchName", ""), "compute_units": prop.multi_processor_count}
    try:
        for path in sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk")):
            for line in open(path).read().splitlines():
                mm = re.search(r"(\d+)\s*Mhz\s*\*", line, re.IGNORECASE)
                if mm:
                    info["sclk_mhz_after_run"] = int(mm.group(1))
                    break
            if "sclk_mhz_after_run" in info:
                break
    except Exception:  # noqa: BLE001 - informational only
        pass
    return info


def parity_on_rows(a, b, out, rows):
    """Compare sampled rows of the device result with the oracle (element-wise and Frobenius)."""
    from oracle import oracle
    c_ref, s_abs = oracle.sgemm_f64(a, b, rows=rows, want_abs=True)
    host = out.cpu().numpy()
    got = host[..., rows, :]
    return oracle.parity_metrics(got, c_ref, s_abs)


def cpu_baseline(a, b, target_seconds=15.0):
    """The oracle as it stands, timed on the host cores, on a bounded number of rows of C."""
    from oracle import oracle
    cores = oracle.host_cores()
    squeeze = a.ndim == 2
    a3 = a[None] if squeeze else a
    b3 = b[None] if squeeze else b
    batch, m, k = a3.shape
    n = b3.shape[2]
    probe_rows = list(range(min(m, max(1, cores))))
    t0 = time.perf_counter()
    oracle.sgemm_f64(a3, b3, rows=probe_rows)
    probe = max(time.perf_counter() - t0, 1e-6)
    rows_per_s = len(probe_rows) / probe
    nrows = int(min(m, max(len(probe_rows), rows_per_s * target_seconds)))
    rows = list(range(nrows))
    t0 = time.perf_counter()
    oracle.sgemm_f64(a3, b3, rows=rows)
    dt = time.perf_counter() - t0
    flops = 2.0 * batch * nrows * n * k
    sample = (f"rows 0..{nrows - 1} of {m} of every problem ({batch} x {nrows}x{n}x{k}), "
              f"{dt:.2f} s wall, fp64 triple loop")
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": sample, "seconds": dt}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c5_4096")
    ap.add_argument("--no-others", action="store_true", help="time only the headline workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--vendor-context", action="store_true",
                    help="also time torch.matmul (the vendor BLAS behind PyTorch) on every GEMM workload, for context")
    ap.add_argument("--tune-reps", type=int, default=5)
    ap.add_argument("--tune-cache", default=None,
                    help="file of tuned configurations: loaded (and tuning skipped) if it exists, else written; "
                         "default: the configurations shipped in paper_1904_03383_amd/tuned_gfx950.txt")
    ap.add_argument("--tune", action="store_true",
                    help="ignore the shipped configurations and tune every workload in this run (tg_tune)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for scaling profiler byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1")

    from oracle import oracle as _oracle
    _oracle.host_cores()
    _oracle._load()          # the CPU oracle is loaded before anything touches the GPU
    import torch
    import paper_1904_03383_amd as tg
    from paper_1904_03383_amd import inputgen as ig
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    tg.load_library()
    if args.workload not in ig.CONFIGS:
        sys.exit(f"bench.py: unknown workload {args.workload}; choose from {list(ig.CONFIGS)}")

    ws_bytes = max(tg.workspace_bytes(*ig.CONFIGS[w][:4]) for w in ig.CONFIGS)
    ws = torch.empty(max(ws_bytes // 4, 4), dtype=torch.float32, device="cuda")
    tg.set_workspace(ws)

    # The tile configurations are the ones tg_tune found on an MI355X, shipped with the package, so that every run
    # times the same kernels as the committed profiles (profiles/ names them); --tune searches again.
    shipped = ROOT / "paper_1904_03383_amd" / "tuned_gfx950.txt"
    cache = pathlib.Path(args.tune_cache) if args.tune_cache else (shipped if shipped.exists() and not args.tune else None)
    if cache and cache.exists():
        tg.load_tune_cache(cache)
        args.tune_reps = 0
        log(f"loaded tuned configurations from {cache}; not tuning")

    log(f"headline workload {args.workload}")
    head, (a, b, out) = time_workload(tg, torch, args.workload, args.steps, args.warmup, args.tune_reps, args.vendor_context)
    dev = device_info(torch)
    log(f"  {head['tile_config']}  {head['device_ms_per_step'] * 1e3:.1f} us  {head['device_tflops']:.1f} TFLOP/s"
        + (f"  (torch.matmul {head['torch_matmul_device_ms_per_step'] * 1e3:.1f} us)" if "torch_matmul_device_ms_per_step" in head else ""))
    log(f"  device: {dev}")

    rows = sorted(set(int(r) for r in np.linspace(0, head["m"] - 1, num=min(head["m"], 128))))
    par = parity_on_rows(a, b, out, rows)
    parity_ok = bool(par["finite"] and par["zero_ok"] and par["max_ratio"] <= ELEM_TOL and par["rel_fro"] <= FRO_TOL)
    log(f"  parity on {len(rows)} sampled rows: max_ratio {par['max_ratio']:.2e} rel_fro {par['rel_fro']:.2e} ok={parity_ok}")

    base = None
    if not args.no_cpu_baseline:
        log("cpu baseline (oracle) ...")
        base = cpu_baseline(a, b)
        log(f"  {base['value'] * 1e3:.2f} GFLOP/s on {base['cores']} cores")
    del a, b, out

    others = []
    if not args.no_others:
        for name in ig.CONFIGS:
            if name == args.workload:
                continue
            steps = args.steps if ig.CONFIGS[name][3] >= 1024 else max(args.steps, 500)
            r, (a2, b2, out2) = time_workload(tg, torch, name, steps, args.warmup, args.tune_reps, args.vendor_context,
                                              min_warm_ms=50.0)
            rows2 = sorted(set(int(x) for x in np.linspace(0, r["m"] - 1, num=min(r["m"], 64))))
            p2 = parity_on_rows(a2, b2, out2, rows2)
            r["parity"] = {"rows_checked": len(rows2), "max_ratio": p2["max_ratio"], "rel_fro": p2["rel_fro"],
                           "ok": bool(p2["finite"] and p2["zero_ok"] and p2["max_ratio"] <= ELEM_TOL and p2["rel_fro"] <= FRO_TOL)}
            parity_ok = parity_ok and r["parity"]["ok"]
            del a2, b2, out2
            extra = f"  (graph replay {r['graph_device_ms_per_step'] * 1e3:.2f} us)" if "graph_device_ms_per_step" in r else ""
            if "abi_call_ms_per_step" in r:
                extra += f"  (through the C ABI directly {r['abi_call_ms_per_step'] * 1e3:.2f} us per call)"
            if "torch_matmul_device_ms_per_step" in r:
                extra += f"  (torch.matmul {r['torch_matmul_device_ms_per_step'] * 1e3:.2f} us)"
            log(f"  {name}: {r['tile_config']}  {r['device_ms_per_step'] * 1e3:.2f} us  {r['device_tflops']:.2f} TFLOP/s{extra}")
            others.append(r)

    if not args.no_others:
        r = time_axpy(tg, torch, min(args.steps, 100), min(args.warmup, 10))
        log(f"  axpy n=2^26: {r['device_ms_per_step'] * 1e3:.1f} us  {r['algorithmic_gbs']:.0f} GB/s  "
            f"({r['frac_hbm_peak'] * 100:.1f}% of HBM peak)  parity_ok={r['parity_ok']}")
        others.append(r)
        # strided matmul (Sec. 5.2) and transposed layouts through tg_sgemm_strided, no workspace
        layouts = [("strided_1024_csa32", 1024, 1024, 1024, "S32", "N", "d64x64x32_w32x32"),
                   ("strided_4096x1024x1024_csa32", 4096, 1024, 1024, "S32", "N", None),
                   ("AT_B_1024", 1024, 1024, 1024, "T", "N", "d64x64x32_w32x32"),
                   ("A_BT_1024", 1024, 1024, 1024, "N", "T", "d64x64x32_w32x32"),
                   ("AT_BT_1024", 1024, 1024, 1024, "T", "T", None),
                   ("AT_B_4096", 4096, 4096, 4096, "T", "N", "t128x256x32_w64x128_acc2"),
                   ("A_BT_4096", 4096, 4096, 4096, "N", "T", None)]
        for lname, lm, ln, lk, la, lb, packed_kernel in layouts:
            r = time_layout(tg, torch, lname, lm, ln, lk, la, lb, min(args.steps, 100), min(args.warmup, 10), ws, packed_kernel)
            extra = ""
            if "packed_with_workspace" in r:
                pw = r["packed_with_workspace"]
                extra = f"  (packing pass + {pw['tile_config']}: {pw['device_ms_per_step'] * 1e3:.1f} us)"
            if "auto_with_workspace" in r:
                aw = r["auto_with_workspace"]
                extra += f"  (automatic choice with a workspace: {aw['tile_config']} {aw['device_ms_per_step'] * 1e3:.1f} us)"
            log(f"  {lname} (A:{la} B:{lb}, no workspace): {r['tile_config']}  {r['device_ms_per_step'] * 1e3:.1f} us  "
                f"{r['device_tflops']:.2f} TFLOP/s  parity_ok={r['parity_ok']}{extra}")
            parity_ok = parity_ok and r["parity_ok"]
            others.append(r)

    if not args.no_others:
        r = time_pieces(tg, torch, args.steps, args.warmup, args.tune_reps, ws)
        log(f"  {r['workload']}: {r['tile_config']}  {r['device_ms_per_step'] * 1e3:.1f} us  {r['device_tflops']:.1f} TFLOP/s fp32-equivalent"
            f"  rel_fro {r['parity']['rel_fro']:.2e}  parity_ok={r['parity']['ok']}")
        parity_ok = parity_ok and r["parity"]["ok"]
        others.append(r)

    if cache and not cache.exists():
        tg.save_tune_cache(cache)

    if args.copy_calibration:
        # a plain streaming kernel of known size: reads 256 MiB, writes 256 MiB
        src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 2.0, out=dst)
        torch.cuda.synchronize()
        log("copy calibration: one elementwise kernel, 256 MiB read + 256 MiB written")
        del src, dst

    # HBM traffic of the dominant kernel per launch comes from committed rocprofv3 counter runs (FETCH_SIZE and
    # WRITE_SIZE cannot be read from inside this process): profiles/hbm_traffic.json lists, per workload, the tile
    # configurations it was measured at.  The figure is only reported when this run timed one of exactly those.
    traffic, traffic_note = None, None
    tfile = ROOT / "profiles" / "hbm_traffic.json"
    if tfile.exists():
        entries = json.loads(tfile.read_text()).get(args.workload, [])
        entries = [entries] if isinstance(entries, dict) else entries
        match = [e for e in entries if e.get("tile_config") == head["tile_config"]]
        if match:
            traffic = match[0].get("bytes_per_launch")
            traffic_note = f"rocprofv3 FETCH_SIZE + WRITE_SIZE at {head['tile_config']}, profiles/hbm_traffic.json"
        elif entries:
            traffic_note = ("not measured at the configuration timed here (" + head["tile_config"] + "); profiles/hbm_traffic.json has "
                            + ", ".join(f"{e.get('tile_config')}: {e.get('bytes_per_launch', 0) / 1e6:.1f} MB" for e in entries))

    if head["bound"] == "mfma":
        roof = {"bound": "mfma", "achieved": head["device_tflops"], "peak": PEAK_MFMA_F32_TFLOPS, "unit": "TFLOP/s",
                "frac": head["frac_mfma_peak"], "traffic": traffic}
    else:
        roof = {"bound": "hbm", "achieved": head["algorithmic_gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": head["frac_hbm_peak"], "traffic": traffic}
    roof["traffic_note"] = traffic_note
    roof["kernel"] = head["tile_config"]
    roof["avg_launch_ms"] = head["device_ms_per_step"]

    line = {
        "metric": "fp32 GEMM TFLOP/s (2mnk/t)", "value": head["tflops"], "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.workload, "batch": head["batch"], "m": head["m"], "n": head["n"], "k": head["k"],
                   "layout": "row-major", "distribution": head["dist"], "tile_config": head["tile_config"]},
        "roofline": roof,
        "cpu_baseline": base,
        "parity": {"rows_checked": len(rows), "max_ratio": par["max_ratio"], "rel_fro": par["rel_fro"], "ok": parity_ok},
        "device": dev,
        "workloads": [head] + others,
    }
    print(json.dumps(line), flush=True)
    if not parity_ok:
        sys.exit("bench.py: the timed result does not match the oracle")


if __name__ == "__main__":
    main()

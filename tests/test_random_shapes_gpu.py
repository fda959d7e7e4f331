"""Seeded random shapes, leading dimensions, base offsets and batch strides through tg_sgemm / tg_sgemm_batched,
integer-valued inputs, every element compared with the CPU oracle bit for bit.  The draw favours the
boundaries the kernels care about: multiples of 4 / 16 / 32 / 64 / 128 and their neighbours, so that the
exact-fit kernels' ragged-edge and K-remainder paths, the predicated kernels and the one-wave kernel all
get hit, with and without a split-K workspace."""
import numpy as np
import pytest

import paper_1904_03383_amd as tg
from paper_1904_03383_amd import inputgen as ig

from gpu_common import say

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def _clean_library_state():
    tg.force_config(None)
    tg.set_workspace(None)
    yield
    tg.force_config(None)
    tg.set_workspace(None)


def _draw_dim(rng, hi):
    kind = rng.integers(0, 4)
    if kind == 0:
        return int(rng.integers(1, hi + 1))
    base = int(rng.choice([4, 16, 32, 64, 128, 256]))
    mult = int(rng.integers(1, max(hi // base, 1) + 1))
    return max(1, min(hi, base * mult + int(rng.choice([-4, -1, 0, 0, 1, 4]))))


def _cases(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        batch = int(rng.choice([1, 1, 1, 2, 3]))
        m, n, k = _draw_dim(rng, 300), _draw_dim(rng, 300), _draw_dim(rng, 1200 if rng.integers(0, 5) == 0 else 200)
        pads = tuple(int(rng.choice([0, 0, 4, 8, 1, 3])) for _ in range(3))          # lda-k, ldb-n, ldc-n
        offs = tuple(int(rng.choice([0, 0, 0, 4, 1])) for _ in range(3))             # element offset of each base
        gaps = tuple(int(rng.choice([0, 0, 4, 7])) for _ in range(3))                # extra batch stride
        out.append((batch, m, n, k, pads, offs, gaps, bool(rng.integers(0, 2))))
    return out


CASES = _cases(20241127, 80)


def _place(host, ld_pad, off, gap, fill):
    """Copy a (batch, rows, cols) host array into a flat device buffer with the given leading-dimension pad,
    base offset and extra batch stride; returns (flat device tensor, strided device view)."""
    import torch
    batch, rows, cols = host.shape
    ld = cols + ld_pad
    stride = rows * ld + gap
    flat = torch.full((off + batch * stride + 8,), fill, dtype=torch.float32, device="cuda")
    view = torch.as_strided(flat, (batch, rows, cols), (stride, ld, 1), off)
    view.copy_(torch.from_numpy(host))
    return flat, view


@pytest.mark.parametrize("chunk", range(8))
def test_random_shapes_are_bit_exact(chunk):
    import torch
    from oracle import oracle
    for idx in range(chunk * 10, chunk * 10 + 10):
        batch, m, n, k, pads, offs, gaps, with_ws = CASES[idx]
        say(f"random case {idx}: batch {batch} {m}x{n}x{k} pads {pads} offsets {offs} gaps {gaps} workspace {with_ws}")
        a = ig.small_int(9000 + idx, (batch, m, k))
        b = ig.small_int(9500 + idx, (batch, k, n))
        ws = None
        if with_ws:
            ws = torch.empty(max(tg.workspace_bytes(batch, m, n, k) // 4, 4), device="cuda")
            tg.set_workspace(ws)
        else:
            tg.set_workspace(None)
        _, da = _place(a, pads[0], offs[0], gaps[0], float("nan"))
        _, db = _place(b, pads[1], offs[1], gaps[1], float("nan"))
        cflat, dc = _place(np.zeros((batch, m, n), np.float32), pads[2], offs[2], gaps[2], 7.0)
        cflat.fill_(7.0)
        if batch == 1:
            tg.sgemm(da[0], db[0], out=dc[0])
        else:
            tg.sgemm_batched(da, db, out=dc)
        torch.cuda.synchronize()
        cfg = tg.last_config()
        ref = oracle.sgemm_f64(a, b)
        got = dc.cpu().numpy()
        assert np.array_equal(got.astype(np.float64), ref), f"case {idx} ({cfg}): result differs from the oracle"
        # nothing outside the m x n regions was written
        mask = torch.ones_like(cflat, dtype=torch.bool)
        torch.as_strided(mask, (batch, m, n), dc.stride(), offs[2]).fill_(False)
        assert bool((cflat[mask] == 7.0).all()), f"case {idx} ({cfg}): stores outside the output"
        del ws


def _strided_operand(rng, host, fill=float("nan")):
    """Device view of a (rows, cols) host matrix with a random layout: row-major with a pad, column-major with a
    pad, or an element stride along its rows."""
    import torch
    rows, cols = host.shape
    kind = int(rng.integers(0, 3))
    if kind == 0:
        ld = cols + int(rng.choice([0, 4, 3]))
        flat = torch.full((rows * ld + 8,), fill, device="cuda")
        view = torch.as_strided(flat, (rows, cols), (ld, 1))
    elif kind == 1:
        ld = rows + int(rng.choice([0, 4, 3]))
        flat = torch.full((cols * ld + 8,), fill, device="cuda")
        view = torch.as_strided(flat, (rows, cols), (1, ld))
    else:
        cs = int(rng.integers(2, 6))
        ld = cols * cs + int(rng.choice([0, 1, 5]))
        flat = torch.full((rows * ld + 8,), fill, device="cuda")
        view = torch.as_strided(flat, (rows, cols), (ld, cs))
    view.copy_(torch.from_numpy(host))
    return flat, view


@pytest.mark.parametrize("chunk", range(4))
def test_random_strided_layouts_are_bit_exact(chunk):
    import torch
    from oracle import oracle
    rng = np.random.default_rng(7700 + chunk)
    for idx in range(10):
        m, n, k = _draw_dim(rng, 300), _draw_dim(rng, 300), _draw_dim(rng, 200)
        with_ws = bool(rng.integers(0, 2))
        a = ig.small_int(9800 + 10 * chunk + idx, (m, k))
        b = ig.small_int(9900 + 10 * chunk + idx, (k, n))
        keep_a, da = _strided_operand(rng, a)
        keep_b, db = _strided_operand(rng, b)
        say(f"random strided case {chunk}.{idx}: {m}x{n}x{k} A strides {tuple(da.stride())} B strides {tuple(db.stride())} workspace {with_ws}")
        ws = None
        if with_ws:
            ws = torch.full((tg.strided_workspace_bytes(m, n, k, 2, 2) // 4 + 4,), float("nan"), device="cuda")
            tg.set_workspace(ws)
        else:
            tg.set_workspace(None)
        out = torch.full((m, n), float("nan"), device="cuda")
        tg.sgemm_strided(da, db, out=out)
        torch.cuda.synchronize()
        cfg = tg.last_config()
        assert np.array_equal(out.cpu().numpy().astype(np.float64), oracle.sgemm_f64(a, b)), f"case {chunk}.{idx} ({cfg})"
        del ws, keep_a, keep_b


EXTREME = [
    (1, 1 << 21, 4, 8), (1, 3, 1 << 20, 5), (1, 8, 8, 1 << 18), (1, 1 << 16, 1, 33), (1, 1, 1 << 16, 64),
    (100000, 4, 4, 4), (3000, 1, 33, 7), (1, 65536 + 3, 36, 4), (2, 40, 8, 40000),
]


@pytest.mark.parametrize("case", EXTREME, ids=str)
@pytest.mark.parametrize("with_ws", [False, True], ids=["nows", "ws"])
def test_extreme_aspect_ratios(case, with_ws):
    """Very tall, very wide, very deep and very many: grid sizes, 64-bit offsets and split-K plans at their edges."""
    import torch
    from oracle import oracle
    batch, m, n, k = case
    say(f"extreme {case} workspace={with_ws}")
    a = ig.small_int(9950, (batch, m, k))
    b = ig.small_int(9951, (batch, k, n))
    ws = None
    if with_ws:
        ws = torch.empty(max(tg.workspace_bytes(batch, m, n, k) // 4, 4), device="cuda")
        tg.set_workspace(ws)
    out = torch.full((batch, m, n), float("nan"), device="cuda")
    tg.sgemm_batched(torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda(), out=out)
    torch.cuda.synchronize()
    cfg = tg.last_config()
    ref = oracle.sgemm_f64(a, b)
    assert np.array_equal(out.cpu().numpy().astype(np.float64), ref), f"{case} ({cfg})"
    del ws


@pytest.mark.parametrize("chunk", range(4))
def test_untuned_choices_with_a_workspace_in_both_math_modes(chunk):
    """Mid-size random shapes with a large workspace set and nothing tuned: the static heuristic then picks
    among every family (register-staged, direct-to-LDS, predicated, split-K, tail splits and, in the piece
    mode, the bf16-piece kernels cutting in the loop or ahead).  Integer inputs, sampled rows, bit for bit."""
    import torch
    from oracle import oracle
    rng = np.random.default_rng(8800 + chunk)
    ws = torch.empty(1 << 27, device="cuda")      # 512 MiB
    families = set()
    try:
        for it in range(14):
            batch = int(rng.choice([1, 1, 1, 2, 3]))
            m = int(rng.integers(200, 3500))
            n = int(rng.integers(50, 900)) * 4
            k = int(rng.choice([rng.integers(32, 3000), 32 * rng.integers(1, 100), 4 * rng.integers(8, 700)]))
            if batch > 1:
                m, n = min(m, 1200), min(n, 1200)
            mode = int(rng.integers(0, 2))
            tg.set_math(mode)
            tg.set_workspace(ws)
            a = ig.small_int(9900 + 100 * chunk + it, (batch, m, k))
            b = ig.small_int(9950 + 100 * chunk + it, (batch, k, n))
            da, db = torch.from_numpy(a).cuda(), torch.from_numpy(b).cuda()
            out = torch.full((batch, m, n), float("nan"), device="cuda")
            say(f"untuned case {chunk}.{it}: mode {mode} batch {batch} {m}x{n}x{k}")
            if batch == 1:
                tg.sgemm(da[0], db[0], out=out[0])
            else:
                tg.sgemm_batched(da, db, out=out)
            torch.cuda.synchronize()
            cfg = tg.last_config()
            families.add(cfg[0] + ("+tail" if ":t" in cfg else "") + ("+split" if ":s1:" not in cfg + ":" else ""))
            rows = np.unique(rng.integers(0, m, 32))
            got = out.cpu().numpy()
            assert np.isfinite(got).all(), cfg
            for i in range(batch):
                assert np.array_equal(got[i][rows].astype(np.float64), oracle.sgemm_f64(a[i][rows], b[i])), \
                    f"case {chunk}.{it} ({cfg}): result differs from the oracle"
    finally:
        tg.set_math(tg.MATH_FP32_MFMA)
    say(f"  families used: {sorted(families)}")

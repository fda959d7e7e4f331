"""GPU parity of the bf16-piece kernels (names starting with "e": every fp32 product formed from six or
nine products of bf16 pieces on the bf16 matrix instructions, summed in fp32) against the CPU oracle.
Same bar as the fp32 kernels: per element 1e-5 * sum|a||b|, relative Frobenius 1e-6, integer-valued
inputs bit exact; plus the cases that are particular to cutting operands into pieces (wide exponent
ranges, integers that need all three pieces, non-finite inputs) and the math-mode switch."""
import numpy as np
import pytest

import paper_1904_03383_amd as tg
from paper_1904_03383_amd import inputgen as ig

from gpu_common import check_against_oracle, run_hip, say, to_dev

pytestmark = pytest.mark.gpu

X6, X9 = "e128x256x32_w64x128_x6", "e128x256x32_w64x128_x9"
E128, E64 = "e128x128x32_w64x64_x6", "e64x64x32_w32x32_x6"     # smaller tiles of the same kernel
C6, C9 = "c128x256x32_w64x128_x6", "c128x256x32_w64x128_x9"   # operands cut ahead into the workspace


@pytest.fixture(autouse=True)
def _clean_library_state():
    tg.force_config(None)
    tg.set_workspace(None)
    tg.set_math(tg.MATH_FP32_MFMA)
    yield
    tg.force_config(None)
    tg.set_workspace(None)
    tg.set_math(tg.MATH_FP32_MFMA)
    tg.clear_tune_cache()


SHAPES = [(128, 256, 32), (1, 4, 32), (100, 200, 64), (129, 260, 128), (257, 516, 96), (384, 768, 1024), (1000, 1000, 992)]


@pytest.mark.parametrize("name", [X6, X9, E128, E64])
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_forced_piece_kernel_matches_oracle(name, shape):
    m, n, k = shape
    say(f"{name} on {m}x{n}x{k}")
    tg.force_config(name)
    for dist in ("uniform", "normal", "int"):
        a, b = ig.make_operands(1, m, n, k, dist, 701, 702)
        c = run_hip(a[0], b[0])
        assert tg.last_config().startswith(name)
        check_against_oracle(c, a[0], b[0], exact=(dist == "int"), what=f"{name} {shape} {dist}")


@pytest.mark.parametrize("name", [X6, X9])
def test_headline_size_all_elements(name):
    """4096^3 with the benchmark's operands: every element against the oracle."""
    say(f"{name} at 4096^3")
    a, b = ig.make_config("c5_4096")
    tg.force_config(name)
    c = run_hip(a[0], b[0])
    m = check_against_oracle(c, a[0], b[0], what=name + " 4096^3")
    say(f"  rel_fro {m['rel_fro']:.2e} max_ratio {m['max_ratio']:.2e}")
    # the leading chain rounds once per 16 terms: better than the fp32 kernels' 5.7e-7 here
    assert m["rel_fro"] < 5e-7


@pytest.mark.parametrize("name", [X6, X9, E128, E64])
def test_wide_exponent_range(name):
    """Entries spread over 2^-30 .. 2^30: the pieces keep fp32's exponent range, nothing is scaled."""
    say(f"{name}, wide exponents")
    rng = np.random.default_rng(711)
    m, n, k = 200, 260, 512
    a = (rng.standard_normal((m, k)) * np.exp2(rng.integers(-30, 31, (m, k)))).astype(np.float32)
    b = (rng.standard_normal((k, n)) * np.exp2(rng.integers(-30, 31, (k, n)))).astype(np.float32)
    tg.force_config(name)
    check_against_oracle(run_hip(a, b), a, b, what=name + " wide exponents")


@pytest.mark.parametrize("name", [X6, X9])
@pytest.mark.parametrize("log2_scale", [-45, 55])
def test_uniformly_tiny_and_huge_operands(name, log2_scale):
    """Both operands scaled by 2^-45 (products near 2^-90: every piece product still above the underflow
    threshold) and by 2^55 (sums near 2^120, below overflow): same bar as at unit scale."""
    say(f"{name}, operands scaled by 2^{log2_scale}")
    a, b = ig.make_operands(1, 200, 260, 512, "normal", 715, 716)
    a = (a[0] * np.float32(2.0 ** log2_scale)).astype(np.float32)
    b = (b[0] * np.float32(2.0 ** log2_scale)).astype(np.float32)
    tg.force_config(name)
    check_against_oracle(run_hip(a, b), a, b, what=f"{name} scale 2^{log2_scale}")


@pytest.mark.parametrize("name", [X6, X9])
def test_integers_that_need_every_piece(name):
    """Integers up to 2^11 use two pieces (all four cross products are among the six); up to 2^23 with
    zero low bits in one operand they use three; sums kept below 2^24 so that fp32 holds them exactly."""
    say(f"{name}, multi-piece integers")
    rng = np.random.default_rng(713)
    tg.force_config(name)
    a = rng.integers(-2047, 2048, (130, 32)).astype(np.float32)
    b = rng.integers(-120, 121, (32, 260)).astype(np.float32)
    check_against_oracle(run_hip(a, b), a, b, exact=True, what=name + " 11-bit x 7-bit")
    if name == X9:
        # 23-bit integers times +-1/0: every piece of A matters, only the nine-product form keeps them all
        a = rng.integers(-(2 ** 22), 2 ** 22, (130, 32)).astype(np.float32)
        b = np.zeros((32, 260), np.float32)
        b[rng.integers(0, 32, 260), np.arange(260)] = rng.choice([-1.0, 1.0], 260)
        check_against_oracle(run_hip(a, b), a, b, exact=True, what=name + " 23-bit selection")


def test_batched_padded_and_split_k():
    import torch
    say("piece kernel: batch of 3, padded leading dimensions, split-K")
    batch, m, n, k = 3, 130, 260, 256
    a, b = ig.make_operands(batch, m, n, k, "int", 721, 722)
    tg.force_config(X6)
    c = run_hip(a, b)
    for i in range(batch):
        check_against_oracle(c[i], a[i], b[i], exact=True, what=f"batched {i}")
    # padded rows: operands and result are views into wider buffers
    da = torch.zeros((m, k + 12), device="cuda"); da[:, :k] = to_dev(a[0])
    db = torch.zeros((k, n + 8), device="cuda"); db[:, :n] = to_dev(b[0])
    out = torch.full((m, n + 4), float("nan"), device="cuda")
    tg.sgemm(da[:, :k], db[:, :n], out=out[:, :n])
    torch.cuda.synchronize()
    assert tg.last_config().startswith(X6)
    check_against_oracle(out[:, :n].cpu().numpy(), a[0], b[0], exact=True, what="padded")
    assert torch.isnan(out[:, n:]).all()
    ws = torch.empty(4 * m * n, device="cuda")
    tg.set_workspace(ws)
    tg.force_config(X6 + ":s4")
    check_against_oracle(run_hip(a[0], b[0]), a[0], b[0], exact=True, what="split-K")
    assert tg.last_config().startswith(X6 + ":s4")


def test_k_range_limit_and_validity_messages():
    import torch
    say("piece kernel: validity")
    tg.force_config(X6)
    a = torch.zeros((128, 48), device="cuda"); b = torch.zeros((48, 256), device="cuda")
    with pytest.raises(tg.TgemmError, match="multiple of the K tile"):
        tg.sgemm(a, b)
    a = torch.zeros((8, 16384), device="cuda"); b = torch.zeros((16384, 8), device="cuda")
    with pytest.raises(tg.TgemmError, match="K range too long"):
        tg.sgemm(a, b)
    ws = torch.empty(2 * 8 * 8, device="cuda")
    tg.set_workspace(ws)
    tg.force_config(X6 + ":s2")     # two ranges of 8192
    a.fill_(1.0); b.fill_(1.0)
    c = tg.sgemm(a, b)
    torch.cuda.synchronize()
    assert (c == 16384.0).all()


def test_non_finite_inputs_poison_their_row_or_column():
    """NaN behaves as in fp32.  An infinite input gives NaN (its remainder inf - inf is NaN), documented as
    the one difference from fp32 arithmetic on non-finite values."""
    import torch
    say("piece kernel: NaN / inf")
    m, n, k = 128, 256, 64
    a = torch.ones((m, k), device="cuda"); b = torch.ones((k, n), device="cuda")
    a[5, 7] = float("nan"); b[9, 100] = float("inf")
    tg.force_config(X6)
    c = tg.sgemm(a, b)
    torch.cuda.synchronize()
    bad = torch.isnan(c)
    expect = torch.zeros_like(bad); expect[5, :] = True; expect[:, 100] = True
    assert torch.equal(bad, expect)
    assert (c[~bad] == float(k)).all()


def test_math_mode_switch_and_tuning():
    import torch
    say("math mode: candidates, tuning, cache per mode")
    m = n = k = 2048
    names = lambda: [s.split(":")[0] for s, _, _ in tg.candidates(1, m, n, k)]
    assert tg.get_math() == tg.MATH_FP32_MFMA and not any(x.startswith("e") for x in names())
    a, b = ig.make_operands(1, m, n, k, "normal", 731, 732)
    da, db = to_dev(a[0]), to_dev(b[0])
    tg.tune(da, db, reps=2)
    tuned_fp32 = tg.last_config()
    assert not tuned_fp32.startswith("e")
    tg.set_math(tg.MATH_BF16_PIECES)
    assert tg.get_math() == tg.MATH_BF16_PIECES and X6 in names() and X9 in names()
    c = tg.tune(da, db, reps=2)
    tuned = tg.last_config()
    say(f"  fp32 mode: {tuned_fp32}; piece mode: {tuned}")
    check_against_oracle(c.cpu().numpy(), a[0], b[0], what="tuned in piece mode " + tuned)
    assert tg.get_config(1, m, n, k) == tuned
    # back in fp32 mode the entry tuned there is used again, never a piece kernel
    tg.set_math(tg.MATH_FP32_MFMA)
    assert tg.get_config(1, m, n, k) == tuned_fp32
    c2 = tg.sgemm(da, db)
    torch.cuda.synchronize()
    assert tg.last_config() == tuned_fp32
    check_against_oracle(c2.cpu().numpy(), a[0], b[0], what="fp32 mode after piece mode")


# ---- kernels that cut the operands ahead (separate passes into a workspace image) ----------------

CUT_AHEAD_SHAPES = [(1, 4, 1), (7, 12, 5), (129, 260, 100), (128, 256, 32), (257, 516, 97), (1000, 1000, 1000), (300, 516, 2052)]


@pytest.mark.parametrize("name", [C6, C9])
@pytest.mark.parametrize("shape", CUT_AHEAD_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_cut_ahead_kernel_any_k(name, shape):
    """The cutting passes pad with zeros: any m and k (n a multiple of 4 for the vector stores)."""
    import torch
    m, n, k = shape
    say(f"{name} on {m}x{n}x{k}")
    ws = torch.empty(tg.workspace_bytes(1, m, n, k) // 4 + (1 << 22), device="cuda")
    tg.set_workspace(ws)
    tg.force_config(name)
    for dist in ("normal", "int"):
        a, b = ig.make_operands(1, m, n, k, dist, 741, 742)
        c = run_hip(a[0], b[0])
        assert tg.last_config().startswith(name)
        check_against_oracle(c, a[0], b[0], exact=(dist == "int"), what=f"{name} {shape} {dist}")


def test_cut_ahead_workspace_rules_unaligned_operands_batches_and_split_k():
    import torch
    say("cut-ahead kernel: workspace, unaligned A and B, batch, split-K")
    m, n, k = 130, 260, 250
    a, b = ig.make_operands(1, m, n, k, "int", 751, 752)
    tg.force_config(C6)
    with pytest.raises(tg.TgemmError) as err:         # no workspace: a workspace error that says why
        tg.sgemm(to_dev(a[0]), to_dev(b[0]))
    assert err.value.status_name == "TG_ERR_WORKSPACE" and "piece images" in str(err.value)
    # images: 2 tile rows of 128 and 2 tile columns of 256 over 8 K tiles, 3 planes of 4 chunks of 16 bytes
    images = 8 * (2 * 128 + 2 * 256) * 3 * 4 * 16
    tg.set_math(tg.MATH_BF16_PIECES)
    assert tg.workspace_bytes(1, m, n, k) >= images
    tg.set_math(tg.MATH_FP32_MFMA)
    ws = torch.empty(images // 4, device="cuda")
    tg.set_workspace(ws)
    check_against_oracle(run_hip(a[0], b[0]), a[0], b[0], exact=True, what="exact-size workspace")
    # A and B views that start 4 bytes into their buffers and have odd leading dimensions
    bufa = torch.zeros(m * (k + 3) + 1, device="cuda"); bufb = torch.zeros(k * (n + 1) + 1, device="cuda")
    da = bufa[1:].view(m, k + 3)[:, :k]; db = bufb[1:].view(k, n + 1)[:, :n]
    da.copy_(to_dev(a[0])); db.copy_(to_dev(b[0]))
    out = torch.full((m, n), float("nan"), device="cuda")
    tg.sgemm(da, db, out=out)
    torch.cuda.synchronize()
    assert tg.last_config().startswith(C6)
    check_against_oracle(out.cpu().numpy(), a[0], b[0], exact=True, what="unaligned A and B")
    # batch of 3 and split-K (partials first, images after them)
    a3, b3 = ig.make_operands(3, m, n, k, "int", 753, 754)
    ws = torch.empty((3 * images + 4 * 3 * m * n * 4 + 1024) // 4, device="cuda")
    tg.set_workspace(ws)
    c = run_hip(a3, b3)
    for i in range(3):
        check_against_oracle(c[i], a3[i], b3[i], exact=True, what=f"batched {i}")
    tg.force_config(C6 + ":s4")
    c = run_hip(a3, b3)
    assert tg.last_config().startswith(C6 + ":s4")
    for i in range(3):
        check_against_oracle(c[i], a3[i], b3[i], exact=True, what=f"batched split-K {i}")
    # n not a multiple of 4 and C at an odd offset with an odd leading dimension: stored element by element
    a5, b5 = ig.make_operands(1, 70, 203, 45, "int", 755, 756)
    bufc = torch.full((70 * 205 + 3,), 7.0, device="cuda")
    dc = bufc[1:1 + 70 * 205].view(70, 205)[:, :203]
    tg.force_config(C9)
    tg.sgemm(to_dev(a5[0]), to_dev(b5[0]), out=dc)
    torch.cuda.synchronize()
    assert tg.last_config().startswith(C9)
    check_against_oracle(dc.cpu().numpy(), a5[0], b5[0], exact=True, what="unaligned C, n = 203")
    mask = torch.ones_like(bufc, dtype=torch.bool)
    torch.as_strided(mask, (70, 203), (205, 1), 1).fill_(False)
    assert bool((bufc[mask] == 7.0).all())


# ---- seeded random shapes and placements through the piece kernels ------------------------------

def _random_piece_cases(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        batch = int(rng.choice([1, 1, 2, 3]))
        m = int(rng.integers(1, 400))
        n = int(rng.choice([4 * rng.integers(1, 150), rng.integers(1, 600)]))
        k = int(rng.choice([rng.integers(1, 700), 32 * rng.integers(1, 20)]))
        pads = (int(rng.choice([0, 4, 1, 3])), int(rng.choice([0, 4, 1, 3])), int(rng.choice([0, 4, 8, 1])))   # lda-k, ldb-n, ldc-n
        offs = (int(rng.choice([0, 4, 1])), int(rng.choice([0, 4, 1])), int(rng.choice([0, 4, 3])))            # element offsets of A, B, C
        gaps = (int(rng.choice([0, 4, 7])), int(rng.choice([0, 4, 7])), int(rng.choice([0, 4, 8, 5])))         # extra batch strides
        out.append((batch, m, n, k, pads, offs, gaps, int(rng.integers(0, 3))))
    return out


PIECE_CASES = _random_piece_cases(20261127, 48)


@pytest.mark.parametrize("chunk", range(6))
def test_random_shapes_and_placements_are_bit_exact(chunk):
    """Any m, n and k, A, B and C anywhere (odd leading dimensions, odd base offsets, odd batch strides): the
    cut-ahead kernels take all of it; the kernel that cuts in its loop is forced too whenever the case meets
    its rules (16-byte aligned operands, k a multiple of 32)."""
    import torch
    from oracle import oracle
    from test_random_shapes_gpu import _place
    ws = torch.empty(1 << 24, device="cuda")       # 64 MiB
    for idx in range(chunk * 8, chunk * 8 + 8):
        batch, m, n, k, pads, offs, gaps, pick = PIECE_CASES[idx]
        a = ig.small_int(9100 + idx, (batch, m, k))
        b = ig.small_int(9300 + idx, (batch, k, n))
        aligned = all(x % 4 == 0 for x in pads + offs + gaps) and k % 4 == 0 and n % 4 == 0
        specs = [(C6, C9, C6 + ":s2")[pick]]
        if specs[0].endswith(":s2") and k <= 96:        # each K range needs at least two K tiles
            specs = [C6]
        if aligned and k % 32 == 0:
            specs.append((X6, E128, E64)[idx % 3])
        _, da = _place(a, pads[0], offs[0], gaps[0], float("nan"))
        _, db = _place(b, pads[1], offs[1], gaps[1], float("nan"))
        ref = oracle.sgemm_f64(a, b)
        for spec in specs:
            say(f"random piece case {idx}: {spec} batch {batch} {m}x{n}x{k} pads {pads} offsets {offs} gaps {gaps}")
            tg.set_workspace(ws)
            tg.force_config(spec)
            cflat, dc = _place(np.zeros((batch, m, n), np.float32), pads[2], offs[2], gaps[2], 7.0)
            cflat.fill_(7.0)
            if batch == 1:
                tg.sgemm(da[0], db[0], out=dc[0])
            else:
                tg.sgemm_batched(da, db, out=dc)
            torch.cuda.synchronize()
            assert tg.last_config().startswith(spec)
            assert np.array_equal(dc.cpu().numpy().astype(np.float64), ref), f"case {idx} ({spec}): result differs from the oracle"
            mask = torch.ones_like(cflat, dtype=torch.bool)
            torch.as_strided(mask, (batch, m, n), dc.stride(), offs[2]).fill_(False)
            assert bool((cflat[mask] == 7.0).all()), f"case {idx} ({spec}): stores outside the output"


@pytest.mark.parametrize("name", [X6, X9, C6])
def test_longest_k_range_keeps_the_bar(name):
    """K = 8192 is the longest range one workgroup may take (512 roundings of the leading chain); twice that
    goes through split-K.  Same bar as everywhere."""
    import torch
    say(f"{name} at K = 8192 and 16384")
    ws = torch.empty(1 << 25, device="cuda")
    tg.set_workspace(ws)
    for k, spec in ((8192, name), (16384, name + ":s2")):
        a, b = ig.make_operands(1, 192, 260, k, "normal", 761, 762)
        tg.force_config(spec)
        c = run_hip(a[0], b[0])
        m = check_against_oracle(c, a[0], b[0], what=f"{spec} K={k}")
        say(f"  {spec} K={k}: rel_fro {m['rel_fro']:.2e}")


def test_worst_case_for_the_dropped_terms():
    """Every element has an all-ones significand (2 - 2^-23 times a power of two), all of one sign: the three
    piece products that the six-product form leaves out are then as large as they can be, about 2^-23 of each
    product, and all add up.  Both forms must stay within the bars, and the difference between them must be
    what the dropped terms explain: present, and at most 2^-22 of sum|a||b|."""
    from oracle import oracle
    say("six against nine products, all-ones significands")
    rng = np.random.default_rng(771)
    m, n, k = 130, 260, 4096
    ones = np.float32(2.0) - np.float32(2.0 ** -23)
    a = (ones * np.exp2(rng.integers(-3, 4, (m, k)))).astype(np.float32)
    b = (ones * np.exp2(rng.integers(-3, 4, (k, n)))).astype(np.float32)
    out = {}
    for name in (X6, X9):
        tg.force_config(name)
        out[name] = run_hip(a, b)
        mm = check_against_oracle(out[name], a, b, what=name + " all-ones significands")
        say(f"  {name}: rel_fro {mm['rel_fro']:.2e} max_ratio {mm['max_ratio']:.2e}")
    _, s_abs = oracle.sgemm_f64(a, b, want_abs=True)
    gap = (out[X9].astype(np.float64) - out[X6].astype(np.float64)) / s_abs
    say(f"  (nine - six) / sum|a||b|: mean {gap.mean():.2e} max {gap.max():.2e}")
    assert 2.0 ** -25 < gap.mean() < 2.0 ** -22 and gap.max() < 2.0 ** -21 and gap.min() > -2.0 ** -22

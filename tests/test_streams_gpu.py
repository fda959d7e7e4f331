"""Stream, HIP-graph and host-thread behaviour of the C-ABI entry points on the GPU: calls only enqueue on the
given stream, can be captured into a graph and replayed, and may be issued from several host threads."""
import threading

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


def test_calls_are_ordered_on_a_side_stream():
    """Producer (torch op), tg_sgemm and consumer (torch op) on one non-default stream, no host sync between."""
    import torch
    say("side stream ordering")
    m, n, k = 384, 256, 512
    a = ig.small_int(701, (m, k))
    b = ig.small_int(702, (k, n))
    da, db = to_dev(a), to_dev(b)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        da2 = da * 2.0                                   # producer on the side stream
        out = torch.full((m, n), float("nan"), device="cuda")
        tg.sgemm(da2, db, out=out)                       # picks up torch's current stream
        twice = out + out                                # consumer on the side stream
        out2 = torch.full((m, n), float("nan"), device="cuda")
        tg.sgemm(da2, db, out=out2, stream=side)         # explicit stream argument
    side.synchronize()
    check_against_oracle(out.cpu().numpy(), 2.0 * a, b, exact=True, what="side stream")
    assert torch.equal(twice, out * 2.0) and torch.equal(out, out2)


@pytest.mark.parametrize("case", ["sgemm", "batched", "k0", "saxpy", "strided_packed", "strided_fused", "split_k", "pieces", "pieces_cut_ahead"])
def test_graph_capture_replays_match_eager(case):
    """Every entry point captured into a HIP graph; each of several replays (with eager work and
    synchronisation in between, inputs changed before each) must equal the eager result."""
    import torch
    say(f"graph capture {case}")
    ws = None
    if case == "sgemm":
        x, y = to_dev(ig.small_int(711, (256, 192))), to_dev(ig.small_int(712, (192, 320)))
        out = torch.empty((256, 320), device="cuda")
        fn = lambda: tg.sgemm(x, y, out=out)
    elif case == "batched":
        x, y = to_dev(ig.small_int(713, (6, 32, 64))), to_dev(ig.small_int(714, (6, 64, 32)))
        out = torch.empty((6, 32, 32), device="cuda")
        fn = lambda: tg.sgemm_batched(x, y, out=out)
    elif case == "k0":
        x, y = torch.empty((40, 0), device="cuda"), torch.empty((0, 24), device="cuda")
        out = torch.empty((40, 24), device="cuda")
        fn = lambda: tg.sgemm(x, y, out=out)
    elif case == "saxpy":
        x, y = to_dev(ig.uniform(715, (100003,))), to_dev(ig.uniform(716, (100003,)))
        out = torch.empty_like(x)
        fn = lambda: tg.saxpy(0.75, x, y, out=out)
    elif case == "strided_packed":                # k no multiple of 32: packing pass + plain kernel, two launches
        xs, y = to_dev(ig.small_int(717, (256, 100 * 3))), to_dev(ig.small_int(718, (100, 256)))
        x = xs[:, ::3]
        ws = torch.empty(tg.strided_workspace_bytes(256, 256, 100, 3, 1) // 4 + 4, device="cuda")
        tg.set_workspace(ws)
        out = torch.empty((256, 256), device="cuda")
        fn = lambda: tg.sgemm_strided(x, y, out=out)
    elif case == "strided_fused":                 # gathered inside the product kernel
        xs, y = to_dev(ig.small_int(717, (256, 128 * 3))), to_dev(ig.small_int(718, (128, 256)))
        x = xs[:, ::3]
        out = torch.empty((256, 256), device="cuda")
        fn = lambda: tg.sgemm_strided(x, y, out=out)
    elif case == "pieces":
        x, y = to_dev(ig.small_int(721, (200, 96))), to_dev(ig.small_int(722, (96, 260)))
        tg.force_config("e128x256x32_w64x128_x6")
        out = torch.empty((200, 260), device="cuda")
        fn = lambda: tg.sgemm(x, y, out=out)
    elif case == "pieces_cut_ahead":              # three kernels per call: two cutting passes and the product
        x, y = to_dev(ig.small_int(723, (200, 90))), to_dev(ig.small_int(724, (90, 260)))
        ws = torch.empty(1 << 20, device="cuda")
        tg.set_workspace(ws)
        tg.force_config("c128x256x32_w64x128_x9")
        out = torch.empty((200, 260), device="cuda")
        fn = lambda: tg.sgemm(x, y, out=out)
    else:
        x, y = to_dev(ig.small_int(719, (128, 1024))), to_dev(ig.small_int(720, (1024, 128)))
        ws = torch.empty(4 * 128 * 128 + 4, device="cuda")
        tg.set_workspace(ws)
        tg.force_config("t128x128x16_w64x64:s4")
        out = torch.empty((128, 128), device="cuda")
        fn = lambda: tg.sgemm(x, y, out=out)
    fn()                                                  # eager once: loads code objects before the capture
    torch.cuda.synchronize()
    if case == "strided_packed":
        assert tg.last_config().endswith("+packA")
    if case == "strided_fused":
        assert "_ga" in tg.last_config() and "+pack" not in tg.last_config()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    for rep in range(4):
        if x.numel():
            x.mul_(-1.0 if rep % 2 else 2.0)              # change the input between replays (on the default stream)
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = out.clone()
        out.fill_(float("nan"))
        fn()                                              # the program's own eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(got, out), f"{case}: replay {rep} differs from the eager call"
        assert torch.isfinite(out).all()
    del ws


def test_concurrent_host_threads_on_their_own_streams():
    """Four host threads, each with its own stream and shapes, call into the library at once (no workspace)."""
    import torch
    say("host threads")
    shapes = [(256, 256, 256), (130, 70, 50), (512, 128, 64), (64, 64, 1100)]
    hosts = [(ig.small_int(730 + i, (m, k)), ig.small_int(740 + i, (k, n))) for i, (m, n, k) in enumerate(shapes)]
    devs = [(to_dev(a), to_dev(b)) for a, b in hosts]
    outs = [torch.full((m, n), float("nan"), device="cuda") for (m, n, k) in shapes]
    errors = []
    torch.cuda.synchronize()

    def work(i):
        try:
            s = torch.cuda.Stream()
            for _ in range(25):
                tg.sgemm(devs[i][0], devs[i][1], out=outs[i], stream=s)
            s.synchronize()
        except Exception as ex:  # noqa: BLE001 - reported in the main thread
            errors.append((i, repr(ex)))

    threads = [threading.Thread(target=work, args=(i,)) for i in range(len(shapes))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for i, (a, b) in enumerate(hosts):
        check_against_oracle(outs[i].cpu().numpy(), a, b, exact=True, what=f"thread {i} {shapes[i]}")

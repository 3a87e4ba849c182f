"""The planner's choices, timed: for a grid of history and chunk lengths at the 7B-class layer
shape, the launch plan the library picks by itself (how many pieces the key range is cut into, or
none) must be within 12 % of the best of a set of forced plans -- the unsplit launch and piece
counts from 2 to 32 set through evl_cache_tune.  The grid mixes the lengths the planner's model was
fitted on with lengths in between (100, 350, 750, 1500, 2600 new tokens: chunk sizes whose row tiles
do not fill the XCDs' compute units evenly, where a piece count one off the right one costs a whole
round of work-groups).  tests/test_host_plan_cpu.py pins WHICH plans are chosen; this test checks on
the chip that they are good ones.  Values do not matter here, only time: the caches hold seeded
random numbers (timing depends on the data: all-zero operands run faster)."""
import time

import numpy as np
import pytest
import torch

from synth import page_permutation

pytestmark = pytest.mark.gpu

HQ, HKV, D = 28, 4, 128
GRID = [(C, n) for C in (0, 1000, 6580, 20000, 60000) for n in (40, 100, 204, 350, 750, 1000, 1500, 2000, 2600)
        if not (C == 0 and n < 204)]
PIECES = (2, 3, 4, 5, 6, 8, 10, 12, 16, 20, 26, 32)
BAR = 1.12


def time_us(fn, stream, calls=10, reps=3):
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    best = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(calls):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        best.append(e0.elapsed_time(e1) / calls * 1e3)
    return min(best)


def test_default_plan_is_close_to_the_best_forced_plan():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2512_10310_amd as evl
    evl.load()
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()
    gen = torch.Generator(device=dev)
    gen.manual_seed(20251210)
    ws_bytes = 1 << 30
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    worst = (0.0, None)
    # the chip raises its clocks only after some tenths of a second of work: do that before anything is timed
    a = torch.randn((4096, 4096), device=dev)
    t_end = time.perf_counter() + 0.5
    while time.perf_counter() < t_end:
        for _ in range(10):
            a @ a
        torch.cuda.synchronize()
    del a
    for C, n in GRID:
        L = C + n
        pages = -(-L // 16)
        kp = torch.randn((pages, HKV, 16, D), generator=gen, device=dev).to(torch.bfloat16)
        vp = torch.randn((pages, HKV, D, 16), generator=gen, device=dev).to(torch.bfloat16)
        tbl = torch.from_numpy(page_permutation(pages, 1)).to(dev)
        zeros = torch.zeros((L, HKV, D), device=dev, dtype=torch.bfloat16)
        q = torch.randn((n, HQ, D), generator=gen, device=dev).to(torch.bfloat16)
        out = torch.empty_like(q)
        with_ws = evl.Cache(HQ, HKV, D, 1e6, kp, vp, tbl, pages, pages, stream=stream.cuda_stream, workspace=ws,
                            workspace_bytes=ws_bytes)
        without = evl.Cache(HQ, HKV, D, 1e6, kp, vp, tbl, pages, pages, stream=stream.cuda_stream)
        with_ws.rope_append(zeros, zeros, 0, L)     # bookkeeping; the pools get their values back below
        without.rope_append(zeros, zeros, 0, L)
        torch.cuda.synchronize()
        kp.normal_(generator=gen)
        vp.normal_(generator=gen)
        torch.cuda.synchronize()
        calls = max(2, min(10, int(1500 / (20 + 1.5e-3 * n * L / 64))))      # about a millisecond per timing
        times, base = {}, -(-n * (HQ // HKV) // 256) * HKV      # work-groups of the unsplit launch
        for pieces in PIECES:
            if pieces > -(-L // 64) // 4:        # pieces of fewer than 4 key tiles are not made
                break
            with_ws.tune(base * pieces)
            t = time_us(lambda: with_ws.chunk_attention(q, C, n, out), stream, calls=calls)
            times["%d work-groups, %d pieces" % with_ws.last_plan()[:2]] = t
        times["unsplit"] = time_us(lambda: without.chunk_attention(q, C, n, out), stream, calls=calls)
        with_ws.tune(0)
        own = time_us(lambda: with_ws.chunk_attention(q, C, n, out), stream, calls=calls)
        plan = with_ws.last_plan()[:2]
        if plan[1] > 1 and "%d work-groups, %d pieces" % plan in times:      # timed twice: the better of the two
            own = min(own, times["%d work-groups, %d pieces" % plan])
        elif plan[1] == 1:
            own = min(own, times["unsplit"])
        best = min(min(times.values()), own)
        ratio = own / best
        if ratio > BAR:      # one more look before failing: a noisy neighbour on the box would show up here
            rival = min(times, key=times.get)
            if rival != "unsplit":
                with_ws.tune(int(rival.split()[0]))
                again = time_us(lambda: with_ws.chunk_attention(q, C, n, out), stream, calls=calls)
            else:
                again = time_us(lambda: without.chunk_attention(q, C, n, out), stream, calls=calls)
            with_ws.tune(0)
            own = min(own, time_us(lambda: with_ws.chunk_attention(q, C, n, out), stream, calls=calls))
            times[rival] = max(times[rival], again)      # the rival has to win twice
            best = min(min(times.values()), own)
            ratio = own / best
        print("C=%5d n=%4d: own plan %s %.1f us, best forced %.1f us (%s), ratio %.3f" % (
            C, n, plan, own, min(times.values()), min(times, key=times.get), ratio), flush=True)
        if ratio > worst[0]:
            worst = (ratio, (C, n))
        assert ratio <= BAR, "C=%d n=%d: the library's plan %s takes %.1f us, %s takes %.1f us" % (
            C, n, plan, own, min(times, key=times.get), min(times.values()))
        del with_ws, without, kp, vp, zeros
    print("worst ratio %.3f at %s" % worst)

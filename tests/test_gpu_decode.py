"""GPU parity for chunks of a few tokens over a long cache (the step's action tokens, generated
one at a time after the frame has been processed: paper Sec. 3.1 / 3.2).  These calls take the
path that merges the key-range pieces inside the attention kernel."""
import numpy as np
import pytest
import torch

import oracle
from synth import TINY, LAYER7B, StreamShape, qkv_chunk

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 1e-2, 1e-3


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2512_10310_amd as evl
    evl.load()


def stream_of(shape, lengths, cfg):
    chunks = [qkv_chunk(shape, n, cfg, 0, s) for s, n in enumerate(lengths)]
    ost = oracle.Stream(shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rope_base)
    return chunks, ost


@pytest.mark.parametrize("out_f32", [False, True])
def test_action_tokens_after_a_long_history(out_f32):
    """6000 cached tokens, then chunks of 1, 1, 2, 4, 8, 1 tokens appended and attended one after
    the other (each sees the previous ones)."""
    from harness import GpuLayer, check_close
    shape = LAYER7B
    lengths = [3000, 3000, 1, 1, 2, 4, 8, 1]
    chunks, ost = stream_of(shape, lengths, cfg=60)
    layer = GpuLayer(shape, [sum(lengths)], random_pages=True, out_f32=out_f32)
    plans = []
    for s, (q, k, v) in enumerate(chunks):
        C = layer.cache.len()
        if s < 2:
            ost.append(k, v, C)
            layer.append(k, v, C)
            continue
        want = ost.step(q, k, v, C)
        got = layer.step(q, k, v, C)
        plans.append(layer.cache.last_plan())
        check_close(got, want, MAX_ABS, MEAN_ABS, "chunk %d of %d tokens at %d" % (s, lengths[s], C))
    assert all(p[1] > 8 for p in plans), plans      # the key range really was cut into pieces


def test_with_and_without_room_for_the_counters():
    """Same inputs with a workspace that holds the ticket counters (pieces merged inside the
    attention kernel) and with one too small for them (and for any partial result: one piece,
    written directly)."""
    from harness import GpuLayer, check_close
    shape = StreamShape(28, 4, 128, 1e6, 2500, 1, 0)
    lengths = [2500, 1, 3]
    chunks, ost = stream_of(shape, lengths, cfg=61)
    want = [ost.step(q, k, v, len(ost)) for (q, k, v) in chunks]
    for name, ws, pieces in (("in_kernel", 4 << 20, None), ("no_room", 8000, 1)):
        layer = GpuLayer(shape, [sum(lengths)], out_f32=True, workspace_bytes=ws)
        for s, (q, k, v) in enumerate(chunks):
            C = layer.cache.len()
            got = layer.step(q, k, v, C)
            if s > 0:
                check_close(got, want[s], MAX_ABS, MEAN_ABS, "%s chunk %d" % (name, s))
                if pieces is None:
                    assert layer.cache.last_plan()[1] > 1
                else:
                    assert layer.cache.last_plan()[1] == pieces


def test_repeated_calls_leave_the_counters_clean():
    """Two different decode calls of the same shape (same workspace addresses) by turns, with a
    larger chunk that uses the merge kernel in between: every result equals the first result
    for its input bit for bit, and that one meets the bar against the oracle.  A piece read
    before it was written, or left over from the previous call, would show up here."""
    from harness import GpuLayer, check_close
    shape = LAYER7B
    chunks, ost = stream_of(shape, [4000, 1], cfg=62)
    layer = GpuLayer(shape, [4000 + 204], out_f32=True)
    layer.append(chunks[0][1], chunks[0][2], 0)
    ost.append(chunks[0][1], chunks[0][2], 0)
    inputs = [chunks[1], qkv_chunk(shape, 1, 62, 0, 5)]
    qb, kb, vb = qkv_chunk(shape, 204, 62, 0, 7)
    first = [None, None]
    for it in range(10):
        w = it % 2
        q1, k1, v1 = inputs[w]
        layer.cache.truncate(4000)
        got = layer.step(q1, k1, v1, 4000)
        if first[w] is None:
            first[w] = got
            ost.truncate(4000)
            check_close(got, ost.step(q1, k1, v1, 4000), MAX_ABS, MEAN_ABS, "input %d" % w)
        assert np.array_equal(got, first[w]), "call %d differs from the first with its input" % it
        if it % 3 == 2:
            layer.cache.truncate(4000)
            big = layer.step(qb, kb, vb, 4000)
            assert np.all(np.isfinite(big))
    assert not np.array_equal(first[0], first[1])


def test_action_tokens_over_a_sampled_history():
    """The decode step of the paper's pipeline: a few new tokens attend to the sampler's choice of
    the history (prefix + 16 of 40 frames) plus the frame just processed; pieces are merged inside
    the multi-entry build of the attention kernel."""
    import paper_2512_10310_amd as evl
    from harness import GpuLayer, check_close
    shape = LAYER7B
    frames = 40
    lengths = [shape.prefix] + [shape.step_tokens] * frames + [1, 4, 8]
    chunks = [qkv_chunk(shape, m, 63, 0, s, bf16=True) for s, m in enumerate(lengths)]
    layer = GpuLayer(shape, [sum(lengths)], random_pages=True)
    for (q, k, v) in chunks[:frames + 1]:
        layer.append(k, v, layer.cache.len())
    hist_end = layer.cache.len()
    kept = evl.sample_uniform(frames - 1, 16)            # among the frames before the newest one
    runs = [(0, shape.prefix)] + [(shape.prefix + f * shape.step_tokens, shape.step_tokens) for f in kept]
    runs.append((hist_end - shape.step_tokens, shape.step_tokens))   # the frame just processed
    for (q, k, v) in chunks[frames + 1:]:
        C = layer.cache.len()
        layer.append(k, v, C)
        # earlier action tokens of this step stay visible: they extend the last run
        cur_runs = runs[:-1] + [(runs[-1][0], C - runs[-1][0])]
        got = layer.attend_sampled(q, cur_runs, C)
        k_hist = np.concatenate([c[1] for c in chunks], axis=0)[:C]
        v_hist = np.concatenate([c[2] for c in chunks], axis=0)[:C]
        want = oracle.sampled_reuse(q, k, v, k_hist, v_hist, cur_runs, 0, shape.rope_base)
        check_close(got, want, MAX_ABS, MEAN_ABS, "%d action tokens at %d" % (q.shape[0], C))
        assert layer.cache.last_plan()[1] > 1


@pytest.mark.parametrize("C", [0, 1, 15, 16, 31, 32, 33, 63, 64, 65, 95, 96, 97, 1000])
@pytest.mark.parametrize("n", [1, 3])
def test_decode_kernel_at_page_and_tile_boundaries(C, n):
    """Cache lengths around the 16-token pages and the decode kernel's 32-key tiles, including a
    one-token prefill (nothing cached)."""
    from harness import GpuLayer, check_close
    shape = StreamShape(14, 2, 128, 1.0e6, 0, 0, 0)
    ost = oracle.Stream(14, 2, 128, 1e6)
    layer = GpuLayer(shape, [C + n], random_pages=True, out_f32=True, cfg=64)
    if C:
        _, k, v = qkv_chunk(shape, C, 64, C, 0)
        ost.append(k, v, 0)
        layer.append(k, v, 0)
    q, k, v = qkv_chunk(shape, n, 64, C, 1)
    want = ost.step(q, k, v, C)
    got = layer.step(q, k, v, C)
    check_close(got, want, MAX_ABS, MEAN_ABS, "C=%d n=%d" % (C, n))


@pytest.mark.parametrize("shape", [TINY, LAYER7B], ids=["tiny", "layer7b"])
def test_ragged_batch_of_short_chunks(shape):
    """Several sequences of very different lengths, each with its own short chunk, in one call
    (d = 64 with two query heads per KV head, and the 7B-class head shape)."""
    from harness import GpuLayer, check_close
    per_row = 32 // shape.group
    lens = [0, 7, 333, 2500, 9000]
    ns = [min(per_row, x) for x in (1, 4, 2, 16, 3)]
    layer = GpuLayer(shape, [c + m for c, m in zip(lens, ns)], random_pages=True, out_f32=True, cfg=65)
    osts = [oracle.Stream(shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rope_base) for _ in lens]
    for s, C in enumerate(lens):
        done = 0
        while done < C:                      # history in pieces of at most 3000 tokens
            m = min(3000, C - done)
            _, k, v = qkv_chunk(shape, m, 65, s, done)
            osts[s].append(k, v, 10 + done)
            layer.append_batched([k], [v], [s], [10 + done])
            done += m
    chunks = [qkv_chunk(shape, m, 65, s, 99999) for s, m in enumerate(ns)]
    ids = list(range(len(lens)))
    layer.append_batched([c[1] for c in chunks], [c[2] for c in chunks], ids, [10 + c for c in lens])
    got = layer.attend_batched([c[0] for c in chunks], ids, lens)
    for s in ids:
        q, k, v = chunks[s]
        want = osts[s].step(q, k, v, 10 + lens[s])
        check_close(got[s], want, MAX_ABS, MEAN_ABS, "sequence %d" % s)


def test_long_pieces_and_no_workspace():
    """One wave walks through hundreds of tiles (more than one register of page ids) when the
    split target is tiny; and without a workspace there is one work-group per KV head, written
    directly.  Same inputs, same bar."""
    from harness import GpuLayer, check_close
    shape = LAYER7B
    C = 41000
    hist_chunks = [qkv_chunk(shape, 4100, 66, 0, s) for s in range(10)]
    q, k, v = qkv_chunk(shape, 2, 66, 0, 77)
    ost = oracle.Stream(shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rope_base)
    for (_, kk, vv) in hist_chunks:
        ost.append(kk, vv, len(ost))
    want = ost.step(q, k, v, C)
    for ws, target in ((64 << 20, 1), (0, 0), (64 << 20, 0)):
        layer = GpuLayer(shape, [C + 2], random_pages=True, out_f32=True, workspace_bytes=ws)
        if target:
            layer.cache.tune(target)
        for (_, kk, vv) in hist_chunks:
            layer.append(kk, vv, layer.cache.len())
        got = layer.step(q, k, v, C)
        check_close(got, want, MAX_ABS, MEAN_ABS, "workspace %d target %d" % (ws, target))
        if ws == 0:
            assert layer.cache.last_plan()[1] == 1


def same_pools(a, b, tables, lengths):
    """The tokens of every sequence sit in both layers' pools with the same bits (the layers may
    use different pages for them), and so do the zero-filled slots up to the end of the last
    page; position tags agree."""
    from harness import PAGE
    ka, va, ta = a.pools_host()
    kb, vb, tb = b.pools_host()
    for s, n in enumerate(lengths):
        for pg in range(-(-n // PAGE)):
            pa, pb = tables[0][s][pg], tables[1][s][pg]
            assert np.array_equal(ka[pa].view(np.uint32), kb[pb].view(np.uint32)), (s, pg)
            assert np.array_equal(va[pa].view(np.uint32), vb[pb].view(np.uint32)), (s, pg)
            used = min(PAGE, n - pg * PAGE)
            assert np.array_equal(ta[pa * PAGE:pa * PAGE + used], tb[pb * PAGE:pb * PAGE + used])


@pytest.mark.parametrize("C", [0, 1, 15, 16, 29, 31, 32, 33, 63, 64, 95, 1000, 6000])
@pytest.mark.parametrize("n", [1, 2, 4])
def test_one_call_step_equals_the_two_calls(C, n):
    """evl_step on a short chunk (one launch that appends and attends) against evl_rope_append +
    evl_chunk_attention on a twin cache: outputs bit for bit, cache contents bit for bit, and
    the oracle's result to the usual bar.  Old ends of the sequence at and around page and tile
    boundaries, an empty cache included; then a second short step on top (it reads what the
    first one appended)."""
    from harness import GpuLayer, check_close
    shape = StreamShape(14, 2, 128, 1.0e6, 0, 0, 0)
    ost = oracle.Stream(14, 2, 128, 1e6)
    two = GpuLayer(shape, [C + 2 * n], random_pages=True, out_f32=True, cfg=66)
    one = GpuLayer(shape, [C + 2 * n], random_pages=True, out_f32=True, cfg=67)     # other pages
    if C:
        _, k, v = qkv_chunk(shape, C, 66, C, 0)
        ost.append(k, v, 5)
        two.append(k, v, 5)
        one.append(k, v, 5)
    for rnd in range(2):
        q, k, v = qkv_chunk(shape, n, 66, C, 1 + rnd)
        at = C + rnd * n
        want = ost.step(q, k, v, 5 + at)
        got_two = two.step(q, k, v, 5 + at)
        before = one.cache.launches()
        got_one = one.fused_step(q, k, v, 5 + at)
        # one launch (two the first time a cache object's piece counters are cleared); while the
        # sequence is shorter than 64 tokens the rows go to the few-keys kernel: append + that kernel
        assert one.cache.launches() - before <= (2 if rnd == 0 or at + n < 64 else 1)
        assert one.cache.len() == two.cache.len() == at + n and one.cache.pos0() == 5
        assert np.array_equal(got_one, got_two), "C=%d n=%d round %d" % (C, n, rnd)
        check_close(got_one, want, MAX_ABS, MEAN_ABS, "C=%d n=%d round %d" % (C, n, rnd))
    same_pools(one, two, (one.table_np, two.table_np), [C + 2 * n])


def test_one_call_step_at_the_largest_positions():
    """The same with position ids that end at 2^31 - 2, the largest there is: the rotation of the
    keys (append part) and of the queries and patched keys (attention part) still agree."""
    from harness import GpuLayer, check_close
    shape = StreamShape(14, 2, 128, 1.0e6, 0, 0, 0)
    C, n = 40, 2
    pos0 = 2 ** 31 - 1 - (C + 2 * n)
    ost = oracle.Stream(14, 2, 128, 1e6)
    two = GpuLayer(shape, [C + 2 * n], random_pages=True, out_f32=True, cfg=68)
    one = GpuLayer(shape, [C + 2 * n], random_pages=True, out_f32=True, cfg=69)
    _, k, v = qkv_chunk(shape, C, 68, C, 0)
    ost.append(k, v, pos0)
    two.append(k, v, pos0)
    one.append(k, v, pos0)
    for rnd in range(2):
        q, k, v = qkv_chunk(shape, n, 68, C, 1 + rnd)
        at = C + rnd * n
        want = ost.step(q, k, v, pos0 + at)
        got_two = two.step(q, k, v, pos0 + at)
        got_one = one.fused_step(q, k, v, pos0 + at)
        assert np.array_equal(got_one, got_two), "round %d" % rnd
        check_close(got_one, want, MAX_ABS, MEAN_ABS, "round %d" % rnd)
    assert one.cache.pos0() == pos0 and one.cache.len() == C + 2 * n
    same_pools(one, two, (one.table_np, two.table_np), [C + 2 * n])
    with pytest.raises(Exception) as e:          # one more token would need position id 2^31 - 1
        one.cache.rope_append(0x40, 0x40, pos0 + C + 2 * n, 1)
    assert "EVL_ERR" in str(e.value)


@pytest.mark.parametrize("shape", [TINY, LAYER7B], ids=["tiny", "layer7b"])
def test_one_call_step_on_a_ragged_batch(shape):
    """Several sequences, short chunks, one call; then a call whose chunks are too long for the
    one-launch form, which must behave the same (it takes the two launches)."""
    from harness import GpuLayer, check_close
    per_row = 32 // shape.group
    lens = [0, 7, 333, 2500, 9000]
    ns = [min(per_row, x) for x in (1, 4, 2, 16, 3)]
    long_ns = [40, 3, 70, 1, 300]
    caps = [c + m + l for c, m, l in zip(lens, ns, long_ns)]
    one = GpuLayer(shape, caps, random_pages=True, out_f32=True, cfg=68)
    two = GpuLayer(shape, caps, random_pages=True, out_f32=True, cfg=69)
    osts = [oracle.Stream(shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rope_base) for _ in lens]
    for s, C in enumerate(lens):
        done = 0
        while done < C:
            m = min(3000, C - done)
            _, k, v = qkv_chunk(shape, m, 68, s, done)
            osts[s].append(k, v, 10 + done)
            one.append_batched([k], [v], [s], [10 + done])
            two.append_batched([k], [v], [s], [10 + done])
            done += m
    ids = list(range(len(lens)))
    cur = list(lens)
    for rnd, sizes in enumerate((ns, long_ns)):
        chunks = [qkv_chunk(shape, m, 68, s, 99990 + rnd) for s, m in enumerate(sizes)]
        qs, ks, vs = ([c[i] for c in chunks] for i in range(3))
        pos = [10 + c for c in cur]
        before = one.cache.launches()
        got_one = one.fused_step_batched(qs, ks, vs, ids, pos)
        took = one.cache.launches() - before
        # short chunks: one launch (+ counter fill) -- but two of these sequences are still shorter than
        # 64 tokens, whose rows go to the few-keys kernel: append, that kernel, the rest (+ counter fill)
        assert took <= 4 if rnd == 0 else took >= 2, took
        two.append_batched(ks, vs, ids, pos)
        got_two = two.attend_batched(qs, ids, cur)
        for s in ids:
            want = osts[s].step(*chunks[s], 10 + cur[s])
            assert np.array_equal(got_one[s], got_two[s]), "round %d sequence %d" % (rnd, s)
            check_close(got_one[s], want, MAX_ABS, MEAN_ABS, "round %d sequence %d" % (rnd, s))
        cur = [c + m for c, m in zip(cur, sizes)]
        assert [one.cache.len(s) for s in ids] == cur == [two.cache.len(s) for s in ids]
    same_pools(one, two, (one.table_np, two.table_np), cur)


@pytest.mark.parametrize("n", [1, 3, 40])
def test_one_call_step_over_a_sampled_history(n):
    """evl_step_sampled against evl_rope_append + evl_chunk_attention_sampled on a twin cache (bit
    for bit, outputs and cache contents) and against the oracle: action tokens over a prefix
    and a few retained frames, one run touching the chunk; n = 40 takes the two launches."""
    from harness import GpuLayer, check_close
    shape = StreamShape(28, 4, 128, 1.0e6, 100, 60, 3)
    steps = 9
    hist = [qkv_chunk(shape, m, 71, 0, s) for s, m in enumerate([100] + [63] * steps)]
    C0 = 100 + 63 * steps
    one = GpuLayer(shape, [C0 + 3 * n], random_pages=True, out_f32=True, cfg=72)
    two = GpuLayer(shape, [C0 + 3 * n], random_pages=True, out_f32=True, cfg=73)
    for (_, k, v) in hist:
        one.append(k, v, 9 + one.cache.len())
        two.append(k, v, 9 + two.cache.len())
    kh = np.concatenate([c[1] for c in hist], axis=0)
    vh = np.concatenate([c[2] for c in hist], axis=0)
    runs0 = [(0, 100)] + [(100 + f * 63, 60) for f in (1, 4, 5)] + [(C0 - 63, 63)]
    for rnd in range(3):
        C = C0 + rnd * n
        q, k, v = qkv_chunk(shape, n, 71, 1, rnd)
        runs = runs0 if rnd == 0 else runs0[:-1] + [(C0 - 63, 63 + rnd * n)]     # earlier action tokens stay
        want = oracle.sampled_reuse(q, k, v, kh, vh, runs, 9, shape.rope_base)
        two.append(k, v, 9 + C)
        got_two = two.attend_sampled(q, runs, C)
        before = one.cache.launches()
        got_one = one.fused_step_sampled(q, k, v, runs, 9 + C)
        took = one.cache.launches() - before
        assert (took <= 2) if n <= 4 else (took >= 2), took
        assert np.array_equal(got_one, got_two), "round %d" % rnd
        check_close(got_one, want, MAX_ABS, MEAN_ABS, "n=%d round %d" % (n, rnd))
        kh = np.concatenate([kh, k], axis=0)
        vh = np.concatenate([vh, v], axis=0)
    same_pools(one, two, (one.table_np, two.table_np), [C0 + 3 * n])

"""GPU parity of the batched sampled-history call and of the packed attention under the
action-isolating mask (paper Sec. 3.3) that is built on it.  Same bar as everywhere."""
import numpy as np
import pytest
import torch

import oracle
from synth import LAYER7B, StreamShape, qkv_chunk, episode_chunk_lengths

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 1e-2, 1e-3


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2512_10310_amd as evl
    evl.load()


def test_ragged_batch_of_sampled_episodes():
    """Three episodes of different lengths, each with its own sampler's choice, plus a second
    group on one of them, in one call; every group against the oracle's gather-and-rotate."""
    import paper_2512_10310_amd as evl
    from harness import GpuLayer, check_close, dev_bf16, host_f32
    shape = StreamShape(28, 4, 128, 1e6, 40, 50, 3)
    steps = [30, 9, 18]
    eps = [[qkv_chunk(shape, m, 80 + s, 0, i) for i, m in enumerate(episode_chunk_lengths(shape, st))]
           for s, st in enumerate(steps)]
    layer = GpuLayer(shape, [40 + st * 53 for st in steps], random_pages=True, out_f32=True)
    for s, ep in enumerate(eps):
        for (q, k, v) in ep:
            layer.append_batched([k], [v], [s], [100 * s + layer.cache.len(s)])
    groups = []   # (seq, cache_len, n_new, runs)
    for s, st in enumerate(steps):
        C = 40 + (st - 1) * 53
        frames = evl.sample_uniform(st - 1, 6) if s != 1 else evl.sample_window(st - 1, 4, 2)
        groups.append((s, C, 53, [(0, 40)] + [(40 + f * 53, 50) for f in frames]))
    groups.append((0, 40 + 10 * 53, 53, [(0, 40), (40 + 2 * 53, 53), (40 + 9 * 53, 53)]))   # an earlier step of episode 0
    qs = [eps[s][(C - 40) // 53 + 1][0] for (s, C, n, r) in groups]
    q_dev = dev_bf16(np.concatenate(qs, axis=0))
    out = layer.new_out(sum(g[2] for g in groups))
    layer.cache.chunk_attention_sampled_batched(q_dev, [g[0] for g in groups], [g[1] for g in groups],
                                                [g[2] for g in groups], [g[3] for g in groups], out)
    torch.cuda.synchronize()
    got = host_f32(out)
    off = 0
    for gi, (s, C, n, runs) in enumerate(groups):
        step_idx = (C - 40) // 53 + 1
        q, k, v = eps[s][step_idx]
        kh = np.concatenate([c[1] for c in eps[s][:step_idx]], axis=0)
        vh = np.concatenate([c[2] for c in eps[s][:step_idx]], axis=0)
        want = oracle.sampled_reuse(q, k, v, kh, vh, runs, 100 * s, shape.rope_base)
        check_close(got[off:off + n], want, MAX_ABS, MEAN_ABS, "group %d" % gi)
        off += n


def pack_inputs(shape, prefix, F, A, N, cfg):
    L = prefix + N * (F + A)
    return qkv_chunk(shape, L, cfg, 0, 0)


@pytest.mark.parametrize("dims", [(20, 30, 5, 6), (0, 17, 2, 5), (33, 16, 0, 4), (7, 40, 9, 1)])
def test_isolated_pack_small(dims):
    """Packs with and without instruction prefix / action tokens, a single step; G = 7, d = 128."""
    from harness import GpuLayer, check_close, dev_bf16, host_f32
    prefix, F, A, N = dims
    shape = StreamShape(28, 4, 128, 1e6, prefix, F, A)
    q, k, v = pack_inputs(shape, prefix, F, A, N, 81)
    L = q.shape[0]
    layer = GpuLayer(shape, [L], random_pages=True, out_f32=True)
    layer.append(k, v, 5)
    out = layer.new_out(L)
    layer.cache.isolated_pack_attention(dev_bf16(q), prefix, F, A, N, out)
    torch.cuda.synchronize()
    want = oracle.isolated_pack(q, k, v, prefix, F, A, N, 5, shape.rope_base)
    check_close(host_f32(out), want, MAX_ABS, MEAN_ABS, "pack %s" % (dims,))


def test_isolated_pack_paper_size():
    """Prefix 256, 16 frames of 196 + 8 tokens (3520 tokens), 28 / 4 heads, d = 128: all rows on the
    fp32 output; with bf16 output all rows but the first 32 instruction tokens, which see only a
    handful of keys and have O(1) outputs, where bf16 output rounding alone comes close to the bar."""
    from harness import GpuLayer, check_close, dev_bf16, host_f32
    shape = LAYER7B
    N = 16
    q, k, v = pack_inputs(shape, shape.prefix, shape.frame_tokens, shape.action_tokens, N, 82)
    L = q.shape[0]
    want = oracle.isolated_pack(q, k, v, shape.prefix, shape.frame_tokens, shape.action_tokens, N, 0, shape.rope_base)
    for out_f32 in (True, False):
        layer = GpuLayer(shape, [L], random_pages=True, out_f32=out_f32)
        layer.append(k, v, 0)
        out = layer.new_out(L)
        layer.cache.isolated_pack_attention(dev_bf16(q), shape.prefix, shape.frame_tokens, shape.action_tokens, N, out)
        torch.cuda.synchronize()
        got = host_f32(out)
        head = 0 if out_f32 else 32
        check_close(got[head:], want[head:], MAX_ABS, MEAN_ABS, "pack, out_f32=%s" % out_f32)
        assert np.all(np.isfinite(got))
    print("plan:", layer.cache.last_plan())


@pytest.mark.parametrize("dims,heads,pos0", [
    ((256, 196, 8, 16), (28, 4, 128), 0),        # the paper's pack
    ((63, 60, 4, 9), (28, 4, 128), 11),          # the smallest served shape: steps of 64 tokens, instruction of 63
    ((100, 64, 1, 5), (6, 2, 64), 50000),        # one action token per step, d = 64, G = 3
    ((300, 70, 30, 7), (8, 8, 128), 3),          # long action chunks, G = 1: a tile meets two holes
])
def test_isolated_pack_appended_with_its_own_ids(dims, heads, pos0):
    """evl_isolated_pack_append (keys rotated at the ids the mask implies) followed by
    evl_isolated_pack_attention, which then is one causal launch with the earlier steps' action
    tokens as holes: against the oracle's dense-mask definition on all rows, against the route
    through evl_rope_append (per-run query shifts) to rounding, and again for fewer frames than
    were appended.  The stored keys carry the pack's ids: checked on the cache contents."""
    import paper_2512_10310_amd as evl
    from harness import GpuLayer, check_close, dev_bf16, host_f32, PAGE
    prefix, F, A, N = dims
    Hq, Hkv, d = heads
    shape = StreamShape(Hq, Hkv, d, 1e6, prefix, F, A)
    q, k, v = pack_inputs(shape, prefix, F, A, N, 83)
    L = q.shape[0]
    want = oracle.isolated_pack(q, k, v, prefix, F, A, N, pos0, shape.rope_base)
    packed = GpuLayer(shape, [L], random_pages=True, out_f32=True, cfg=84)
    plain = GpuLayer(shape, [L], random_pages=True, out_f32=True, cfg=85)
    packed.cache.isolated_pack_append(dev_bf16(k), dev_bf16(v), pos0, prefix, F, A, N)
    plain.append(k, v, pos0)
    assert packed.cache.len() == L and packed.cache.pos0() == pos0
    qd = dev_bf16(q)
    out_a, out_b = packed.new_out(L), plain.new_out(L)
    before = packed.cache.launches()
    packed.cache.isolated_pack_attention(qd, prefix, F, A, N, out_a)
    took = packed.cache.launches() - before
    plain.cache.isolated_pack_attention(qd, prefix, F, A, N, out_b)
    torch.cuda.synchronize()
    got_a, got_b = host_f32(out_a), host_f32(out_b)
    print("pack %s: %d launches, plan %s" % (dims, took, packed.cache.last_plan()))
    check_close(got_a, want, MAX_ABS, MEAN_ABS, "pack ids %s" % (dims,))
    check_close(got_a, got_b, MAX_ABS, MEAN_ABS, "pack ids against the shifted-query route %s" % (dims,))
    assert took <= 2        # attention (+ merge of the pieces, if the key range was cut)
    # position tags: instruction and visual tokens numbered without a gap, action tokens behind their frame
    _, _, tags = packed.pools_host()
    for t in sorted({0, prefix - 1, prefix, prefix + F - 1, prefix + F, prefix + F + A - 1, prefix + F + A, L - 1}):
        s = 0 if t < prefix else (t - prefix) // (F + A)
        assert tags[oracle.slot(packed.table_np[0], PAGE, t)] == pos0 + t - A * s, t
    # fewer frames of the same pack
    M = N // 2
    Lm = prefix + M * (F + A)
    out_m = packed.new_out(Lm)
    packed.cache.isolated_pack_attention(qd, prefix, F, A, M, out_m)
    torch.cuda.synchronize()
    check_close(host_f32(out_m), want[:Lm], MAX_ABS, MEAN_ABS, "pack ids, %d of %d frames" % (M, N))
    # a sequence that holds a pack takes nothing else until it is reset
    with pytest.raises(evl.EvlError) as e:
        packed.cache.rope_append(dev_bf16(k[:1]), dev_bf16(v[:1]), pos0 + L, 1)
    assert e.value.status == "EVL_ERR_NONCONTIGUOUS"
    with pytest.raises(evl.EvlError) as e:
        packed.cache.chunk_attention(qd, 0, 4, out_a)
    assert e.value.status == "EVL_ERR_ARG"
    packed.cache.reset()
    assert packed.cache.len() == 0


def random_pack(seed):
    """A served pack shape drawn from the seed: instruction of 63..400 tokens, steps of 64..300 tokens
    (half of them under 100) with 1..48 action tokens among them, 1..10 steps, one of five head shapes, any start position."""
    rng = np.random.default_rng(8300 + seed)
    Hq, Hkv, d = [(28, 4, 128), (8, 8, 128), (6, 2, 64), (16, 2, 128), (12, 4, 64)][int(rng.integers(5))]
    prefix = int(rng.integers(63, 401))
    step = int(rng.integers(64, 301)) if rng.integers(2) else int(rng.integers(64, 100))   # short steps: two holes in a tile
    A = int(rng.integers(1, min(48, step - 1) + 1))
    F = step - A
    N = int(rng.integers(1, 11))
    pos0 = int(rng.integers(0, 60000))
    return (prefix, F, A, N), (Hq, Hkv, d), pos0


@pytest.mark.parametrize("seed", range(10))
def test_isolated_pack_with_its_own_ids_random_shapes(seed):
    """Seeded shapes of the one-launch pack route (holes at every alignment to the 64-key tiles, one or
    two holes per tile, packs that end inside a tile) against the oracle's dense-mask definition."""
    from harness import GpuLayer, check_close, dev_bf16, host_f32
    (prefix, F, A, N), (Hq, Hkv, d), pos0 = random_pack(seed)
    shape = StreamShape(Hq, Hkv, d, 1e6, prefix, F, A)
    q, k, v = pack_inputs(shape, prefix, F, A, N, 8300 + seed)
    L = q.shape[0]
    print("seed %d: prefix %d, %d steps of %d + %d tokens, heads %s, pos0 %d" % (seed, prefix, N, F, A, (Hq, Hkv, d), pos0),
          flush=True)
    want = oracle.isolated_pack(q, k, v, prefix, F, A, N, pos0, shape.rope_base)
    layer = GpuLayer(shape, [L], random_pages=True, out_f32=True, cfg=8400 + seed)
    layer.cache.isolated_pack_append(dev_bf16(k), dev_bf16(v), pos0, prefix, F, A, N)
    out = layer.new_out(L)
    layer.cache.isolated_pack_attention(dev_bf16(q), prefix, F, A, N, out)
    torch.cuda.synchronize()
    check_close(host_f32(out), want, MAX_ABS, MEAN_ABS, "random pack, seed %d" % seed)


def test_isolated_pack_append_refuses_what_it_does_not_serve():
    import paper_2512_10310_amd as evl
    from harness import GpuLayer
    shape = LAYER7B
    layer = GpuLayer(shape, [4000], out_f32=True)
    for args in ((10, 196, 8, 2), (256, 40, 8, 2), (256, 196, 0, 2)):     # short instruction, short steps, no action tokens
        with pytest.raises(evl.EvlError) as e:
            layer.cache.isolated_pack_append(0x1000, 0x1000, 0, *args)
        assert e.value.status == "EVL_ERR_UNSUPPORTED", args
    assert layer.cache.len() == 0 and layer.cache.launches() == 0

"""The entry point that allocates nothing (evl_chunk_attention_static: partial results and ticket
counters in the library's static device array) against evl_chunk_attention on a caller-provided
workspace: same bar as every parity test (max |diff| <= 1e-2, mean |diff| <= 1e-3), and both
against the CPU oracle.  Two calls in a row share the array, the second with a smaller input; a
third goes through the kernel for chunks of a few tokens, which also keeps its ticket counters
there."""
import numpy as np
import pytest
import torch

import oracle
from synth import LAYER7B, qkv_chunk

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 1e-2, 1e-3


def test_static_scratch_entry_point_matches_the_workspace_one():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2512_10310_amd as evl
    evl.load()
    from harness import GpuLayer, check_close, dev_bf16, host_f32
    shape = LAYER7B
    C, n_big, n_small, n_tiny = 1500, 204, 70, 2
    total = C + n_big + n_small + n_tiny
    # a cache WITHOUT a workspace next to one with: the static call must not need the first's
    bare = GpuLayer(shape, [total], random_pages=True, out_f32=True, workspace_bytes=0)
    full = GpuLayer(shape, [total], random_pages=True, out_f32=True)
    ost = oracle.Stream(shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.rope_base)
    _, k0, v0 = qkv_chunk(shape, C, 7, 0, 0)
    for layer in (bare, full):
        layer.append(k0, v0, 0)
    ost.append(k0, v0, 0)
    for step, n in enumerate((n_big, n_small, n_tiny), start=1):
        q, k, v = qkv_chunk(shape, n, 7, 0, step)
        before = len(ost)
        want = ost.step(q, k, v, before)
        for layer in (bare, full):
            layer.append(k, v, before)
        qd = dev_bf16(q)
        out_static, out_ws = bare.new_out(n), full.new_out(n)
        print("static call: %d cached + %d new" % (before, n), flush=True)
        bare.cache.chunk_attention_static(qd, before, n, out_static)
        full.cache.chunk_attention(qd, before, n, out_ws)
        torch.cuda.synchronize()
        got_static, got_ws = host_f32(out_static), host_f32(out_ws)
        check_close(got_static, got_ws, MAX_ABS, MEAN_ABS, "static vs workspace, n=%d" % n)
        check_close(got_static, want, MAX_ABS, MEAN_ABS, "static vs oracle, n=%d" % n)
        if step < 3:
            # the key range was really cut into pieces: the array was in use
            assert bare.cache.last_plan()[1] > 1, bare.cache.last_plan()
            assert bare.cache.last_plan()[2] <= (16 << 20)
    # the size limit is refused with a clear error, and nothing is launched
    launches = bare.cache.launches()
    too_many = 8192 // shape.n_q_heads + 1
    with pytest.raises(evl.EvlError) as err:
        bare.cache.chunk_attention_static(dev_bf16(np.zeros((too_many, shape.n_q_heads, shape.head_dim), np.float32)),
                                          0, too_many, bare.new_out(too_many))
    assert err.value.status == "EVL_ERR_WORKSPACE" and "8192" in str(err.value)
    assert bare.cache.launches() == launches

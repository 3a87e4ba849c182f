"""GPU parity along a full streaming episode (256-token prefix, then 100 steps of 196 frame +
8 action tokens; the cache grows to 20 656 tokens): integer bookkeeping at every step, outputs
against the oracle at sampled steps."""
import numpy as np
import pytest
import torch

import oracle
from synth import LAYER7B, qkv_chunk, episode_chunk_lengths

pytestmark = pytest.mark.gpu
MAX_ABS, MEAN_ABS = 1e-2, 1e-3


@pytest.mark.parametrize("layer_id", [0, 13, 27])
def test_episode_100_steps(layer_id):
    assert torch.cuda.is_available()
    from harness import GpuLayer, check_close, PAGE
    shape = LAYER7B
    lengths = episode_chunk_lengths(shape, 100)
    total = sum(lengths)
    assert total == 20656
    layer = GpuLayer(shape, [total], random_pages=True, out_f32=False, cfg=2, workspace_bytes=128 << 20)
    ost = oracle.Stream(28, 4, 128, 1e6)
    checked = {0, 1, 25, 50, 75, 100}
    rng = np.random.default_rng(layer_id)
    want_len = 0
    for s, n in enumerate(lengths):
        q, k, v = qkv_chunk(shape, n, 2, layer_id, s)
        before = layer.cache.len()
        assert before == want_len == len(ost)
        if s in checked:
            got = layer.step(q, k, v, before)
            ost.append(k, v, before)
            # first and last token, the tokens around which the packed rows (7 heads per token) cross a
            # 256-row tile of the kernel (36.57 tokens per tile), and six seeded ones
            rows = sorted(set([0, n - 1] + [t for t in (36, 73, 109, 146, 182) if t < n] + rng.integers(0, n, 6).tolist()))
            want = ost.attend(q, before, rows=rows)
            check_close(got[rows], want, MAX_ABS, MEAN_ABS, "layer %d step %d" % (layer_id, s))
            assert np.all(np.isfinite(got))
        else:
            layer.append(k, v, before)
            ost.append(k, v, before)
        want_len += n
    assert layer.cache.len() == 20656 and layer.cache.pos0() == 0
    # position tags: exactly contiguous over the whole episode, at the oracle's slots
    _, _, tags = layer.pools_host()
    slots = np.array([oracle.slot(layer.table_np[0], PAGE, t) for t in range(0, total, 97)] +
                     [oracle.slot(layer.table_np[0], PAGE, total - 1)])
    ts = np.array(list(range(0, total, 97)) + [total - 1])
    assert np.array_equal(tags[slots], ts.astype(np.int32))
    assert np.array_equal(np.sort(tags[tags >= 0]), np.arange(total, dtype=np.int32))

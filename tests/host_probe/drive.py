"""Drives the library's host side through seeded random episodes against the checking launchers
of launch_probe.cpp (no GPU, no device memory: every pointer is a made-up address that nothing
dereferences).  Run as a script by tests/test_host_plan_cpu.py:

    python tests/host_probe/drive.py <probe library> <first seed> <number of seeds>
    python tests/host_probe/drive.py <probe library> plans

Prints one line per seed; exits non-zero at the first call that is refused, at the first launch
whose kernel arguments break what the kernels assume, or when the library's bookkeeping differs
from the model kept here."""
import ctypes as C
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from paper_2512_10310_amd import binding  # noqa: E402

Q, K, V, OUT = 0x10000000, 0x20000000, 0x30000000, 0x40000000
KPOOL, VPOOL, TABLE, WS = 0x100000000, 0x200000000, 0x300000000, 0x400000000
KINDS = ["append", "attention", "decode", "combine", "zero_counters", "pages_copy", "few_keys"]


def main(path, seed0, n_seeds):
    probe = binding.declare(C.CDLL(path))
    probe.evl_probe_message.restype = C.c_char_p
    probe.evl_probe_count.restype = C.c_int64
    probe.evl_probe_pending.restype = C.c_int64
    binding._lib = probe              # this process only ever sees the probe
    totals = np.zeros(len(KINDS), dtype=np.int64)
    for seed in range(seed0, seed0 + n_seeds):
        totals += episode(probe, seed)
    print("launches checked:", ", ".join("%s %d" % kv for kv in zip(KINDS, totals)), flush=True)
    # every kind of launch the episodes can reach was reached
    assert all(totals[:5] > 0) and totals[6] > 0, totals
    return 0


def random_runs(rng, limit, max_runs):
    n = int(rng.integers(0, max_runs + 1))
    n = min(n, limit // 2)
    if n == 0:
        return []
    cuts = np.sort(rng.choice(np.arange(0, limit + 1), size=2 * n, replace=False))
    return [(int(cuts[2 * i]), int(cuts[2 * i + 1] - cuts[2 * i])) for i in range(n)]


def episode(probe, seed):
    rng = np.random.default_rng([20251212, seed])
    group = int(rng.choice([1, 2, 4, 7, 8]))
    n_kv = int(rng.choice([1, 2, 4, 8]))
    d = int(rng.choice([64, 128]))
    n_q = group * n_kv
    max_seqs = int(rng.choice([1, 2, 5, 70]))
    cap_tokens = int(rng.choice([400, 5000, 70000]))
    pages_per_seq = (cap_tokens + 15) // 16
    out_f32 = bool(rng.integers(0, 2))
    max_chunk = int(rng.choice([8, 300, 3600]))
    ws_kind = int(rng.integers(0, 4))       # none / a sliver / the documented size / plenty
    ws_need = max(binding.workspace_bytes(n_q, d, max_chunk, max_seqs),
                  binding.workspace_bytes_sampled(n_q, d, max_chunk, 200))
    ws_bytes = [0, 1 << 16, ws_need, 4 * ws_need][ws_kind]
    probe.evl_probe_reset(max_seqs)
    c = binding.Cache(n_q, n_kv, d, float(rng.choice([1e4, 1e6])), KPOOL, VPOOL, TABLE,
                      n_pages=max_seqs * pages_per_seq, max_pages_per_seq=pages_per_seq, max_seqs=max_seqs,
                      workspace=WS if ws_bytes else None, workspace_bytes=ws_bytes,
                      out_dtype=binding.EVL_OUT_F32 if out_f32 else binding.EVL_OUT_BF16)
    if rng.integers(0, 3) == 0:
        c.tune(int(rng.choice([8, 64, 1024])))
    lens = [0] * max_seqs
    pos0 = [None] * max_seqs
    what = "seed %d: %dq/%dkv d=%d, %d sequences of up to %d tokens, workspace %d, out %s" % (
        seed, n_q, n_kv, d, max_seqs, cap_tokens, ws_bytes, "f32" if out_f32 else "bf16")

    def chunk_len():
        return int(rng.choice([1, 2, 3, 4, 17, 64, 204, max_chunk]))

    def next_pos(s):
        if pos0[s] is None:
            pos0[s] = int(rng.choice([0, 1, 1000, 60000]))
        return pos0[s] + lens[s]

    def some_seqs(need_history):
        ok = [s for s in range(max_seqs) if (lens[s] > 0 or not need_history)]
        if not ok:
            return []
        k = int(rng.integers(1, min(len(ok), 66) + 1))
        return [int(s) for s in rng.choice(ok, size=k, replace=False)]

    def room(s, n):
        return lens[s] + n <= cap_tokens

    def call(name, fn, may_lack_workspace=False):
        try:
            fn()
        except binding.EvlError as e:
            msg = probe.evl_probe_message().decode()
            if e.status == "EVL_ERR_WORKSPACE" and may_lack_workspace and ws_kind < 2 and not msg:
                return False
            raise AssertionError("%s\n  %s refused: %s\n  probe: %s" % (what, name, e, msg or "-"))
        msg = probe.evl_probe_message().decode()
        assert not msg, "%s\n  %s: %s" % (what, name, msg)
        assert probe.evl_probe_pending() == 0, "%s\n  %s left partial results unmerged" % (what, name)
        return True

    for op_no in range(60):
        op = int(rng.integers(0, 12)) if op_no > 2 else 0
        if op == 0:                                   # append to some sequences
            ss = [s for s in some_seqs(False)]
            ns = [chunk_len() for _ in ss]
            keep = [(s, n) for s, n in zip(ss, ns) if room(s, n)]
            if not keep:
                continue
            ss, ns = [s for s, _ in keep], [n for _, n in keep]
            ps = [next_pos(s) for s in ss]
            if len(ss) == 1 and ss[0] == 0 and rng.integers(0, 2):
                call("rope_append", lambda: c.rope_append(K, V, ps[0], ns[0]))
            else:
                call("rope_append_batched", lambda: c.rope_append_batched(K, V, ss, ps, ns))
            for s, n in zip(ss, ns):
                lens[s] += n
        elif op in (1, 2):                            # attend some chunks that were appended
            ss = some_seqs(True)
            if not ss:
                continue
            ns = [int(rng.integers(1, min(lens[s], max_chunk) + 1)) if rng.integers(0, 2) else min(lens[s], chunk_len())
                  for s in ss]
            cl = [lens[s] - n if rng.integers(0, 4) else int(rng.integers(0, lens[s] - n + 1)) for s, n in zip(ss, ns)]
            if len(ss) == 1 and ss[0] == 0 and rng.integers(0, 2):
                call("chunk_attention", lambda: c.chunk_attention(Q, cl[0], ns[0], OUT))
            else:
                call("chunk_attention_batched", lambda: c.chunk_attention_batched(Q, ss, cl, ns, OUT))
        elif op in (3, 4):                            # one chunk over retained runs of its history
            ss = some_seqs(True)
            if not ss:
                continue
            s = ss[0]
            n = min(lens[s], chunk_len())
            cache_len = lens[s] - n
            runs = random_runs(rng, cache_len, int(rng.choice([3, 17, 70, 200])))
            call("chunk_attention_sampled (%d runs)" % len(runs),
                 lambda: c.chunk_attention_sampled(Q, runs, cache_len, n, OUT, seq=s), may_lack_workspace=len(runs) >= 64)
        elif op == 5:                                 # several such groups in one call
            ss = some_seqs(True)
            if not ss:
                continue
            groups = [int(s) for s in rng.choice(ss, size=int(rng.integers(1, 40)))]
            ns = [min(lens[s], chunk_len()) for s in groups]
            cl = [lens[s] - n for s, n in zip(groups, ns)]
            runs = [random_runs(rng, x, int(rng.choice([2, 9, 30]))) for x in cl]
            toks = list(np.cumsum([0] + ns[:-1]) * 8) if rng.integers(0, 2) else None
            call("chunk_attention_sampled_batched (%d groups)" % len(groups),
                 lambda: c.chunk_attention_sampled_batched(Q, groups, cl, ns, runs, OUT, tok_offs=toks))
        elif op == 6:                                 # a pack under the action-isolating mask
            ss = some_seqs(True)
            if not ss:
                continue
            s = ss[0]
            ft, at = int(rng.choice([4, 16, 196])), int(rng.choice([0, 2, 8]))
            prefix = int(rng.choice([0, 7, 32, 256]))
            if prefix > lens[s]:
                prefix = 0
            frames = min((lens[s] - prefix) // (ft + at), int(rng.integers(0, 20)))
            if prefix == 0 and frames == 0:
                continue
            call("isolated_pack_attention (%d + %d x (%d + %d))" % (prefix, frames, ft, at),
                 lambda: c.isolated_pack_attention(Q, prefix, ft, at, frames, OUT, seq=s))
            # the same pack appended with its own position ids: one causal launch with holes
            if prefix >= 63 and ft + at >= 64 and at >= 1 and frames >= 1 and rng.integers(0, 2):
                free = [x for x in range(max_seqs) if lens[x] == 0]
                total = prefix + frames * (ft + at)
                if free and total <= cap_tokens:
                    x = free[0]
                    p0 = int(rng.choice([0, 5, 40000]))
                    call("isolated_pack_append", lambda: c.isolated_pack_append(K, V, p0, prefix, ft, at, frames, seq=x))
                    lens[x], pos0[x] = total, p0
                    fewer = int(rng.integers(0, frames + 1))
                    call("isolated_pack_attention on a pack (%d of %d frames)" % (fewer, frames),
                         lambda: c.isolated_pack_attention(Q, prefix, ft, at, fewer, OUT, seq=x))
                    call("reset", lambda: c.reset(x))
                    lens[x], pos0[x] = 0, None
        elif op in (7, 8):                            # append and attend in one call
            ss = some_seqs(False)
            short = bool(rng.integers(0, 2))
            ns = [int(rng.integers(1, 5)) if short else chunk_len() for _ in ss]
            keep = [(s, n) for s, n in zip(ss, ns) if room(s, n)]
            if not keep:
                continue
            ss, ns = [s for s, _ in keep], [n for _, n in keep]
            ps = [next_pos(s) for s in ss]
            if len(ss) == 1 and ss[0] == 0 and rng.integers(0, 2):
                call("step", lambda: c.step(Q, K, V, ps[0], ns[0], OUT))
            else:
                call("step_batched", lambda: c.step_batched(Q, K, V, ss, ps, ns, OUT))
            for s, n in zip(ss, ns):
                lens[s] += n
        elif op == 9:                                 # the same over retained runs
            s = int(rng.integers(0, max_seqs))
            n = int(rng.integers(1, 5)) if rng.integers(0, 2) else chunk_len()
            if not room(s, n):
                continue
            runs = random_runs(rng, lens[s], int(rng.choice([3, 17, 70, 200])))
            p = next_pos(s)
            if call("step_sampled (%d runs)" % len(runs),
                    lambda: c.step_sampled(Q, K, V, runs, p, n, OUT, seq=s), may_lack_workspace=len(runs) >= 64):
                lens[s] += n
        elif op == 10:                                # roll a sequence back
            s = int(rng.integers(0, max_seqs))
            if lens[s] == 0:
                continue
            new_len = int(rng.integers(0, lens[s] + 1))
            call("truncate", lambda: c.truncate(new_len, seq=s))
            lens[s] = new_len
            if new_len == 0 and rng.integers(0, 2):
                call("reset", lambda: c.reset(s))
                pos0[s] = None
        else:                                         # start a sequence over
            s = int(rng.integers(0, max_seqs))
            call("reset", lambda: c.reset(s))
            lens[s], pos0[s] = 0, None
        for s in range(max_seqs):
            assert c.len(s) == lens[s], "%s\n  sequence %d: library length %d, model %d" % (what, s, c.len(s), lens[s])
            if lens[s] > 0:
                assert c.pos0(s) == pos0[s], "%s\n  sequence %d: pos0 %d, model %s" % (what, s, c.pos0(s), pos0[s])
    counts = np.array([probe.evl_probe_count(k) for k in range(len(KINDS))], dtype=np.int64)
    assert c.launches() == counts.sum(), "%s\n  library counted %d launches, probe saw %s" % (what, c.launches(), counts)
    print(what, "->", counts.sum(), "launches", flush=True)
    c.close()
    return counts


def plans(path):
    """Prints the planner's choice (work-groups, pieces) for a few single-sequence launches of the
    7B-class layer shape: "<cached tokens> <new tokens> <work-groups> <pieces>" per line."""
    probe = binding.declare(C.CDLL(path))
    probe.evl_probe_message.restype = C.c_char_p
    binding._lib = probe
    probe.evl_probe_reset(1)
    for cached, new in ((6580, 204), (20452, 204), (65536, 204), (0, 3520), (0, 256), (5000, 1000), (60000, 500),
                        (20000, 4000), (3316, 204), (6580, 40), (60000, 100)):
        pages = (cached + new + 15) // 16
        c = binding.Cache(28, 4, 128, 1e6, KPOOL, VPOOL, TABLE, n_pages=pages, max_pages_per_seq=pages,
                          workspace=WS, workspace_bytes=1 << 30)
        c.rope_append(K, V, 0, cached + new)
        c.chunk_attention(Q, cached, new, OUT)
        assert not probe.evl_probe_message(), probe.evl_probe_message()
        wg, pieces, _ = c.last_plan()
        print(cached, new, wg, pieces, flush=True)
        c.close()
    return 0


if __name__ == "__main__":
    if sys.argv[2] == "plans":
        sys.exit(plans(sys.argv[1]))
    sys.exit(main(sys.argv[1], int(sys.argv[2]), int(sys.argv[3])))

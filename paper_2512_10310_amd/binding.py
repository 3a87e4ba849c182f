"""ctypes binding of the C ABI in include/evl.h.  Same names, same arguments; this module
marshals pointers and sizes and does no arithmetic of the method.  PyTorch tensors are used
only as device-memory handles (data_ptr) and for the current HIP stream."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(PKG, "libevl.so")

EVL_OUT_BF16, EVL_OUT_F32 = 0, 1
PAGE_SIZE = 16

_STATUS = {0: "EVL_OK", -1: "EVL_ERR_NULL", -2: "EVL_ERR_ARG", -3: "EVL_ERR_ALIGN",
           -4: "EVL_ERR_NONCONTIGUOUS", -5: "EVL_ERR_CAPACITY", -6: "EVL_ERR_RANGE",
           -7: "EVL_ERR_UNSUPPORTED", -8: "EVL_ERR_LAUNCH", -9: "EVL_ERR_WORKSPACE"}

EXPORTS = ["evl_cache_create", "evl_cache_destroy", "evl_cache_reset", "evl_cache_truncate",
           "evl_cache_len", "evl_cache_pos0", "evl_cache_set_stream", "evl_workspace_bytes",
           "evl_last_error", "evl_rope_append", "evl_chunk_attention",
           "evl_rope_append_batched", "evl_chunk_attention_batched", "evl_last_plan",
           "evl_timing_enable", "evl_timing_read", "evl_cache_tune",
           "evl_chunk_attention_sampled", "evl_workspace_bytes_sampled", "evl_sample_uniform",
           "evl_sample_window", "evl_chunk_attention_sampled_batched", "evl_isolated_pack_attention",
           "evl_pages_copy", "evl_step", "evl_step_batched", "evl_step_sampled",
           "evl_cache_launches", "evl_chunk_attention_static", "evl_isolated_pack_append"]


def status_name(code: int) -> str:
    return _STATUS.get(int(code), "EVL_ERR_%d" % code)


class EvlError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("%s: %s" % (status_name(code), msg))
        self.code = int(code)
        self.status = status_name(code)


class Run(C.Structure):
    _fields_ = [("start", C.c_int32), ("len", C.c_int32)]


class CacheDesc(C.Structure):
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("page_size", C.c_int32), ("n_pages", C.c_int32),
                ("max_pages_per_seq", C.c_int32), ("max_seqs", C.c_int32),
                ("out_dtype", C.c_int32), ("rope_base", C.c_double),
                ("k_pool", C.c_void_p), ("v_pool", C.c_void_p), ("block_table", C.c_void_p),
                ("pos_tags", C.c_void_p), ("workspace", C.c_void_p),
                ("workspace_bytes", C.c_size_t), ("stream", C.c_void_p)]


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Load libevl.so.  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError("libevl.so is not built (run `python -c 'import __graft_entry__ as g; "
                           "g.build()'` or `python paper_2512_10310_amd/build.py`)")
    _lib = declare(C.CDLL(_LIB_PATH))
    return _lib


def declare(L):
    """Sets the argument and result types of the C ABI's functions on a loaded library."""
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    pi32, pi64 = C.POINTER(C.c_int32), C.POINTER(C.c_int64)
    L.evl_cache_create.argtypes = [C.POINTER(CacheDesc), C.POINTER(vp)]
    L.evl_cache_destroy.argtypes = [vp]
    L.evl_cache_reset.argtypes = [vp, i32]
    L.evl_cache_truncate.argtypes = [vp, i32, i32]
    L.evl_cache_len.argtypes = [vp, i32]
    L.evl_cache_pos0.argtypes = [vp, i32]
    L.evl_cache_pos0.restype = i64
    L.evl_cache_set_stream.argtypes = [vp, vp]
    L.evl_workspace_bytes.argtypes = [C.POINTER(CacheDesc), i32, i32]
    L.evl_workspace_bytes.restype = C.c_size_t
    L.evl_last_error.restype = C.c_char_p
    L.evl_rope_append.argtypes = [vp, vp, vp, i64, i32]
    L.evl_chunk_attention.argtypes = [vp, vp, i32, i32, vp]
    L.evl_chunk_attention_static.argtypes = [vp, vp, i32, i32, vp]
    L.evl_rope_append_batched.argtypes = [vp, vp, vp, pi32, pi64, pi32, i32]
    L.evl_chunk_attention_batched.argtypes = [vp, vp, pi32, pi32, pi32, i32, vp]
    L.evl_last_plan.argtypes = [vp, pi32, pi32, C.POINTER(C.c_size_t)]
    L.evl_cache_tune.argtypes = [vp, i32]
    L.evl_timing_enable.argtypes = [vp, i32]
    L.evl_timing_read.argtypes = [vp, C.POINTER(C.c_float), i32, pi32]
    L.evl_chunk_attention_sampled.argtypes = [vp, vp, i32, C.POINTER(Run), i32, i32, i32, vp]
    L.evl_chunk_attention_sampled_batched.argtypes = [vp, vp, i32, pi32, pi32, pi32, pi32, pi32,
                                                      C.POINTER(Run), vp]
    L.evl_isolated_pack_attention.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp]
    L.evl_isolated_pack_append.argtypes = [vp, i32, vp, vp, i64, i32, i32, i32, i32]
    L.evl_pages_copy.argtypes = [vp, vp, vp, pi32, i32, vp, vp, pi32, i32, i32]
    L.evl_step.argtypes = [vp, vp, vp, vp, i64, i32, vp]
    L.evl_step_sampled.argtypes = [vp, vp, vp, vp, i32, C.POINTER(Run), i32, i64, i32, vp]
    L.evl_cache_launches.argtypes = [vp]
    L.evl_cache_launches.restype = i64
    L.evl_step_batched.argtypes = [vp, vp, vp, vp, pi32, pi64, pi32, i32, vp]
    L.evl_workspace_bytes_sampled.argtypes = [C.POINTER(CacheDesc), i32, i32]
    L.evl_workspace_bytes_sampled.restype = C.c_size_t
    L.evl_sample_uniform.argtypes = [i32, i32, pi32]
    L.evl_sample_window.argtypes = [i32, i32, i32, pi32]
    for name in EXPORTS:
        fn = getattr(L, name)
        if name not in ("evl_cache_pos0", "evl_workspace_bytes", "evl_workspace_bytes_sampled",
                        "evl_last_error", "evl_cache_launches"):
            fn.restype = C.c_int32
    return L


def _check(code: int) -> None:
    if code != 0:
        raise EvlError(code, load().evl_last_error().decode())


def _ptr(x) -> Optional[int]:
    """Device (or fake) address of a tensor-like, an int, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _arr(vals: Sequence[int], ct):
    return (ct * len(vals))(*[int(v) for v in vals])


def workspace_bytes(n_q_heads: int, head_dim: int, max_n_new: int, max_seqs: int) -> int:
    d = CacheDesc(n_q_heads=n_q_heads, n_kv_heads=1, head_dim=head_dim)
    return int(load().evl_workspace_bytes(C.byref(d), max_n_new, max_seqs))


def workspace_bytes_sampled(n_q_heads: int, head_dim: int, max_n_new: int, max_runs: int) -> int:
    d = CacheDesc(n_q_heads=n_q_heads, n_kv_heads=1, head_dim=head_dim)
    return int(load().evl_workspace_bytes_sampled(C.byref(d), max_n_new, max_runs))


def sample_uniform(n_frames: int, n_keep: int):
    buf = (C.c_int32 * max(int(n_keep), 1))()
    n = load().evl_sample_uniform(int(n_frames), int(n_keep), buf)
    return [int(buf[i]) for i in range(n)]


def sample_window(n_frames: int, n_keep: int, stride: int):
    buf = (C.c_int32 * max(int(n_keep), 1))()
    n = load().evl_sample_window(int(n_frames), int(n_keep), int(stride), buf)
    return [int(buf[i]) for i in range(n)]


def make_runs(runs):
    """[(start, len), ...] -> (ctypes array of evl_run, count), accepted by chunk_attention_sampled."""
    return (Run * max(len(runs), 1))(*[Run(int(a), int(b)) for a, b in runs]), len(runs)


class Cache:
    """One layer's paged GQA KV cache: the host-side evl_cache object.  Device memory is the
    caller's (pools, block table, tags, workspace are tensors or raw addresses)."""

    def __init__(self, n_q_heads: int, n_kv_heads: int, head_dim: int, rope_base: float,
                 k_pool, v_pool, block_table, n_pages: int, max_pages_per_seq: int,
                 max_seqs: int = 1, pos_tags=None, workspace=None, workspace_bytes: int = 0,
                 out_dtype: int = EVL_OUT_BF16, stream: Optional[int] = None,
                 page_size: int = PAGE_SIZE):
        L = load()
        self._keep = (k_pool, v_pool, block_table, pos_tags, workspace)
        d = CacheDesc(n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, head_dim=head_dim,
                      page_size=page_size, n_pages=n_pages, max_pages_per_seq=max_pages_per_seq,
                      max_seqs=max_seqs, out_dtype=out_dtype, rope_base=float(rope_base),
                      k_pool=_ptr(k_pool), v_pool=_ptr(v_pool), block_table=_ptr(block_table),
                      pos_tags=_ptr(pos_tags), workspace=_ptr(workspace),
                      workspace_bytes=int(workspace_bytes), stream=stream)
        h = C.c_void_p()
        _check(L.evl_cache_create(C.byref(d), C.byref(h)))
        self._h = h

    def close(self) -> None:
        if getattr(self, "_h", None):
            load().evl_cache_destroy(self._h)
            self._h = None

    def __del__(self):
        # (at interpreter shutdown the module's globals may already be gone: the process's memory goes with them)
        if load is not None:
            self.close()

    def reset(self, seq: int = 0) -> None:
        _check(load().evl_cache_reset(self._h, seq))

    def truncate(self, new_len: int, seq: int = 0) -> None:
        _check(load().evl_cache_truncate(self._h, seq, new_len))

    def len(self, seq: int = 0) -> int:
        n = load().evl_cache_len(self._h, seq)
        if n < 0:
            _check(n)
        return n

    def pos0(self, seq: int = 0) -> int:
        return int(load().evl_cache_pos0(self._h, seq))

    def launches(self) -> int:
        return int(load().evl_cache_launches(self._h))

    def set_stream(self, stream: Optional[int]) -> None:
        _check(load().evl_cache_set_stream(self._h, stream))

    def rope_append(self, k_new, v_new, pos_offset: int, n_new: int) -> None:
        _check(load().evl_rope_append(self._h, _ptr(k_new), _ptr(v_new), int(pos_offset), int(n_new)))

    def chunk_attention(self, q_new, cache_len: int, n_new: int, out) -> None:
        _check(load().evl_chunk_attention(_ptr(q_new), self._h, int(cache_len), int(n_new), _ptr(out)))

    def chunk_attention_static(self, q_new, cache_len: int, n_new: int, out) -> None:
        _check(load().evl_chunk_attention_static(_ptr(q_new), self._h, int(cache_len), int(n_new), _ptr(out)))

    def step(self, q_new, k_new, v_new, pos_offset: int, n_new: int, out) -> None:
        _check(load().evl_step(self._h, _ptr(q_new), _ptr(k_new), _ptr(v_new), int(pos_offset), int(n_new),
                               _ptr(out)))

    def step_batched(self, q_new, k_new, v_new, seq_ids, pos_offsets, n_new, out) -> None:
        n = len(seq_ids)
        _check(load().evl_step_batched(
            self._h, _ptr(q_new), _ptr(k_new), _ptr(v_new), _arr(seq_ids, C.c_int32),
            _arr(pos_offsets, C.c_int64), _arr(n_new, C.c_int32), n, _ptr(out)))

    def rope_append_batched(self, k_new, v_new, seq_ids, pos_offsets, n_new) -> None:
        n = len(seq_ids)
        _check(load().evl_rope_append_batched(
            self._h, _ptr(k_new), _ptr(v_new), _arr(seq_ids, C.c_int32),
            _arr(pos_offsets, C.c_int64), _arr(n_new, C.c_int32), n))

    def chunk_attention_batched(self, q_new, seq_ids, cache_lens, n_new, out) -> None:
        n = len(seq_ids)
        _check(load().evl_chunk_attention_batched(
            _ptr(q_new), self._h, _arr(seq_ids, C.c_int32), _arr(cache_lens, C.c_int32),
            _arr(n_new, C.c_int32), n, _ptr(out)))

    def chunk_attention_sampled(self, q_new, runs, cache_len: int, n_new: int, out, seq: int = 0) -> None:
        """runs: [(start, len), ...] retained runs of the stored sequence, or the array that
        make_runs built from such a list (saves the conversion when the same runs are used again)."""
        arr, n = runs if isinstance(runs, tuple) and len(runs) == 2 and isinstance(runs[1], int) and \
            not isinstance(runs[0], int) else make_runs(runs)
        _check(load().evl_chunk_attention_sampled(_ptr(q_new), self._h, int(seq), arr, n,
                                                  int(cache_len), int(n_new), _ptr(out)))

    def step_sampled(self, q_new, k_new, v_new, runs, pos_offset: int, n_new: int, out, seq: int = 0) -> None:
        """runs as for chunk_attention_sampled."""
        arr, n = runs if isinstance(runs, tuple) and len(runs) == 2 and isinstance(runs[1], int) and \
            not isinstance(runs[0], int) else make_runs(runs)
        _check(load().evl_step_sampled(self._h, _ptr(q_new), _ptr(k_new), _ptr(v_new), int(seq), arr, n,
                                       int(pos_offset), int(n_new), _ptr(out)))

    def chunk_attention_sampled_batched(self, q_new, seq_ids, cache_lens, n_new, runs_per_group, out,
                                        tok_offs=None) -> None:
        """runs_per_group: one list of (start, len) per group."""
        flat = [r for g in runs_per_group for r in g]
        offs = [0]
        for g in runs_per_group:
            offs.append(offs[-1] + len(g))
        arr, _ = make_runs(flat)
        n = len(seq_ids)
        _check(load().evl_chunk_attention_sampled_batched(
            _ptr(q_new), self._h, n, _arr(seq_ids, C.c_int32), _arr(cache_lens, C.c_int32),
            _arr(n_new, C.c_int32), _arr(tok_offs, C.c_int32) if tok_offs is not None else None,
            _arr(offs, C.c_int32), arr, _ptr(out)))

    def isolated_pack_attention(self, q_packed, prefix: int, frame_tokens: int, action_tokens: int,
                                n_frames: int, out_packed, seq: int = 0) -> None:
        _check(load().evl_isolated_pack_attention(_ptr(q_packed), self._h, int(seq), int(prefix),
                                                  int(frame_tokens), int(action_tokens), int(n_frames),
                                                  _ptr(out_packed)))

    def isolated_pack_append(self, k_packed, v_packed, pos0: int, prefix: int, frame_tokens: int,
                             action_tokens: int, n_frames: int, seq: int = 0) -> None:
        _check(load().evl_isolated_pack_append(self._h, int(seq), _ptr(k_packed), _ptr(v_packed), int(pos0),
                                               int(prefix), int(frame_tokens), int(action_tokens), int(n_frames)))

    def pages_copy(self, dst_k, dst_v, dst_pages, dst_pool_pages: int, src_k, src_v, src_pages,
                   src_pool_pages: int) -> None:
        n = len(src_pages)
        assert len(dst_pages) == n
        _check(load().evl_pages_copy(self._h, _ptr(dst_k), _ptr(dst_v), _arr(dst_pages, C.c_int32),
                                     int(dst_pool_pages), _ptr(src_k), _ptr(src_v),
                                     _arr(src_pages, C.c_int32), int(src_pool_pages), n))

    def tune(self, target_workgroups: int = 0) -> None:
        _check(load().evl_cache_tune(self._h, int(target_workgroups)))

    def timing_enable(self, n_pairs: int) -> None:
        _check(load().evl_timing_enable(self._h, int(n_pairs)))

    def timing_read(self, max_n: int = 65536):
        """Elapsed milliseconds of the bracketed attention kernel launches, oldest first."""
        buf = (C.c_float * max_n)()
        n = C.c_int32()
        _check(load().evl_timing_read(self._h, buf, max_n, C.byref(n)))
        return [float(buf[i]) for i in range(n.value)]

    def last_plan(self):
        """(attention work-groups, largest split count, workspace bytes used) of the last call."""
        a, b, w = C.c_int32(), C.c_int32(), C.c_size_t()
        _check(load().evl_last_plan(self._h, C.byref(a), C.byref(b), C.byref(w)))
        return a.value, b.value, w.value

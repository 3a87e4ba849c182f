/*
 * evl.h -- C ABI of the MI355X (gfx950) library for KV-cache reuse with contiguous RoPE.
 *
 * The operation is the one the paper states in Sec. 3.2 (and draws in Fig. 1, left): at
 * every navigation step only the newly observed frame's tokens, plus that step's
 * text/action tokens, are processed.  The combined sequence "cached tokens + new chunk"
 * carries contiguous position ids; RoPE is applied at those ids; the new keys/values join a
 * per-layer KV cache; and the new chunk's queries attend over cache + chunk (causal inside
 * the chunk).  This library rotates keys when they are written, which equals rotating at
 * read time as long as no cached token is dropped or reordered.
 *
 * Conventions fixed by this library (the paper leaves them open):
 *   theta_j = rope_base^(-2j/d); element j pairs with element j + d/2 ("rotate-half");
 *   values are never rotated; query head h reads KV head h / (Hq/Hkv); scores are scaled by
 *   1/sqrt(d); chunk token i sees cached tokens 0..cache_len-1 and chunk tokens 0..i.
 *
 * Memory and execution model
 *   - Every pointer marked DEVICE is device memory owned by the caller (e.g. a PyTorch
 *     tensor).  The library never allocates or frees device memory, moves bytes only where
 *     a call says so, and never synchronises: every call only enqueues kernels on `stream`
 *     and returns (so a sequence of calls can be captured into a HIP graph).
 *   - Every pointer marked HOST is ordinary host memory, read during the call only.
 *   - Input buffers must stay alive and unchanged until the stream has run the kernels.
 *   - An evl_cache is a small HOST object (lengths and geometry of one layer's cache).  It
 *     is not thread-safe; use one thread per cache.
 *   - All functions return EVL_OK (0) or a negative evl_status, and evl_last_error() describes
 *     the problem.  Every argument is checked before anything is enqueued: a call refused for
 *     its arguments (any status but EVL_ERR_LAUNCH) has enqueued nothing and changed nothing.
 *     EVL_ERR_LAUNCH comes from the HIP runtime in mid-call: a call that takes several launches
 *     (more than 64 sequences, an attention call with its merge) may by then have enqueued
 *     some of them, and an append has recorded exactly the sequences whose launch went out.
 *   - Under HIP graph capture: calls that use the ticket counters at the end of the workspace
 *     (chunks of a few tokens, see evl_workspace_bytes) clear them with a small kernel the
 *     first time a cache object needs them.  Make that first call outside the capture (one
 *     eager call on the cache does it); otherwise the clearing is only recorded and runs with
 *     the first replay, and eager calls made before that replay would find the counters
 *     uncleared.
 *
 * Layouts (row-major, bf16 unless stated)
 *   q_new [n][Hq][d], k_new / v_new [n][Hkv][d], out [n][Hq][d]: token-major, as a QKV
 *   projection emits them; q_new and k_new arrive UNROTATED.
 *   k_pool [n_pages][Hkv][page_size][d]   rotated keys.
 *   v_pool [n_pages][Hkv][d][page_size]   values, transposed inside each page so that the
 *                                         attention kernel reads 8 consecutive keys of one
 *                                         channel as one 16-byte word.
 *   block_table [max_seqs][max_pages_per_seq] int32: entry k of row s is the pool page that
 *   holds tokens k*page_size .. (k+1)*page_size-1 of sequence s.  The caller fills the
 *   entries a sequence can reach before the first call that touches them; any page order
 *   is allowed.  Page ids outside [0, n_pages) are clamped into range by the kernels (a
 *   guard against wild accesses, not a feature).
 */
#ifndef EVL_H
#define EVL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct evl_cache evl_cache;

typedef enum {
    EVL_OK = 0,
    EVL_ERR_NULL = -1,          /* a required pointer is NULL                               */
    EVL_ERR_ARG = -2,           /* a size or count is out of its domain                     */
    EVL_ERR_ALIGN = -3,         /* a device pointer is not 16-byte aligned                  */
    EVL_ERR_NONCONTIGUOUS = -4, /* pos_offset does not continue the cached sequence         */
    EVL_ERR_CAPACITY = -5,      /* the sequence would outgrow its block-table row           */
    EVL_ERR_RANGE = -6,         /* cache_len + n_new exceeds what has been appended         */
    EVL_ERR_UNSUPPORTED = -7,   /* head shape / page size the kernels are not built for     */
    EVL_ERR_LAUNCH = -8,        /* the HIP runtime refused a launch (no device, bad stream) */
    EVL_ERR_WORKSPACE = -9      /* the workspace cannot hold the partial results that must be merged */
} evl_status;

enum { EVL_OUT_BF16 = 0, EVL_OUT_F32 = 1 };

typedef struct {
    int32_t n_q_heads;         /* Hq                                                         */
    int32_t n_kv_heads;        /* Hkv, Hq % Hkv == 0                                         */
    int32_t head_dim;          /* d, 64 or 128                                               */
    int32_t page_size;         /* tokens per page, must be 16                                */
    int32_t n_pages;           /* pages in k_pool / v_pool                                   */
    int32_t max_pages_per_seq; /* row length of block_table; a sequence holds at most
                                  max_pages_per_seq * page_size tokens                      */
    int32_t max_seqs;          /* rows of block_table                                        */
    int32_t out_dtype;         /* EVL_OUT_BF16 or EVL_OUT_F32: element type of `out`         */
    double rope_base;          /* e.g. 1e4, 1e6                                              */
    void *k_pool;              /* DEVICE bf16, 16-byte aligned                               */
    void *v_pool;              /* DEVICE bf16, 16-byte aligned                               */
    int32_t *block_table;      /* DEVICE int32                                               */
    int32_t *pos_tags;         /* DEVICE int32 [n_pages*page_size] or NULL: if given, the
                                  append kernel records each written slot's position id      */
    void *workspace;           /* DEVICE scratch for split-KV partial results, or NULL       */
    size_t workspace_bytes;    /* 0 is legal: attention then runs without splitting the keys */
    void *stream;              /* hipStream_t (NULL = the default stream)                    */
} evl_cache_desc;

/* Host-side object for one layer's cache.  Copies *desc; allocates host memory only. */
evl_status evl_cache_create(const evl_cache_desc *desc, evl_cache **out);
evl_status evl_cache_destroy(evl_cache *cache);
/* Forget sequence `seq`: length 0, first position id unset. */
evl_status evl_cache_reset(evl_cache *cache, int32_t seq);
/* Drop the tokens new_len .. len-1 of `seq` (bookkeeping only; pool contents stay).  Used
 * to hold a fixed-length window when one step is measured repeatedly. */
evl_status evl_cache_truncate(evl_cache *cache, int32_t seq, int32_t new_len);
/* Tokens appended to `seq` so far; negative evl_status on error. */
int32_t evl_cache_len(const evl_cache *cache, int32_t seq);
/* Position id of the first token of `seq` (set by its first append); -1 if unset. */
int64_t evl_cache_pos0(const evl_cache *cache, int32_t seq);
/* Change the stream later calls enqueue on. */
evl_status evl_cache_set_stream(evl_cache *cache, void *stream);

/* Recommended workspace size for chunks of up to max_n_new tokens on up to max_seqs
 * sequences at once.  Smaller workspaces are legal: the key range is then split less.
 * If the workspace is at least 8 KB, its last 4 KB hold counters that the library zeroes
 * before their first use and that every call leaves at zero (chunks of a few tokens -- at
 * most 32 (token, query head) pairs per KV head -- take a kernel that merges its pieces
 * itself with their help): the caller must not write there between calls, and caches that
 * share a workspace must be used from one stream. */
size_t evl_workspace_bytes(const evl_cache_desc *desc, int32_t max_n_new, int32_t max_seqs);

/* Text of the calling thread's last error ("" if none). */
const char *evl_last_error(void);

/*
 * Sec. 3.2 (position ids run without a gap over cache + new chunk, and the rotation is
 * applied at those ids): append a chunk of n_new tokens to sequence 0.  Token i takes position id
 * pos_offset + i; k_new[i] is rotated at that id and stored, v_new[i] is stored as given,
 * both at the paged slot of sequence index len + i.  The first append after a reset fixes
 * pos0 = pos_offset; later appends must satisfy pos_offset == pos0 + len, else
 * EVL_ERR_NONCONTIGUOUS.  k_new, v_new: DEVICE bf16, 16-byte aligned.
 */
evl_status evl_rope_append(evl_cache *cache, const void *k_new, const void *v_new,
                           int64_t pos_offset, int32_t n_new);

/*
 * Sec. 3.2 (per step, only the new frame's tokens go through the transformer; everything
 * older is read from the cache): attention of the chunk's queries over cache + chunk for
 * sequence 0.  cache_len is the number of tokens
 * that precede the chunk; the chunk's own keys/values must already be appended
 * (evl_cache_len >= cache_len + n_new, else EVL_ERR_RANGE).  q_new[i] is rotated at
 * pos0 + cache_len + i and sees tokens 0 .. cache_len + i.  cache_len == 0 is a plain
 * causal prefill.  q_new: DEVICE bf16; out: DEVICE, out_dtype; both 16-byte aligned.
 */
evl_status evl_chunk_attention(const void *q_new, evl_cache *cache, int32_t cache_len,
                               int32_t n_new, void *out);

/*
 * evl_chunk_attention for callers that cannot allocate device memory -- code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc -- and so cannot hand the cache
 * a workspace: the partial results of the key-range pieces and the ticket counters live in a
 * static device array of the library (16 MiB + 4 KiB per GPU, held until the process ends)
 * instead of cache->workspace, which this call neither reads nor writes.  Same arguments, same
 * checks and the same result as evl_chunk_attention on a cache whose workspace has that size
 * (the key range is cut into as many pieces as fit); sequence 0.  Chunks of more than 8192
 * (token, query head) rows (n_new * n_q_heads) are refused with EVL_ERR_WORKSPACE.  The call
 * allocates and frees nothing, on the device or through any library.  All calls on one GPU
 * share that GPU's array: calls that overlap in time on one GPU (two streams, two threads)
 * race; calls on one stream are safe.  Whatever must start at zero is cleared by the call
 * itself, with a fill kernel on the stream.
 */
evl_status evl_chunk_attention_static(const void *q_new, evl_cache *cache, int32_t cache_len,
                                      int32_t n_new, void *out);

/*
 * Ragged batch: the same two operations for n_seqs independent sequences in one launch
 * sequence.  Inputs and outputs are concatenated along the token axis in the order of the
 * arrays (sequence seq_ids[0]'s n_new[0] tokens first, and so on).  seq_ids, pos_offsets,
 * cache_lens, n_new: HOST arrays of n_seqs entries; seq_ids must be distinct.
 */
evl_status evl_rope_append_batched(evl_cache *cache, const void *k_new, const void *v_new,
                                   const int32_t *seq_ids, const int64_t *pos_offsets,
                                   const int32_t *n_new, int32_t n_seqs);
evl_status evl_chunk_attention_batched(const void *q_new, evl_cache *cache,
                                       const int32_t *seq_ids, const int32_t *cache_lens,
                                       const int32_t *n_new, int32_t n_seqs, void *out);

/*
 * Sec. 3.2, frame sampler (the history that a step attends to is a sampled subset of the
 * frames seen so far, and position ids run without a gap over that subset plus the new
 * chunk): attention of the chunk's queries over the retained runs of sequence `seq` plus the
 * chunk, with the rotation the combined sequence's contiguous ids define.
 *
 * The cache stays append-only: every frame is appended once with evl_rope_append and no
 * stored key is ever re-rotated or moved.  runs[0 .. n_runs-1] (HOST; sequence indices,
 * non-empty, ascending, disjoint, inside [0, cache_len)) name what the sampler keeps; the
 * chunk occupies sequence indices cache_len .. cache_len + n_new - 1 and must already be
 * appended.  With R = sum of the runs' lengths, the u-th retained token takes id pos0 + u,
 * chunk token i takes id pos0 + R + i and sees every retained token and chunk tokens 0 .. i.
 * The result equals rotating the unrotated keys of the gathered sequence at those ids; the
 * library reaches it by shifting the rotation of the queries per run (RoPE scores depend on
 * the difference of the two ids only).  Runs that keep everything reproduce
 * evl_chunk_attention.
 *
 * The key range is split over work-groups as in the plain call (workspace as there; none is
 * needed when it is not split).  More than 64 runs with different shifts take several
 * launches whose results are merged through the workspace: EVL_ERR_WORKSPACE if it cannot
 * hold one partial result per launch; evl_workspace_bytes_sampled sizes it.
 * q_new: DEVICE bf16; out: DEVICE, out_dtype; both 16-byte aligned.
 */
typedef struct {
    int32_t start; /* sequence index of the run's first token */
    int32_t len;   /* tokens in the run                        */
} evl_run;
evl_status evl_chunk_attention_sampled(const void *q_new, evl_cache *cache, int32_t seq,
                                       const evl_run *runs, int32_t n_runs, int32_t cache_len,
                                       int32_t n_new, void *out);
/*
 * The same for several independent (sequence, runs, chunk) groups in one call: a ragged batch
 * of episodes that each run their own sampler, or several chunks of one packed sequence that
 * see different parts of it.  Group g uses sequence seq_ids[g] (sequences may repeat: the call
 * only reads the cache), the runs runs[run_offsets[g] .. run_offsets[g+1]-1], the chunk at
 * sequence indices cache_lens[g] .. +n_new[g]-1; its queries are the n_new[g] tokens of q_new
 * that start at token tok_offs[g], its results go to the same tokens of `out` (tok_offs NULL:
 * groups are concatenated in order).  All arrays HOST; run_offsets has n_groups + 1 entries.
 * A group may have at most 64 runs with different shifts (EVL_ERR_UNSUPPORTED beyond).
 */
evl_status evl_chunk_attention_sampled_batched(const void *q_new, evl_cache *cache, int32_t n_groups,
                                               const int32_t *seq_ids, const int32_t *cache_lens,
                                               const int32_t *n_new, const int32_t *tok_offs,
                                               const int32_t *run_offsets, const evl_run *runs,
                                               void *out);
/*
 * Sec. 3.3 (packed training sequences with the action-isolating mask), forward attention:
 * sequence `seq` holds a pack of `prefix` instruction tokens followed by n_frames times
 * (frame_tokens visual tokens, action_tokens action tokens), appended with evl_rope_append as
 * one sequence.  Instruction and visual tokens attend to the instruction and the visual
 * tokens up to themselves; the action tokens of step t attend to the instruction, the visual
 * tokens of steps <= t and their own chunk up to themselves; no token sees another step's
 * actions.  Position ids are contiguous over what a token sees, i.e. those of the single-step
 * example the chunk stands for.  q_packed / out_packed: [prefix + n_frames * (frame_tokens +
 * action_tokens)][Hq][d], rows in pack order.  Built on evl_chunk_attention_sampled_batched:
 * one group for the instruction and one per step of the pack.
 */
evl_status evl_isolated_pack_attention(const void *q_packed, evl_cache *cache, int32_t seq,
                                       int32_t prefix, int32_t frame_tokens, int32_t action_tokens,
                                       int32_t n_frames, void *out_packed);
/*
 * Sec. 3.3, the faster way to the same result: append the whole pack to the EMPTY sequence `seq`
 * with the position ids the action-isolating mask implies -- instruction and visual tokens are
 * numbered without a gap from pos0 (action tokens skipped), the action tokens of step t continue
 * right behind frame t -- instead of the contiguous ids of evl_rope_append.  Keys are rotated at
 * those ids and stored, values stored as given, at the sequence indices 0 .. L-1 of the pack
 * order (L = prefix + n_frames * (frame_tokens + action_tokens)).  evl_isolated_pack_attention on
 * such a sequence (same prefix / frame_tokens / action_tokens, any n_frames up to the appended
 * ones) then runs as ONE causal launch in which the action tokens of earlier steps are holes of
 * the key range: no run list, no per-run shift of the queries; results agree with the route
 * through evl_rope_append to rounding.  Served shapes: action_tokens >= 1, frame_tokens +
 * action_tokens >= 64, prefix >= 63 (EVL_ERR_UNSUPPORTED otherwise: use evl_rope_append).  A
 * sequence that holds a pack takes no further appends and no other attention call until
 * evl_cache_reset (EVL_ERR_NONCONTIGUOUS / EVL_ERR_ARG).  k_packed, v_packed: DEVICE bf16
 * [L][Hkv][d], 16-byte aligned.
 */
evl_status evl_isolated_pack_append(evl_cache *cache, int32_t seq, const void *k_packed,
                                    const void *v_packed, int64_t pos0, int32_t prefix,
                                    int32_t frame_tokens, int32_t action_tokens, int32_t n_frames);
/* Workspace that serves evl_chunk_attention_sampled for chunks of up to max_n_new tokens and
 * up to max_runs runs (it also serves the plain calls on one sequence). */
size_t evl_workspace_bytes_sampled(const evl_cache_desc *desc, int32_t max_n_new,
                                   int32_t max_runs);

/*
 * Sec. 3.2, the two frame samplers, on frame indices 0 .. n_frames-1 (HOST only).  idx (room
 * for n_keep entries) receives the retained frames in ascending order; the count is returned.
 *   uniform: n_keep frames spread evenly over the whole history, oldest and newest included:
 *            the nearest integer to j (n_frames-1)/(n_keep-1), j = 0 .. n_keep-1 (all frames
 *            while n_frames <= n_keep).
 *   window : the newest frame and every stride-th frame before it, at most n_keep of them.
 * How frames map to runs of tokens is the caller's business (a frame is usually one chunk).
 */
int32_t evl_sample_uniform(int32_t n_frames, int32_t n_keep, int32_t *idx);
int32_t evl_sample_window(int32_t n_frames, int32_t n_keep, int32_t stride, int32_t *idx);

/*
 * Sec. 3.2, one navigation step as one call: exactly evl_rope_append[_batched] followed by
 * evl_chunk_attention[_batched] with cache_len = the sequence's length before the append
 * (same arguments, same checks, same results bit for bit, same state afterwards; a refused
 * call changes nothing).  When every chunk of the call is a few tokens long (at most 32 rows
 * of (token, query head) pairs per KV head: the action tokens of a step) both parts run in
 * ONE kernel launch, the attention reading the chunk's keys and values from k_new / v_new
 * while other work-groups of the same launch write them to the cache; longer chunks take the
 * two calls one after the other.
 */
evl_status evl_step(evl_cache *cache, const void *q_new, const void *k_new, const void *v_new,
                    int64_t pos_offset, int32_t n_new, void *out);
evl_status evl_step_batched(evl_cache *cache, const void *q_new, const void *k_new, const void *v_new,
                            const int32_t *seq_ids, const int64_t *pos_offsets, const int32_t *n_new,
                            int32_t n_seqs, void *out);
/* The same for a sampled history: evl_rope_append_batched for sequence seq followed by
 * evl_chunk_attention_sampled with cache_len = the length before the append; runs as there.
 * Every error of either part, EVL_ERR_WORKSPACE included, is reported before anything is
 * appended. */
evl_status evl_step_sampled(evl_cache *cache, const void *q_new, const void *k_new, const void *v_new,
                            int32_t seq, const evl_run *runs, int32_t n_runs, int64_t pos_offset,
                            int32_t n_new, void *out);

/*
 * Sec. 3.2, memory management (the cache is offloaded to host memory and only the segments the
 * sampler selects are brought back): copies n whole pages -- the K block and the V block of
 * all KV heads -- from one page pool to another on the cache's stream.  A pool is a pair of
 * arrays laid out like k_pool / v_pool; it may be DEVICE memory or pinned HOST memory that the
 * device can address (hipHostMalloc, a pinned PyTorch tensor); src / dst may be the same pool
 * if the page lists do not overlap.  Page i of the list goes from src page src_pages[i] to dst
 * page dst_pages[i]; both lists HOST, ids checked against the pool sizes (EVL_ERR_RANGE).
 * A pool pointer the device cannot address (pageable host memory) is refused with EVL_ERR_ARG,
 * a pool larger than its allocation with EVL_ERR_RANGE, before anything is launched.
 * Offloading a segment = copying its pages out and handing the device pages to other tokens;
 * reloading = copying them into any free device pages and pointing the block-table entries of
 * the segment at those pages: sequence indices and position ids do not change, so
 * evl_chunk_attention_sampled works on reloaded segments as on resident ones.
 */
evl_status evl_pages_copy(evl_cache *cache, void *dst_k, void *dst_v, const int32_t *dst_pages,
                          int32_t dst_pool_pages, const void *src_k, const void *src_v,
                          const int32_t *src_pages, int32_t src_pool_pages, int32_t n);

/* =========================================================================================
 * DIAGNOSTICS.  Everything from here to the end of the header serves measurement and tests
 * (bench.py, the planner tests): none of it is part of the method, none of it is needed to use
 * the library, and none of it changes a result beyond rounding order.
 * ========================================================================================= */

/*
 * How the last evl_chunk_attention[_batched] call on `cache` was (or the next identical one
 * would be) partitioned: number of attention work-groups, largest split count of any
 * sequence, and workspace bytes used.  Any pointer may be NULL.  Host-only.
 */
evl_status evl_last_plan(const evl_cache *cache, int32_t *n_workgroups, int32_t *max_splits,
                         size_t *workspace_used);

/*
 * Tuning knob of the attention launch: target_workgroups is the number of work-groups the
 * key-range splitting aims for; the split it leads to is then made as asked.  0 returns to the
 * default, in which the library prices the candidate piece counts of every launch with a model of
 * the chip (how work-groups are dealt to XCDs and shader engines, what a key tile, a work-group's
 * start and end and the merge of the pieces cost) and takes the cheapest, which may be no split at
 * all (a long chunk over a short history); launches of the short-chunk kernel aim at about 140
 * work-groups.  Results do not depend on it beyond rounding order.
 */
evl_status evl_cache_tune(evl_cache *cache, int32_t target_workgroups);

/* Number of kernels the calls on this cache have enqueued so far (-1 for a NULL cache): lets a
 * caller or a test see how many launches a call took. */
int64_t evl_cache_launches(const evl_cache *cache);

/*
 * Measurement aid (not part of the method).  With n_pairs > 0 every later
 * evl_chunk_attention[_batched / _sampled] call launches its attention kernel -- the dense
 * contraction, without the combine kernel -- with a pair of HIP events attached to that
 * dispatch (hipExtLaunchKernel): the pair receives the begin and the end time of the kernel
 * itself, the interval a kernel trace reports.  The pairs come from a ring of n_pairs that the
 * library creates on the cache's stream's device.  n_pairs == 0 switches this off and destroys
 * the events.  Events are host-side handles: no device memory is allocated.
 */
evl_status evl_timing_enable(evl_cache *cache, int32_t n_pairs);
/*
 * Waits for the recorded pairs to complete, writes their elapsed times (milliseconds, oldest
 * first, at most `max`) to the HOST array ms_out, stores the count in *n_out and empties the
 * ring.  If more than n_pairs calls were bracketed since the last read, only the newest
 * n_pairs are kept.
 */
evl_status evl_timing_read(evl_cache *cache, float *ms_out, int32_t max, int32_t *n_out);

#ifdef __cplusplus
}
#endif
#endif /* EVL_H */

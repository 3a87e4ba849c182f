// Host side of the C ABI declared in include/evl.h: argument checking, the integer
// bookkeeping of the contiguous position ids (paper Sec. 3.2), and the partitioning of the
// attention work over the chip.  No device memory is allocated or touched here.
#include "evl.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "evl_internal.h"

namespace {

thread_local char g_err[512] = "";

evl_status fail(evl_status st, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Work-groups the attention launch aims for: enough to give each of the 256 CUs a few.
constexpr int kDefaultTargetItems = 240;
constexpr int kMinTilesPerSplit = 4;   // 256 keys: below this the prologue dominates
constexpr int kDecodeTargetGroups = 140;  // work-groups a launch of the short-chunk kernel aims at
constexpr int kMaxSplits = 256;  // pieces of one key range (a single long sequence can fill the chip by itself)

struct Plan {
    int32_t n_items = 0, max_splits = 1;
    size_t workspace_used = 0;
};

}  // namespace

// Shape of a pack under the action-isolating mask: `prefix` instruction tokens, then steps of
// frame_tokens visual + action_tokens action tokens.  action_tokens == 0: not a pack.
struct PackShape {
    int32_t prefix = 0, frame_tokens = 0, action_tokens = 0;
};

struct evl_cache {
    evl_cache_desc d;
    int group;
    int target_items;  // work-groups the key-range splitting aims for
    bool tuned = false;  // the caller set the target: splits are then made as asked, not priced
    double rev_freq[evl::kMaxHalfDim];  // theta_j / (2 pi)
    std::vector<int64_t> len, pos0;
    std::vector<char> has_pos0;
    std::vector<PackShape> pack;  // per sequence: set by evl_isolated_pack_append (position ids skip action tokens)
    Plan last_plan;
    bool counters_zeroed = false;  // the ticket counters at the end of the workspace are ready
    // measurement aid: ring of event pairs around the attention kernel
    std::vector<hipEvent_t> ev_start, ev_stop;
    int64_t ev_count = 0;  // pairs recorded since the last read
    int64_t n_launches = 0;  // kernels enqueued so far (evl_cache_launches)
};

static evl_status check_desc(const evl_cache_desc *d) {
    if (!d) return fail(EVL_ERR_NULL, "desc is NULL");
    if (d->n_q_heads <= 0 || d->n_kv_heads <= 0 || d->n_q_heads % d->n_kv_heads)
        return fail(EVL_ERR_ARG, "need n_q_heads %% n_kv_heads == 0 (got %d / %d)", d->n_q_heads,
                    d->n_kv_heads);
    if (d->head_dim != 64 && d->head_dim != 128)
        return fail(EVL_ERR_UNSUPPORTED, "head_dim %d: kernels exist for 64 and 128", d->head_dim);
    if (d->page_size != evl::kPage)
        return fail(EVL_ERR_UNSUPPORTED, "page_size %d: kernels exist for 16", d->page_size);
    if (d->n_pages <= 0 || d->max_pages_per_seq <= 0 || d->max_seqs <= 0)
        return fail(EVL_ERR_ARG, "n_pages, max_pages_per_seq and max_seqs must be positive");
    if ((int64_t)d->max_pages_per_seq * d->page_size > INT32_MAX / 2)
        return fail(EVL_ERR_ARG, "max_pages_per_seq too large");
    if (d->out_dtype != EVL_OUT_BF16 && d->out_dtype != EVL_OUT_F32)
        return fail(EVL_ERR_ARG, "out_dtype must be EVL_OUT_BF16 or EVL_OUT_F32");
    if (!(d->rope_base > 1.0) || !std::isfinite(d->rope_base))
        return fail(EVL_ERR_ARG, "rope_base must be finite and > 1");
    if (!d->k_pool || !d->v_pool || !d->block_table)
        return fail(EVL_ERR_NULL, "k_pool, v_pool and block_table are required");
    if (!aligned16(d->k_pool) || !aligned16(d->v_pool))
        return fail(EVL_ERR_ALIGN, "k_pool / v_pool must be 16-byte aligned");
    if (d->workspace_bytes && !d->workspace)
        return fail(EVL_ERR_NULL, "workspace_bytes > 0 with a NULL workspace");
    if (d->workspace && !aligned16(d->workspace))
        return fail(EVL_ERR_ALIGN, "workspace must be 16-byte aligned");
    return EVL_OK;
}

extern "C" {

const char *evl_last_error(void) { return g_err; }

evl_status evl_cache_create(const evl_cache_desc *desc, evl_cache **out) {
    if (!out) return fail(EVL_ERR_NULL, "out is NULL");
    *out = nullptr;
    evl_status st = check_desc(desc);
    if (st != EVL_OK) return st;
    evl_cache *c = new (std::nothrow) evl_cache();
    if (!c) return fail(EVL_ERR_ARG, "out of host memory");
    c->d = *desc;
    c->group = desc->n_q_heads / desc->n_kv_heads;
    c->target_items = kDefaultTargetItems;
    for (int j = 0; j < desc->head_dim / 2; ++j)
        c->rev_freq[j] = std::pow(desc->rope_base, -2.0 * (double)j / (double)desc->head_dim) /
                         6.283185307179586476925286766559;
    c->len.assign(desc->max_seqs, 0);
    c->pos0.assign(desc->max_seqs, 0);
    c->has_pos0.assign(desc->max_seqs, 0);
    c->pack.assign(desc->max_seqs, PackShape());
    *out = c;
    return EVL_OK;
}

static void destroy_events(evl_cache *c) {
    for (hipEvent_t e : c->ev_start) (void)hipEventDestroy(e);
    for (hipEvent_t e : c->ev_stop) (void)hipEventDestroy(e);
    c->ev_start.clear();
    c->ev_stop.clear();
    c->ev_count = 0;
}

evl_status evl_cache_destroy(evl_cache *cache) {
    if (!cache) return fail(EVL_ERR_NULL, "cache is NULL");
    destroy_events(cache);
    delete cache;
    return EVL_OK;
}

static evl_status check_seq(const evl_cache *c, int32_t seq) {
    if (!c) return fail(EVL_ERR_NULL, "cache is NULL");
    if (seq < 0 || seq >= c->d.max_seqs)
        return fail(EVL_ERR_ARG, "sequence %d outside [0, %d)", seq, c->d.max_seqs);
    return EVL_OK;
}

evl_status evl_cache_reset(evl_cache *cache, int32_t seq) {
    evl_status st = check_seq(cache, seq);
    if (st != EVL_OK) return st;
    cache->len[seq] = 0;
    cache->has_pos0[seq] = 0;
    cache->pack[seq] = PackShape();
    return EVL_OK;
}

evl_status evl_cache_truncate(evl_cache *cache, int32_t seq, int32_t new_len) {
    evl_status st = check_seq(cache, seq);
    if (st != EVL_OK) return st;
    if (new_len < 0 || new_len > cache->len[seq])
        return fail(EVL_ERR_RANGE, "truncate to %d: sequence %d holds %lld tokens", new_len, seq,
                    (long long)cache->len[seq]);
    cache->len[seq] = new_len;
    if (new_len == 0) {
        cache->has_pos0[seq] = 0;
        cache->pack[seq] = PackShape();
    }
    return EVL_OK;
}

int32_t evl_cache_len(const evl_cache *cache, int32_t seq) {
    evl_status st = check_seq(cache, seq);
    if (st != EVL_OK) return (int32_t)st;
    return (int32_t)cache->len[seq];
}

int64_t evl_cache_pos0(const evl_cache *cache, int32_t seq) {
    if (check_seq(cache, seq) != EVL_OK || !cache->has_pos0[seq]) return -1;
    return cache->pos0[seq];
}

int64_t evl_cache_launches(const evl_cache *cache) { return cache ? cache->n_launches : -1; }

evl_status evl_cache_set_stream(evl_cache *cache, void *stream) {
    if (!cache) return fail(EVL_ERR_NULL, "cache is NULL");
    cache->d.stream = stream;
    return EVL_OK;
}

size_t evl_workspace_bytes(const evl_cache_desc *desc, int32_t max_n_new, int32_t max_seqs) {
    if (!desc || max_n_new <= 0 || max_seqs <= 0 || desc->head_dim <= 0 || desc->n_q_heads <= 0)
        return 0;
    // room for 16 splits of every sequence -- more for short chunks, whose key range is cut finer:
    // as many pieces as make one work-group per CU (at most 64), and 64 for chunks of a few
    // tokens --: d outputs (at most 4 bytes each) and two floats per (split, token, head); then
    // the ticket counters
    const int64_t row_tiles = ((int64_t)max_n_new * desc->n_q_heads + evl::kAttnRows - 1) / evl::kAttnRows;
    const size_t pieces = (size_t)std::min<int64_t>(64, std::max<int64_t>(16, 256 / row_tiles + 1));
    const size_t per_seq = std::max<size_t>(pieces * max_n_new, (size_t)64 * std::min(max_n_new, 16));
    const size_t rows = per_seq * max_seqs * desc->n_q_heads;
    return rows * (size_t)(desc->head_dim + 2) * sizeof(float) + evl::kCounterBytes;
}

// ------------------------------------------------------------------------------------------
// RoPE + append
// ------------------------------------------------------------------------------------------
// Everything an append can be refused for; touches no state.
static evl_status check_append(evl_cache *c, const void *k_new, const void *v_new, const int32_t *seq_ids,
                               const int64_t *pos_offsets, const int32_t *n_new, int32_t n_seqs) {
    if (!c) return fail(EVL_ERR_NULL, "cache is NULL");
    if (!k_new || !v_new) return fail(EVL_ERR_NULL, "k_new / v_new is NULL");
    if (!seq_ids || !pos_offsets || !n_new) return fail(EVL_ERR_NULL, "a host array is NULL");
    if (!aligned16(k_new) || !aligned16(v_new))
        return fail(EVL_ERR_ALIGN, "k_new / v_new must be 16-byte aligned");
    if (n_seqs <= 0 || n_seqs > c->d.max_seqs)
        return fail(EVL_ERR_ARG, "n_seqs %d outside [1, %d]", n_seqs, c->d.max_seqs);
    const int64_t cap = (int64_t)c->d.max_pages_per_seq * c->d.page_size;
    std::vector<char> seen(c->d.max_seqs, 0);
    for (int i = 0; i < n_seqs; ++i) {
        const int32_t s = seq_ids[i];
        evl_status st = check_seq(c, s);
        if (st != EVL_OK) return st;
        if (seen[s]) return fail(EVL_ERR_ARG, "sequence %d listed twice", s);
        seen[s] = 1;
        if (n_new[i] <= 0) return fail(EVL_ERR_ARG, "n_new[%d] = %d must be positive", i, n_new[i]);
        if (pos_offsets[i] < 0 || pos_offsets[i] + n_new[i] > (int64_t)INT32_MAX)
            return fail(EVL_ERR_ARG, "position ids of entry %d leave [0, 2^31)", i);
        if (c->pack[s].action_tokens > 0)
            return fail(EVL_ERR_NONCONTIGUOUS,
                        "sequence %d holds a pack (evl_isolated_pack_append), whose position ids skip action "
                        "tokens: reset it before appending", s);
        if (c->has_pos0[s] && pos_offsets[i] != c->pos0[s] + c->len[s])
            return fail(EVL_ERR_NONCONTIGUOUS,
                        "sequence %d: pos_offset %lld does not continue the cache (expected %lld)",
                        s, (long long)pos_offsets[i], (long long)(c->pos0[s] + c->len[s]));
        if (c->len[s] + n_new[i] > cap)
            return fail(EVL_ERR_CAPACITY, "sequence %d: %lld + %d tokens exceed capacity %lld", s,
                        (long long)c->len[s], n_new[i], (long long)cap);
    }
    return EVL_OK;
}

// Kernel arguments for appending entries [base, base + cnt) of the call; *tok_off: tokens of the
// concatenated inputs before them (advanced).
static void fill_append(const evl_cache *c, const void *k_new, const void *v_new, const int32_t *seq_ids,
                        const int64_t *pos_offsets, const int32_t *n_new, int base, int cnt, int64_t *tok_off,
                        evl::AppendParams *pp) {
    evl::AppendParams &p = *pp;
    std::memset(&p, 0, sizeof(p));
    p.k_new = k_new;
    p.v_new = v_new;
    p.k_pool = c->d.k_pool;
    p.v_pool = c->d.v_pool;
    p.block_table = c->d.block_table;
    p.pos_tags = c->d.pos_tags;
    p.n_kv_heads = c->d.n_kv_heads;
    p.n_pages = c->d.n_pages;
    p.max_pages_per_seq = c->d.max_pages_per_seq;
    p.n_seqs = cnt;
    std::memcpy(p.rev_freq, c->rev_freq, sizeof(p.rev_freq));
    int items = 0;
    for (int i = 0; i < cnt; ++i) {
        const int32_t s = seq_ids[base + i];
        const int64_t t0 = c->len[s], t1 = t0 + n_new[base + i];
        evl::AppendSeq &q = p.seq[i];
        q.bt_row = s;
        q.t_begin = (int32_t)t0;
        q.n_new = n_new[base + i];
        q.tok_off = (int32_t)*tok_off;
        q.item_begin = items;
        q.pos_begin = pos_offsets[base + i];
        const int pages = (int)((t1 - 1) / evl::kPage - t0 / evl::kPage + 1);
        items += pages * c->d.n_kv_heads;
        *tok_off += n_new[base + i];
    }
    p.n_items = items;
}

// The bookkeeping of an append that has been enqueued.
static void commit_append(evl_cache *c, const int32_t *seq_ids, const int64_t *pos_offsets, const int32_t *n_new,
                          int base, int cnt) {
    for (int i = 0; i < cnt; ++i) {
        const int32_t s = seq_ids[base + i];
        if (!c->has_pos0[s]) {
            c->pos0[s] = pos_offsets[base + i];
            c->has_pos0[s] = 1;
        }
        c->len[s] += n_new[base + i];
    }
}

evl_status evl_rope_append_batched(evl_cache *c, const void *k_new, const void *v_new,
                                   const int32_t *seq_ids, const int64_t *pos_offsets,
                                   const int32_t *n_new, int32_t n_seqs) {
    // validate everything before touching any state
    evl_status st = check_append(c, k_new, v_new, seq_ids, pos_offsets, n_new, n_seqs);
    if (st != EVL_OK) return st;
    int64_t tok_off = 0;
    for (int base = 0; base < n_seqs; base += evl::kMaxSeqs) {
        const int cnt = std::min(evl::kMaxSeqs, n_seqs - base);
        evl::AppendParams p;
        fill_append(c, k_new, v_new, seq_ids, pos_offsets, n_new, base, cnt, &tok_off, &p);
        hipError_t e = evl::launch_rope_append(p, c->d.head_dim, (hipStream_t)c->d.stream);
        if (e == hipSuccess) ++c->n_launches;
        if (e != hipSuccess)
            return fail(EVL_ERR_LAUNCH, "rope_append launch failed: %s", hipGetErrorString(e));
        commit_append(c, seq_ids, pos_offsets, n_new, base, cnt);
    }
    return EVL_OK;
}

evl_status evl_rope_append(evl_cache *cache, const void *k_new, const void *v_new,
                           int64_t pos_offset, int32_t n_new) {
    const int32_t seq = 0;
    return evl_rope_append_batched(cache, k_new, v_new, &seq, &pos_offset, &n_new, 1);
}

// ------------------------------------------------------------------------------------------
// Chunk attention
// ------------------------------------------------------------------------------------------
// The last kCounterBytes of a workspace of at least twice that size hold the ticket counters;
// the partial results use what lies before them.
static size_t partials_capacity(const evl_cache *c) {
    return c->d.workspace_bytes >= 2 * evl::kCounterBytes ? c->d.workspace_bytes - evl::kCounterBytes
                                                         : c->d.workspace_bytes;
}
static int32_t *counters_of(const evl_cache *c) {
    if (!c->d.workspace || c->d.workspace_bytes < 2 * evl::kCounterBytes) return nullptr;
    const size_t off = (c->d.workspace_bytes - evl::kCounterBytes) & ~(size_t)15;
    return (int32_t *)((char *)c->d.workspace + off);
}
// Zeroes the counters once per cache object (every launch leaves them at zero).
static evl_status ready_counters(evl_cache *c) {
    if (c->counters_zeroed) return EVL_OK;
    hipError_t e = evl::launch_zero_counters(counters_of(c), evl::kCounters, (hipStream_t)c->d.stream);
    if (e == hipSuccess) ++c->n_launches;
    if (e != hipSuccess)
        return fail(EVL_ERR_LAUNCH, "counter initialisation failed: %s", hipGetErrorString(e));
    c->counters_zeroed = true;
    return EVL_OK;
}

// Fields of the kernel arguments that do not depend on the entries.
static void init_params(const evl_cache *c, const void *q_new, void *out, void *part_o,
                        float *part_ml, evl::AttnParams *p, evl::CombineParams *cp) {
    const int D = c->d.head_dim, G = c->group;
    const int MT = evl::attention_rows_per_workgroup();
    std::memset(p, 0, sizeof(*p));
    std::memset(cp, 0, sizeof(*cp));
    p->q = q_new;
    p->k_pool = c->d.k_pool;
    p->v_pool = c->d.v_pool;
    p->block_table = c->d.block_table;
    p->out = out;
    p->part_o = part_o;
    p->part_ml = part_ml;
    p->n_q_heads = c->d.n_q_heads;
    p->n_kv_heads = c->d.n_kv_heads;
    p->group = G;
    p->n_pages = c->d.n_pages;
    p->max_pages_per_seq = c->d.max_pages_per_seq;
    p->out_f32 = c->d.out_dtype == EVL_OUT_F32;
    // cos/sin table: the tokens of 256 packed rows, if that stays within 48 KB of LDS
    p->tab_tokens = std::min(MT / G + 2, (48 * 1024) / (evl::attention_tab_stride(D) * 8));
    p->q_scale = (float)(1.4426950408889634 / std::sqrt((double)D));
    std::memcpy(p->rev_freq, c->rev_freq, sizeof(p->rev_freq));
    cp->part_o = part_o;
    cp->part_ml = part_ml;
    cp->out = out;
    cp->n_q_heads = c->d.n_q_heads;
    cp->out_f32 = p->out_f32;
}

// How an entry's work items (groups x m_tiles) are cut into XCD chunks (see evl_internal.h), and
// what the cut puts on the fullest shader engine of the chip.
struct Chunking {
    int rows, pad;   // AttnSeq::chunk_rows, chunk_pad
    int engine;      // real work-groups on the fullest shader engine (of an entry dealt from XCD 0)
};

// Real work-groups on the fullest shader engine for one way of cutting.  The chunks go to the
// XCDs in turn; an XCD deals its slots (padding included) to its four engines in turn.
static int engine_load(int groups, int m_tiles, int rows, int pad) {
    const int chunks = evl::xcd_chunks(groups, m_tiles, rows, pad);
    int worst = 0;
    if (!pad) {  // all slots real except the tail of the entry's last chunk
        for (int x = 0; x < 8 && x < chunks; ++x) {
            int w = (chunks - x + 7) / 8 * rows;
            if ((chunks - 1) % 8 == x) w -= chunks * rows - groups * m_tiles;
            worst = std::max(worst, (w + evl::kEnginesPerXcd - 1) / evl::kEnginesPerXcd);
        }
        return worst;
    }
    // padded: a chunk's slots are a multiple of 4 (asserted by the caller's choice of 8), so slot i of any
    // chunk goes to engine i % 4: a full chunk puts rows / 4 on each, a group's last chunk of
    // `last` real items (last + 3) / 4 on the fullest.  Group g's last chunk is chunk g * cpg + cpg - 1.
    const int cpg = (m_tiles + rows - 1) / rows, last = m_tiles - (cpg - 1) * rows;
    int lasts[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int g = 0; g < groups; ++g) ++lasts[(g * cpg + cpg - 1) % 8];
    for (int x = 0; x < 8 && x < chunks; ++x) {
        const int here = (chunks - x + 7) / 8;
        worst = std::max(worst, (here - lasts[x]) * (rows / evl::kEnginesPerXcd) +
                                    lasts[x] * ((last + evl::kEnginesPerXcd - 1) / evl::kEnginesPerXcd));
    }
    return worst;
}

// The cut for an entry: groups of at most kXcdChunkRowTiles row tiles are chunks by themselves.
// Otherwise the candidates are, in order of preference, chunks of 8 cut group by group with
// padding, dense chunks of a divisor of m_tiles between 7 and 4 (no padding, no straddling),
// and dense chunks of 8 down to 4 that straddle groups.  What decides is the load of the fullest
// shader engine: first its rounds of 8 work-groups, then -- work-groups that run at the same
// time share their XCD's L2 and clock -- the load itself (220 equal work-groups in one round:
// 263 us with 32 on the fullest XCD, 250 with 30, 240 to 247 with 28); candidates within 3 % of
// the lightest count as equal and the preferred one of them is taken (a 4000-token prefill in
// many rounds: 138 us padded, 147 us dense by 8, 153 us by 5).
static Chunking choose_chunking(int groups, int m_tiles) {
    const int cus = evl::kCusPerXcd / evl::kEnginesPerXcd;
    if (m_tiles <= evl::kXcdChunkRowTiles) {
        const int rows = std::max(m_tiles, 1);
        return Chunking{rows, 0, engine_load(groups, m_tiles, rows, 0)};
    }
    Chunking cand[1 + 2 * (evl::kXcdChunkRowTiles / 2 + 1)];
    int n = 0;
    cand[n++] = Chunking{evl::kXcdChunkRowTiles, 1, 0};
    for (int rows = evl::kXcdChunkRowTiles - 1; rows >= evl::kXcdChunkRowTiles / 2; --rows)
        if (m_tiles % rows == 0) cand[n++] = Chunking{rows, 0, 0};
    for (int rows = evl::kXcdChunkRowTiles; rows >= evl::kXcdChunkRowTiles / 2; --rows)
        if (m_tiles % rows != 0) cand[n++] = Chunking{rows, 0, 0};
    int lightest = 0;
    for (int i = 0; i < n; ++i) {
        cand[i].engine = engine_load(groups, m_tiles, cand[i].rows, cand[i].pad);
        if (cand[i].engine < cand[lightest].engine) lightest = i;
    }
    const int rounds = (cand[lightest].engine + cus - 1) / cus;
    for (int i = 0; i < n; ++i)
        if ((cand[i].engine + cus - 1) / cus == rounds && cand[i].engine * 100 <= cand[lightest].engine * 103)
            return cand[i];
    return cand[lightest];
}

// An unsplit entry with more work items than compute units -- a long chunk whose row tiles see
// different numbers of keys under the causal mask -- is dealt row tile after row tile, all groups'
// longest work items first, in dense chunks of 8: with the groups one after the other the last
// groups' longest work items start a round late, and they are the launch's critical path (3520
// tokens on an empty cache: 129 -> 111 us; 5000: 232 -> 185 us; 4000 new over 6580 cached: 452 ->
// 437 us; never slower in any unsplit launch tried).  Launches cut into pieces lose 3 to 15 % with it.
static bool tile_major_pays(int n_splits, int groups, int m_tiles) {
    return n_splits == 1 && groups * m_tiles > 256;
}

// Work-groups an entry of a launch puts on each XCD: its chunks go round-robin over the 8 XCDs,
// starting at XCD *next, where the entry before it stopped; the kernel recomputes the same
// assignment from (XCD, slot) and the entry's xcd_first.
static void add_xcd_load(int per_xcd[8], int *next, evl::AttnSeq *q, int groups, int m_tiles, const Chunking &ck) {
    const int chunks = evl::xcd_chunks(groups, m_tiles, ck.rows, ck.pad);
    q->chunk_rows = ck.rows;
    q->chunk_pad = ck.pad;
    q->xcd_first = *next;
    for (int x = 0; x < 8; ++x) {
        const int r = (x - *next) & 7;
        per_xcd[x] += (chunks > r ? (chunks - r + 7) / 8 : 0) * ck.rows;
    }
    *next = (*next + chunks) & 7;
}

// Splitting a key range buys balance and pays for it: more work-groups with their fixed cost,
// partial rows written and read back, one more kernel.  With long chunks over short histories (a
// prefill: thousands of rows, each piece a full copy of them) the price is the larger part.
// Constants of the launch-time model below, in microseconds, fitted (least squares on the
// logarithm) to 1600 timings of forced plans: 8 histories from 0 to 60 000 cached tokens x 15
// chunk lengths from 40 to 4000, 4 short histories (256 to 868) x 6 chunk lengths, up to 13 piece
// counts each; 7B-class heads (28 / 4, d = 128).
struct PlanModel {
    double tile = 1.393;            // a key tile of a work-group ...
    double tile_few_rows = -0.197;  // ... less when few row tiles share the keys (x min(1, 6 / row tiles))
    double tile_busy = 0.174;       // ... more when every compute unit is busy (x share of them in use)
    double tile_unsplit = -0.081;   // ... a little less in a launch without pieces
    double fixed = 3.2;             // a work-group's start and end
    double fixed_unsplit = 8.0;     // ... more without pieces: the whole causal end of the chunk sits in every work-group
    double merge = 11.625;          // the merge launch
    double per_mb = 0.423;          // partial rows written and read back, per MB
    double tail = 0.325;            // unequal work-groups leave a tail: x (1 - shortest / longest)
    double tail_longest_first = 0.5;  // ... a smaller one when the longest are dealt first (tile_major_pays)
    double unsplit_margin = 1.05;   // a split has to beat the unsplit launch by this factor
    // Heads of 64 channels: a key tile is about this fraction of the work (not fitted: set so that the
    // choices for 16 / 4 heads of 64 channels come out within a few percent of the best forced plans)
    explicit PlanModel(int head_dim) {
        const double scale = head_dim == 64 ? kTileScaleD64 : 1.0;
        tile *= scale;
        tile_few_rows *= scale;
        tile_busy *= scale;
        tile_unsplit *= scale;
    }
    static constexpr double kTileScaleD64 = 0.5;
};

// Number of pieces for a launch that serves ONE set of rows (one sequence's chunk): every
// candidate is priced with a model of how the chip runs the launch, fitted to timings of forced
// plans over a grid of history and chunk lengths (8 histories from 0 to 60 000 tokens, 15 chunk
// lengths from 40 to 4000, up to 13 piece counts each; 7B-class heads).  What the model knows:
//  * Work-groups run one per compute unit, and the hardware deals them to the 8 XCDs in turn and,
//    inside an XCD, to its 4 shader engines of 8 compute units in turn: the fullest shader
//    engine's work-groups, in rounds of 8, set the pace (252 equal work-groups that put 33 on
//    one XCD take two rounds, 240 that put 30 on each take one).  The load of the fullest XCD
//    follows from the work-item map (xcd_chunks, xcd_chunk_rows).
//  * Equal pieces come in whole rounds; the unequal items of a causal chunk over a short history
//    pack better than that, the more so the less uniform they are, but leave a tail.
//  * A key tile costs a work-group 1.2 to 1.5 us: less when few row tiles share the keys, more
//    when every compute unit is busy (the clock is lower then).
//  * A split costs the merge launch and the partial rows, written once and read once; a launch
//    without pieces pays about 8 us more per work-group (PlanModel).
// see[mt]: key tiles row tile mt sees under the causal mask, non-decreasing; tiles: key tiles of
// the whole range (the longest work item without a split); rows * row_bytes: one copy of the
// partial rows; capacity: room for them.  A split has to beat the unsplit launch by 5 % of the
// model's time to be taken (where the two are close the model errs towards splitting, and the
// unsplit launch needs no workspace).  Returns the number of pieces (1 = no split), their length
// in key tiles in *tps_out.
static int pick_pieces(const std::vector<int> &see, int n_kv_heads, int head_dim, int64_t tiles, size_t rows,
                       size_t row_bytes, size_t capacity, int *tps_out) {
    const PlanModel k(head_dim);
    const int m_tiles = (int)see.size();
    double work = 0.0;
    for (int v : see) work += v;
    const int see_min = see.front(), see_max = see.back();
    int best_n = 1, best_tps = (int)tiles;
    double best_t = 0.0, unsplit_t = 0.0;
    const int64_t most = std::min<int64_t>(kMaxSplits, tiles);
    for (int64_t want = 1; want <= most; want += want < 32 ? 1 : want / 8) {
        const int64_t tps = (tiles + want - 1) / want, n = (tiles + tps - 1) / tps;
        if (n != want && want <= 32) continue;  // the same plan as a smaller `want`
        if (n > 1 && (tps < kMinTilesPerSplit || (size_t)n * rows * row_bytes > capacity)) continue;
        // work items that see any key: piece s of row tile mt does if see[mt] > s * tps
        int64_t live = 0;
        for (int64_t sp = 0; sp < n; ++sp) {
            if (sp * tps < see_min)
                live += m_tiles;
            else
                live += see.end() - std::upper_bound(see.begin(), see.end(), (int)(sp * tps));
        }
        const double longest = (double)std::min<int64_t>(tps, see_max);
        const double mean = work / ((double)m_tiles * (double)n);
        const double uniform = n == 1 ? (double)see_min / (double)see_max : mean / longest;
        const double busy = std::min(1.0, (double)(live * n_kv_heads) / 256.0);
        // work-groups on the fullest shader engine, in rounds of its 8 compute units
        const int groups = (int)n * n_kv_heads;
        const double engine = (double)choose_chunking(groups, m_tiles).engine / 8.0;
        // (whole rounds matter for the first two; with many rounds the in-order dispatch evens the end out)
        const double rounds = engine + (std::ceil(engine) - engine) * uniform * std::min(1.0, 2.0 / engine);
        const double tile_us = k.tile + k.tile_few_rows * std::min(1.0, 6.0 / m_tiles) + k.tile_busy * busy +
                               (n == 1 ? k.tile_unsplit : 0.0);
        const double fixed = k.fixed + (n == 1 ? k.fixed_unsplit : 0.0);
        // (an unsplit launch of several rounds is dealt longest work items first: half the tail)
        const double tail = k.tail * (tile_major_pays((int)n, groups, m_tiles) ? k.tail_longest_first : 1.0);
        double t = std::max(longest * tile_us + fixed,
                            rounds * (mean * tile_us + fixed) * (1.0 + tail * (1.0 - uniform)));
        if (n > 1) t += k.merge + k.per_mb * (double)((size_t)n * rows * row_bytes) * 1e-6;
        if (n == 1) unsplit_t = t;
        if (want == 1 || t < best_t) {
            best_t = t;
            best_n = (int)n;
            best_tps = (int)tps;
        }
    }
    if (best_n > 1 && unsplit_t > 0.0 && unsplit_t <= k.unsplit_margin * best_t) {
        best_n = 1;
        best_tps = (int)tiles;
    }
    *tps_out = best_tps;
    return best_n;
}

// The same pricing for a launch that serves several sequences.  All sequences share one piece
// length T (in key tiles), so that work-groups carry about the same amount of work whatever
// their sequence's length; the candidates are the lengths that cut the longest sequence into
// 1, 2, 3 ... pieces.  The chunks of the launch go round the XCDs entry after entry, so the
// fullest XCD holds the launch's chunks / 8, rounded up, and its fullest shader engine a quarter
// of that.  m_tiles, tiles, mean_see (key tiles a row tile of the sequence sees on average under
// the causal mask), rows (token x head rows) per sequence.  Fills n_splits / tps per sequence;
// returns the partial rows the plan needs.
static size_t pick_piece_length(const std::vector<int> &m_tiles, const std::vector<int> &tiles,
                                const std::vector<double> &mean_see, const std::vector<size_t> &rows, int n_kv_heads,
                                int head_dim, size_t row_bytes, size_t capacity, std::vector<int> *n_splits, std::vector<int> *tps) {
    const PlanModel k(head_dim);
    const int n = (int)m_tiles.size();
    const int longest_seq = *std::max_element(tiles.begin(), tiles.end());
    std::vector<int> ns(n), len(n), best_ns(n, 1), best_len(tiles);
    double best_t = 0.0, unsplit_t = 0.0;
    size_t best_rows = 0;
    std::vector<int> unsplit_len(tiles);
    const int most = std::min<int>(kMaxSplits, std::max(1, longest_seq / kMinTilesPerSplit));
    for (int want = 1; want <= most; want += want < 16 ? 1 : want / 4) {
        const int T = std::max((longest_seq + want - 1) / want, want > 1 ? kMinTilesPerSplit : 1);
        size_t ws_rows = 0;
        double items = 0.0, work = 0.0, longest = 0.0, shortest = 1e30, rows_weighted = 0.0;
        int per_xcd[8] = {0, 0, 0, 0, 0, 0, 0, 0}, next = 0;
        for (int i = 0; i < n; ++i) {
            ns[i] = std::max(1, std::min(kMaxSplits, (tiles[i] + T - 1) / T));
            len[i] = (tiles[i] + ns[i] - 1) / ns[i];
            ns[i] = (tiles[i] + len[i] - 1) / len[i];
            if (ns[i] > 1) ws_rows += (size_t)ns[i] * rows[i];
            const int groups = ns[i] * n_kv_heads;
            const Chunking ck = choose_chunking(groups, m_tiles[i]);
            const int chunks = evl::xcd_chunks(groups, m_tiles[i], ck.rows, ck.pad);
            for (int x = 0; x < 8; ++x) {
                const int r = (x - next) & 7;
                per_xcd[x] += (chunks > r ? (chunks - r + 7) / 8 : 0) * ck.rows;
            }
            next = (next + chunks) & 7;
            const double it = (double)m_tiles[i] * groups;
            items += it;
            work += mean_see[i] * m_tiles[i] * n_kv_heads;
            rows_weighted += it * std::min(1.0, 6.0 / m_tiles[i]);
            longest = std::max<double>(longest, std::min<double>(len[i], tiles[i]));
            shortest = std::min<double>(shortest, mean_see[i] / ns[i]);
        }
        if (want > 1 && ws_rows == 0) break;             // pieces longer than every sequence: the unsplit plan again
        if (ws_rows * row_bytes > capacity) continue;
        const double mean = work / items, uniform = std::min(1.0, std::min(shortest, mean) / longest);
        const double engine = (double)((*std::max_element(per_xcd, per_xcd + 8) + evl::kEnginesPerXcd - 1) /
                                       evl::kEnginesPerXcd) / 8.0;
        // (whole rounds matter for the first two; with many rounds the in-order dispatch evens the end out)
        const double rounds = engine + (std::ceil(engine) - engine) * uniform * std::min(1.0, 2.0 / engine);
        const double tile_us = k.tile + k.tile_few_rows * rows_weighted / items + k.tile_busy * std::min(1.0, items / 256.0) +
                               (ws_rows == 0 ? k.tile_unsplit : 0.0);
        const double fixed = k.fixed + (ws_rows == 0 ? k.fixed_unsplit : 0.0);
        double t = std::max(longest * tile_us + fixed,
                            rounds * (mean * tile_us + fixed) * (1.0 + k.tail * (1.0 - uniform)));
        if (ws_rows > 0) t += k.merge + k.per_mb * (double)(ws_rows * row_bytes) * 1e-6;
        if (want == 1) unsplit_t = t;
        if (want == 1 || t < best_t) {
            best_t = t;
            best_ns = ns;
            best_len = len;
            best_rows = ws_rows;
        }
    }
    if (best_rows > 0 && unsplit_t > 0.0 && unsplit_t <= k.unsplit_margin * best_t) {
        best_ns.assign(n, 1);
        best_len = unsplit_len;
        best_rows = 0;
    }
    *n_splits = best_ns;
    *tps = best_len;
    return best_rows;
}

// Enqueue the attention kernel; when timing is switched on, an event pair takes the begin and
// end time of that dispatch.
static evl_status launch_attention(evl_cache *c, const evl::AttnParams &p) {
    const bool timed = !c->ev_start.empty();
    const size_t slot = timed ? (size_t)(c->ev_count % (int64_t)c->ev_start.size()) : 0;
    hipError_t e = evl::launch_chunk_attention(p, c->d.head_dim, (hipStream_t)c->d.stream,
                                               timed ? c->ev_start[slot] : nullptr,
                                               timed ? c->ev_stop[slot] : nullptr);
    if (e == hipSuccess) ++c->n_launches;
    if (e != hipSuccess)
        return fail(EVL_ERR_LAUNCH, "chunk_attention launch failed: %s", hipGetErrorString(e));
    if (timed) ++c->ev_count;
    return EVL_OK;
}

// One key range the rows attend to, with the position at which the queries are rotated for it.
struct Entry { int32_t begin, stop, causal; int64_t q_pos; int tiles; };

// ------------------------------------------------------------------------------------------
// Rows that see fewer than kFewKeys keys (the first tokens of a sequence, or of a sparsely
// sampled history) are served by a kernel of their own, in fp32; every call peels them off its
// chunks before it plans the matrix kernels, and hands those the rest of each chunk as a chunk
// that starts that many tokens later (the same result: how a chunk is cut never matters).
// ------------------------------------------------------------------------------------------
// Number of leading tokens of a chunk whose rows see fewer than kFewKeys keys, if `before` keys
// are visible to all of the chunk's tokens: token i sees before + i + 1.
static int32_t few_tokens(int64_t before, int32_t n_new) {
    return (int32_t)std::max<int64_t>(0, std::min<int64_t>(n_new, evl::kFewKeys - 1 - before));
}

struct FewGroup {
    int32_t bt_row, cache_len, n_few, tok_off;  // the group's first n_few tokens are served here
    std::vector<Entry> ent;                     // its key ranges, the causal one last
};

// Writes group g's entries into the launch's entry table from index `at` on.
static void fill_few_group(const evl_cache *c, evl::AttnParams *p, int at, const FewGroup &g) {
    for (size_t i = 0; i < g.ent.size(); ++i) {
        evl::AttnSeq &q = p->seq[at + (int)i];
        std::memset(&q, 0, sizeof(q));
        q.bt_row = g.bt_row;
        q.cache_len = g.cache_len;
        q.n_new = g.n_few;
        q.tok_off = g.tok_off;
        q.k_begin = g.ent[i].begin;
        // (the causal range ends with the last token served here)
        q.k_stop = g.ent[i].causal ? std::min(g.ent[i].stop, g.cache_len + g.n_few) : g.ent[i].stop;
        q.causal = g.ent[i].causal;
        q.q_pos = (int32_t)g.ent[i].q_pos;
        q.n_ent = i == 0 ? (int32_t)g.ent.size() : 0;
    }
}

// The groups from *next on ride along with an attention launch, as many as its entry table still
// has room for (behind the launch's own p->n_seqs entries, which must be final); *next advances.
static void attach_few(const evl_cache *c, evl::AttnParams *p, const std::vector<FewGroup> &groups, size_t *next) {
    int at = p->n_seqs;
    p->few_first = at;
    while (*next < groups.size() && at + (int)groups[*next].ent.size() <= evl::kMaxEntries) {
        const FewGroup &g = groups[*next];
        fill_few_group(c, p, at, g);
        at += (int)g.ent.size();
        p->few_rows += g.n_few * c->d.n_q_heads;
        ++*next;
    }
    p->few_entries = at - p->few_first;
}

// The groups from `next` on in launches of their own.
static evl_status few_keys_attention(evl_cache *c, const void *q_new, void *out, const std::vector<FewGroup> &groups,
                                     size_t next = 0) {
    while (next < groups.size()) {
        evl::AttnParams p;
        evl::CombineParams cp;
        // (partial results and counters are not used: every row is finished by its own wave)
        init_params(c, q_new, out, nullptr, nullptr, &p, &cp);
        attach_few(c, &p, groups, &next);
        hipError_t e = evl::launch_few_keys(p, c->d.head_dim, (hipStream_t)c->d.stream);
        if (e == hipSuccess) ++c->n_launches;
        if (e != hipSuccess)
            return fail(EVL_ERR_LAUNCH, "few-keys attention launch failed: %s", hipGetErrorString(e));
    }
    return EVL_OK;
}

// ------------------------------------------------------------------------------------------
// Chunks of a few tokens (at most 32 packed rows per KV head): the decode kernel, one wave per
// piece of the key range.  `ents`: the key ranges the rows attend to (one per sequence in the
// plain call; the retained runs and the chunk in the sampled call), grouped by rows: group g
// covers ents[first[g]] .. ents[first[g+1]-1].  Returns EVL_OK with *done = false if this launch
// is not one for the decode kernel (the caller then takes the general path).
// ------------------------------------------------------------------------------------------
struct DecodeEntry {
    int32_t bt_row, cache_len, n_new, tok_off, k_begin, k_stop, causal;
    int64_t q_pos;
    int64_t k_pos = 0;  // fused step only: position id of the chunk's first token
};
constexpr int kMinDecodeTilesPerPiece = 2;  // 64 keys

static evl_status decode_attention(evl_cache *c, const void *q_new, void *out,
                                   const std::vector<DecodeEntry> &ents, const std::vector<int> &first,
                                   bool *done, const evl::AppendParams *fused = nullptr) {
    *done = false;
    const int D = c->d.head_dim, Hq = c->d.n_q_heads, Hkv = c->d.n_kv_heads, G = c->group;
    const int n_groups = (int)first.size() - 1, E = (int)ents.size();
    if (E > evl::kMaxSeqs || n_groups * Hkv > evl::kCounters) return EVL_OK;
    int max_new = 0;
    for (const DecodeEntry &e : ents) {
        if (e.n_new * G > evl::kDecodeRows) return EVL_OK;
        max_new = std::max(max_new, e.n_new);
    }
    if (evl::decode_lds_bytes(D, max_new) > 160 * 1024) return EVL_OK;

    const int KT = evl::kDecodeTileKeys, W = evl::kDecodeWavesPerGroup;
    const size_t esz = c->d.out_dtype == EVL_OUT_F32 ? 4 : 2;
    const size_t row_bytes = (size_t)D * esz + 2 * sizeof(float);
    std::vector<int> tiles(E), pieces(E), tps(E), wgs(n_groups);
    int64_t all_tiles = 0;
    for (int i = 0; i < E; ++i) {
        tiles[i] = (ents[i].k_stop + KT - 1) / KT - ents[i].k_begin / KT;
        all_tiles += tiles[i];
    }
    // one piece length for the launch: about 140 work-groups of W pieces unless the caller set a target
    // (timed over 3520 / 20 656 / 65 536 cached tokens, 1 and 4 new: 110 to 150 work-groups are the
    // fastest everywhere -- 240, one per compute unit, cost 4 to 13 % more at the two longer histories,
    // more work-groups than that 20 to 35 %, 60 or fewer 15 to 60 %)
    const int64_t target = (int64_t)(c->tuned ? c->target_items : kDecodeTargetGroups) * W;
    // short histories (up to 64 work-groups' worth of single tiles): one tile per wave, so that the
    // few compute units in use pull less each; beyond that two tiles per piece keep the merge small
    const int64_t min_tiles = all_tiles * Hkv <= 64 * W ? 1 : kMinDecodeTilesPerPiece;
    int64_t T = std::max<int64_t>(min_tiles, (all_tiles * Hkv + target - 1) / target);
    size_t ws_rows = 0;
    for (;;) {
        ws_rows = 0;
        bool split = false;
        for (int g = 0; g < n_groups; ++g) {
            int np = 0;
            for (int i = first[g]; i < first[g + 1]; ++i) {
                const int n = (int)std::max<int64_t>(1, (tiles[i] + T - 1) / T);
                tps[i] = (tiles[i] + n - 1) / n;
                pieces[i] = (tiles[i] + tps[i] - 1) / tps[i];
                np += pieces[i];
            }
            wgs[g] = (np + W - 1) / W;
            if (wgs[g] > 1) {
                ws_rows += (size_t)wgs[g] * ents[first[g]].n_new * Hq;
                split = true;
            }
        }
        if (!split) break;
        if (counters_of(c) && ws_rows * row_bytes <= partials_capacity(c)) break;
        T *= 2;  // no room for the partial results (or for the counters): fewer, longer pieces
        if (T > (int64_t)1 << 40) return EVL_OK;
    }
    // A group's pieces are dealt to work-groups of W waves: with 9 pieces two work-groups would run
    // with 7 idle waves.  The group's pieces are made shorter until its work-groups are full (the
    // number of work-groups, and with it the partial rows, stays as it is).
    for (int g = 0; g < n_groups; ++g) {
        const int64_t budget = (int64_t)wgs[g] * W;
        auto pieces_at = [&](int64_t len) {
            int64_t np = 0;
            for (int i = first[g]; i < first[g + 1]; ++i) np += std::max<int64_t>(1, (tiles[i] + len - 1) / len);
            return np;
        };
        int64_t lo = min_tiles, hi = T;  // the shortest piece length whose pieces still fit the work-groups
        if (pieces_at(hi) > budget) continue;  // (pieces were counted after rounding: leave the group alone)
        while (lo < hi) {
            const int64_t mid = (lo + hi) / 2;
            if (pieces_at(mid) <= budget)
                hi = mid;
            else
                lo = mid + 1;
        }
        for (int i = first[g]; i < first[g + 1]; ++i) {
            const int n = (int)std::max<int64_t>(1, (tiles[i] + hi - 1) / hi);
            tps[i] = (tiles[i] + n - 1) / n;
            pieces[i] = (tiles[i] + tps[i] - 1) / tps[i];
        }
    }
    if (ws_rows > 0) {
        evl_status st = ready_counters(c);
        if (st != EVL_OK) return st;
    }

    void *part_o = c->d.workspace;
    float *part_ml = part_o ? (float *)((char *)part_o + ws_rows * D * esz) : nullptr;
    evl::AttnParams p;
    evl::CombineParams cp;
    init_params(c, q_new, out, part_o, part_ml, &p, &cp);
    p.n_seqs = E;
    p.tab_tokens = max_new;
    p.counters = ws_rows > 0 ? counters_of(c) : nullptr;
    if (fused) {
        p.k_new = fused->k_new;
        p.v_new = fused->v_new;
    }
    Plan plan;
    plan.workspace_used = ws_rows * row_bytes;
    size_t part_off = 0;
    int n_wg = 0;
    for (int g = 0; g < n_groups; ++g) {
        int pieces_before = 0;
        for (int i = first[g]; i < first[g + 1]; ++i) {
            const DecodeEntry &e = ents[i];
            evl::AttnSeq &q = p.seq[i];
            q.bt_row = e.bt_row;
            q.cache_len = e.cache_len;
            q.n_new = e.n_new;
            q.tok_off = e.tok_off;
            q.k_begin = e.k_begin;
            q.k_stop = e.k_stop;
            q.causal = e.causal;
            q.q_pos = (int32_t)e.q_pos;
            q.k_pos = (int32_t)e.k_pos;
            q.n_ent = i == first[g] ? first[g + 1] - first[g] : 0;
            q.n_splits = pieces[i];
            q.tiles_per_split = tps[i];
            q.m_tiles = 1;
            q.split_base = pieces_before;
            pieces_before += pieces[i];
            q.total_splits = wgs[g];
            q.cnt_base = g * Hkv;
            q.part_off = (int64_t)part_off;
        }
        if (wgs[g] > 1) part_off += (size_t)wgs[g] * ents[first[g]].n_new * Hq;
        n_wg += wgs[g] * Hkv;
        plan.max_splits = std::max(plan.max_splits, wgs[g]);
    }
    p.n_items = n_wg;
    plan.n_items = n_wg;
    const bool timed = !c->ev_start.empty();
    const size_t slot = timed ? (size_t)(c->ev_count % (int64_t)c->ev_start.size()) : 0;
    hipError_t e = evl::launch_decode_attention(p, D, n_wg, (hipStream_t)c->d.stream,
                                                timed ? c->ev_start[slot] : nullptr,
                                                timed ? c->ev_stop[slot] : nullptr, fused);
    if (e == hipSuccess) ++c->n_launches;
    if (e != hipSuccess)
        return fail(EVL_ERR_LAUNCH, "decode attention launch failed: %s", hipGetErrorString(e));
    if (timed) ++c->ev_count;
    c->last_plan = plan;
    *done = true;
    return EVL_OK;
}

static evl_status attention_batched_core(const void *q_new, evl_cache *c, const int32_t *seq_ids,
                                         const int32_t *cache_lens, const int32_t *n_new, const int32_t *tok_offs_in,
                                         int32_t n_seqs, void *out, const std::vector<FewGroup> &few,
                                         const PackShape *pack = nullptr);

evl_status evl_chunk_attention_batched(const void *q_new, evl_cache *c, const int32_t *seq_ids,
                                       const int32_t *cache_lens, const int32_t *n_new,
                                       int32_t n_seqs, void *out) {
    if (!c) return fail(EVL_ERR_NULL, "cache is NULL");
    if (!q_new || !out) return fail(EVL_ERR_NULL, "q_new / out is NULL");
    if (!seq_ids || !cache_lens || !n_new) return fail(EVL_ERR_NULL, "a host array is NULL");
    if (!aligned16(q_new) || !aligned16(out))
        return fail(EVL_ERR_ALIGN, "q_new / out must be 16-byte aligned");
    if (n_seqs <= 0 || n_seqs > c->d.max_seqs)
        return fail(EVL_ERR_ARG, "n_seqs %d outside [1, %d]", n_seqs, c->d.max_seqs);
    std::vector<char> seen(c->d.max_seqs, 0);
    for (int i = 0; i < n_seqs; ++i) {
        const int32_t s = seq_ids[i];
        evl_status st = check_seq(c, s);
        if (st != EVL_OK) return st;
        if (seen[s]) return fail(EVL_ERR_ARG, "sequence %d listed twice", s);
        seen[s] = 1;
        if (c->pack[s].action_tokens > 0)
            return fail(EVL_ERR_ARG, "sequence %d holds a pack: use evl_isolated_pack_attention", s);
        if (n_new[i] <= 0) return fail(EVL_ERR_ARG, "n_new[%d] = %d must be positive", i, n_new[i]);
        if (cache_lens[i] < 0) return fail(EVL_ERR_ARG, "cache_lens[%d] is negative", i);
        if ((int64_t)cache_lens[i] + n_new[i] > c->len[s])
            return fail(EVL_ERR_RANGE,
                        "sequence %d: cache_len %d + n_new %d exceeds the %lld appended tokens", s,
                        cache_lens[i], n_new[i], (long long)c->len[s]);
    }

    // rows that see fewer than kFewKeys keys go to their own kernel; the matrix kernels get what
    // is left of each chunk
    std::vector<int32_t> ids, lens, ns, offs;
    std::vector<FewGroup> few;
    int64_t off = 0;
    for (int i = 0; i < n_seqs; ++i) {
        const int32_t a = few_tokens(cache_lens[i], n_new[i]);
        if (a > 0)
            few.push_back(FewGroup{seq_ids[i], cache_lens[i], a, (int32_t)off,
                                   {Entry{0, cache_lens[i] + a, 1, c->pos0[seq_ids[i]] + cache_lens[i], 0}}});
        if (a < n_new[i]) {
            ids.push_back(seq_ids[i]);
            lens.push_back(cache_lens[i] + a);
            ns.push_back(n_new[i] - a);
            offs.push_back((int32_t)(off + a));
        }
        off += n_new[i];
    }
    if (ids.empty()) {
        c->last_plan = Plan();
        return few_keys_attention(c, q_new, out, few);
    }
    return attention_batched_core(q_new, c, ids.data(), lens.data(), ns.data(), offs.data(), (int32_t)ids.size(), out,
                                  few);
}

// The plain call on chunks whose rows all see at least kFewKeys keys (arguments checked by the
// caller); tok_offs[i]: first token of chunk i in q_new / out.  few: the rows that were peeled
// off, which travel with the first attention launch(es) or, behind the decode kernel, alone.
static evl_status attention_batched_core(const void *q_new, evl_cache *c, const int32_t *seq_ids,
                                         const int32_t *cache_lens, const int32_t *n_new, const int32_t *tok_offs_in,
                                         int32_t n_seqs, void *out, const std::vector<FewGroup> &few,
                                         const PackShape *pack) {
    const int D = c->d.head_dim, Hq = c->d.n_q_heads, Hkv = c->d.n_kv_heads, G = c->group;
    const int MT = evl::attention_rows_per_workgroup();
    const int KN = evl::kKeyTile;

    // chunks of a few tokens everywhere: the decode kernel (which knows nothing of packs)
    if (!pack) {
        std::vector<DecodeEntry> ents(n_seqs);
        std::vector<int> first(n_seqs + 1);
        for (int i = 0; i < n_seqs; ++i) {
            ents[i] = DecodeEntry{seq_ids[i], cache_lens[i], n_new[i], tok_offs_in[i], 0, cache_lens[i] + n_new[i], 1,
                                  c->pos0[seq_ids[i]] + cache_lens[i]};
            first[i] = i;
        }
        first[n_seqs] = n_seqs;
        bool done = false;
        evl_status st = decode_attention(c, q_new, out, ents, first, &done);
        if (st != EVL_OK) return st;
        if (done) return few_keys_attention(c, q_new, out, few);
    }

    // ---- partition: one split length (in key tiles) for the whole launch, so that every
    // work-group has about the same amount of work whatever its sequence's length ----
    std::vector<int> m_tiles(n_seqs), tiles(n_seqs);
    int64_t base_items = 0, work = 0;
    for (int i = 0; i < n_seqs; ++i) {
        m_tiles[i] = (n_new[i] * G + MT - 1) / MT;
        tiles[i] = (cache_lens[i] + n_new[i] + KN - 1) / KN;
        base_items += (int64_t)m_tiles[i] * Hkv;
        work += (int64_t)m_tiles[i] * Hkv * tiles[i];
    }
    // a partial row: d outputs in the output's element type, then (reference, sum) as floats
    const size_t esz = c->d.out_dtype == EVL_OUT_F32 ? 4 : 2;
    const size_t row_bytes = (size_t)D * esz + 2 * sizeof(float);
    // One split length T (in key tiles) for the whole launch, so that work-groups carry about
    // the same amount of work whatever their sequence's length.  A launch that already has more
    // row tiles than the target (a ragged batch) aims for eight work-groups per CU instead, so
    // that the hardware's in-order dispatch can even out what is left of the imbalance.
    const int64_t target = base_items > c->target_items ? std::max<int64_t>(c->target_items, 2048)
                                                        : c->target_items;
    int64_t T = std::max<int64_t>(kMinTilesPerSplit, (work + target - 1) / target);
    std::vector<int> n_splits(n_seqs), tps(n_seqs);
    size_t ws_rows = 0;
    for (;;) {
        ws_rows = 0;
        for (int i = 0; i < n_seqs; ++i) {
            int ns = (int)std::min<int64_t>(kMaxSplits, (tiles[i] + T - 1) / T);
            ns = std::max(ns, 1);
            tps[i] = (tiles[i] + ns - 1) / ns;
            n_splits[i] = (tiles[i] + tps[i] - 1) / tps[i];
            if (n_splits[i] > 1) ws_rows += (size_t)n_splits[i] * n_new[i] * Hq;
        }
        if (ws_rows * row_bytes <= partials_capacity(c) || ws_rows == 0) break;
        T *= 2;  // workspace too small: split less
    }
    // unless the caller set a target, the plan is priced instead: how many pieces, if any (with long
    // chunks over short histories -- a prefill -- a split costs more than it brings)
    if (!c->tuned) {
        if (n_seqs == 1) {  // one set of rows: the number of pieces is searched, not derived from a target
            std::vector<int> see(m_tiles[0]);  // key tiles row tile mt sees under the causal mask
            for (int mt = 0; mt < m_tiles[0]; ++mt)
                see[mt] = (cache_lens[0] + (std::min((mt + 1) * MT, n_new[0] * G) - 1) / G + 1 + KN - 1) / KN;
            n_splits[0] = pick_pieces(see, Hkv, D, tiles[0], (size_t)n_new[0] * Hq, row_bytes,
                                      c->d.workspace ? partials_capacity(c) : 0, &tps[0]);
            ws_rows = n_splits[0] > 1 ? (size_t)n_splits[0] * n_new[0] * Hq : 0;
        } else {  // several sequences: one piece length for all of them, priced the same way
            std::vector<double> mean_see(n_seqs);
            std::vector<size_t> rows(n_seqs);
            for (int i = 0; i < n_seqs; ++i) {
                double sum = 0.0;
                for (int mt = 0; mt < m_tiles[i]; ++mt)
                    sum += (cache_lens[i] + (std::min((mt + 1) * MT, n_new[i] * G) - 1) / G + 1 + KN - 1) / KN;
                mean_see[i] = sum / std::max(m_tiles[i], 1);
                rows[i] = (size_t)n_new[i] * Hq;
            }
            ws_rows = pick_piece_length(m_tiles, tiles, mean_see, rows, Hkv, D, row_bytes,
                                        c->d.workspace ? partials_capacity(c) : 0, &n_splits, &tps);
        }
    }

    // Longest sequences first: their work-groups are dispatched first and the short ones fill
    // the gaps at the end.  Inputs and outputs keep the caller's order (tok_offs).
    std::vector<int> order(n_seqs);
    std::vector<int64_t> tok_offs(n_seqs);
    {
        for (int i = 0; i < n_seqs; ++i) {
            order[i] = i;
            tok_offs[i] = tok_offs_in[i];
        }
        std::stable_sort(order.begin(), order.end(),
                         [&](int a, int b) { return tiles[a] > tiles[b]; });
    }

    void *part_o = c->d.workspace;
    // all O partials first, then all (m, l) pairs; both regions stay 16-byte aligned
    float *part_ml = part_o ? (float *)((char *)part_o + ws_rows * D * esz) : nullptr;

    Plan plan;
    plan.workspace_used = ws_rows * row_bytes;
    size_t part_off = 0, few_next = 0;
    for (int base = 0; base < n_seqs; base += evl::kMaxSeqs) {
        const int cnt = std::min(evl::kMaxSeqs, n_seqs - base);
        evl::AttnParams p;
        evl::CombineParams cp;
        init_params(c, q_new, out, part_o, part_ml, &p, &cp);
        p.n_seqs = cnt;
        if (pack) {
            p.hole_first = pack->prefix;
            p.hole_period = pack->frame_tokens + pack->action_tokens;
            p.hole_width = pack->action_tokens;
        }
        attach_few(c, &p, few, &few_next);
        int items = 0, crow = 0, cseqs = 0;
        int per_xcd[8] = {0, 0, 0, 0, 0, 0, 0, 0}, xcd_next = 0;
        for (int i = 0; i < cnt; ++i) {
            const int k = order[base + i];
            const int64_t tok_off = tok_offs[k];
            evl::AttnSeq &q = p.seq[i];
            q.bt_row = seq_ids[k];
            q.cache_len = cache_lens[k];
            q.n_new = n_new[k];
            q.tok_off = (int32_t)tok_off;
            q.k_begin = 0;
            q.k_stop = cache_lens[k] + n_new[k];
            q.causal = 1;
            q.n_ent = 1;
            q.n_splits = n_splits[k];
            q.split_base = 0;
            q.total_splits = n_splits[k];
            q.tiles_per_split = tps[k];
            q.m_tiles = m_tiles[k];
            q.part_off = (int64_t)part_off;
            q.q_pos = (int32_t)(c->pos0[seq_ids[k]] + cache_lens[k]);
            const int groups = n_splits[k] * Hkv;
            Chunking ck = choose_chunking(groups, m_tiles[k]);
            if (tile_major_pays(n_splits[k], groups, m_tiles[k])) {
                ck = Chunking{evl::kXcdChunkRowTiles, 0, 0};
                q.tile_major = 1;
            }
            add_xcd_load(per_xcd, &xcd_next, &q, groups, m_tiles[k], ck);
            items += m_tiles[k] * groups;
            plan.max_splits = std::max(plan.max_splits, n_splits[k]);
            if (n_splits[k] > 1) {
                evl::CombineSeq &cs = cp.seq[cseqs++];
                cs.n_new = n_new[k];
                cs.tok_off = (int32_t)tok_off;
                cs.n_splits = n_splits[k];
                cs.row_begin = crow;
                cs.part_off = (int64_t)part_off;
                crow += n_new[k] * Hq;
                part_off += (size_t)n_splits[k] * n_new[k] * Hq;
            }
        }
        p.n_items = items;
        p.items_per_xcd = *std::max_element(per_xcd, per_xcd + 8);
        cp.n_seqs = cseqs;
        cp.n_rows = crow;
        plan.n_items += items;
        evl_status st = launch_attention(c, p);
        if (st != EVL_OK) return st;
        if (crow > 0) {
            hipError_t e = evl::launch_combine(cp, D, (hipStream_t)c->d.stream);
            if (e == hipSuccess) ++c->n_launches;
            if (e != hipSuccess)
                return fail(EVL_ERR_LAUNCH, "combine launch failed: %s", hipGetErrorString(e));
        }
    }
    c->last_plan = plan;
    return few_keys_attention(c, q_new, out, few, few_next);
}

evl_status evl_chunk_attention(const void *q_new, evl_cache *cache, int32_t cache_len,
                               int32_t n_new, void *out) {
    const int32_t seq = 0;
    return evl_chunk_attention_batched(q_new, cache, &seq, &cache_len, &n_new, 1, out);
}

// The same call for callers that cannot allocate device memory: partial results and ticket
// counters live in the library's own static device array instead of the cache's workspace.
evl_status evl_chunk_attention_static(const void *q_new, evl_cache *c, int32_t cache_len, int32_t n_new,
                                      void *out) {
    if (!c) return fail(EVL_ERR_NULL, "cache is NULL");
    if (n_new > 0 && (int64_t)n_new * c->d.n_q_heads > evl::kStaticScratchMaxRows)
        return fail(EVL_ERR_WORKSPACE,
                    "evl_chunk_attention_static serves chunks of at most %d (token, query head) rows; "
                    "%d tokens x %d heads = %lld", evl::kStaticScratchMaxRows, n_new, c->d.n_q_heads,
                    (long long)n_new * c->d.n_q_heads);
    void *ptr = nullptr;
    size_t bytes = 0;
    hipError_t e = evl::static_scratch(&ptr, &bytes);
    if (e != hipSuccess)
        return fail(EVL_ERR_LAUNCH, "the static scratch array is not available: %s", hipGetErrorString(e));
    // The array is shared by every call on this GPU and keeps what the last one left: the ticket
    // counters are cleared (by a fill kernel on the stream) whenever this call is going to use them.
    void *const ws = c->d.workspace;
    const size_t ws_bytes = c->d.workspace_bytes;
    const bool zeroed = c->counters_zeroed;
    c->d.workspace = ptr;
    c->d.workspace_bytes = bytes;
    c->counters_zeroed = false;
    const int32_t seq = 0;
    const evl_status st = evl_chunk_attention_batched(q_new, c, &seq, &cache_len, &n_new, 1, out);
    c->d.workspace = ws;
    c->d.workspace_bytes = ws_bytes;
    c->counters_zeroed = zeroed;
    return st;
}

// ------------------------------------------------------------------------------------------
// A whole step: append, then attend from the appended chunk
// ------------------------------------------------------------------------------------------
evl_status evl_step_batched(evl_cache *c, const void *q_new, const void *k_new, const void *v_new,
                            const int32_t *seq_ids, const int64_t *pos_offsets, const int32_t *n_new,
                            int32_t n_seqs, void *out) {
    if (!q_new || !out) return fail(EVL_ERR_NULL, "q_new / out is NULL");
    if (!aligned16(q_new) || !aligned16(out)) return fail(EVL_ERR_ALIGN, "q_new / out must be 16-byte aligned");
    evl_status st = check_append(c, k_new, v_new, seq_ids, pos_offsets, n_new, n_seqs);
    if (st != EVL_OK) return st;
    std::vector<int32_t> cache_lens(n_seqs);
    for (int i = 0; i < n_seqs; ++i) cache_lens[i] = (int32_t)c->len[seq_ids[i]];
    // chunks of a few tokens everywhere: one launch appends and attends (unless some sequence is
    // still so short that its rows go to the few-keys kernel)
    bool short_history = false;
    for (int i = 0; i < n_seqs; ++i) short_history = short_history || few_tokens(cache_lens[i], n_new[i]) > 0;
    if (n_seqs <= evl::kMaxSeqs && !short_history) {
        std::vector<DecodeEntry> ents(n_seqs);
        std::vector<int> first(n_seqs + 1);
        int64_t off = 0;
        for (int i = 0; i < n_seqs; ++i) {
            ents[i] = DecodeEntry{seq_ids[i], cache_lens[i], n_new[i], (int32_t)off, 0, cache_lens[i] + n_new[i], 1,
                                  pos_offsets[i], pos_offsets[i]};
            first[i] = i;
            off += n_new[i];
        }
        first[n_seqs] = n_seqs;
        evl::AppendParams a;
        int64_t tok_off = 0;
        fill_append(c, k_new, v_new, seq_ids, pos_offsets, n_new, 0, n_seqs, &tok_off, &a);
        bool done = false;
        st = decode_attention(c, q_new, out, ents, first, &done, &a);
        if (st != EVL_OK) return st;
        if (done) {
            commit_append(c, seq_ids, pos_offsets, n_new, 0, n_seqs);
            return EVL_OK;
        }
    }
    // otherwise the two calls, one after the other
    st = evl_rope_append_batched(c, k_new, v_new, seq_ids, pos_offsets, n_new, n_seqs);
    if (st != EVL_OK) return st;
    return evl_chunk_attention_batched(q_new, c, seq_ids, cache_lens.data(), n_new, n_seqs, out);
}

evl_status evl_step(evl_cache *cache, const void *q_new, const void *k_new, const void *v_new,
                    int64_t pos_offset, int32_t n_new, void *out) {
    const int32_t seq = 0;
    return evl_step_batched(cache, q_new, k_new, v_new, &seq, &pos_offset, &n_new, 1, out);
}

// ------------------------------------------------------------------------------------------
// Chunk attention over a sampled history
// ------------------------------------------------------------------------------------------
// Key tiles of the attention kernel that cover an entry's key range: the tiles start at the page
// that holds the range's first key (the kernel derives the same from the range).
static int entry_tiles(int32_t begin, int32_t stop) {
    const int KN = evl::kKeyTile, PG = evl::kPage;
    const int sh = (begin / PG % (KN / PG)) * PG;
    return (stop - sh + KN - 1) / KN - begin / KN;
}

// Checks one (sequence, runs, chunk) and turns it into entries: runs that touch each other share
// a shift and merge; a run that ends where the chunk begins merges with the chunk.
// appended: the chunk already sits in the cache behind cache_len (the attention calls); otherwise
// it is about to be appended at the sequence's end (the one-call step), whose first token gets
// position id pos_chunk.
static evl_status build_entries(const evl_cache *c, int32_t seq, const evl_run *runs, int32_t n_runs,
                                int32_t cache_len, int32_t n_new, std::vector<Entry> *out, bool appended = true,
                                int64_t pos_chunk = 0) {
    std::vector<Entry> &ent = *out;
    ent.clear();
    if (n_runs < 0 || (n_runs > 0 && !runs)) return fail(EVL_ERR_NULL, "runs is NULL");
    evl_status st = check_seq(c, seq);
    if (st != EVL_OK) return st;
    if (c->pack[seq].action_tokens > 0)
        return fail(EVL_ERR_ARG, "sequence %d holds a pack: use evl_isolated_pack_attention", seq);
    if (n_new <= 0) return fail(EVL_ERR_ARG, "n_new = %d must be positive", n_new);
    if (cache_len < 0) return fail(EVL_ERR_ARG, "cache_len is negative");
    if (appended && (int64_t)cache_len + n_new > c->len[seq])
        return fail(EVL_ERR_RANGE, "sequence %d: cache_len %d + n_new %d exceeds the %lld appended tokens",
                    seq, cache_len, n_new, (long long)c->len[seq]);
    const int64_t pos0 = appended ? c->pos0[seq] : pos_chunk - cache_len;
    int64_t retained = 0, prev_end = 0;
    for (int r = 0; r < n_runs; ++r) {
        if (runs[r].len <= 0 || runs[r].start < prev_end || (int64_t)runs[r].start + runs[r].len > cache_len)
            return fail(EVL_ERR_ARG,
                        "run %d = [%d, +%d): runs must be non-empty, ascending, disjoint and "
                        "inside [0, cache_len = %d)", r, runs[r].start, runs[r].len, cache_len);
        prev_end = (int64_t)runs[r].start + runs[r].len;
        retained += runs[r].len;
    }
    int64_t u = 0;  // combined index of the next run's first token
    for (int r = 0; r <= n_runs; ++r) {
        const int32_t start = r < n_runs ? runs[r].start : cache_len;
        const int32_t len = r < n_runs ? runs[r].len : n_new;
        if (!ent.empty() && ent.back().stop == start) {
            ent.back().stop = start + len;
        } else {
            Entry e;
            e.begin = start;
            e.stop = start + len;
            e.causal = 0;
            e.q_pos = pos0 + retained + (start - u);
            e.tiles = 0;
            ent.push_back(e);
        }
        u += len;
    }
    ent.back().causal = 1;
    if (ent.back().q_pos + n_new > INT32_MAX) return fail(EVL_ERR_ARG, "position ids beyond 2^31");
    return EVL_OK;
}

// The stored key of sequence index t carries the rotation of id pos0 + t.  In the combined
// sequence "retained runs + chunk" the token at index t of a run that starts at `start` and
// lands at combined index u_start sits at id pos0 + u_start + (t - start).  Scores depend on
// the difference of the two ids only, so rotating the query of chunk token i at
//     pos0 + R + i + (start - u_start)          (R = retained tokens)
// against the stored key gives the score the combined sequence's contiguous ids define.
// Each run with its own shift is one entry of the launch; a work-group walks through the
// entries of its piece of the key tiles and shifts its queries' rotation from one to the next.
evl_status evl_chunk_attention_sampled(const void *q_new, evl_cache *c, int32_t seq,
                                       const evl_run *runs, int32_t n_runs, int32_t cache_len,
                                       int32_t n_new, void *out) {
    if (!c) return fail(EVL_ERR_NULL, "cache is NULL");
    if (!q_new || !out) return fail(EVL_ERR_NULL, "q_new / out is NULL");
    if (!aligned16(q_new) || !aligned16(out))
        return fail(EVL_ERR_ALIGN, "q_new / out must be 16-byte aligned");
    evl_status st;
    std::vector<Entry> ent;
    st = build_entries(c, seq, runs, n_runs, cache_len, n_new, &ent);
    if (st != EVL_OK) return st;
    const int E = (int)ent.size();

    // rows that see fewer than kFewKeys keys (a sparse history and the chunk's first tokens) go to
    // their own kernel; what follows sees the rest of the chunk, which starts tok0 tokens later
    int32_t tok0 = 0;
    std::vector<FewGroup> few;
    size_t few_next = 0;
    {
        int64_t retained = 0;
        for (int r = 0; r < n_runs; ++r) retained += runs[r].len;
        tok0 = few_tokens(retained, n_new);
        if (tok0 > 0) {
            few.push_back(FewGroup{seq, cache_len, tok0, 0, ent});
            if (tok0 == n_new) {
                c->last_plan = Plan();
                return few_keys_attention(c, q_new, out, few);
            }
            for (Entry &e : ent) e.q_pos += tok0;
            cache_len += tok0;
            n_new -= tok0;
        }
    }

    const int D = c->d.head_dim, Hq = c->d.n_q_heads, Hkv = c->d.n_kv_heads, G = c->group;
    const int MT = evl::attention_rows_per_workgroup();
    const int m_tiles = (n_new * G + MT - 1) / MT;

    // a chunk of a few tokens: the decode kernel, every run a key range with its own query position
    {
        std::vector<DecodeEntry> dents(E);
        for (int i = 0; i < E; ++i)
            dents[i] = DecodeEntry{seq, cache_len, n_new, tok0, ent[i].begin, ent[i].stop, ent[i].causal, ent[i].q_pos};
        const std::vector<int> first = {0, E};
        bool done = false;
        st = decode_attention(c, q_new, out, dents, first, &done);
        if (st != EVL_OK) return st;
        if (done) return few_keys_attention(c, q_new, out, few);
    }

    // ---- partition.  The entries' key tiles are laid end to end and cut into pieces of one
    // length; a work-group walks through the entries of its piece, so a piece costs about the
    // same whatever it is made of.  One launch describes at most kMaxSeqs entries: more
    // entries make several groups, each cut into its own pieces. ----
    const int n_groups = (E + evl::kMaxSeqs - 1) / evl::kMaxSeqs;
    std::vector<int64_t> g_tiles(n_groups, 0);
    int64_t all_tiles = 0;
    for (int i = 0; i < E; ++i) {
        ent[i].tiles = entry_tiles(ent[i].begin, ent[i].stop);
        g_tiles[i / evl::kMaxSeqs] += ent[i].tiles;
        all_tiles += ent[i].tiles;
    }
    const int64_t base_items = (int64_t)m_tiles * Hkv * n_groups;
    const int64_t work = (int64_t)m_tiles * Hkv * all_tiles;
    const size_t esz = c->d.out_dtype == EVL_OUT_F32 ? 4 : 2;
    const size_t row_bytes = (size_t)D * esz + 2 * sizeof(float);
    const int64_t target = base_items > c->target_items ? std::max<int64_t>(c->target_items, 2048)
                                                        : c->target_items;
    int64_t T = std::max<int64_t>(kMinTilesPerSplit, (work + target - 1) / target);
    std::vector<int> g_splits(n_groups), g_tps(n_groups);
    int total_splits = 0;
    size_t ws_rows = 0;
    for (;;) {
        total_splits = 0;
        for (int g = 0; g < n_groups; ++g) {
            int ns = (int)std::min<int64_t>(kMaxSplits, (g_tiles[g] + T - 1) / T);
            ns = std::max(ns, 1);
            g_tps[g] = (int)((g_tiles[g] + ns - 1) / ns);
            g_splits[g] = (int)((g_tiles[g] + g_tps[g] - 1) / g_tps[g]);
            total_splits += g_splits[g];
        }
        ws_rows = total_splits > 1 ? (size_t)total_splits * n_new * Hq : 0;
        if (ws_rows * row_bytes <= partials_capacity(c)) break;
        if (total_splits == n_groups)
            return fail(EVL_ERR_WORKSPACE,
                        "%d runs take %d launches, whose results need %zu workspace bytes to be merged; "
                        "the cache has room for %zu", E, n_groups, ws_rows * row_bytes, partials_capacity(c));
        T *= 2;
    }

    // one group and no target set by the caller: the number of pieces is priced like the plain call's
    // (a history handed over as one run then gets the plain call's plan, and its bits)
    if (n_groups == 1 && !c->tuned) {
        std::vector<int> see(m_tiles);  // key tiles row tile mt sees: all of the runs, the chunk up to its own tokens
        const Entry &last = ent.back();
        for (int mt = 0; mt < m_tiles; ++mt) {
            const int last_tok = (std::min((mt + 1) * MT, n_new * G) - 1) / G;
            const int64_t stop = std::min<int64_t>(last.stop, (int64_t)cache_len + last_tok + 1);
            see[mt] = (int)(all_tiles - last.tiles + entry_tiles(last.begin, (int32_t)std::max<int64_t>(stop, last.begin + 1)));
        }
        g_splits[0] = pick_pieces(see, Hkv, D, all_tiles, (size_t)n_new * Hq, row_bytes,
                                  c->d.workspace ? partials_capacity(c) : 0, &g_tps[0]);
        total_splits = g_splits[0];
        ws_rows = total_splits > 1 ? (size_t)total_splits * n_new * Hq : 0;
    }

    void *part_o = c->d.workspace;
    float *part_ml = part_o ? (float *)((char *)part_o + ws_rows * D * esz) : nullptr;
    Plan plan;
    plan.workspace_used = ws_rows * row_bytes;
    evl::CombineParams cp;
    int split_base = 0;
    for (int g = 0; g < n_groups; ++g) {
        const int base = g * evl::kMaxSeqs;
        const int cnt = std::min(evl::kMaxSeqs, E - base);
        evl::AttnParams p;
        init_params(c, q_new, out, part_o, part_ml, &p, &cp);
        p.n_seqs = cnt;
        p.multi_entry = cnt > 1;
        attach_few(c, &p, few, &few_next);
        for (int i = 0; i < cnt; ++i) {
            const Entry &e = ent[base + i];
            evl::AttnSeq &q = p.seq[i];
            q.bt_row = seq;
            q.cache_len = cache_len;
            q.n_new = n_new;
            q.tok_off = tok0;
            q.k_begin = e.begin;
            q.k_stop = e.stop;
            q.causal = e.causal;
            q.q_pos = (int32_t)e.q_pos;
            q.n_ent = i == 0 ? cnt : 0;
            q.n_splits = i == 0 ? g_splits[g] : 0;
            q.tiles_per_split = g_tps[g];
            q.m_tiles = m_tiles;
            q.split_base = split_base;
            q.total_splits = total_splits;
            q.part_off = 0;
        }
        int per_xcd[8] = {0, 0, 0, 0, 0, 0, 0, 0}, xcd_next = 0;
        add_xcd_load(per_xcd, &xcd_next, &p.seq[0], g_splits[g] * Hkv, m_tiles, choose_chunking(g_splits[g] * Hkv, m_tiles));
        p.n_items = m_tiles * g_splits[g] * Hkv;
        p.items_per_xcd = *std::max_element(per_xcd, per_xcd + 8);
        plan.n_items += p.n_items;
        split_base += g_splits[g];
        st = launch_attention(c, p);
        if (st != EVL_OK) return st;
    }
    if (total_splits > 1) {
        cp.n_seqs = 1;
        cp.n_rows = n_new * Hq;
        cp.seq[0].n_new = n_new;
        cp.seq[0].tok_off = tok0;
        cp.seq[0].n_splits = total_splits;
        cp.seq[0].row_begin = 0;
        cp.seq[0].part_off = 0;
        hipError_t e = evl::launch_combine(cp, D, (hipStream_t)c->d.stream);
        if (e == hipSuccess) ++c->n_launches;
        if (e != hipSuccess)
            return fail(EVL_ERR_LAUNCH, "combine launch failed: %s", hipGetErrorString(e));
    }
    plan.max_splits = total_splits;
    c->last_plan = plan;
    return few_keys_attention(c, q_new, out, few, few_next);
}

// The sampled call as a whole step: append, then attend over the retained runs and the chunk.
evl_status evl_step_sampled(evl_cache *c, const void *q_new, const void *k_new, const void *v_new, int32_t seq,
                            const evl_run *runs, int32_t n_runs, int64_t pos_offset, int32_t n_new, void *out) {
    if (!q_new || !out) return fail(EVL_ERR_NULL, "q_new / out is NULL");
    if (!aligned16(q_new) || !aligned16(out)) return fail(EVL_ERR_ALIGN, "q_new / out must be 16-byte aligned");
    evl_status st = check_append(c, k_new, v_new, &seq, &pos_offset, &n_new, 1);
    if (st != EVL_OK) return st;
    const int32_t cache_len = (int32_t)c->len[seq];
    std::vector<Entry> ent;
    st = build_entries(c, seq, runs, n_runs, cache_len, n_new, &ent, false, pos_offset);
    if (st != EVL_OK) return st;
    const int E = (int)ent.size();
    int64_t retained = 0;
    for (int r = 0; r < n_runs; ++r) retained += runs[r].len;
    if (E <= evl::kMaxSeqs && few_tokens(retained, n_new) == 0) {
        std::vector<DecodeEntry> dents(E);
        for (int i = 0; i < E; ++i)
            dents[i] = DecodeEntry{seq, cache_len, n_new, 0, ent[i].begin, ent[i].stop, ent[i].causal, ent[i].q_pos,
                                   pos_offset};
        const std::vector<int> first = {0, E};
        evl::AppendParams a;
        int64_t tok_off = 0;
        fill_append(c, k_new, v_new, &seq, &pos_offset, &n_new, 0, 1, &tok_off, &a);
        bool done = false;
        st = decode_attention(c, q_new, out, dents, first, &done, &a);
        if (st != EVL_OK) return st;
        if (done) {
            commit_append(c, &seq, &pos_offset, &n_new, 0, 1);
            return EVL_OK;
        }
    }
    // More runs than one launch describes: their results are merged through the workspace.  If it
    // cannot hold them the attention call would refuse; say so before anything is appended.
    const int n_launches = (E + evl::kMaxSeqs - 1) / evl::kMaxSeqs;
    if (n_launches > 1) {
        const size_t esz = c->d.out_dtype == EVL_OUT_F32 ? 4 : 2;
        const size_t need = (size_t)n_launches * n_new * c->d.n_q_heads * ((size_t)c->d.head_dim * esz + 2 * sizeof(float));
        if (need > partials_capacity(c))
            return fail(EVL_ERR_WORKSPACE,
                        "%d runs take %d launches, whose results need %zu workspace bytes to be merged; "
                        "the cache has room for %zu", E, n_launches, need, partials_capacity(c));
    }
    st = evl_rope_append_batched(c, k_new, v_new, &seq, &pos_offset, &n_new, 1);
    if (st != EVL_OK) return st;
    return evl_chunk_attention_sampled(q_new, c, seq, runs, n_runs, cache_len, n_new, out);
}

// Several (sequence, runs, chunk) groups in one call.  A group's entries stay together in one
// launch (at most kMaxEntries entries and kMaxSeqs groups per launch); all groups share one
// piece length.
evl_status evl_chunk_attention_sampled_batched(const void *q_new, evl_cache *c, int32_t n_groups_in,
                                               const int32_t *seq_ids_in, const int32_t *cache_lens_in,
                                               const int32_t *n_new_in, const int32_t *tok_offs,
                                               const int32_t *run_offsets, const evl_run *runs, void *out) {
    if (!c) return fail(EVL_ERR_NULL, "cache is NULL");
    if (!q_new || !out) return fail(EVL_ERR_NULL, "q_new / out is NULL");
    if (!seq_ids_in || !cache_lens_in || !n_new_in || !run_offsets) return fail(EVL_ERR_NULL, "a host array is NULL");
    if (!aligned16(q_new) || !aligned16(out))
        return fail(EVL_ERR_ALIGN, "q_new / out must be 16-byte aligned");
    if (n_groups_in <= 0) return fail(EVL_ERR_ARG, "n_groups = %d must be positive", n_groups_in);

    const int D = c->d.head_dim, Hq = c->d.n_q_heads, Hkv = c->d.n_kv_heads, G = c->group;
    const int MT = evl::attention_rows_per_workgroup();
    struct Group { int first, count, m_tiles, n_splits, tps; int64_t tiles; int32_t tok_off; };
    std::vector<Entry> ent;       // all groups' entries, group after group
    std::vector<Group> grp;
    std::vector<FewGroup> few;    // the leading tokens of groups whose rows see fewer than kFewKeys keys
    std::vector<int32_t> g_seq, g_len, g_new;  // the groups the matrix kernels serve (what is left of each chunk)
    int64_t tok = 0;
    for (int g = 0; g < n_groups_in; ++g) {
        if (run_offsets[g + 1] < run_offsets[g])
            return fail(EVL_ERR_ARG, "run_offsets must not decrease (group %d)", g);
        std::vector<Entry> e;
        const evl_run *g_runs = runs ? runs + run_offsets[g] : nullptr;
        const int32_t g_n_runs = run_offsets[g + 1] - run_offsets[g];
        evl_status st = build_entries(c, seq_ids_in[g], g_runs, g_n_runs, cache_lens_in[g], n_new_in[g], &e);
        if (st != EVL_OK) return st;
        if ((int)e.size() > evl::kMaxSeqs)
            return fail(EVL_ERR_UNSUPPORTED, "group %d has %d runs with different shifts; a batched call takes "
                                             "at most %d per group", g, (int)e.size(), evl::kMaxSeqs);
        if (tok_offs && (tok_offs[g] < 0 || ((int64_t)tok_offs[g] * Hq * D * 2) % 16))
            return fail(EVL_ERR_ARG, "tok_offs[%d] = %d", g, tok_offs[g]);
        const int32_t g_tok = tok_offs ? tok_offs[g] : (int32_t)tok;
        tok += n_new_in[g];
        int64_t retained = 0;
        for (int r = 0; r < g_n_runs; ++r) retained += g_runs[r].len;
        const int32_t a = few_tokens(retained, n_new_in[g]);
        if (a > 0) few.push_back(FewGroup{seq_ids_in[g], cache_lens_in[g], a, g_tok, e});
        if (a == n_new_in[g]) continue;
        Group gr;
        gr.first = (int)ent.size();
        gr.count = (int)e.size();
        gr.m_tiles = ((n_new_in[g] - a) * G + MT - 1) / MT;
        gr.tok_off = g_tok + a;
        gr.tiles = 0;
        gr.n_splits = 1;
        gr.tps = 0;
        for (Entry &x : e) {
            x.q_pos += a;
            x.tiles = entry_tiles(x.begin, x.stop);
            gr.tiles += x.tiles;
        }
        ent.insert(ent.end(), e.begin(), e.end());
        grp.push_back(gr);
        g_seq.push_back(seq_ids_in[g]);
        g_len.push_back(cache_lens_in[g] + a);
        g_new.push_back(n_new_in[g] - a);
    }
    if (grp.empty()) {
        c->last_plan = Plan();
        return few_keys_attention(c, q_new, out, few);
    }
    size_t few_next = 0;
    const int n_groups = (int)grp.size();
    const int32_t *seq_ids = g_seq.data(), *cache_lens = g_len.data(), *n_new = g_new.data();

    // chunks of a few tokens everywhere: the decode kernel
    if ((int)ent.size() <= evl::kMaxSeqs) {
        std::vector<DecodeEntry> dents(ent.size());
        std::vector<int> first(n_groups + 1);
        for (int g = 0; g < n_groups; ++g) {
            first[g] = grp[g].first;
            for (int i = grp[g].first; i < grp[g].first + grp[g].count; ++i)
                dents[i] = DecodeEntry{seq_ids[g], cache_lens[g], n_new[g], grp[g].tok_off, ent[i].begin,
                                       ent[i].stop, ent[i].causal, ent[i].q_pos};
        }
        first[n_groups] = (int)ent.size();
        bool done = false;
        evl_status st = decode_attention(c, q_new, out, dents, first, &done);
        if (st != EVL_OK) return st;
        if (done) return few_keys_attention(c, q_new, out, few);
    }

    // ---- partition: one piece length for all groups, as in the plain batched call ----
    int64_t base_items = 0, work = 0;
    for (const Group &g : grp) {
        base_items += (int64_t)g.m_tiles * Hkv;
        work += (int64_t)g.m_tiles * Hkv * g.tiles;
    }
    const size_t esz = c->d.out_dtype == EVL_OUT_F32 ? 4 : 2;
    const size_t row_bytes = (size_t)D * esz + 2 * sizeof(float);
    const int64_t target = base_items > c->target_items ? std::max<int64_t>(c->target_items, 2048)
                                                        : c->target_items;
    int64_t T = std::max<int64_t>(kMinTilesPerSplit, (work + target - 1) / target);
    size_t ws_rows = 0;
    for (;;) {
        ws_rows = 0;
        for (int g = 0; g < n_groups; ++g) {
            int ns = (int)std::max<int64_t>(1, std::min<int64_t>(kMaxSplits, (grp[g].tiles + T - 1) / T));
            grp[g].tps = (int)((grp[g].tiles + ns - 1) / ns);
            grp[g].n_splits = (int)((grp[g].tiles + grp[g].tps - 1) / grp[g].tps);
            if (grp[g].n_splits > 1) ws_rows += (size_t)grp[g].n_splits * n_new[g] * Hq;
        }
        if (ws_rows * row_bytes <= partials_capacity(c) || ws_rows == 0) break;
        T *= 2;
    }
    if (!c->tuned) {  // no target set by the caller: the common piece length is priced, as in the plain batched call
        std::vector<int> g_m(n_groups), g_tiles(n_groups), g_ns, g_tps;
        std::vector<double> g_see(n_groups);
        std::vector<size_t> g_rows(n_groups);
        for (int g = 0; g < n_groups; ++g) {
            g_m[g] = grp[g].m_tiles;
            g_tiles[g] = (int)grp[g].tiles;
            g_see[g] = (double)grp[g].tiles;  // (the causal cut inside the chunk's own entry is not counted)
            g_rows[g] = (size_t)n_new[g] * Hq;
        }
        ws_rows = pick_piece_length(g_m, g_tiles, g_see, g_rows, Hkv, D, row_bytes,
                                    c->d.workspace ? partials_capacity(c) : 0, &g_ns, &g_tps);
        for (int g = 0; g < n_groups; ++g) {
            grp[g].n_splits = g_ns[g];
            grp[g].tps = g_tps[g];
        }
    }
    void *part_o = c->d.workspace;
    float *part_ml = part_o ? (float *)((char *)part_o + ws_rows * D * esz) : nullptr;

    Plan plan;
    plan.workspace_used = ws_rows * row_bytes;
    size_t part_off = 0;
    for (int g0 = 0; g0 < n_groups;) {
        // as many whole groups as one launch can describe
        int g1 = g0, n_ent = 0;
        while (g1 < n_groups && g1 - g0 < evl::kMaxSeqs && n_ent + grp[g1].count <= evl::kMaxEntries)
            n_ent += grp[g1++].count;
        evl::AttnParams p;
        evl::CombineParams cp;
        init_params(c, q_new, out, part_o, part_ml, &p, &cp);
        p.n_seqs = n_ent;
        p.multi_entry = 1;
        attach_few(c, &p, few, &few_next);
        int items = 0, crow = 0, cseqs = 0, at = 0;
        int per_xcd[8] = {0, 0, 0, 0, 0, 0, 0, 0}, xcd_next = 0;
        for (int g = g0; g < g1; ++g) {
            const Group &gr = grp[g];
            for (int i = 0; i < gr.count; ++i) {
                const Entry &e = ent[gr.first + i];
                evl::AttnSeq &q = p.seq[at + i];
                q.bt_row = seq_ids[g];
                q.cache_len = cache_lens[g];
                q.n_new = n_new[g];
                q.tok_off = gr.tok_off;
                q.k_begin = e.begin;
                q.k_stop = e.stop;
                q.causal = e.causal;
                q.q_pos = (int32_t)e.q_pos;
                q.n_ent = i == 0 ? gr.count : 0;
                q.n_splits = i == 0 ? gr.n_splits : 0;
                q.tiles_per_split = gr.tps;
                q.m_tiles = gr.m_tiles;
                q.split_base = 0;
                q.total_splits = gr.n_splits;
                q.part_off = (int64_t)part_off;
            }
            add_xcd_load(per_xcd, &xcd_next, &p.seq[at], gr.n_splits * Hkv, gr.m_tiles,
                         choose_chunking(gr.n_splits * Hkv, gr.m_tiles));
            items += gr.m_tiles * gr.n_splits * Hkv;
            plan.max_splits = std::max(plan.max_splits, gr.n_splits);
            if (gr.n_splits > 1) {
                evl::CombineSeq &cs = cp.seq[cseqs++];
                cs.n_new = n_new[g];
                cs.tok_off = gr.tok_off;
                cs.n_splits = gr.n_splits;
                cs.row_begin = crow;
                cs.part_off = (int64_t)part_off;
                crow += n_new[g] * Hq;
                part_off += (size_t)gr.n_splits * n_new[g] * Hq;
            }
            at += gr.count;
        }
        p.n_items = items;
        p.items_per_xcd = *std::max_element(per_xcd, per_xcd + 8);
        cp.n_seqs = cseqs;
        cp.n_rows = crow;
        plan.n_items += items;
        evl_status st = launch_attention(c, p);
        if (st != EVL_OK) return st;
        if (crow > 0) {
            hipError_t e = evl::launch_combine(cp, D, (hipStream_t)c->d.stream);
            if (e == hipSuccess) ++c->n_launches;
            if (e != hipSuccess)
                return fail(EVL_ERR_LAUNCH, "combine launch failed: %s", hipGetErrorString(e));
        }
        g0 = g1;
    }
    c->last_plan = plan;
    return few_keys_attention(c, q_new, out, few, few_next);
}

// Packed sequence under the action-isolating mask: the instruction and every step of the pack
// (a frame's visual tokens followed by its action tokens) are groups of the batched sampled
// call, whose runs are what the mask lets the step see; the contiguous ids over those runs are
// the ids the corresponding single-step example would have.
// Appends a whole pack to an empty sequence with the position ids of the action-isolating mask:
// instruction and visual tokens are numbered without a gap, the action tokens of a step continue
// behind their frame, so that a later attention call needs no per-run shift of its queries.
evl_status evl_isolated_pack_append(evl_cache *c, int32_t seq, const void *k_packed, const void *v_packed,
                                    int64_t pos0, int32_t prefix, int32_t frame_tokens, int32_t action_tokens,
                                    int32_t n_frames) {
    if (!c) return fail(EVL_ERR_NULL, "cache is NULL");
    if (prefix < 0 || frame_tokens <= 0 || action_tokens < 0 || n_frames < 0 || (prefix == 0 && n_frames == 0))
        return fail(EVL_ERR_ARG, "bad pack shape: prefix %d, %d frames of %d + %d tokens", prefix, n_frames,
                    frame_tokens, action_tokens);
    const int64_t step = (int64_t)frame_tokens + action_tokens, total = (int64_t)prefix + n_frames * step;
    if (total > INT32_MAX / 2) return fail(EVL_ERR_ARG, "pack too long");
    if (action_tokens < 1 || step < evl::kKeyTile || prefix < evl::kFewKeys - 1)
        return fail(EVL_ERR_UNSUPPORTED,
                    "evl_isolated_pack_append serves packs with action tokens, at least %d tokens per step and an "
                    "instruction of at least %d tokens (got %d + %d, %d): append with evl_rope_append instead",
                    evl::kKeyTile, evl::kFewKeys - 1, frame_tokens, action_tokens, prefix);
    evl_status st = check_seq(c, seq);
    if (st != EVL_OK) return st;
    if (c->len[seq] != 0)
        return fail(EVL_ERR_NONCONTIGUOUS, "sequence %d holds %lld tokens: a pack goes into an empty sequence", seq,
                    (long long)c->len[seq]);
    const int32_t n_new = (int32_t)total;
    st = check_append(c, k_packed, v_packed, &seq, &pos0, &n_new, 1);
    if (st != EVL_OK) return st;
    evl::AppendParams p;
    int64_t tok_off = 0;
    fill_append(c, k_packed, v_packed, &seq, &pos0, &n_new, 0, 1, &tok_off, &p);
    p.hole_first = prefix;
    p.hole_period = (int32_t)step;
    p.hole_width = action_tokens;
    hipError_t e = evl::launch_rope_append(p, c->d.head_dim, (hipStream_t)c->d.stream);
    if (e == hipSuccess) ++c->n_launches;
    if (e != hipSuccess) return fail(EVL_ERR_LAUNCH, "rope_append launch failed: %s", hipGetErrorString(e));
    commit_append(c, &seq, &pos0, &n_new, 0, 1);
    c->pack[seq].prefix = prefix;
    c->pack[seq].frame_tokens = frame_tokens;
    c->pack[seq].action_tokens = action_tokens;
    return EVL_OK;
}

evl_status evl_isolated_pack_attention(const void *q_packed, evl_cache *c, int32_t seq, int32_t prefix,
                                       int32_t frame_tokens, int32_t action_tokens, int32_t n_frames,
                                       void *out_packed) {
    if (!c) return fail(EVL_ERR_NULL, "cache is NULL");
    if (prefix < 0 || frame_tokens <= 0 || action_tokens < 0 || n_frames < 0 ||
        (prefix == 0 && n_frames == 0))
        return fail(EVL_ERR_ARG, "bad pack shape: prefix %d, %d frames of %d + %d tokens", prefix, n_frames,
                    frame_tokens, action_tokens);
    const int64_t step = (int64_t)frame_tokens + action_tokens;
    if ((int64_t)prefix + n_frames * step > INT32_MAX / 2) return fail(EVL_ERR_ARG, "pack too long");
    // A sequence appended with the pack's own ids: one causal launch in which the action tokens of
    // earlier steps are holes of the key range; no run list, no shifted queries.
    if (check_seq(c, seq) == EVL_OK && c->pack[seq].action_tokens > 0) {
        const PackShape &ps = c->pack[seq];
        if (ps.prefix != prefix || ps.frame_tokens != frame_tokens || ps.action_tokens != action_tokens)
            return fail(EVL_ERR_ARG, "sequence %d holds a pack of shape %d + n x (%d + %d), asked for %d + n x (%d + %d)",
                        seq, ps.prefix, ps.frame_tokens, ps.action_tokens, prefix, frame_tokens, action_tokens);
        if (!q_packed || !out_packed) return fail(EVL_ERR_NULL, "q_packed / out_packed is NULL");
        if (!aligned16(q_packed) || !aligned16(out_packed))
            return fail(EVL_ERR_ALIGN, "q_packed / out_packed must be 16-byte aligned");
        const int64_t total = (int64_t)prefix + n_frames * step;
        if (total > c->len[seq])
            return fail(EVL_ERR_RANGE, "sequence %d: the pack has %lld tokens, %lld were appended", seq,
                        (long long)total, (long long)c->len[seq]);
        // the first 63 tokens (inside the instruction: prefix >= 63) see fewer than 64 keys
        const int32_t a = (int32_t)std::min<int64_t>(evl::kFewKeys - 1, total);
        std::vector<FewGroup> few;
        few.push_back(FewGroup{seq, 0, a, 0, {Entry{0, a, 1, c->pos0[seq], 0}}});
        if (total == a) {
            c->last_plan = Plan();
            return few_keys_attention(c, q_packed, out_packed, few);
        }
        const int32_t rest = (int32_t)(total - a);
        return attention_batched_core(q_packed, c, &seq, &a, &rest, &a, 1, out_packed, few, &ps);
    }
    std::vector<int32_t> seqs, lens, ns, toks, offs(1, 0);
    std::vector<evl_run> runs;
    auto add_group = [&](int32_t begin, int32_t n, int frames_visible) {
        // runs: the instruction and the visual tokens of the first frames_visible frames
        if (prefix > 0) runs.push_back(evl_run{0, prefix});
        for (int f = 0; f < frames_visible; ++f)
            runs.push_back(evl_run{(int32_t)(prefix + f * step), frame_tokens});
        seqs.push_back(seq);
        lens.push_back(begin);
        ns.push_back(n);
        toks.push_back(begin);
        offs.push_back((int32_t)runs.size());
    };
    if (prefix > 0) {   // the instruction itself: plain causal, no runs
        seqs.push_back(seq);
        lens.push_back(0);
        ns.push_back(prefix);
        toks.push_back(0);
        offs.push_back(0);
    }
    // Step t: its visual tokens and its action tokens are one chunk.  Causal order inside the
    // chunk gives the action tokens the whole frame and their own predecessors, and keeps the
    // action tokens away from the visual ones, which come first; the runs are the instruction and
    // the visual tokens of the earlier frames.
    for (int t = 0; t < n_frames; ++t) add_group((int32_t)(prefix + t * step), (int32_t)step, t);
    return evl_chunk_attention_sampled_batched(q_packed, c, (int32_t)seqs.size(), seqs.data(), lens.data(),
                                               ns.data(), toks.data(), offs.data(), runs.data(), out_packed);
}

size_t evl_workspace_bytes_sampled(const evl_cache_desc *desc, int32_t max_n_new, int32_t max_runs) {
    if (!desc || max_n_new <= 0 || max_runs < 0 || desc->head_dim <= 0 || desc->n_q_heads <= 0)
        return 0;
    // 16 pieces of the key tiles, and one more per launch that the runs take
    const size_t pieces = 16 + ((size_t)max_runs + 1 + evl::kMaxSeqs - 1) / evl::kMaxSeqs;
    return pieces * (size_t)max_n_new * desc->n_q_heads * ((size_t)desc->head_dim + 2) * 4 +
           evl::kCounterBytes;
}

// Frame samplers of Sec. 3.2 on frame indices 0 .. n_frames-1 (HOST only, integer arithmetic).
int32_t evl_sample_uniform(int32_t n_frames, int32_t n_keep, int32_t *idx) {
    if (n_frames <= 0 || n_keep <= 0 || !idx) return 0;
    if (n_frames <= n_keep) {
        for (int32_t j = 0; j < n_frames; ++j) idx[j] = j;
        return n_frames;
    }
    if (n_keep == 1) {
        idx[0] = n_frames - 1;
        return 1;
    }
    // nearest integer to j (n_frames - 1) / (n_keep - 1), halves upwards
    const int64_t num = n_frames - 1, den = n_keep - 1;
    for (int64_t j = 0; j < n_keep; ++j) idx[j] = (int32_t)((2 * j * num + den) / (2 * den));
    return n_keep;
}

int32_t evl_sample_window(int32_t n_frames, int32_t n_keep, int32_t stride, int32_t *idx) {
    if (n_frames <= 0 || n_keep <= 0 || stride <= 0 || !idx) return 0;
    const int32_t n = std::min<int64_t>(n_keep, ((int64_t)n_frames - 1) / stride + 1);
    for (int32_t j = 0; j < n; ++j) idx[j] = n_frames - 1 - (n - 1 - j) * stride;
    return n;
}

// ------------------------------------------------------------------------------------------
// Page copies: offload to / reload from another pool
// ------------------------------------------------------------------------------------------
evl_status evl_pages_copy(evl_cache *c, void *dst_k, void *dst_v, const int32_t *dst_pages,
                          int32_t dst_pool_pages, const void *src_k, const void *src_v,
                          const int32_t *src_pages, int32_t src_pool_pages, int32_t n) {
    if (!c) return fail(EVL_ERR_NULL, "cache is NULL");
    if (!dst_k || !dst_v || !src_k || !src_v) return fail(EVL_ERR_NULL, "a pool pointer is NULL");
    if (n < 0 || (n > 0 && (!dst_pages || !src_pages))) return fail(EVL_ERR_NULL, "a page list is NULL");
    if (!aligned16(dst_k) || !aligned16(dst_v) || !aligned16(src_k) || !aligned16(src_v))
        return fail(EVL_ERR_ALIGN, "pool pointers must be 16-byte aligned");
    if (dst_pool_pages <= 0 || src_pool_pages <= 0) return fail(EVL_ERR_ARG, "pool sizes must be positive");
    for (int i = 0; i < n; ++i) {
        if (src_pages[i] < 0 || src_pages[i] >= src_pool_pages)
            return fail(EVL_ERR_RANGE, "src_pages[%d] = %d outside the source pool of %d pages", i, src_pages[i],
                        src_pool_pages);
        if (dst_pages[i] < 0 || dst_pages[i] >= dst_pool_pages)
            return fail(EVL_ERR_RANGE, "dst_pages[%d] = %d outside the destination pool of %d pages", i,
                        dst_pages[i], dst_pool_pages);
    }
    const int page_bytes = c->d.n_kv_heads * evl::kPage * c->d.head_dim * 2;
    if (n == 0) return EVL_OK;
    // The kernel dereferences all four pools: each must be memory the device can address (device
    // memory or pinned host memory), and, where the runtime knows the allocation, large enough.
    const struct { const void *p; int32_t pages; const char *name; } pools[4] = {
        {dst_k, dst_pool_pages, "dst_k"}, {dst_v, dst_pool_pages, "dst_v"},
        {src_k, src_pool_pages, "src_k"}, {src_v, src_pool_pages, "src_v"}};
    for (const auto &pool : pools) {
        // (for memory the runtime does not know, the attribute query succeeds and reports the
        // type "unregistered" with no device pointer; the range query fails)
        hipPointerAttribute_t attr;
        hipDeviceptr_t base_ptr = nullptr;
        size_t size = 0;
        const bool known = hipPointerGetAttributes(&attr, pool.p) == hipSuccess &&
                           (attr.type == hipMemoryTypeDevice || attr.type == hipMemoryTypeHost ||
                            attr.type == hipMemoryTypeManaged) &&
                           attr.devicePointer != nullptr &&
                           hipMemGetAddressRange(&base_ptr, &size, (hipDeviceptr_t)pool.p) == hipSuccess;
        if (!known) {
            (void)hipGetLastError();
            return fail(EVL_ERR_ARG, "%s is neither device memory nor pinned host memory", pool.name);
        }
        const size_t off = (size_t)((const char *)pool.p - (const char *)base_ptr);
        if (off > size || (size_t)pool.pages * page_bytes > size - off)
            return fail(EVL_ERR_RANGE, "%s: %d pages of %d bytes do not fit its allocation (%zu bytes from there)",
                        pool.name, pool.pages, page_bytes, size - off);
    }
    for (int base = 0; base < n; base += evl::kMaxPagesPerCopy) {
        evl::PageCopyParams p;
        p.src_k = src_k;
        p.src_v = src_v;
        p.dst_k = dst_k;
        p.dst_v = dst_v;
        p.n = std::min(evl::kMaxPagesPerCopy, n - base);
        p.page_bytes = page_bytes;
        std::memcpy(p.src_page, src_pages + base, sizeof(int32_t) * p.n);
        std::memcpy(p.dst_page, dst_pages + base, sizeof(int32_t) * p.n);
        hipError_t e = evl::launch_pages_copy(p, (hipStream_t)c->d.stream);
        if (e == hipSuccess) ++c->n_launches;
        if (e != hipSuccess) return fail(EVL_ERR_LAUNCH, "page copy launch failed: %s", hipGetErrorString(e));
    }
    return EVL_OK;
}

evl_status evl_cache_tune(evl_cache *c, int32_t target_workgroups) {
    if (!c) return fail(EVL_ERR_NULL, "cache is NULL");
    if (target_workgroups < 0) return fail(EVL_ERR_ARG, "target_workgroups must be >= 0");
    if (target_workgroups) {
        c->target_items = target_workgroups;
        c->tuned = true;
    } else {
        c->target_items = kDefaultTargetItems;
        c->tuned = false;
    }
    return EVL_OK;
}

evl_status evl_timing_enable(evl_cache *c, int32_t n_pairs) {
    if (!c) return fail(EVL_ERR_NULL, "cache is NULL");
    if (n_pairs < 0 || n_pairs > (1 << 16)) return fail(EVL_ERR_ARG, "n_pairs %d outside [0, 65536]", n_pairs);
    destroy_events(c);
    for (int i = 0; i < n_pairs; ++i) {
        hipEvent_t a = nullptr, b = nullptr;
        if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
            if (a) (void)hipEventDestroy(a);
            destroy_events(c);
            return fail(EVL_ERR_LAUNCH, "hipEventCreate failed");
        }
        c->ev_start.push_back(a);
        c->ev_stop.push_back(b);
    }
    return EVL_OK;
}

evl_status evl_timing_read(evl_cache *c, float *ms_out, int32_t max, int32_t *n_out) {
    if (!c) return fail(EVL_ERR_NULL, "cache is NULL");
    if (!ms_out || !n_out) return fail(EVL_ERR_NULL, "ms_out / n_out is NULL");
    *n_out = 0;
    const int64_t ring = (int64_t)c->ev_start.size();
    if (ring == 0) return fail(EVL_ERR_ARG, "timing is not enabled on this cache");
    const int64_t have = std::min(c->ev_count, ring);
    const int64_t first = c->ev_count - have;
    int32_t n = 0;
    for (int64_t k = first; k < c->ev_count && n < max; ++k) {
        const size_t slot = (size_t)(k % ring);
        float ms = 0.f;
        if (hipEventSynchronize(c->ev_stop[slot]) != hipSuccess ||
            hipEventElapsedTime(&ms, c->ev_start[slot], c->ev_stop[slot]) != hipSuccess)
            return fail(EVL_ERR_LAUNCH, "reading a timing event failed");
        ms_out[n++] = ms;
    }
    c->ev_count = 0;
    *n_out = n;
    return EVL_OK;
}

evl_status evl_last_plan(const evl_cache *cache, int32_t *n_workgroups, int32_t *max_splits,
                         size_t *workspace_used) {
    if (!cache) return fail(EVL_ERR_NULL, "cache is NULL");
    if (n_workgroups) *n_workgroups = cache->last_plan.n_items;
    if (max_splits) *max_splits = cache->last_plan.max_splits;
    if (workspace_used) *workspace_used = cache->last_plan.workspace_used;
    return EVL_OK;
}

}  // extern "C"

// Internal interface between the host side of the library (argument checking, integer
// bookkeeping, work partitioning) and its gfx950 kernels.  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace evl {

constexpr int kPage = 16;           // tokens per page (the only page size the kernels support)
constexpr int kMaxSeqs = 64;        // sequences one launch can describe in its kernel arguments
constexpr int kMaxEntries = 160;    // entries (key ranges) one attention launch can describe
constexpr int kMaxHalfDim = 64;     // head_dim / 2 at most
constexpr int kKeyTile = 64;        // keys staged in LDS per iteration of the attention loop
constexpr int kThreads = 256;       // work-group size of every kernel (4 wavefronts)

// ---- fused RoPE + append ------------------------------------------------------------------
struct AppendSeq {
    int32_t bt_row;      // row of the block table
    int32_t t_begin;     // sequence index of the chunk's first token (= length before the append)
    int32_t n_new;       // tokens in the chunk
    int32_t tok_off;     // first token of this sequence's chunk in the concatenated inputs
    int32_t item_begin;  // first work-group of this sequence
    int32_t pad_;
    int64_t pos_begin;   // position id of the chunk's first token
};

struct AppendParams {
    const void *k_new, *v_new;
    void *k_pool, *v_pool;
    const int32_t *block_table;
    int32_t *pos_tags;   // may be null
    int32_t n_kv_heads, n_pages, max_pages_per_seq, n_seqs, n_items, pad_;
    // Packed sequence under the action-isolating mask (hole_width > 0; one sequence per launch):
    // the token at sequence index t belongs to step s(t) = (t - hole_first) / hole_period (0 before
    // hole_first), the last hole_width tokens of every step are that step's action tokens, and
    // position ids skip the action tokens of earlier steps: id(t) = pos_begin + t - hole_width * s(t).
    int32_t hole_first, hole_period, hole_width, pad2_;
    double rev_freq[kMaxHalfDim];  // theta_j / (2 pi): turns per position
    AppendSeq seq[kMaxSeqs];
};

// ---- chunk attention ----------------------------------------------------------------------
// One entry of an attention launch: a key range of one sequence that the chunk's queries attend
// to, with the position at which the queries are rotated for it.  Entries that serve the same
// output rows form a group of consecutive entries; the key tiles of a group's entries, taken
// one entry after the other, are cut into n_splits pieces of tiles_per_split tiles, and one
// work-group handles one (row tile, KV head, piece), walking from entry to entry and shifting
// its queries' rotation on the way.  The plain call has one entry per sequence (all keys,
// causal); the sampled call has one per retained run of the history plus one for the chunk.
// The group's first entry carries the partition; the others have n_ent = n_splits = 0.
struct AttnSeq {
    int32_t bt_row;
    int32_t cache_len;        // tokens that precede the chunk (causal limit of row i: cache_len + i)
    int32_t n_new;            // chunk tokens
    int32_t tok_off;          // first token of this sequence's chunk in q_new / out
    int32_t k_begin;          // first key (sequence index) of this entry's range
    int32_t k_stop;           // end (exclusive) of this entry's key range; never empty
    int32_t causal;           // 1: row i sees keys <= cache_len + i only (the entry holding the chunk)
    int32_t q_pos;            // position at which chunk token 0's query is rotated for this entry
    int32_t n_ent;            // entries in the group (first entry of a group only)
    int32_t n_splits;         // pieces the group's key tiles are cut into
    int32_t tiles_per_split;  // key tiles per piece
    int32_t m_tiles;          // row tiles of the chunk
    int32_t split_base;       // index of this group's first piece among all pieces of the rows
    int32_t total_splits;     // pieces over all groups of the rows (1 = write `out` directly)
    int32_t cnt_base;         // decode kernel: first ticket counter of the rows (one per KV head)
    int32_t k_pos;            // fused step: position id of the chunk's first token (the key side)
    int32_t chunk_rows;       // attention kernel: work items per XCD chunk (first entry of a group), ...
    int32_t chunk_pad;        // ... and 1 if every (KV head, piece) group is cut and padded by itself
    int32_t xcd_first;        // ... and the XCD its first chunk goes to (the launch's chunks go round the XCDs entry after entry)
    int32_t tile_major;       // ... and 1 if the dense cut counts items row tile after row tile (all groups' longest first)
    int64_t part_off;         // first partial row of the rows' block in the workspace
};

struct AttnParams {
    const void *q;
    const void *k_new, *v_new;  // the chunks' raw keys / values: fused step of the decode kernel only
    const void *k_pool, *v_pool;
    const int32_t *block_table;
    void *out;
    void *part_o;    // [partial rows][d] normalised partial outputs, in the output's element type
    float *part_ml;  // [partial rows][2] exponent reference (log2 domain) and sum
    int32_t *counters;  // ticket counters of the decode kernel's in-kernel merge, or null
    int32_t n_q_heads, n_kv_heads, group, n_pages, max_pages_per_seq, out_f32, n_seqs, n_items;
    int32_t items_per_xcd;  // largest number of work items any XCD gets (grid = 8 x this)
    int32_t tab_tokens;  // tokens the LDS cos/sin table of a work-group has room for
    float q_scale;   // log2(e) / sqrt(d), folded into the rotated queries
    int32_t multi_entry;  // 1 if some group of this launch has more than one entry
    // Groups of rows that see fewer than kFewKeys keys: entries seq[few_first .. few_first +
    // few_entries), few_rows (token, query head) rows in all.  In an attention launch they ride
    // along as extra work-groups behind the 8 * items_per_xcd of the matrix part.
    int32_t few_first, few_entries, few_rows;
    // Packed sequence under the action-isolating mask (hole_width > 0; the launch serves one
    // sequence, plain build): steps and position ids as in AppendParams; the action tokens of a step
    // are visible to the rows of that step only (a "hole" in what later steps see).  The kernel
    // handles at most two holes per key tile: hole_period >= kKeyTile.
    int32_t hole_first, hole_period, hole_width;
    double rev_freq[kMaxHalfDim];  // theta_j / (2 pi): turns per position
    AttnSeq seq[kMaxEntries];
};

struct CombineSeq {
    int32_t n_new, tok_off, n_splits, row_begin;  // row_begin: first (token, head) row handled
    int64_t part_off;
};

struct CombineParams {
    const void *part_o;
    const float *part_ml;
    void *out;
    int32_t n_q_heads, out_f32, n_seqs, n_rows;
    CombineSeq seq[kMaxSeqs];
};

// Geometry of the chunk-attention kernel that the host side plans with.
constexpr int kAttnRows = 256;   // packed (token, query-head-in-group) rows per work-group
constexpr int kAttnStages = 3;   // K/V tile buffers of the kernel's LDS ring
constexpr size_t attention_stage_bytes(int head_dim) {  // one K tile + one V tile, bf16
    return (size_t)2 * kKeyTile * head_dim * 2;
}
inline int attention_rows_per_workgroup() { return kAttnRows; }
// Work items of an entry -- its (KV head, piece) groups of m_tiles row tiles each -- are dealt to
// the XCDs in chunks of chunk_rows items that take consecutive slots of one XCD, where they share
// keys in the L2.  Two ways of cutting, chosen by the host per entry (AttnSeq::chunk_rows,
// chunk_pad) and obeyed by the kernel's work-item map:
//  * padded (chunk_pad = 1): every group is cut by itself; a group's last chunk is padded to
//    chunk_rows slots with work items that exit at once.  No chunk straddles two groups.
//  * dense (chunk_pad = 0): the items of all groups, laid end to end, are cut; only the entry's
//    last chunk can be short.  A chunk straddles groups unless chunk_rows divides m_tiles.
// The hardware deals an XCD's work-groups to its four shader engines in turn, so padding in the
// middle of an XCD's list leaves the engines with unequal numbers of real work-groups: with equal
// items in one or two rounds that costs a whole round, which is what the dense cut is for.
constexpr int kXcdChunkRowTiles = 8;
constexpr int kCusPerXcd = 32, kEnginesPerXcd = 4;
// chunks of an entry with `groups` groups
__host__ __device__ inline int xcd_chunks(int groups, int m_tiles, int chunk_rows, int chunk_pad) {
    if (m_tiles < 1 || chunk_rows < 1) return 0;
    return chunk_pad ? groups * ((m_tiles + chunk_rows - 1) / chunk_rows)
                     : (groups * m_tiles + chunk_rows - 1) / chunk_rows;
}
// Dynamic LDS bytes the attention kernel needs: the tile ring, then a region that first holds
// the cos/sin table of the prologue (tab_tokens tokens) and, in launches whose work-groups walk
// through several entries, afterwards the rounding residuals of the rotated queries.
// A token's row of the table is head_dim / 2 (cos, sin) pairs plus kTabPad pairs of padding: the
// lanes of a wave read the rows of five or six different tokens at once, and rows a multiple of
// 256 bytes apart would all start in the same LDS bank.
constexpr int kTabPad = 2;
constexpr int attention_tab_stride(int head_dim) { return head_dim / 2 + kTabPad; }
inline size_t attention_lds_bytes(int head_dim, int tab_tokens, bool multi_entry) {
    const size_t tab = (size_t)tab_tokens * attention_tab_stride(head_dim) * 2 * sizeof(float);
    const size_t residuals = multi_entry ? (size_t)kAttnRows * head_dim * 2 : 0;
    return (size_t)kAttnStages * attention_stage_bytes(head_dim) + (tab > residuals ? tab : residuals);
}

hipError_t launch_rope_append(const AppendParams &p, int head_dim, hipStream_t stream);
// ev_start / ev_stop: both null, or a pair of events that receive the begin and end time of the
// dispatch itself
hipError_t launch_chunk_attention(const AttnParams &p, int head_dim, hipStream_t stream,
                                  hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);
// Attention for chunks of at most kDecodeRows packed rows per KV head: one wave per piece of
// kDecodeTile-key tiles, kDecodeWavesPerGroup pieces per work-group.
constexpr int kDecodeRows = 32;
constexpr int kDecodeTileKeys = 32;
constexpr int kDecodeWavesPerGroup = 8;
// LDS bytes of the decode kernel.  Per wave: a K tile and a V tile (together also the fp32
// partial output of 32 rows), a cos/sin table for the chunk's tokens (tab_tokens: the longest
// chunk of the launch), and (reference, sum) of its 32 rows.
inline size_t decode_lds_bytes(int head_dim, int tab_tokens) {
    return (size_t)kDecodeWavesPerGroup * ((size_t)2 * kDecodeTileKeys * head_dim * 2 +
                                           (size_t)tab_tokens * (head_dim / 2) * 8 + kDecodeRows * 8) +
           16;
}
// fused: if given, the same launch also appends the chunks (whose keys and values the attention
// part then takes from p.k_new / p.v_new instead of from the cache)
hipError_t launch_decode_attention(const AttnParams &p, int head_dim, int n_workgroups, hipStream_t stream,
                                   hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr,
                                   const AppendParams *fused = nullptr);
hipError_t launch_combine(const CombineParams &p, int head_dim, hipStream_t stream);
// Rows that see fewer than kFewKeys keys (the first tokens of a sequence) do not go through the
// bf16 matrix pipes: with so few keys nothing averages out the rounding of the rotated queries
// and of the probabilities to bf16, so those rows get plain fp32 arithmetic, one wave per row
// (the rotated keys in the cache stay what they are).  Entries as in an attention launch (groups
// of key ranges with their query positions; n_new = the group's tokens served here, all of which
// see fewer than kFewKeys keys), named by few_first / few_entries / few_rows.  This launcher
// starts the kernel on its own; launch_chunk_attention takes such groups along with its matrix
// work, as extra work-groups of the same launch.
constexpr int kFewKeys = 64;
hipError_t launch_few_keys(const AttnParams &p, int head_dim, hipStream_t stream);
hipError_t launch_zero_counters(int *counters, int n, hipStream_t stream);

// ---- page copies between pools ---------------------------------------------------------------
constexpr int kMaxPagesPerCopy = 960;  // page pairs one launch carries in its kernel arguments
struct PageCopyParams {
    const void *src_k, *src_v;
    void *dst_k, *dst_v;
    int32_t n, page_bytes;  // page_bytes: Hkv * 16 * d * 2, the size of a page's K block (= V block)
    int32_t src_page[kMaxPagesPerCopy], dst_page[kMaxPagesPerCopy];
};
hipError_t launch_pages_copy(const PageCopyParams &p, hipStream_t stream);

constexpr int kCounters = 1024;         // ticket counters kept in the last 4 KB of the workspace
constexpr size_t kCounterBytes = 4096;

// ---- the library's own scratch array (for callers that cannot allocate) ------------------------
// A file-scope device array that stands in for the caller's workspace: room for the partial rows
// of one chunk plus the ticket counters.  Every GPU the library runs on holds one copy until the
// process ends.
constexpr size_t kStaticScratchBytes = ((size_t)16 << 20) + kCounterBytes;
constexpr int kStaticScratchMaxRows = 8192;  // (token, query head) rows of a chunk served from it
// Device address and size of the current device's copy of the array (looked up once per device).
hipError_t static_scratch(void **ptr, size_t *bytes);

}  // namespace evl

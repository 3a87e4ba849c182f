// Stand-ins for the kernel launchers, for tests of the library's host side on a machine without a
// GPU.  Linked with evl_api.cpp in place of the kernel file, every call of the C ABI runs its
// argument checks, its integer bookkeeping and its work partitioning as in the product, and then
// hands the kernel arguments to the checks below instead of to the GPU.  Each check restates, from
// the kernels' point of view, what a kernel takes for granted about its arguments: that every work
// item of the grid exists, that the pieces of a key range cover its tiles exactly once, that
// partial results stay inside the workspace and are merged completely, that the tables fit.  A
// launch that breaks one of them is refused with hipErrorInvalidValue and the first such message
// is kept for the test to read.  Test infrastructure only: nothing of this is part of libevl.so.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <set>
#include <vector>

#include "evl_internal.h"

namespace {

char g_msg[512] = "";
int64_t g_count[7] = {0, 0, 0, 0, 0, 0, 0};
int g_max_seqs = 1;

// rows (of one launch sequence of attention kernels) whose partial results wait for a combine
struct Pending {
    int n_new, total_splits;
    int64_t rows_begin, rows_end;             // its partial rows in the workspace
    std::vector<std::pair<int, int>> pieces;  // [split_base, split_base + n_splits) of each group
};
std::map<std::pair<int64_t, int>, Pending> g_pending;  // key: (part_off, tok_off)

hipError_t refuse(const char *fmt, ...) {
    if (!g_msg[0]) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(g_msg, sizeof(g_msg), fmt, ap);
        va_end(ap);
    }
    return hipErrorInvalidValue;
}

#define REQUIRE(cond, ...) \
    do {                   \
        if (!(cond)) return refuse(__VA_ARGS__); \
    } while (0)

size_t partial_rows(const void *part_o, const float *part_ml, int D, bool out_f32) {
    if (!part_o || !part_ml) return 0;
    return (size_t)((const char *)part_ml - (const char *)part_o) / ((size_t)D * (out_f32 ? 4 : 2));
}

hipError_t check_common(const evl::AttnParams &p, int D, const char *who) {
    REQUIRE(D == 64 || D == 128, "%s: head_dim %d", who, D);
    REQUIRE(p.q && p.k_pool && p.v_pool && p.block_table && p.out, "%s: a null pointer", who);
    REQUIRE(p.n_kv_heads >= 1 && p.group >= 1 && p.group * p.n_kv_heads == p.n_q_heads,
            "%s: heads %d / %d / group %d", who, p.n_q_heads, p.n_kv_heads, p.group);
    REQUIRE(p.n_pages >= 1 && p.max_pages_per_seq >= 1, "%s: pool shape", who);
    REQUIRE(std::fabs(p.q_scale * std::sqrt((double)D) - 1.4426950408889634) < 1e-6, "%s: q_scale %g", who,
            (double)p.q_scale);
    REQUIRE(p.rev_freq[0] > 0.159 && p.rev_freq[0] < 0.1592, "%s: rev_freq[0] = %g", who, p.rev_freq[0]);
    for (int j = 1; j < D / 2; ++j)
        REQUIRE(p.rev_freq[j] > 0 && p.rev_freq[j] < p.rev_freq[j - 1], "%s: rev_freq not decreasing at %d", who, j);
    return hipSuccess;
}

// what both attention kernels assume of one entry's key range
hipError_t check_range(const evl::AttnParams &p, const evl::AttnSeq &head, const evl::AttnSeq &en, int x,
                       const char *who) {
    REQUIRE(en.k_begin >= 0 && en.k_begin < en.k_stop, "%s: entry %d has the empty range [%d, %d)", who, x,
            en.k_begin, en.k_stop);
    REQUIRE((int64_t)en.k_stop <= (int64_t)p.max_pages_per_seq * evl::kPage,
            "%s: entry %d ends at key %d, past the block-table row", who, x, en.k_stop);
    if (en.causal)
        REQUIRE(en.k_stop == head.cache_len + head.n_new && en.k_begin <= head.cache_len,
                "%s: causal entry %d = [%d, %d) does not end with the chunk (%d + %d)", who, x, en.k_begin,
                en.k_stop, head.cache_len, head.n_new);
    else
        REQUIRE(en.k_stop <= head.cache_len, "%s: entry %d = [%d, %d) reaches into the chunk at %d", who, x,
                en.k_begin, en.k_stop, head.cache_len);
    REQUIRE(en.q_pos >= 0 && (int64_t)en.q_pos + head.n_new <= INT32_MAX, "%s: entry %d q_pos %d", who, x, en.q_pos);
    return hipSuccess;
}

}  // namespace

extern "C" {
void evl_probe_reset(int32_t max_seqs) {
    g_msg[0] = 0;
    std::memset(g_count, 0, sizeof(g_count));
    g_pending.clear();
    g_max_seqs = max_seqs;
}
const char *evl_probe_message(void) { return g_msg; }
int64_t evl_probe_count(int32_t kind) { return kind >= 0 && kind < 7 ? g_count[kind] : -1; }
int64_t evl_probe_pending(void) { return (int64_t)g_pending.size(); }
}

namespace evl {

hipError_t launch_rope_append(const AppendParams &p, int head_dim, hipStream_t) {
    const char *who = "append";
    ++g_count[0];
    REQUIRE(head_dim == 64 || head_dim == 128, "%s: head_dim %d", who, head_dim);
    REQUIRE(p.k_new && p.v_new && p.k_pool && p.v_pool && p.block_table, "%s: a null pointer", who);
    REQUIRE(p.n_seqs >= 1 && p.n_seqs <= kMaxSeqs, "%s: n_seqs %d", who, p.n_seqs);
    REQUIRE(p.n_kv_heads >= 1 && p.n_pages >= 1 && p.max_pages_per_seq >= 1, "%s: shape", who);
    REQUIRE(p.rev_freq[0] > 0.159 && p.rev_freq[0] < 0.1592, "%s: rev_freq[0] = %g", who, p.rev_freq[0]);
    int items = 0;
    int64_t tok = p.seq[0].tok_off;  // (a call with many sequences takes several launches)
    REQUIRE(tok >= 0, "%s: tok_off %lld", who, (long long)tok);
    std::set<int> rows;
    for (int s = 0; s < p.n_seqs; ++s) {
        const AppendSeq &q = p.seq[s];
        REQUIRE(q.bt_row >= 0 && q.bt_row < g_max_seqs && rows.insert(q.bt_row).second,
                "%s: sequence %d: block-table row %d out of range or listed twice", who, s, q.bt_row);
        REQUIRE(q.n_new >= 1 && q.t_begin >= 0, "%s: sequence %d: t_begin %d, n_new %d", who, s, q.t_begin, q.n_new);
        REQUIRE((int64_t)q.t_begin + q.n_new <= (int64_t)p.max_pages_per_seq * kPage,
                "%s: sequence %d grows past its block-table row", who, s);
        REQUIRE(q.tok_off == tok, "%s: sequence %d: tok_off %d, expected %lld", who, s, q.tok_off, (long long)tok);
        REQUIRE(q.item_begin == items, "%s: sequence %d: item_begin %d, expected %d", who, s, q.item_begin, items);
        REQUIRE(q.pos_begin >= 0 && q.pos_begin + q.n_new <= INT32_MAX, "%s: sequence %d: positions", who, s);
        const int pages = (q.t_begin + q.n_new + kPage - 1) / kPage - q.t_begin / kPage;
        items += pages * p.n_kv_heads;
        tok += q.n_new;
    }
    REQUIRE(p.n_items == items, "%s: n_items %d, the sequences touch %d (page, head) pairs", who, p.n_items, items);
    if (p.hole_width != 0)  // a pack: one sequence, from its first token, steps no shorter than their action tokens
        REQUIRE(p.n_seqs == 1 && p.seq[0].t_begin == 0 && p.hole_width > 0 && p.hole_first >= 0 &&
                    p.hole_period > p.hole_width,
                "%s: pack of %d sequences from token %d, steps of %d with %d action tokens after %d", who, p.n_seqs,
                p.seq[0].t_begin, p.hole_period, p.hole_width, p.hole_first);
    return hipSuccess;
}

hipError_t check_few(const AttnParams &p, const char *who);

hipError_t launch_chunk_attention(const AttnParams &p, int D, hipStream_t, hipEvent_t, hipEvent_t) {
    const char *who = "attention";
    ++g_count[1];
    if (hipError_t e = check_common(p, D, who)) return e;
    // rows with few keys that ride along: entries behind the launch's own
    REQUIRE(p.few_entries == 0 || p.few_first == p.n_seqs, "%s: few-keys entries start at %d, own entries end at %d",
            who, p.few_first, p.n_seqs);
    if (hipError_t e = check_few(p, who)) return e;
    const int G = p.group, Hq = p.n_q_heads, Hkv = p.n_kv_heads, KN = kKeyTile;
    REQUIRE(p.n_seqs >= 1 && p.n_seqs <= kMaxEntries, "%s: n_seqs %d", who, p.n_seqs);
    const size_t ws_rows = partial_rows(p.part_o, p.part_ml, D, p.out_f32 != 0);
    int items = 0, per_xcd[8] = {0, 0, 0, 0, 0, 0, 0, 0}, xcd_next = 0;
    bool multi = false;
    for (int e = 0; e < p.n_seqs;) {
        const AttnSeq &sq = p.seq[e];
        REQUIRE(sq.n_ent >= 1 && e + sq.n_ent <= p.n_seqs, "%s: entry %d: group of %d entries", who, e, sq.n_ent);
        REQUIRE(sq.n_ent <= 64, "%s: entry %d: a group of %d entries does not fit a wave's lanes", who, e, sq.n_ent);
        multi = multi || sq.n_ent > 1;
        REQUIRE(sq.bt_row >= 0 && sq.bt_row < g_max_seqs, "%s: entry %d: block-table row %d", who, e, sq.bt_row);
        REQUIRE(sq.n_new >= 1 && sq.cache_len >= 0 && sq.tok_off >= 0, "%s: entry %d: chunk", who, e);
        REQUIRE(sq.m_tiles == (sq.n_new * G + kAttnRows - 1) / kAttnRows, "%s: entry %d: m_tiles %d for %d rows", who,
                e, sq.m_tiles, sq.n_new * G);
        int64_t tiles = 0;
        int n_causal = 0;
        for (int x = e; x < e + sq.n_ent; ++x) {
            const AttnSeq &en = p.seq[x];
            if (x > e)
                REQUIRE(en.n_ent == 0 && en.n_splits == 0, "%s: entry %d inside a group claims work items", who, x);
            if (hipError_t err = check_range(p, sq, en, x, who)) return err;
            n_causal += en.causal != 0;
            REQUIRE(!en.causal || x == e + sq.n_ent - 1, "%s: causal entry %d is not the group's last", who, x);
            // the kernel's own count for the work-group with the chunk's last rows
            const int sh = (en.k_begin / kPage % (KN / kPage)) * kPage;
            tiles += (en.k_stop - sh + KN - 1) / KN - en.k_begin / KN;
        }
        REQUIRE(n_causal <= 1, "%s: entry %d: several causal entries", who, e);
        REQUIRE(sq.n_splits >= 1 && sq.tiles_per_split >= 1, "%s: entry %d: %d pieces of %d tiles", who, e,
                sq.n_splits, sq.tiles_per_split);
        REQUIRE((int64_t)(sq.n_splits - 1) * sq.tiles_per_split < tiles &&
                    tiles <= (int64_t)sq.n_splits * sq.tiles_per_split,
                "%s: entry %d: %d pieces of %d tiles for %lld tiles", who, e, sq.n_splits, sq.tiles_per_split,
                (long long)tiles);
        REQUIRE(sq.split_base >= 0 && sq.split_base + sq.n_splits <= sq.total_splits,
                "%s: entry %d: pieces %d + %d of %d", who, e, sq.split_base, sq.n_splits, sq.total_splits);
        if (sq.total_splits > 1) {
            REQUIRE(p.part_o && p.part_ml, "%s: entry %d splits without a workspace", who, e);
            REQUIRE(sq.part_off >= 0 && (size_t)sq.part_off + (size_t)sq.total_splits * sq.n_new * Hq <= ws_rows,
                    "%s: entry %d: partial rows %lld + %d x %d beyond the %zu of the workspace", who, e,
                    (long long)sq.part_off, sq.total_splits, sq.n_new * Hq, ws_rows);
            const int64_t r0 = sq.part_off, r1 = sq.part_off + (int64_t)sq.total_splits * sq.n_new * Hq;
            if (!g_pending.count({sq.part_off, sq.tok_off}))  // new rows: away from all rows still waiting
                for (auto &kv : g_pending)
                    REQUIRE(r1 <= kv.second.rows_begin || kv.second.rows_end <= r0,
                            "%s: entry %d: partial rows %lld..%lld overlap those of other rows", who, e, (long long)r0,
                            (long long)r1);
            Pending &pd = g_pending[{sq.part_off, sq.tok_off}];
            if (pd.pieces.empty()) {
                pd.n_new = sq.n_new;
                pd.total_splits = sq.total_splits;
                pd.rows_begin = r0;
                pd.rows_end = r1;
            }
            REQUIRE(pd.n_new == sq.n_new && pd.total_splits == sq.total_splits,
                    "%s: entry %d disagrees with an earlier group of the same rows", who, e);
            pd.pieces.push_back({sq.split_base, sq.split_base + sq.n_splits});
        }
        // work items per XCD, as the kernel recomputes them from (XCD, slot): the entry's chunking is the
        // host's choice among padded chunks (cut group by group) and dense ones (all groups end to end)
        const int groups = sq.n_splits * Hkv;
        const int chunk_rows = sq.chunk_rows;
        REQUIRE(chunk_rows >= 1 && chunk_rows <= kXcdChunkRowTiles && (sq.chunk_pad == 0 || sq.chunk_pad == 1),
                "%s: entry %d: chunks of %d work items, pad flag %d", who, e, chunk_rows, sq.chunk_pad);
        REQUIRE((sq.tile_major == 0 || sq.tile_major == 1) && !(sq.tile_major && sq.chunk_pad),
                "%s: entry %d: row-tile-major order needs the dense cut (flags %d, %d)", who, e, sq.tile_major, sq.chunk_pad);
        REQUIRE(!sq.chunk_pad || chunk_rows % kEnginesPerXcd == 0,
                "%s: entry %d: padded chunks of %d slots do not keep the shader engines in step", who, e, chunk_rows);
        const int chunks = sq.chunk_pad ? groups * ((sq.m_tiles + chunk_rows - 1) / chunk_rows)
                                        : (groups * sq.m_tiles + chunk_rows - 1) / chunk_rows;
        REQUIRE(sq.xcd_first == xcd_next, "%s: entry %d: first chunk on XCD %d, the entry before it stopped at %d", who, e,
                sq.xcd_first, xcd_next);
        for (int x = 0; x < 8; ++x) {
            const int r = (x - sq.xcd_first) & 7;
            per_xcd[x] += (chunks > r ? (chunks - r + 7) / 8 : 0) * chunk_rows;
        }
        xcd_next = (xcd_next + chunks) & 7;
        items += groups * sq.m_tiles;
        e += sq.n_ent;
    }
    REQUIRE(p.n_items == items, "%s: n_items %d, entries describe %d", who, p.n_items, items);
    {   // the kernel's work-group -> work-item map, replayed: every (entry, group, row tile) exactly once
        std::vector<std::vector<char>> seen(p.n_seqs);
        for (int e = 0; e < p.n_seqs; ++e)
            if (p.seq[e].n_ent > 0) seen[e].assign((size_t)p.seq[e].n_splits * Hkv * p.seq[e].m_tiles, 0);
        int64_t mapped = 0;
        for (int b = 0; b < p.items_per_xcd * 8; ++b) {
            const int xcd = b % 8;
            int local = b / 8, s = -1, gs = 0;
            for (int e = 0; e < p.n_seqs; ++e) {
                const AttnSeq &en = p.seq[e];
                const int r = (xcd - en.xcd_first) & 7, mtl = en.chunk_rows > 1 ? en.chunk_rows : 1;
                const int chunks = xcd_chunks(en.n_splits * Hkv, en.m_tiles, en.chunk_rows, en.chunk_pad);
                const int here = (chunks > r ? (chunks - r + 7) / 8 : 0) * mtl;
                if (local < here) {
                    s = e;
                    gs = r + 8 * (local / mtl);
                    break;
                }
                local -= here;
            }
            if (s < 0) continue;
            const AttnSeq &sq = p.seq[s];
            const int mtl = sq.chunk_rows > 1 ? sq.chunk_rows : 1;
            int grp, mt_up;
            if (sq.chunk_pad) {
                const int cpg = (sq.m_tiles + mtl - 1) / mtl;
                grp = gs / cpg;
                mt_up = (gs - grp * cpg) * mtl + local % mtl;
                if (mt_up >= sq.m_tiles) continue;
            } else {
                const int u = gs * mtl + local % mtl;
                if (u >= sq.n_splits * Hkv * sq.m_tiles) continue;
                if (sq.tile_major) {
                    mt_up = u / (sq.n_splits * Hkv);
                    grp = u - mt_up * (sq.n_splits * Hkv);
                } else {
                    grp = u / sq.m_tiles;
                    mt_up = u - grp * sq.m_tiles;
                }
            }
            REQUIRE(grp >= 0 && grp < sq.n_splits * Hkv, "%s: work-group %d lands in group %d of entry %d", who, b, grp, s);
            char &mark = seen[s][(size_t)grp * sq.m_tiles + mt_up];
            REQUIRE(!mark, "%s: work-groups meet at entry %d, group %d, row tile %d", who, s, grp, mt_up);
            mark = 1;
            ++mapped;
        }
        REQUIRE(mapped == items, "%s: the work-item map reaches %lld of %d work items", who, (long long)mapped, items);
    }
    REQUIRE(p.items_per_xcd == *std::max_element(per_xcd, per_xcd + 8), "%s: items_per_xcd %d, fullest XCD has %d",
            who, p.items_per_xcd, *std::max_element(per_xcd, per_xcd + 8));
    if (p.hole_width != 0) {  // a pack: one causal key range, at most two holes per key tile, rows of a few keys inside the instruction
        REQUIRE(p.hole_width > 0 && p.hole_period >= KN && p.hole_period > p.hole_width && p.hole_first >= kFewKeys - 1,
                "%s: pack with steps of %d tokens, %d of them action tokens, after %d", who, p.hole_period, p.hole_width,
                p.hole_first);
        REQUIRE(!multi && !p.multi_entry && p.n_seqs == 1 && p.seq[0].k_begin == 0, "%s: a pack is one causal key range", who);
    }
    // (the multi-entry build also serves groups of one entry; the plain build serves nothing else)
    REQUIRE(p.multi_entry || !multi, "%s: groups of several entries given to the plain build", who);
    // (a work-group whose tokens outnumber the table computes its rotations without it)
    REQUIRE(p.tab_tokens >= 0, "%s: tab_tokens %d", who, p.tab_tokens);
    REQUIRE(attention_lds_bytes(D, p.tab_tokens, p.multi_entry != 0) <= 160 * 1024, "%s: LDS", who);
    return hipSuccess;
}

// The few-keys part of a launch gives every row one wave and every visible key one lane: all rows
// of a group must see fewer than 64 keys, counted through the group's entries, and the entries
// must be the ones an attention launch would take.
hipError_t check_few(const AttnParams &p, const char *who) {
    REQUIRE(p.few_rows >= 0 && p.few_entries >= 0, "%s: few-keys part %d rows, %d entries", who, p.few_rows,
            p.few_entries);
    if (p.few_entries == 0) {
        REQUIRE(p.few_rows == 0, "%s: %d few-keys rows without entries", who, p.few_rows);
        return hipSuccess;
    }
    REQUIRE(p.few_first >= 0 && p.few_first + p.few_entries <= kMaxEntries, "%s: few-keys entries %d + %d", who,
            p.few_first, p.few_entries);
    int rows = 0;
    for (int e = p.few_first; e < p.few_first + p.few_entries;) {
        const AttnSeq &sq = p.seq[e];
        REQUIRE(sq.n_ent >= 1 && e + sq.n_ent <= p.few_first + p.few_entries, "%s: few-keys entry %d: group of %d entries",
                who, e, sq.n_ent);
        REQUIRE(sq.bt_row >= 0 && sq.bt_row < g_max_seqs, "%s: few-keys entry %d: block-table row %d", who, e, sq.bt_row);
        REQUIRE(sq.n_new >= 1 && sq.cache_len >= 0 && sq.tok_off >= 0, "%s: few-keys entry %d: chunk", who, e);
        int64_t before = 0;  // keys every row of the group sees
        int n_causal = 0;
        for (int x = e; x < e + sq.n_ent; ++x) {
            const AttnSeq &en = p.seq[x];
            if (x > e) REQUIRE(en.n_ent == 0, "%s: few-keys entry %d inside a group heads a group", who, x);
            if (hipError_t err = check_range(p, sq, en, x, who)) return err;
            n_causal += en.causal != 0;
            REQUIRE(!en.causal || x == e + sq.n_ent - 1, "%s: causal few-keys entry %d is not the group's last", who, x);
            before += (en.causal ? sq.cache_len : en.k_stop) - en.k_begin;
        }
        REQUIRE(n_causal == 1, "%s: few-keys entry %d: %d causal entries", who, e, n_causal);
        REQUIRE(before + sq.n_new < kFewKeys, "%s: few-keys entry %d: the last of %d rows sees %lld keys", who, e,
                sq.n_new, (long long)(before + sq.n_new));
        rows += sq.n_new * p.n_q_heads;
        e += sq.n_ent;
    }
    REQUIRE(p.few_rows == rows, "%s: few_rows %d, groups hold %d rows", who, p.few_rows, rows);
    return hipSuccess;
}

hipError_t launch_few_keys(const AttnParams &p, int D, hipStream_t) {
    const char *who = "few keys";
    ++g_count[6];
    if (hipError_t e = check_common(p, D, who)) return e;
    REQUIRE(p.few_rows >= 1 && p.few_first == 0 && p.n_seqs == 0, "%s: %d rows, entries from %d, %d other entries", who,
            p.few_rows, p.few_first, p.n_seqs);
    return check_few(p, who);
}

hipError_t launch_combine(const CombineParams &p, int D, hipStream_t) {
    const char *who = "combine";
    ++g_count[3];
    REQUIRE(p.part_o && p.part_ml && p.out, "%s: a null pointer", who);
    REQUIRE(p.n_seqs >= 1 && p.n_seqs <= kMaxSeqs, "%s: n_seqs %d", who, p.n_seqs);
    const size_t ws_rows = partial_rows(p.part_o, p.part_ml, D, p.out_f32 != 0);
    int rows = 0;
    for (int s = 0; s < p.n_seqs; ++s) {
        const CombineSeq &q = p.seq[s];
        REQUIRE(q.n_new >= 1 && q.n_splits >= 2 && q.tok_off >= 0, "%s: sequence %d", who, s);
        REQUIRE(q.row_begin == rows, "%s: sequence %d: row_begin %d, expected %d", who, s, q.row_begin, rows);
        REQUIRE(q.part_off >= 0 && (size_t)q.part_off + (size_t)q.n_splits * q.n_new * p.n_q_heads <= ws_rows,
                "%s: sequence %d reads past the workspace", who, s);
        // exactly the rows some attention launch left in pieces, all of whose pieces were written
        auto it = g_pending.find({q.part_off, q.tok_off});
        REQUIRE(it != g_pending.end(), "%s: sequence %d: no attention launch wrote these partial rows", who, s);
        Pending &pd = it->second;
        REQUIRE(pd.n_new == q.n_new && pd.total_splits == q.n_splits, "%s: sequence %d: %d x %d, written %d x %d", who,
                s, q.n_splits, q.n_new, pd.total_splits, pd.n_new);
        std::sort(pd.pieces.begin(), pd.pieces.end());
        int next = 0;
        for (auto &iv : pd.pieces) {
            REQUIRE(iv.first == next, "%s: sequence %d: pieces %d..%d missing or written twice", who, s, next, iv.first);
            next = iv.second;
        }
        REQUIRE(next == q.n_splits, "%s: sequence %d: pieces from %d on were never written", who, s, next);
        g_pending.erase(it);
        rows += q.n_new * p.n_q_heads;
    }
    REQUIRE(p.n_rows == rows, "%s: n_rows %d, sequences hold %d", who, p.n_rows, rows);
    return hipSuccess;
}

hipError_t launch_decode_attention(const AttnParams &p, int D, int n_workgroups, hipStream_t, hipEvent_t, hipEvent_t,
                                   const AppendParams *fused) {
    const char *who = fused ? "decode step" : "decode";
    ++g_count[2];
    if (hipError_t e = check_common(p, D, who)) return e;
    const int G = p.group, Hq = p.n_q_heads, Hkv = p.n_kv_heads, KT = kDecodeTileKeys, W = kDecodeWavesPerGroup;
    REQUIRE(p.n_seqs >= 1 && p.n_seqs <= kMaxSeqs, "%s: n_seqs %d", who, p.n_seqs);
    const size_t ws_rows = partial_rows(p.part_o, p.part_ml, D, p.out_f32 != 0);
    int wgs = 0, max_new = 0, n_groups = 0;
    std::set<int> counters;
    std::vector<std::pair<int64_t, int64_t>> regions;
    for (int e = 0; e < p.n_seqs;) {
        const AttnSeq &sq = p.seq[e];
        REQUIRE(sq.n_ent >= 1 && e + sq.n_ent <= p.n_seqs, "%s: entry %d: group of %d entries", who, e, sq.n_ent);
        REQUIRE(sq.bt_row >= 0 && sq.bt_row < g_max_seqs, "%s: entry %d: block-table row %d", who, e, sq.bt_row);
        REQUIRE(sq.n_new >= 1 && sq.n_new * G <= kDecodeRows, "%s: entry %d: %d rows", who, e, sq.n_new * G);
        REQUIRE(sq.cache_len >= 0 && sq.tok_off >= 0, "%s: entry %d: chunk", who, e);
        max_new = std::max(max_new, sq.n_new);
        int pieces = 0;
        for (int x = e; x < e + sq.n_ent; ++x) {
            const AttnSeq &en = p.seq[x];
            if (x > e) REQUIRE(en.n_ent == 0, "%s: entry %d inside a group heads a group", who, x);
            if (hipError_t err = check_range(p, sq, en, x, who)) return err;
            REQUIRE(en.bt_row == sq.bt_row && en.n_new == sq.n_new && en.cache_len == sq.cache_len &&
                        en.tok_off == sq.tok_off,
                    "%s: entry %d does not carry its group's rows", who, x);
            const int tiles = (en.k_stop + KT - 1) / KT - en.k_begin / KT;
            REQUIRE(en.n_splits >= 1 && en.tiles_per_split >= 1 &&
                        (int64_t)(en.n_splits - 1) * en.tiles_per_split < tiles &&
                        tiles <= (int64_t)en.n_splits * en.tiles_per_split,
                    "%s: entry %d: %d pieces of %d tiles for %d tiles", who, x, en.n_splits, en.tiles_per_split, tiles);
            REQUIRE(en.split_base == pieces, "%s: entry %d: %d pieces before it, split_base %d", who, x, pieces,
                    en.split_base);
            pieces += en.n_splits;
            REQUIRE(en.total_splits == sq.total_splits && en.cnt_base == sq.cnt_base && en.part_off == sq.part_off,
                    "%s: entry %d disagrees with its group", who, x);
            if (fused && en.causal)
                REQUIRE(en.k_pos >= 0 && (int64_t)en.k_pos + sq.n_new <= INT32_MAX, "%s: entry %d: k_pos", who, x);
        }
        REQUIRE(sq.total_splits == (pieces + W - 1) / W, "%s: entry %d: %d pieces in %d work-groups", who, e, pieces,
                sq.total_splits);
        if (sq.total_splits > 1) {
            REQUIRE(p.counters && p.part_o && p.part_ml, "%s: entry %d splits without counters or workspace", who, e);
            REQUIRE(sq.cnt_base >= 0 && sq.cnt_base + Hkv <= kCounters, "%s: entry %d: counters %d..", who, e, sq.cnt_base);
            for (int h = 0; h < Hkv; ++h)
                REQUIRE(counters.insert(sq.cnt_base + h).second, "%s: entry %d shares a ticket counter", who, e);
            const int64_t n = (int64_t)sq.total_splits * sq.n_new * Hq;
            REQUIRE(sq.part_off >= 0 && (size_t)(sq.part_off + n) <= ws_rows, "%s: entry %d: partial rows beyond the workspace",
                    who, e);
            regions.push_back({sq.part_off, sq.part_off + n});
        }
        wgs += sq.total_splits * Hkv;
        ++n_groups;
        e += sq.n_ent;
    }
    std::sort(regions.begin(), regions.end());
    for (size_t i = 1; i < regions.size(); ++i)
        REQUIRE(regions[i].first >= regions[i - 1].second, "%s: two groups share partial rows", who);
    REQUIRE(p.n_items == wgs && n_workgroups == wgs, "%s: %d work-groups launched, n_items %d, entries describe %d", who,
            n_workgroups, p.n_items, wgs);
    REQUIRE(p.tab_tokens >= max_new, "%s: rotation table of %d tokens, longest chunk %d", who, p.tab_tokens, max_new);
    REQUIRE(decode_lds_bytes(D, p.tab_tokens) <= 160 * 1024, "%s: LDS", who);
    if (fused) {
        REQUIRE(p.k_new == fused->k_new && p.v_new == fused->v_new && p.k_new && p.v_new, "%s: chunk inputs", who);
        REQUIRE(fused->n_seqs == n_groups, "%s: %d sequences appended, %d attended", who, fused->n_seqs, n_groups);
        // every group's chunk is the one being appended to the same sequence, at the same place
        for (int e = 0; e < p.n_seqs; ++e) {
            const AttnSeq &sq = p.seq[e];
            if (sq.n_ent == 0) continue;
            const AttnSeq &last = p.seq[e + sq.n_ent - 1];
            REQUIRE(last.causal, "%s: entry %d: the group does not end with the chunk", who, e);
            bool found = false;
            for (int s = 0; s < fused->n_seqs; ++s) {
                const AppendSeq &a = fused->seq[s];
                if (a.bt_row != sq.bt_row) continue;
                found = a.t_begin == sq.cache_len && a.n_new == sq.n_new && a.tok_off == sq.tok_off &&
                        a.pos_begin == last.k_pos;
            }
            REQUIRE(found, "%s: entry %d: no matching append", who, e);
        }
        --g_count[0];  // (counted below as part of this launch)
        if (hipError_t e = launch_rope_append(*fused, D, nullptr)) return e;
    } else {
        REQUIRE(!p.k_new && !p.v_new, "%s: chunk inputs without an append", who);
    }
    return hipSuccess;
}

hipError_t launch_zero_counters(int *counters, int n, hipStream_t) {
    ++g_count[4];
    REQUIRE(counters && n == kCounters && ((uintptr_t)counters & 15) == 0, "zero_counters: %p, %d", (void *)counters, n);
    return hipSuccess;
}

// (a host array of the real size stands in for the device array: the checks above only compare
// addresses and sizes)
hipError_t static_scratch(void **ptr, size_t *bytes) {
    static std::vector<unsigned char> fake(kStaticScratchBytes + 256);
    *ptr = (void *)(((uintptr_t)fake.data() + 255) & ~(uintptr_t)255);
    *bytes = kStaticScratchBytes;
    return hipSuccess;
}

hipError_t launch_pages_copy(const PageCopyParams &p, hipStream_t) {
    ++g_count[5];
    REQUIRE(p.n >= 1 && p.n <= kMaxPagesPerCopy && p.page_bytes > 0 && p.page_bytes % 16 == 0, "pages_copy: %d pages of %d bytes",
            p.n, p.page_bytes);
    return hipSuccess;
}

}  // namespace evl

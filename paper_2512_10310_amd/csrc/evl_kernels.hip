// gfx950 (CDNA4) kernels for KV-cache reuse with contiguous RoPE (paper Sec. 3.2):
//   rope_append_kernel : rotate the new keys at their contiguous position ids and scatter
//                        keys / values into the paged per-layer cache.
//   attn_kernel        : flash-style attention of the new chunk's queries over cache + chunk
//                        (bf16 MFMA, fp32 accumulation, online softmax), GQA rows packed.  A
//                        second build walks through several key ranges with different query
//                        rotations (history chosen by a frame sampler).
//   combine_kernel     : merge the per-key-range partial results of attn_kernel.
//   decode_kernel      : attention for chunks of a few tokens (the action tokens that follow a
//                        frame): one wave per piece of the key range, merged in the kernel;
//                        decode_step_kernel appends the chunk in the same launch.
//   pages_copy_kernel  : whole pages between two pools (cache offload to host memory).
//
// 64-wide wavefronts, v_mfma_f32_32x32x16_bf16.  The attention kernel computes the scores
// transposed (keys along M, queries along N), so that each lane owns one query column: the
// row maximum and row sum of the softmax then need a single exchange between lane l and
// lane l+32, the probabilities are already in the register layout the second contraction
// wants for its B operand, and the running rescale of the output is a per-lane scalar.
#include "evl_internal.h"

#include <hip/hip_ext.h>

#include <mutex>
#include <type_traits>

namespace evl {

typedef __bf16 bf16;
typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// cos / sin of the rotary angle position * theta_j.  rev_freq = theta_j / (2 pi) arrives in
// double; the product is formed and reduced to a fraction of a turn in [-0.5, 0.5] in double
// (positions reach ~6.6e4 and theta_0 = 1, so a float angle would be off by ~4e-3 rad), and
// the fraction goes to the hardware sine / cosine, which take their argument in turns.
// Keys (at append) and queries (in the attention prologue) both use this one function, so
// the relative-position property holds to rounding.
__device__ __forceinline__ float2 rope_cos_sin(int pos, double rev_freq) {
    const double a = (double)pos * rev_freq;
    const float frac = (float)(a - rint(a));
    return make_float2(__builtin_amdgcn_cosf(frac), __builtin_amdgcn_sinf(frac));
}

// A key's channel pair (a, b) turned by (cos, sin), rounded to bf16: the one place where keys are
// rotated.  The append stores these bits and the fused step's attention rebuilds them from the
// inputs, so both must round alike: each product and sum is a separate fp32 operation here,
// whatever the surrounding code would let the compiler contract.
__device__ __forceinline__ void rotate_key_pair(float a, float b, float2 cs, bf16 &lo, bf16 &hi) {
#pragma clang fp contract(off)
    const float ac = a * cs.x, bs = b * cs.y, bc = b * cs.x, as = a * cs.y;
    lo = (bf16)(ac - bs);
    hi = (bf16)(bc + as);
}

__device__ __forceinline__ int clamp_page(int page, int n_pages) {
    return (int)min((unsigned)page, (unsigned)(n_pages - 1));
}

// 8-byte stores and loads that are coherent across the chip's XCDs (each XCD has its own L2):
// relaxed atomics at device scope, i.e. accesses that go past the non-coherent L2 lines.  Used
// for partial results that another work-group of the same launch reads.
__device__ __forceinline__ void store_coherent8(void *p, uint64_t bits) {
    __hip_atomic_store((uint64_t *)p, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t load_coherent8(const void *p) {
    return __hip_atomic_load((const uint64_t *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename V>
__device__ __forceinline__ V load_vec(const V *p, bool coherent) {
    static_assert(sizeof(V) % 8 == 0, "whole 8-byte words only");
    if (!coherent) return *p;
    union { uint64_t u[sizeof(V) / 8]; V v; } x;
#pragma unroll
    for (size_t w = 0; w < sizeof(V) / 8; ++w) x.u[w] = load_coherent8((const uint64_t *)p + w);
    return x.v;
}
__device__ __forceinline__ float2 load_f2(const float2 *p, bool coherent) {
    if (!coherent) return *p;
    union { uint64_t u; float2 v; } x;
    x.u = load_coherent8(p);
    return x.v;
}

// Merge of the per-piece partial results of one output row: out = sum_s w_s O_s / sum_s w_s with
// w_s = 2^(m_s - m) l_s, m = max_s m_s, over the normalised partials O_s.  Called by D/8 lanes
// per row, lane `sub` handling 8 channels.  Piece s of the row sits `stride` partial rows
// after piece s-1; o_idx: element index of the row in `out`.
template <int D, typename PT>
__device__ __forceinline__ void merge_row(const void *part_o, const float *part_ml, size_t prow0,
                                          size_t stride, int n_splits, void *out, bool out_f32,
                                          size_t o_idx, int sub) {
    // pieces in flight per lane: all of them for up to 16 (8 with fp32 partials), so that a row
    // costs one memory round trip; longer lists go chunk by chunk with a running reference
    constexpr int U = sizeof(PT) == 2 ? 16 : 8;
    typedef PT ptx8 __attribute__((ext_vector_type(8)));
    const float2 *ml = (const float2 *)part_ml + prow0;
    const ptx8 *po = (const ptx8 *)((const PT *)part_o + prow0 * D) + sub;
    const size_t ostride = stride * (D / 8);
    float m = -INFINITY, wsum = 0.f, acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    for (int sp = 0; sp < n_splits; sp += U) {
        float2 q[U];
        ptx8 o[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (sp + u < n_splits) {
                q[u] = ml[(sp + u) * stride];
                o[u] = po[(sp + u) * ostride];
            } else {
                q[u] = make_float2(-INFINITY, 0.f);
#pragma unroll
                for (int e = 0; e < 8; ++e) o[u][e] = (PT)0.f;
            }
        }
        float m_new = m;
#pragma unroll
        for (int u = 0; u < U; ++u) m_new = fmaxf(m_new, q[u].x);
        const float keep = __builtin_amdgcn_exp2f(m - m_new);  // 0 for the first chunk
        m = m_new;
        wsum *= keep;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] *= keep;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float w = __builtin_amdgcn_exp2f(q[u].x - m) * q[u].y;
            wsum += w;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += w * (float)o[u][e];
        }
    }
    const float inv = 1.0f / wsum;
    if (out_f32) {
#pragma unroll
        for (int e = 0; e < 8; e += 4) {
            f32x4 v;
#pragma unroll
            for (int c = 0; c < 4; ++c) v[c] = acc[e + c] * inv;
            *(f32x4 *)((float *)out + o_idx + sub * 8 + e) = v;
        }
    } else {
        bf16x8 ob;
#pragma unroll
        for (int e = 0; e < 8; ++e) ob[e] = (bf16)(acc[e] * inv);
        *(bf16x8 *)((bf16 *)out + o_idx + sub * 8) = ob;
    }
}

// The same merge for a handful of rows, done by a whole work-group of NT threads: with few
// rows, one thread per (row, 8-channel slice) would walk through the pieces one memory round
// trip after the other.  Here the pieces are dealt to as many thread groups as fit (group sg
// takes pieces sg*U .. sg*U+U-1, then n_par*U further on, ...), each thread keeps a running
// (reference, weight sum, 8 outputs), and the groups' results meet in LDS.  `scratch`: NT * 10
// floats of LDS, free for use; all NT threads must call (two barriers inside).  Row rr of the
// n_rows rows has its pieces at partial row prow0(rr) + s * stride and goes to element
// o_idx(rr) of `out`; reads go past the L2 (pieces come from other work-groups of the launch).
template <int D, typename PT, int NT, typename RowFn>
__device__ __forceinline__ void merge_rows_parallel(const void *part_o, const float *part_ml, size_t stride,
                                                    int n_splits, int n_rows, void *out, bool out_f32,
                                                    float *scratch, RowFn row_fn) {
    constexpr int LPR = D / 8, U = 8;  // U: pieces in flight per thread
    typedef PT ptx8 __attribute__((ext_vector_type(8)));
    const int tid = threadIdx.x;
    const int per_group = n_rows * LPR;
    const int n_par = max(1, min(NT / per_group, (n_splits + U - 1) / U));
    const int sg = tid / per_group, rem = tid - sg * per_group;
    const int rr = rem / LPR, sub = rem - rr * LPR;
    const bool active = sg < n_par;
    float m = -INFINITY, wsum = 0.f, acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    size_t prow0 = 0, o_idx = 0;
    if (active) {
        row_fn(rr, prow0, o_idx);
        const float2 *ml = (const float2 *)part_ml + prow0;
        const ptx8 *po = (const ptx8 *)((const PT *)part_o + prow0 * D) + sub;
        const size_t ostride = stride * (D / 8);
        for (int base = sg * U; base < n_splits; base += n_par * U) {
            float2 q[U];
            ptx8 o[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                // (clamped, not skipped: unconditional loads go out together)
                const int si = min(base + u, n_splits - 1);
                q[u] = load_f2(ml + si * stride, true);
                o[u] = load_vec(po + si * ostride, true);
            }
            float mx = m;
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (base + u < n_splits) mx = fmaxf(mx, q[u].x);
            const float a = __builtin_amdgcn_exp2f(m - mx);  // m = -inf at first: a = 0
            m = mx;
            wsum *= a;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] *= a;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float w = base + u < n_splits ? __builtin_amdgcn_exp2f(q[u].x - m) * q[u].y : 0.f;
                wsum += w;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] += w * (float)o[u][e];
            }
        }
    }
    if (n_par > 1) {
        __syncthreads();
        if (active) {
            float *mine = scratch + (size_t)tid * 10;
            mine[0] = m;
            mine[1] = wsum;
#pragma unroll
            for (int e = 0; e < 8; ++e) mine[2 + e] = acc[e];
        }
        __syncthreads();
        if (active && sg == 0) {
            for (int g2 = 1; g2 < n_par; ++g2) {
                const float *o2 = scratch + (size_t)(tid + g2 * per_group) * 10;
                const float m2 = o2[0];
                const float mx = fmaxf(m, m2);
                const float a = mx == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m - mx);
                const float b = mx == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m2 - mx);
                m = mx;
                wsum = wsum * a + o2[1] * b;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] = acc[e] * a + o2[2 + e] * b;
            }
        }
    }
    if (active && sg == 0) {
        const float inv = 1.0f / wsum;
        if (out_f32) {
#pragma unroll
            for (int e = 0; e < 8; e += 4) {
                f32x4 v;
#pragma unroll
                for (int c = 0; c < 4; ++c) v[c] = acc[e + c] * inv;
                *(f32x4 *)((float *)out + o_idx + sub * 8 + e) = v;
            }
        } else {
            bf16x8 ob;
#pragma unroll
            for (int e = 0; e < 8; ++e) ob[e] = (bf16)(acc[e] * inv);
            *(bf16x8 *)((bf16 *)out + o_idx + sub * 8) = ob;
        }
    }
}

// =========================================================================================
// Fused RoPE + append.  One work-group per (sequence, touched page, KV head).
//   threads [0, 16 * D/16): one token x one 8-channel slice pair (j, j + D/2) of the key.
//   all threads: stage the page's value rows in LDS, write them back transposed.
// =========================================================================================
// (the body serves two kernels: work-group `item` of the append, done by the first kThreads
// threads of the work-group; vt: LDS staging for the page's value rows)
template <int D>
__device__ __forceinline__ void rope_append_body(const AppendParams &p, const int item, bf16 (*vt)[D + 8]) {
    constexpr int NPAIR = D / 16;  // 8-channel slices in half a head vector
    if (item >= p.n_items) return;
    int s = 0;
    while (s + 1 < p.n_seqs && item >= p.seq[s + 1].item_begin) ++s;
    const AppendSeq sq = p.seq[s];
    const int Hkv = p.n_kv_heads;
    const int local = item - sq.item_begin;
    const int kvh = local % Hkv;
    const int page_idx = sq.t_begin / kPage + local / Hkv;  // index into the block-table row
    const int t_end = sq.t_begin + sq.n_new;

    // threads past the first kThreads (a larger work-group of another kernel) only meet the barrier
    const int tid = threadIdx.x < kThreads ? (int)threadIdx.x : 1 << 20;
    const bf16 *k_new = (const bf16 *)p.k_new;
    const bf16 *v_new = (const bf16 *)p.v_new;

    // All input loads go out first and without conditions (threads with nothing to do read a
    // clamped address), the block-table entry right behind them: the page id is needed for the
    // stores only, so its round trip runs beside those of the inputs instead of before them.
    constexpr int VPIECES = kPage * (D / 8);  // 16-byte pieces of the page's value rows
    static_assert(VPIECES <= kThreads, "one value piece per thread");
    const int v_tl = (tid % VPIECES) / (D / 8), v_c = tid % (D / 8);
    const int v_t = page_idx * kPage + v_tl;
    const bool v_mine = tid < VPIECES && v_t >= sq.t_begin && v_t < t_end;
    const int v_i = max(min(v_t - sq.t_begin, sq.n_new - 1), 0);
    const bf16x8 v_in = *(const bf16x8 *)(v_new + ((size_t)(sq.tok_off + v_i) * Hkv + kvh) * D + 8 * v_c);
    const int k_tl = (tid % (kPage * NPAIR)) / NPAIR, k_c = tid % NPAIR;
    const int k_t = page_idx * kPage + k_tl;
    const bool k_mine = tid < kPage * NPAIR && k_t >= sq.t_begin && k_t < t_end;
    const int k_i = max(min(k_t - sq.t_begin, sq.n_new - 1), 0);
    const bf16 *k_src = k_new + ((size_t)(sq.tok_off + k_i) * Hkv + kvh) * D + 8 * k_c;
    const bf16x8 k_lo = *(const bf16x8 *)k_src;
    const bf16x8 k_hi = *(const bf16x8 *)(k_src + D / 2);
    double k_rf[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) k_rf[e] = p.rev_freq[8 * k_c + e];
    __builtin_amdgcn_sched_barrier(0);
    const int pid =
        clamp_page(p.block_table[(size_t)sq.bt_row * p.max_pages_per_seq + page_idx], p.n_pages);
    __builtin_amdgcn_sched_barrier(0);
    if (v_mine) *(bf16x8 *)&vt[v_tl][8 * v_c] = v_in;  // (the first load to return)
    bf16 *k_page = (bf16 *)p.k_pool + ((size_t)pid * Hkv + kvh) * kPage * D;
    bf16 *v_page = (bf16 *)p.v_pool + ((size_t)pid * Hkv + kvh) * D * kPage;

    // ---- keys: rotate and store ----
    if (tid < kPage * NPAIR) {
        const int tl = k_tl, c = k_c;
        const int t = k_t;
        if (k_mine) {
            const int i = t - sq.t_begin;
            int pos = (int)sq.pos_begin + i;
            if (p.hole_width > 0) {  // a pack: ids skip the action tokens of earlier steps
                const int st = t < p.hole_first ? 0 : (t - p.hole_first) / p.hole_period;
                const int s0 = sq.t_begin < p.hole_first ? 0 : (sq.t_begin - p.hole_first) / p.hole_period;
                pos -= p.hole_width * (st - s0);
            }
            const bf16x8 lo = k_lo, hi = k_hi;
            bf16x8 rlo, rhi;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float2 cs = rope_cos_sin(pos, k_rf[e]);
                bf16 r0, r1;
                rotate_key_pair((float)lo[e], (float)hi[e], cs, r0, r1);
                rlo[e] = r0;
                rhi[e] = r1;
            }
            bf16 *dst = k_page + (size_t)tl * D + 8 * c;
            *(bf16x8 *)dst = rlo;
            *(bf16x8 *)(dst + D / 2) = rhi;
            if (p.pos_tags && kvh == 0 && c == 0) p.pos_tags[(size_t)pid * kPage + tl] = (int32_t)pos;
        } else if (t >= t_end) {
            // slots of this page past the sequence's end: keep them finite (zero), because the
            // attention kernel multiplies masked probabilities (exact zeros) with whatever
            // the page holds there
            bf16x8 z;
#pragma unroll
            for (int e = 0; e < 8; ++e) z[e] = (bf16)0.f;
            bf16 *dst = k_page + (size_t)tl * D + 8 * c;
            *(bf16x8 *)dst = z;
            *(bf16x8 *)(dst + D / 2) = z;
        }
    }

    // ---- values: [token][d] rows -> [d][token] page ----
    __syncthreads();
    for (int ch = tid; ch < D * 2; ch += kThreads) {
        const int dd = ch / 2, half = ch % 2;
        const int t0 = page_idx * kPage + half * 8;
        bf16 *dst = v_page + (size_t)dd * kPage + half * 8;
        if (t0 >= sq.t_begin) {
            bf16x8 w;
#pragma unroll
            for (int e = 0; e < 8; ++e) w[e] = t0 + e < t_end ? vt[half * 8 + e][dd] : (bf16)0.f;
            *(bf16x8 *)dst = w;
        } else {
            // columns of earlier tokens stay as they are; new tokens are written, slots past
            // the end are zeroed
            for (int e = 0; e < 8; ++e)
                if (t0 + e >= sq.t_begin) dst[e] = t0 + e < t_end ? vt[half * 8 + e][dd] : (bf16)0.f;
        }
    }
}

template <int D>
__global__ __launch_bounds__(kThreads) void rope_append_kernel(const AppendParams p) {
    __shared__ bf16 vt[kPage][D + 8];
    rope_append_body<D>(p, blockIdx.x, vt);
}

// =========================================================================================
// Rows that see fewer than 64 keys.  One wave per (token, query head) row, everything in fp32:
// lane f rotates the query's channel pair of frequency f (per entry, at that entry's query
// position) into a wave-private LDS row; lane j owns the j-th visible key, counted through the
// group's entries, and forms its score as a plain dot product with the stored (rotated) key;
// maximum and sum go over the lanes; then lane c accumulates channels c (and c + 64) of the
// output over the keys.  No barrier: waves are independent.
// =========================================================================================
// (the body serves two kernels: row = index of the wave's row among the launch's few-keys rows;
// qs: D floats of LDS of the wave's own)
template <int D>
__device__ __forceinline__ void few_keys_body(const AttnParams &p, int row, float *qs) {
    const int lane = threadIdx.x & 63;
    const int G = p.group, Hq = p.n_q_heads, Hkv = p.n_kv_heads;
    if (row >= p.few_rows) return;
    int s = p.few_first;  // first entry of the row's group
    for (;;) {
        if (s >= p.few_first + p.few_entries || p.seq[s].n_ent <= 0) return;  // (few_rows is the groups' row count: never taken)
        const int rows_here = p.seq[s].n_new * Hq;
        if (row < rows_here) break;
        row -= rows_here;
        s += p.seq[s].n_ent;
    }
    const AttnSeq sq = p.seq[s];
    const int i = row / Hq, hq = row - i * Hq, kvh = hq / G;
    const int f = lane & (D / 2 - 1);  // (D = 64: the upper half of the wave repeats the lower)
    const bf16 *qrow = (const bf16 *)p.q + ((size_t)(sq.tok_off + i) * Hq + hq) * D;
    const float qa = (float)qrow[f], qb = (float)qrow[f + D / 2];
    const double rev_freq = p.rev_freq[f];
    const int32_t *bt = p.block_table + (size_t)sq.bt_row * p.max_pages_per_seq;

    int n_keys = 0, my_t = 0, my_pid = 0;
    bool mine = false, is_first = false;  // is_first: the first key of its range
    float score = -INFINITY;  // log2 domain
    for (int e = s; e < s + sq.n_ent; ++e) {
        const int kb = p.seq[e].k_begin;
        const int ks = p.seq[e].causal ? min(p.seq[e].k_stop, sq.cache_len + i + 1) : p.seq[e].k_stop;
        const int len = ks - kb;
        if (len <= 0) continue;
        const float2 cs = rope_cos_sin(p.seq[e].q_pos + i, rev_freq);
        // (a wave's LDS accesses are served in order: the reads below see these writes, and the
        // next entry's writes come after this entry's reads)
        qs[f] = qa * cs.x - qb * cs.y;
        qs[f + D / 2] = qb * cs.x + qa * cs.y;
        asm volatile("" ::: "memory");
        const int jj = lane - n_keys;
        if (jj >= 0 && jj < len) {
            mine = true;
            is_first = jj == 0;
            my_t = kb + jj;
            my_pid = clamp_page(bt[my_t / kPage], p.n_pages);
            const bf16 *krow =
                (const bf16 *)p.k_pool + (((size_t)my_pid * Hkv + kvh) * kPage + my_t % kPage) * D;
            float acc = 0.f;
#pragma unroll
            for (int c = 0; c < D / 8; ++c) {
                const bf16x8 kk = *(const bf16x8 *)(krow + 8 * c);
#pragma unroll
                for (int x = 0; x < 8; ++x) acc = fmaf(qs[8 * c + x], (float)kk[x], acc);
            }
            score = acc * p.q_scale;
        }
        asm volatile("" ::: "memory");
        n_keys += len;
    }
    n_keys = min(n_keys, 64);  // (the host sends only rows with fewer than 64 keys)

    float m = score;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    const float pj = mine ? __builtin_amdgcn_exp2f(score - m) : 0.f;
    float l = pj;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) l += __shfl_xor(l, off);

    // Values: [page][head][channel][16 tokens], so the (up to 16) keys that share a page are 32
    // contiguous bytes per channel.  The visible keys fall into page segments (a segment starts
    // where a key range starts or a page does); lane c takes channel c (and c + 64) and walks
    // through the segments four at a time, all loads of a round first.  Which lane holds a
    // segment's first key comes from a ballot; its page, first token and the weights are read
    // from that lane and its successors (wave-uniform reads, no memory access).
    const bool head_of_segment = mine && (my_t % kPage == 0 || is_first);
    unsigned long long heads = __ballot(head_of_segment);
    constexpr int CB = D == 128 ? 2 : 1;  // 64-channel blocks per lane
    float o[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) o[cb] = 0.f;
    const bf16 *v_pool = (const bf16 *)p.v_pool;
    const int pj_bits = __float_as_int(pj);
    while (heads) {
        int h0[4], cnt[4], slot0[4];
        bf16x8 w0[4][CB], w1[4][CB];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const bool any = heads != 0;
            h0[u] = any ? __ffsll(heads) - 1 : 0;
            heads &= heads - 1;
            const int next = heads ? __ffsll(heads) - 1 : n_keys;
            cnt[u] = any ? next - h0[u] : 0;
            const int pid = __builtin_amdgcn_readlane(my_pid, h0[u]);
            slot0[u] = __builtin_amdgcn_readlane(my_t, h0[u]) % kPage;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                const bf16 *src = v_pool + (((size_t)pid * Hkv + kvh) * D + lane + 64 * cb) * kPage;
                w0[u][cb] = *(const bf16x8 *)src;
                w1[u][cb] = *(const bf16x8 *)(src + 8);
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int sl = 0; sl < kPage; ++sl) {
                const int k = sl - slot0[u];  // which key of the segment sits in this slot
                const bool on = k >= 0 && k < cnt[u];
                const float w = __int_as_float(__builtin_amdgcn_readlane(pj_bits, on ? h0[u] + k : 0));
                // (slots outside the segment are other tokens' or unused: selected away, not multiplied by zero)
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
                    o[cb] += on ? w * (float)(sl < 8 ? w0[u][cb][sl] : w1[u][cb][sl - 8]) : 0.f;
            }
    }
    const float o0 = o[0], o1 = o[CB - 1];
    const float inv = 1.0f / l;
    const size_t o_idx = ((size_t)(sq.tok_off + i) * Hq + hq) * D;
    if (p.out_f32) {
        ((float *)p.out)[o_idx + lane] = o0 * inv;
        if (D == 128) ((float *)p.out)[o_idx + lane + 64] = o1 * inv;
    } else {
        ((bf16 *)p.out)[o_idx + lane] = (bf16)(o0 * inv);
        if (D == 128) ((bf16 *)p.out)[o_idx + lane + 64] = (bf16)(o1 * inv);
    }
}

constexpr int kFewRowsPerGroup = 4;  // waves (rows) per work-group of the kernel on its own

template <int D>
__global__ __launch_bounds__(kFewRowsPerGroup * 64) void few_keys_kernel(const AttnParams p) {
    __shared__ float q_rot[kFewRowsPerGroup][D];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    few_keys_body<D>(p, blockIdx.x * kFewRowsPerGroup + wave, q_rot[wave]);
}

// =========================================================================================
// Chunk attention.
//
// Work item = (sequence, KV head, key-range split, row tile).  Rows are the packed pairs
// (chunk token i, query head g of the KV head's group), row = i * G + g, so that the G query
// heads sharing a KV head sit in the same tile and every K / V byte staged in LDS is used by
// all of them.  A work-group has 8 wavefronts (two per SIMD); each owns a block of 32 rows and
// walks the key range in tiles of 64 keys (4 pages):
//
//   S^T[key][row]  = K[key][:] . Q^T[:][row]        A = K tile (LDS), B = Q (registers)
//   O^T[ch][row]  += V^T[ch][key] . P^T[key][row]    A = V^T tile (LDS), B = P (registers)
//
// Lane l = (j, h) with j = l % 32, h = l / 32 owns row j of its block.  The 32x32 result of
// a 32-key block leaves lane (j, h) with 16 scores; the K rows are fed to the MFMA in a
// permuted order chosen so that those 16 scores belong to keys 16*(v/8) + 8*h + v%8
// (v = 0..15): score registers 8s..8s+7 are then 8 consecutive keys, exactly the 8
// contraction slots lane (j, h) supplies to the k-step s of the second MFMA, and the
// matching A operand is one 16-byte read of 8 consecutive keys of one channel of V^T.
//
// K/V tiles travel HBM -> LDS directly (global_load_lds_dwordx4, no register staging) into
// a ring of kStages tile buffers, two tiles ahead of the math, with one barrier per tile.
// Two waves share the fetch of each of a tile's four pages.  A direct load writes lane i's 16 bytes at
// base + 16*i, so the LDS layout is fixed per 1 KB instruction and bank conflicts are
// avoided by choosing which global chunk each lane fetches:
//   K: rows of D bf16, 16-byte chunk c of row R sits at chunk position c ^ g(R);
//   V: per (page, 32-channel block) 1 KB = [key half][32 channels][8 keys].
// =========================================================================================

constexpr int kStages = kAttnStages;

template <int D>
struct Tile {
    static constexpr int KN = kKeyTile;
    static constexpr int CH = D / 8;               // 16-byte chunks per K row
    static constexpr int ROWS_PER_LOAD = 64 / CH;  // K rows one wave-wide direct load covers
    static constexpr int ITS = D / 32;             // direct loads per page, for K and for V
    static constexpr int K_BYTES = KN * D * 2;
    static constexpr int V_PAGE_BYTES = D * kPage * 2;
    static constexpr int V_BYTES = (KN / kPage) * V_PAGE_BYTES;
    static constexpr int STAGE_BYTES = K_BYTES + V_BYTES;
};

// Every work-group covers 256 packed rows: 8 wavefronts (two per SIMD) x 1 block of 32 rows.
constexpr int kRowsPerWorkgroup = kAttnRows;
static_assert(Tile<128>::STAGE_BYTES == attention_stage_bytes(128) &&
                  Tile<64>::STAGE_BYTES == attention_stage_bytes(64),
              "the host side sizes the LDS ring from attention_stage_bytes");

// One wave-wide 16-byte-per-lane load from global memory straight into LDS: lane i fetches the
// 16 bytes at base + off (base: wave-uniform 64-bit address in SGPRs, off: per-lane byte
// offset) and its data lands at lds_base + 16*i.  Written as asm so that the compiler does not
// serialise the ring with full vmcnt waits; completion is awaited explicitly (wait_loads)
// before the barrier.
__device__ __forceinline__ void load_to_lds_16(const void *base, unsigned off, unsigned lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_base), "v"(off), "s"(base)
                 : "memory");
}

// s_waitcnt vmcnt(N) only (expcnt / lgkmcnt fields left at "no wait"); N is an immediate.
template <int N>
__device__ __forceinline__ void wait_loads() {
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// MULTI: built for groups of several entries (the sampled call); the plain build has one
// entry per group and none of the entry-to-entry machinery.
// HOLES: the sequence is a pack under the action-isolating mask (see AttnParams::hole_*).
template <int D, int QB, bool MULTI, bool HOLES = false>
__global__ __launch_bounds__(kRowsPerWorkgroup / (32 * QB) * 64) void attn_kernel(const AttnParams p) {
    static_assert(!(MULTI && HOLES), "a pack is one causal key range");
    using T = Tile<D>;
    constexpr int KN = T::KN;
    constexpr int KS = D / 16;   // k-steps of the score contraction
    constexpr int DB = D / 32;   // 32-channel blocks of the output
    constexpr int MT = kRowsPerWorkgroup;
    constexpr int NW = MT / (32 * QB);          // wavefronts
    constexpr int PARTS = NW / 4;               // wavefronts sharing the fetch of one page
    constexpr int WITS = T::ITS / PARTS;        // direct loads per wave per page, K and V each
    static_assert(T::ITS % PARTS == 0, "page fetch must split evenly over its waves");
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)smem;

    // Work-groups behind the matrix part serve the rows that see fewer than 64 keys, one per wave.
    if ((int)blockIdx.x >= p.items_per_xcd * 8) {
        const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        few_keys_body<D>(p, ((int)blockIdx.x - p.items_per_xcd * 8) * NW + w, (float *)smem + w * D);
        return;
    }

    // XCD-aware work-group -> work-item map.  The hardware deals work-groups round-robin to
    // the 8 XCDs, each with its own L2: work-group b runs on XCD b % 8 and is that XCD's
    // slot b / 8.  An entry's work items -- its (KV head, split) groups of m_tiles row tiles --
    // are cut into chunks of chunk_rows items (group by group, or all groups end to end: the
    // host's choice per entry); the row tiles of one group read the same K/V, so a chunk takes
    // consecutive slots of one XCD -- chunks of at most kXcdChunkRowTiles items, so that a group
    // of many row tiles (a long prefill) is not pinned to one XCD; the chunks of the launch go
    // round the XCDs entry after entry (an entry's first chunk to XCD xcd_first, where the entry
    // before it stopped), which spreads every sequence -- long or short -- over the whole chip
    // and loads the XCDs evenly to within one chunk.  Sequences are listed longest first.
    const int G = p.group, Hq = p.n_q_heads, Hkv = p.n_kv_heads;
    const int xcd = blockIdx.x % 8;
    int local = blockIdx.x / 8;
    int s = -1, gs = 0;
    if (p.n_seqs <= 4) {  // a few entries: a scalar walk is the shortest
        for (int e = 0; e < p.n_seqs; ++e) {
            const int r = (xcd - p.seq[e].xcd_first) & 7;  // first chunk of entry e that lands on this XCD
            const int mtl = max(p.seq[e].chunk_rows, 1);
            const int chunks = xcd_chunks(p.seq[e].n_splits * Hkv, p.seq[e].m_tiles, p.seq[e].chunk_rows, p.seq[e].chunk_pad);
            const int here = (chunks > r ? (chunks - r + 7) / 8 : 0) * mtl;
            if (local < here) {
                s = e;
                gs = r + 8 * (local / mtl);
                break;
            }
            local -= here;
        }
    }
    // Many entries: the search runs over 64 entries at a time, one per lane (one load per lane
    // instead of a chain of dependent scalar loads): items each entry puts on this XCD, an
    // inclusive prefix sum over the lanes, and the first lane whose sum exceeds this
    // work-group's slot.
    for (int e0 = 0; p.n_seqs > 4 && e0 < p.n_seqs; e0 += 64) {
        const int ln = threadIdx.x & 63, e = e0 + ln;
        int here = 0, r = 0, mtl = 1;
        if (e < p.n_seqs) {
            const int chunks = xcd_chunks(p.seq[e].n_splits * Hkv, p.seq[e].m_tiles, p.seq[e].chunk_rows, p.seq[e].chunk_pad);
            mtl = max(p.seq[e].chunk_rows, 1);
            r = (xcd - p.seq[e].xcd_first) & 7;  // first chunk of entry e that lands on this XCD
            here = (chunks > r ? (chunks - r + 7) / 8 : 0) * mtl;
        }
        int incl = here;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int up = __shfl_up(incl, off);
            if (ln >= off) incl += up;
        }
        const int total = __shfl(incl, 63);
        if (local < total) {
            const int hit = __ffsll((unsigned long long)__ballot(incl > local)) - 1;
            s = e0 + hit;
            local -= __shfl(incl - here, hit);
            gs = __shfl(r, hit) + 8 * (local / __shfl(mtl, hit));
            break;
        }
        local -= total;
    }
    if (s < 0) return;  // this XCD has fewer items than the fullest one
    s = __builtin_amdgcn_readfirstlane(s);
    gs = __builtin_amdgcn_readfirstlane(gs);
    local = __builtin_amdgcn_readfirstlane(local);
    const AttnSeq sq = p.seq[s];
    // gs counts the entry's chunks.  Padded cut: chunk gs % cpg of group gs / cpg.  Dense cut: the
    // chunk holds items gs * mtl .. of the entry, item u being row tile u % m_tiles (counted from
    // the last) of group u / m_tiles.
    const int mtl = max(sq.chunk_rows, 1);
    int grp, mt_up;
    if (sq.chunk_pad) {
        const int cpg = (sq.m_tiles + mtl - 1) / mtl;
        grp = gs / cpg;
        mt_up = (gs - grp * cpg) * mtl + local % mtl;
        if (mt_up >= sq.m_tiles) return;  // padding of a group's last chunk
    } else {
        const int u = gs * mtl + local % mtl;
        if (u >= sq.n_splits * Hkv * sq.m_tiles) return;  // padding of the entry's last chunk
        if (sq.tile_major) {  // row tile after row tile: the groups' longest work items come first
            const int groups = sq.n_splits * Hkv;
            mt_up = u / groups;
            grp = u - mt_up * groups;
        } else {
            grp = u / sq.m_tiles;
            mt_up = u - grp * sq.m_tiles;
        }
    }
    // last row tile first: under the causal mask it sees the most keys, and the longest
    // work-groups should not be the ones that start last
    const int mt = sq.m_tiles - 1 - mt_up;
    const int split = grp % sq.n_splits;
    const int kvh = grp / sq.n_splits;

    const int R = sq.n_new * G;  // packed rows of this sequence
    const int C = sq.cache_len;
    const int row0 = mt * MT;
    // Pack (HOLES): step of a sequence index, and the id offset of chunk token `tok` from the
    // chunk's first token (ids skip the action tokens of the steps in between).
    const int h_first = HOLES ? p.hole_first : 0, h_period = HOLES ? p.hole_period : 1;
    const int h_width = HOLES ? p.hole_width : 0;
    auto step_of = [&](int t) __attribute__((always_inline)) -> int {
        return t < h_first ? 0 : (t - h_first) / h_period;
    };
    auto chunk_pos = [&](int tok) __attribute__((always_inline)) -> int {
        return HOLES ? tok - h_width * (step_of(C + tok) - step_of(C)) : tok;
    };
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 31, h = lane >> 5;

    // ---- Loads of the prologue, in the order they are issued (a wave's loads return in order):
    // the frequency this thread fills into the rotation table, the block-table entries of the
    // first tiles, then the queries.  The two small ones are not held up behind the 8 KB of
    // queries: the table is built and the first tiles are requested while the queries arrive.
    // (the table's row length divides the work-group size, so a thread always meets the same
    // frequency)
    const double my_rev_freq = p.rev_freq[tid & (D / 2 - 1)];
    const int wrow0 = row0 + wave * 32 * QB;
    bf16x8 Q[QB][KS];
    int row_tok[QB], row_head[QB];
    bool row_ok[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int rb = wrow0 + qb * 32;
        const int r = min(rb + j, R - 1);
        const int tok = r / G, g = r - tok * G;
        row_ok[qb] = rb + j < R;
        row_tok[qb] = tok;
        row_head[qb] = kvh * G + g;
    }

    // keys this work-group may need: everything up to its last row's own token
    const int wg_last_tok = (min(row0 + MT, R) - 1) / G;
    // Entry e of the group: its key range [k_lo, k_hi) (cut by causality where the entry holds
    // the chunk itself) and the key tiles t0 .. t0 + nt - 1 that cover it.  Keys of the first
    // and last tile that fall outside the range are masked.
    const int e_end = s + sq.n_ent;
    // Multi-entry build: the group's entries (at most 64) sit in registers, lane x holding entry
    // s + x, fetched with one load per field for all entries at once; a walk through the entries
    // then reads lanes instead of waiting for one scalar load after the other.
    int ent_begin = 0, ent_stop = 0, ent_q_pos = 0, ent_causal = 0;
    if (MULTI) {
        const int x = s + min(lane, sq.n_ent - 1);
        ent_begin = p.seq[x].k_begin;
        ent_stop = p.seq[x].k_stop;
        ent_q_pos = p.seq[x].q_pos;
        ent_causal = p.seq[x].causal;
    }
    auto entry_causal = [&](int e) __attribute__((always_inline)) -> int {
        return MULTI ? __builtin_amdgcn_readlane(ent_causal, e - s) : sq.causal;
    };
    auto entry_q_pos = [&](int e) __attribute__((always_inline)) -> int {
        return MULTI ? __builtin_amdgcn_readlane(ent_q_pos, e - s) : sq.q_pos;
    };
    // Tile i of an entry covers the keys (t0 + i) * KN + sh .. + KN - 1, where sh (0, 16, 32 or
    // 48) lets the entry's tiles start at the page that holds its first key instead of at a
    // multiple of KN keys: a retained frame of 204 tokens then always takes 4 tiles.  (The plain
    // call's one entry starts at key 0: sh = 0.)
    auto span = [&](int e, int &k_lo, int &k_hi, int &t0, int &nt, int &sh) __attribute__((always_inline)) {
        // (the plain build has one entry per group: the one already loaded)
        const int kb = MULTI ? __builtin_amdgcn_readlane(ent_begin, e - s) : sq.k_begin;
        const int ks = MULTI ? __builtin_amdgcn_readlane(ent_stop, e - s) : sq.k_stop;
        const int causal = entry_causal(e);
        k_lo = kb;
        k_hi = causal ? min(ks, C + wg_last_tok + 1) : ks;
        t0 = kb / KN;
        sh = (kb / kPage % (KN / kPage)) * kPage;
        nt = max((k_hi - sh + KN - 1) / KN - t0, 0);
    };
    // This item's piece: tiles split * tiles_per_split .. + tiles_per_split - 1 of the group's
    // tiles counted entry after entry.  e0: entry in which the piece starts, after first_skip
    // of its tiles; n_tiles: tiles of the piece (fewer than tiles_per_split at the end of the
    // group; 0 if the rows of this work-group see nothing of the piece).
    int e0 = s, first_skip = 0, n_tiles = 0;
    {
        int skip = split * sq.tiles_per_split, budget = sq.tiles_per_split;
        bool started = false;
        for (int e = s; e < e_end && budget > 0; ++e) {
            int kl, kh, t0, nt, sh;
            span(e, kl, kh, t0, nt, sh);
            if (!started) {
                if (skip >= nt) {
                    skip -= nt;
                    continue;
                }
                started = true;
                e0 = e;
                first_skip = skip;
                nt -= skip;
            }
            const int take = min(nt, budget);
            n_tiles += take;
            budget -= take;
        }
    }
    // The entry the current tile belongs to: tile i of the piece is key tile i + cur_off (first
    // key (i + cur_off) * KN + cur_sh) as long as i < cur_end.
    int cur_e = e0, cur_off, cur_end, cur_k_lo, cur_k_hi, cur_sh;
    {
        int t0, nt;
        span(e0, cur_k_lo, cur_k_hi, t0, nt, cur_sh);
        cur_off = t0 + first_skip;
        cur_end = min(nt - first_skip, n_tiles);
    }
    const int q_pos0 = entry_q_pos(e0);
    const int causal0 = entry_causal(e0);

    // ---- tile fetch: wave w brings in (its part of) page w / PARTS of the tile ----
    const int fpage = wave / PARTS;             // page of the tile this wave fetches
    const int fit0 = (wave % PARTS) * WITS;     // first of its 1 KB loads inside that page
    const int32_t *bt = p.block_table + (size_t)sq.bt_row * p.max_pages_per_seq;
    // Pages past an entry's last visible key are fetched as copies of the page that holds it
    // (finite, masked), so that every tile issues the same load count.
    // Block-table entries of this wave's page in 64 consecutive tiles sit in one VGPR (lane l:
    // tile pid_base + l of this work-group's range) and are picked out with v_readlane: no
    // scalar or LDS access in the loop competes with the LDS operand reads for lgkmcnt.
    int pid_base = 0;
    auto load_pids = [&](int rel0) __attribute__((always_inline)) -> int {
        const int f = rel0 + lane;  // this lane's tile, counted from the piece's first
        int idx = 0, fs = 0;
        for (int e = e0; e < e_end && fs < n_tiles; ++e) {
            int kl, kh, t0, nt, sh;
            span(e, kl, kh, t0, nt, sh);
            if (e == e0) {
                t0 += first_skip;
                nt -= first_skip;
            }
            // lanes past the end of the piece end up with the last entry's last page
            if (e == e0 || f >= fs)
                idx = min((t0 + f - fs) * (KN / kPage) + sh / kPage + fpage, (kh - 1) / kPage);
            fs += nt;
        }
        return bt[idx];
    };
    int klim[QB];  // row sees keys < klim
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) klim[qb] = causal0 ? min(C + row_tok[qb] + 1, cur_k_hi) : cur_k_hi;
    int pid_vec = n_tiles > 0 ? load_pids(0) : 0;
    __builtin_amdgcn_sched_barrier(0);  // the small loads are out: now the queries
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const bf16 *qrow = (const bf16 *)p.q + ((size_t)(sq.tok_off + row_tok[qb]) * Hq + row_head[qb]) * D;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) Q[qb][ks] = *(const bf16x8 *)(qrow + 16 * ks + 8 * h);
    }
    __builtin_amdgcn_sched_barrier(0);
    // Rotation factors.  The G query heads of a token share them, so the work-group computes
    // cos / sin once per (token, frequency) into an LDS table behind the tile ring and every
    // lane picks its own 2 * D/4 values; if the work-group's tokens do not fit the table (tiny
    // groups: many tokens per 256 rows), each lane computes its own.
    const int tok_first = row0 / G;
    const bool use_tab = wg_last_tok - tok_first + 1 <= p.tab_tokens;
    float2 *tab = (float2 *)(smem + kStages * T::STAGE_BYTES);
    if (use_tab) {
        const int ntok = wg_last_tok - tok_first + 1;
        for (int e = tid; e < ntok * (D / 2); e += NW * 64) {
            const int tk = e / (D / 2), f = e - tk * (D / 2);
            const float2 cs = rope_cos_sin(q_pos0 + chunk_pos(tok_first + tk), my_rev_freq);
            // (the score scale rides along)
            tab[tk * attention_tab_stride(D) + f] = make_float2(cs.x * p.q_scale, cs.y * p.q_scale);
        }
    }
    // Work-groups that walk through several entries keep, per lane, the rounding residuals of
    // their rotated queries in the table's place once the table has been used (see
    // shift_queries), and the frequency lane % (D/2), whose shift factors the lane computes.
    constexpr bool multi = MULTI;
    bf16x8 *resid = (bf16x8 *)(smem + kStages * T::STAGE_BYTES) + (size_t)wave * (QB * KS * 64) + lane;
    bf16x8 Qres[QB][KS];
    asm volatile("" : "+v"(pid_vec));
    // raw entry for tile rel of the piece (rel never decreases); clamped where it is used
    auto page_id = [&](int rel) __attribute__((always_inline)) -> int {
        if (__builtin_expect(rel - pid_base >= 64, 0)) {
            pid_base += 64;
            pid_vec = load_pids(pid_base);
            // make the load complete here, inside the rare branch: otherwise its wait lands
            // after the branch and would drain the tile fetches in flight on every step
            asm volatile("" : "+v"(pid_vec));
        }
        return __builtin_amdgcn_readlane(pid_vec, rel - pid_base);
    };
    const char *k_pool = (const char *)p.k_pool;
    const char *v_pool = (const char *)p.v_pool;
    // per-lane byte offsets inside a (page, head) block, for load `it` add it * 1024
    //   K block [16 tokens][D]: lane -> row lane / CH, chunk position lane % CH holds
    //   chunk (lane % CH) ^ g(row in tile); g depends on the row's low 4 bits only.
    int k_lane_off[WITS];
#pragma unroll
    for (int it = 0; it < WITS; ++it) {
        const int r = (fit0 + it) * T::ROWS_PER_LOAD + lane / T::CH;  // row in page == row in tile mod 16
        const int jj = (r & 3) | ((r & 4) << 1) | ((r & 8) >> 1);  // swap bits 2 and 3
        const int g = D == 128 ? jj : (jj >> 1);
        k_lane_off[it] = r * (D * 2) + (((lane % T::CH) ^ g) & (T::CH - 1)) * 16;
    }
    //   V block [D channels][16 tokens]: lane -> key half lane / 32, channel it*32 + lane % 32
    const int v_lane_off = (lane & 31) * (kPage * 2) + (lane >> 5) * 16;
    // K ring: kStages buffers of K_BYTES at lds0; V ring: kStages buffers of V_BYTES behind it.
    auto issue_k = [&](int pid, int stage) __attribute__((always_inline)) {
        const size_t blk = ((size_t)clamp_page(pid, p.n_pages) * Hkv + kvh) * (size_t)(kPage * D * 2);
        const unsigned dst = lds0 + stage * T::K_BYTES + fpage * (kPage * D * 2) + fit0 * 1024;
#pragma unroll
        for (int it = 0; it < WITS; ++it)
            load_to_lds_16(k_pool + blk, k_lane_off[it], dst + it * 1024);
    };
    auto issue_v = [&](int pid, int stage) __attribute__((always_inline)) {
        const size_t blk = ((size_t)clamp_page(pid, p.n_pages) * Hkv + kvh) * (size_t)(kPage * D * 2);
        const unsigned dst =
            lds0 + kStages * T::K_BYTES + stage * T::V_BYTES + fpage * T::V_PAGE_BYTES + fit0 * 1024;
#pragma unroll
        for (int it = 0; it < WITS; ++it)
            load_to_lds_16(v_pool + blk, (fit0 + it) * 1024 + v_lane_off, dst + it * 1024);
    };

    // Fetch schedule (see the loop below): iteration i reads K of tile lo+i+1 and V of tile
    // lo+i, and requests K of tile lo+i+3 and V of tile lo+i+2; the first tiles are requested
    // here.
    int pid_a = 0, pid_b = 0;  // page ids for the next K fetch and the next V fetch
    if (n_tiles > 0) {
        // K of the first two tiles and V of the first: all the first scores and the first
        // iteration need; V of the second and K of the third follow once the first K is in, so
        // that the start-up burst of every work-group asking at once stays small
        const int p0 = page_id(0);
        issue_k(p0, 0);
        issue_v(p0, 0);
        if (n_tiles > 1) {
            pid_b = page_id(1);
            issue_k(pid_b, 1);
        }
        if (n_tiles > 2) pid_a = page_id(2);
    }
    // Rotate the queries (the table was filled above; see there).
    {
        if (use_tab) __syncthreads();
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const int pos = q_pos0 + chunk_pos(row_tok[qb]);
            const float2 *trow = tab + (size_t)(row_tok[qb] - tok_first) * attention_tab_stride(D) + 8 * h;
#pragma unroll
            for (int ks = 0; ks < KS / 2; ++ks) {
                const bf16x8 lo = Q[qb][ks], hi = Q[qb][ks + KS / 2];
                bf16x8 rlo, rhi;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float2 cs;
                    if (use_tab) {
                        cs = trow[16 * ks + e];
                    } else {
                        cs = rope_cos_sin(pos, p.rev_freq[16 * ks + 8 * h + e]);
                        cs.x *= p.q_scale;
                        cs.y *= p.q_scale;
                    }
                    const float a = (float)lo[e], b = (float)hi[e];
                    const float x = a * cs.x - b * cs.y;
                    const float y = b * cs.x + a * cs.y;
                    rlo[e] = (bf16)x;
                    rhi[e] = (bf16)y;
                    if (multi) {
                        Qres[qb][ks][e] = (bf16)(x - (float)rlo[e]);
                        Qres[qb][ks + KS / 2][e] = (bf16)(y - (float)rhi[e]);
                    }
                }
                Q[qb][ks] = rlo;
                Q[qb][ks + KS / 2] = rhi;
            }
        }
    }

    // The scores are kept with the row's exponent reference already taken off: the MFMA chain
    // of a score block starts from the accumulator negm = -m_run instead of zero, which saves
    // one subtraction per score in the softmax.
    f32x16 O[QB][DB], negm[QB];
    float m_run[QB], l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m_run[qb] = 0.f;
        l_run[qb] = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) negm[qb][v] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) O[qb][db][v] = 0.f;
    }

    // LDS read offsets.  K: A-row j of a 32-key block reads tile row krow (see above), whose
    // chunk c sits at position c ^ gj.  V: lane (j, h) reads [page][block][h][j].
    const int krow = 16 * (j >> 4) + 8 * ((j >> 2) & 1) + 4 * ((j >> 3) & 1) + (j & 3);
    const int gj = D == 128 ? (j & 15) : ((j & 15) >> 1);
    int k_read_off[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        k_read_off[ks] = krow * (D * 2) + (((2 * ks + h) ^ gj) & (T::CH - 1)) * 16;
    const int v_read_off = kStages * T::K_BYTES + h * 512 + j * 16;

    // S^T = K Q^T for the tile in K stage `stage`
    // The two 32-key blocks are advanced alternately: consecutive MFMAs then never depend on
    // each other (a dependent back-to-back MFMA costs about twice an independent one).
    auto scores = [&](int stage, f32x16 (&S)[QB][2]) __attribute__((always_inline)) {
        const unsigned char *kst = smem + stage * T::K_BYTES;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            bf16x8 a[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
                a[kb] = *(const bf16x8 *)(kst + kb * 32 * (D * 2) + k_read_off[ks]);
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    if (ks == 0) {
                        S[qb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kb], Q[qb][ks], negm[qb], 0, 0, 0);
                    } else {
                        S[qb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kb], Q[qb][ks], S[qb][kb], 0, 0, 0);
                    }
                }
        }
    };

    // first tile of this wave that needs the causal / range mask: tiles ending at or below
    // the smallest key limit of the wave's rows are fully visible
    const bool wave_active = wrow0 < R;
    auto first_masked_tile = [&](int e, int k_hi, int sh) __attribute__((always_inline)) -> int {
        return ((entry_causal(e) ? min(C + min(wrow0, R - 1) / G + 1, k_hi) : k_hi) - sh) / KN;
    };
    int t_mask = first_masked_tile(e0, cur_k_hi, cur_sh);
    // The softmax side moves on to the next entry (the queries moved one tile earlier).
    auto next_entry = [&]() __attribute__((always_inline)) {
        ++cur_e;
        int t0, nt;
        span(cur_e, cur_k_lo, cur_k_hi, t0, nt, cur_sh);
        cur_off = t0 - cur_end;
        cur_end = min(cur_end + nt, n_tiles);
        t_mask = first_masked_tile(cur_e, cur_k_hi, cur_sh);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
            klim[qb] = entry_causal(cur_e) ? min(C + row_tok[qb] + 1, cur_k_hi) : cur_k_hi;
    };
    // The next tile opens the next entry: rotate the (already rotated and scaled) queries on by
    // the difference of the two entries' query positions.  Lane l computes the factors of
    // frequency l % (D/2) and the lanes exchange them.  The queries sit in registers as bf16;
    // to keep a chain of such shifts from piling up rounding errors, what each rounding cut off
    // is kept (as bf16, lane-private in LDS) and added back before the next shift.
    // (The new residuals are only formed if the piece goes on to a third entry: they serve the
    // next shift and nothing else.)
    auto shift_queries = [&]() __attribute__((always_inline)) {
        const float2 f = rope_cos_sin(entry_q_pos(cur_e + 1) - entry_q_pos(cur_e),
                                      p.rev_freq[lane & (D / 2 - 1)]);
        bool shifts_again;
        {
            int kl, kh, t0, nt, sh;
            span(cur_e + 1, kl, kh, t0, nt, sh);
            shifts_again = cur_end + nt < n_tiles;
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int ks = 0; ks < KS / 2; ++ks) {
                const bf16x8 lo = Q[qb][ks], hi = Q[qb][ks + KS / 2];
                const bf16x8 el = resid[(qb * KS + ks) * 64], eh = resid[(qb * KS + ks + KS / 2) * 64];
                bf16x8 rlo, rhi, nel, neh;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int src = 16 * ks + 8 * h + e;
                    const float c = __shfl(f.x, src), sn = __shfl(f.y, src);
                    const float a = (float)lo[e] + (float)el[e], b = (float)hi[e] + (float)eh[e];
                    const float x = a * c - b * sn, y = b * c + a * sn;
                    rlo[e] = (bf16)x;
                    rhi[e] = (bf16)y;
                    if (shifts_again) {
                        nel[e] = (bf16)(x - (float)rlo[e]);
                        neh[e] = (bf16)(y - (float)rhi[e]);
                    }
                }
                Q[qb][ks] = rlo;
                Q[qb][ks + KS / 2] = rhi;
                if (shifts_again) {
                    resid[(qb * KS + ks) * 64] = nel;
                    resid[(qb * KS + ks + KS / 2) * 64] = neh;
                }
                __builtin_amdgcn_sched_barrier(0);  // one slice at a time: few registers in flight
            }
    };

    // scores of the tile being normalised and of the next one, by turns in SA and SB
    f32x16 SA[QB][2], SB[QB][2];
    bf16x8 P[QB][2][2];
    typedef bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 ones;
    ones[0] = (bf16)1.0f;
    ones[1] = (bf16)1.0f;

    // ---- softmax of tile t, from its scores S (log2 domain: scale and log2(e) are folded into Q) ----
    // The exponent reference m_run of a row is NOT the running maximum: it stays where it is as
    // long as the row's probabilities stay small, so the per-tile maximum search, reference
    // update and rescale of O drop out of the common path (any reference gives the same O / l;
    // it only has to keep the numbers in range).  The scores arrive with the reference already
    // subtracted (see negm).  Common path per score: exp2, round to bf16, add to the tile sum.
    // If a lane's tile sum is not below the bound (which also catches inf and NaN), or the row
    // has no weight yet (its first visible keys), the wave redoes the tile the classic way
    // before its probabilities are used: the reference moves to the tile maximum, O, l and the
    // scores in flight move with it, the probabilities are recomputed.
    constexpr float kSumBound = 1048576.0f;  // 2^20 for the 32 probabilities a lane holds
    float tsum[QB];                          // tile sum of the probabilities in P
    // probabilities of scores 2*pr and 2*pr+1 (pr = 0..15 walks the lane's 32 scores in pairs)
    auto softmax_pair = [&](f32x16 (&S_cur)[QB][2], int pr) __attribute__((always_inline)) {
        const int kb = pr >> 3, v = (pr & 7) * 2;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            bf16x2 e;
            e[0] = (bf16)__builtin_amdgcn_exp2f(S_cur[qb][kb][v]);
            e[1] = (bf16)__builtin_amdgcn_exp2f(S_cur[qb][kb][v + 1]);
            tsum[qb] = __builtin_amdgcn_fdot2_f32_bf16(e, ones, tsum[qb], false);
            P[qb][kb][v >> 3][v & 7] = e[0];
            P[qb][kb][v >> 3][(v & 7) + 1] = e[1];
        }
    };
    // Pack (HOLES): hole_lo / hole_step follow the tiles as the loop advances -- the first hole
    // (a step's action tokens) that ends behind the current tile's first key, and its step.  With
    // hole_period >= KN a tile meets at most that hole and the next one.  A hole is hidden from the
    // rows of later steps only.
    int hole_lo = 0, hole_step = 0, row_step[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) row_step[qb] = HOLES ? step_of(C + row_tok[qb]) : 0;
    auto seek_hole = [&](int t) __attribute__((always_inline)) -> bool {  // true: tile t meets a hole
        const int k0 = t * KN + cur_sh;
        while (hole_lo + h_width <= k0) {
            hole_lo += h_period;
            ++hole_step;
        }
        return hole_lo < k0 + KN;
    };
    // bits [lo, lo + w) of a 64-bit word, clipped to the word
    auto bit_range = [](int lo, int w) __attribute__((always_inline)) -> unsigned long long {
        const int a = max(lo, 0), b = min(lo + w, 64);
        if (b <= a) return 0ull;
        return (b - a >= 64 ? ~0ull : (1ull << (b - a)) - 1ull) << a;
    };
    auto apply_mask = [&](f32x16 (&S_cur)[QB][2], int t) __attribute__((always_inline)) {
        if (HOLES) {
            // A pack masks about every third tile: the hidden keys of the tile are gathered in a 64-bit
            // word per row (bit x = key x of the tile) -- the two holes (wave-uniform words, dropped for
            // rows of the hole's own step or an earlier one), the causal limit, the range's lower end --
            // and every score then costs one bit test.
            const int k0 = t * KN + cur_sh;
            const unsigned long long hole_a = bit_range(hole_lo - k0, h_width);
            const unsigned long long hole_b = bit_range(hole_lo + h_period - k0, h_width);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                unsigned long long hidden = (hole_step < row_step[qb] ? hole_a : 0ull) |
                                            (hole_step + 1 < row_step[qb] ? hole_b : 0ull);
                hidden |= ~bit_range(0, klim[qb] - k0);   // keys at or past the row's limit
                hidden |= bit_range(0, cur_k_lo - k0);    // keys before the range
                // this lane's keys are 32 kb + 16 (v / 8) + 8 h + v % 8
                const unsigned w[2] = {(unsigned)hidden >> (8 * h), (unsigned)(hidden >> 32) >> (8 * h)};
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        if ((w[kb] >> (16 * (v >> 3) + (v & 7))) & 1u) S_cur[qb][kb][v] = -INFINITY;
            }
            return;
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const int lim = klim[qb] - t * KN - cur_sh - 8 * h;  // local key index bounds for this lane
            const int low = cur_k_lo - t * KN - cur_sh - 8 * h;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int kl = 32 * kb + 16 * (v >> 3) + (v & 7);
                    if (kl >= lim || kl < low) S_cur[qb][kb][v] = -INFINITY;
                }
        }
    };
    // the rare slow path, then l += tile sum.  S_next: the next tile's scores, computed from the
    // old reference while this tile was normalised (has_next), which move along with it.
    auto finish_softmax = [&](f32x16 (&S_cur)[QB][2], f32x16 (&S_next)[QB][2], bool has_next)
                              __attribute__((always_inline)) {
        bool redo = false;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) redo |= !(tsum[qb] < kSumBound) || l_run[qb] == 0.f;
        if (__any(redo)) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                float mx = S_cur[qb][0][0];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) mx = fmaxf(mx, S_cur[qb][kb][v]);
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                // The scores are relative to the old reference, which moves by delta: up to the
                // tile maximum, or, as long as the row has no weight yet (O and l still zero),
                // to wherever the tile maximum is.
                const bool massless = l_run[qb] + __shfl_xor(l_run[qb], 32) == 0.f;
                const float delta = massless ? (mx > -INFINITY ? mx : 0.f) : fmaxf(mx, 0.f);
                const float alpha = massless ? 1.0f : __builtin_amdgcn_exp2f(-delta);
                m_run[qb] += delta;
                l_run[qb] *= alpha;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int v = 0; v < 16; ++v) O[qb][db][v] *= alpha;
#pragma unroll
                for (int v = 0; v < 16; ++v) negm[qb][v] = -m_run[qb];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        S_cur[qb][kb][v] -= delta;
                        if (has_next) S_next[qb][kb][v] -= delta;
                    }
                tsum[qb] = 0.f;
            }
#pragma unroll
            for (int pr = 0; pr < 16; ++pr) softmax_pair(S_cur, pr);
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) l_run[qb] += tsum[qb];
    };

    // One iteration handles tile i of the piece.  Each wavefront interleaves its own MFMAs with its own
    // softmax arithmetic (a second wavefront on the SIMD gets no VALU issue slots while this one
    // streams MFMAs, so the overlap has to come from within the instruction stream), and the
    // order is pinned with scheduling barriers:
    //   block A: the 2*KS MFMAs of the scores of tile i+1, each followed by the softmax of one
    //            pair of scores of tile i, LDS operand reads 4 MFMAs ahead
    //   block B: the 4*DB MFMAs of O += P V of tile i, LDS operand reads 4 MFMAs ahead
    int ring = 0;  // i % kStages
    // `mask`: std::integral_constant (decided at compile time) or bool.  S_cur: scores of tile i
    // (consumed); S_next: receives the scores of tile i+1.
    auto iteration = [&](int i, auto mask, auto last_tag, f32x16 (&S_cur)[QB][2],
                         f32x16 (&S_next)[QB][2]) __attribute__((always_inline)) {
        constexpr bool LAST = decltype(last_tag)::value;
        const bool do_mask = mask;
        const int t = i + cur_off;
        // this wave's part of K(i+1) and V(i) has landed; younger fetches may be in flight
        if (i + 2 < n_tiles)
            wait_loads<2 * WITS>();
        else if (i + 1 < n_tiles)
            wait_loads<WITS>();
        else
            wait_loads<0>();
        // ... and so has every other wave's; also everyone is done with iteration i-1, whose
        // K and V buffers are the ones refilled during this iteration
        __syncthreads();
        const int r1 = ring + 1 == kStages ? 0 : ring + 1;
        const int r2 = r1 + 1 == kStages ? 0 : r1 + 1;
        if (i + 3 < n_tiles) issue_k(pid_a, ring);
        // A wave whose 32 rows lie past the end of the chunk (short chunks: a few action tokens)
        // only takes part in the fetches and barriers.
        if (wave_active) {
        if (do_mask) apply_mask(S_cur, t);
        if (multi && !LAST && __builtin_expect(i + 1 == cur_end, 0)) shift_queries();  // the next tile opens the next entry
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) tsum[qb] = 0.f;

        // ---- block A ----
        constexpr int NA = 2 * KS;  // MFMA slots; slot u: k-step u / 2 of key block u % 2
        if (!LAST) {
            const unsigned char *kst = smem + r1 * T::K_BYTES;
            bf16x8 a[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                a[u] = *(const bf16x8 *)(kst + (u & 1) * 32 * (D * 2) + k_read_off[u >> 1]);
            __builtin_amdgcn_sched_barrier(0);
            // Inside the two MFMA blocks the wave asks for the highest issue priority, outside
            // (waits, barrier, fetch requests, mask, bookkeeping) for the lowest: the SIMD's other
            // wave, when it is in a block, is not held up by this one's housekeeping.  Worth 0.8 %.
            __builtin_amdgcn_s_setprio(3);
#pragma unroll
            for (int u = 0; u < NA; ++u) {
                const int ks = u >> 1, kb = u & 1;
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    if (ks == 0) {
                        S_next[qb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u & 3], Q[qb][ks], negm[qb], 0, 0, 0);
                    } else {
                        S_next[qb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u & 3], Q[qb][ks], S_next[qb][kb], 0, 0, 0);
                    }
                }
                if (u + 4 < NA)
                    a[u & 3] = *(const bf16x8 *)(kst + ((u + 4) & 1) * 32 * (D * 2) + k_read_off[(u + 4) >> 1]);
                // 16 score pairs over NA MFMA slots
#pragma unroll
                for (int pr = u * 16 / NA; pr < (u + 1) * 16 / NA; ++pr) softmax_pair(S_cur, pr);
                __builtin_amdgcn_sched_barrier(0);
            }
            __builtin_amdgcn_s_setprio(0);
        } else {
#pragma unroll
            for (int pr = 0; pr < 16; ++pr) softmax_pair(S_cur, pr);
        }
        finish_softmax(S_cur, S_next, !LAST);
        }
        if (i + 2 < n_tiles) issue_v(pid_b, r2);
        pid_b = pid_a;
        if (i + 4 < n_tiles) pid_a = page_id(i + 4);

        // ---- block B ----
        if (wave_active) {
            constexpr int NB = 4 * DB;  // MFMA slots; slot u: key 16-block u / DB, channel block u % DB
            const unsigned char *vst = smem + v_read_off + ring * T::V_BYTES;
            bf16x8 a[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                a[u] = *(const bf16x8 *)(vst + (u / DB) * T::V_PAGE_BYTES + (u % DB) * 1024);
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_setprio(3);
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                const int pg = u / DB, db = u % DB;
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
                    O[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u & 3], P[qb][pg >> 1][pg & 1], O[qb][db], 0, 0, 0);
                if (u + 4 < NB)
                    a[u & 3] = *(const bf16x8 *)(vst + ((u + 4) / DB) * T::V_PAGE_BYTES + ((u + 4) % DB) * 1024);
                __builtin_amdgcn_sched_barrier(0);
            }
            __builtin_amdgcn_s_setprio(0);
        }
        ring = r1;
    };

    if (n_tiles > 0) {
        typedef std::integral_constant<bool, true> yes;
        typedef std::integral_constant<bool, false> no;
        // only K of the first tile has to be there for the first scores
        if (n_tiles >= 2)
            wait_loads<2 * WITS>();
        else
            wait_loads<WITS>();
        __syncthreads();
        if (multi) {  // everyone is done with the cos/sin table: its place takes the residuals
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) resid[(qb * KS + ks) * 64] = Qres[qb][ks];
        }
        if (n_tiles > 1) issue_v(pid_b, 1);
        if (n_tiles > 2) {
            issue_k(pid_a, 2);
            pid_b = pid_a;
        }
        if (n_tiles > 3) pid_a = page_id(3);
        if (wave_active) scores(0, SA);
        // a tile needs the mask if it starts below its entry's key range or reaches past the
        // smallest key limit of the wave's rows
        auto needs_mask = [&](int i) __attribute__((always_inline)) -> bool {
            const int t = i + cur_off;
            return t * KN + cur_sh < cur_k_lo || t >= t_mask;
        };
        auto to_a = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) SA[qb][kb] = SB[qb][kb];
        };
        int i = 0;
        if (HOLES) {
            // a pack: tiles that meet a hole are scattered over the key range
            {   // the first hole that can matter for this piece's first tile
                const int k0 = cur_off * KN + cur_sh;
                hole_step = step_of(max(k0, h_first));
                hole_lo = h_first + hole_step * h_period + (h_period - h_width);
            }
            for (; i + 2 < n_tiles; i += 2) {  // two per round: the score buffers swap roles without copies
                const bool hole0 = seek_hole(i + cur_off);
                iteration(i, needs_mask(i) || hole0, no(), SA, SB);
                const bool hole1 = seek_hole(i + 1 + cur_off);
                iteration(i + 1, needs_mask(i + 1) || hole1, no(), SB, SA);
            }
            for (; i < n_tiles - 1; ++i) {
                const bool hole = seek_hole(i + cur_off);
                iteration(i, needs_mask(i) || hole, no(), SA, SB);
                to_a();
            }
            const bool hole = seek_hole(i + cur_off);
            iteration(i, needs_mask(i) || hole, yes(), SA, SB);
        } else if (!multi) {
            // one entry: the tiles that need a mask are the first (if the entry starts inside
            // it) and the last few; the fully visible ones in between get a loop of their own
            const int i_mask = t_mask - cur_off;
            const bool low_mask = needs_mask(0) && i_mask > 0;
            if (low_mask && n_tiles > 1) {
                iteration(0, yes(), no(), SA, SB);
                to_a();
                i = 1;
            }
            // the fully visible tiles, two per round so that the two score buffers swap roles
            // without being copied
            const int stop = min(i_mask, n_tiles - 1);
            for (; i + 1 < stop; i += 2) {
                iteration(i, no(), no(), SA, SB);
                iteration(i + 1, no(), no(), SB, SA);
            }
            for (; i < stop; ++i) {
                iteration(i, no(), no(), SA, SB);
                to_a();
            }
            for (; i < n_tiles - 1; ++i) {
                iteration(i, yes(), no(), SA, SB);
                to_a();
            }
            if (i >= i_mask || (i == 0 && low_mask))
                iteration(i, yes(), yes(), SA, SB);
            else
                iteration(i, no(), yes(), SA, SB);
        } else {
            for (; i < n_tiles - 1; ++i) {
                if (__builtin_expect(i == cur_end, 0)) next_entry();
                iteration(i, needs_mask(i), no(), SA, SB);
                to_a();
            }
            if (i == cur_end) next_entry();
            iteration(i, needs_mask(i), yes(), SA, SB);
        }
    }

    // ---- epilogue ----
    // Lane (j, h) holds, for output block db and register v, channel db*32 + 8*(v/4) + 4*h + v%4.
    // bf16 rows (the final output, or partial results that a later launch merges) go through
    // LDS once, so that each store instruction writes whole 256-byte rows instead of 8-byte
    // pieces of 32 different rows.
    const bool staged = !p.out_f32;
    if (staged) {
        constexpr int RS = D * 2 + 16;  // staging row stride: rows shifted by 4 banks
        __syncthreads();                // every wave is done with the tile rings
        unsigned char *stg = smem + wave * (32 * QB * RS);
        const bool direct = sq.total_splits == 1;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32);
            const float inv = direct ? 1.0f / l_tot : (l_tot > 0.f ? 1.0f / l_tot : 0.f);
            // destination row of this lane's row j (in rows of D elements); -1: none
            long long drow = -1;
            if (row_ok[qb])
                drow = direct ? (long long)(sq.tok_off + row_tok[qb]) * Hq + row_head[qb]
                              : sq.part_off + ((long long)(sq.split_base + split) * sq.n_new + row_tok[qb]) * Hq +
                                    row_head[qb];
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    bf16x4 ob;
#pragma unroll
                    for (int e = 0; e < 4; ++e) ob[e] = (bf16)(O[qb][db][4 * a + e] * inv);
                    *(bf16x4 *)(stg + (qb * 32 + j) * RS + (db * 32 + 8 * a + 4 * h) * 2) = ob;
                }
            if (!direct && row_ok[qb] && h == 0)
                *(float2 *)(p.part_ml + drow * 2) = make_float2(l_tot > 0.f ? m_run[qb] : -1.0e30f, l_tot);
            bf16 *base = (bf16 *)(direct ? p.out : p.part_o);
            constexpr int LPR = D / 8;          // lanes per row
            constexpr int RPI = 64 / LPR;       // rows per store instruction
#pragma unroll
            for (int it = 0; it < 32 / RPI; ++it) {
                const int r = it * RPI + lane / LPR, c = lane % LPR;
                const long long dr = __shfl(drow, r);
                const bf16x8 val = *(const bf16x8 *)(stg + (qb * 32 + r) * RS + c * 16);
                // (partial rows are read once, by another kernel: streamed past the L2, so that the end of
                // this kernel has less to write back; measured -0.8 us per launch at the 7B step's shape)
                if (dr >= 0) {
                    if (direct)
                        *(bf16x8 *)(base + dr * D + c * 8) = val;
                    else
                        __builtin_nontemporal_store(val, (bf16x8 *)(base + dr * D + c * 8));
                }
            }
        }
    }
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        if (staged) break;
        const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32);
        if (!row_ok[qb]) continue;
        const size_t orow = (size_t)(sq.tok_off + row_tok[qb]) * Hq + row_head[qb];
        if (sq.total_splits == 1) {
            const float inv = 1.0f / l_tot;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const int ch = db * 32 + 8 * a + 4 * h;
                    f32x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = O[qb][db][4 * a + e] * inv;
                    if (p.out_f32) {
                        *(f32x4 *)((float *)p.out + orow * D + ch) = o;
                    } else {
                        bf16x4 ob;
#pragma unroll
                        for (int e = 0; e < 4; ++e) ob[e] = (bf16)o[e];
                        *(bf16x4 *)((bf16 *)p.out + orow * D + ch) = ob;
                    }
                }
        } else {
            // partial row index: [split][token][head] inside this sequence's block.  Partials
            // are stored normalised (O / l) in the element type of the final output, next to
            // the pair (exponent reference, l); a split that saw no key stores zeros and l = 0.
            const size_t prow = (size_t)sq.part_off +
                                ((size_t)(sq.split_base + split) * sq.n_new + row_tok[qb]) * Hq + row_head[qb];
            const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const int ch = db * 32 + 8 * a + 4 * h;
                    f32x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = O[qb][db][4 * a + e] * inv;
                    if (p.out_f32) {
                        *(f32x4 *)((float *)p.part_o + prow * D + ch) = o;
                    } else {
                        bf16x4 ob;
#pragma unroll
                        for (int e = 0; e < 4; ++e) ob[e] = (bf16)o[e];
                        *(bf16x4 *)((bf16 *)p.part_o + prow * D + ch) = ob;
                    }
                }
            if (h == 0) *(float2 *)(p.part_ml + prow * 2) = make_float2(l_tot > 0.f ? m_run[qb] : -1.0e30f, l_tot);
        }
    }
}

// =========================================================================================
// Attention for chunks of a few tokens (at most 32 packed rows per KV head: the action tokens
// that follow a frame).  There is too little arithmetic to share: reading the keys and values
// once is all the work, so every WAVE is a worker of its own.  A wave takes one piece of one
// entry's key range, keeps a private 32-key tile buffer in LDS (filled by direct loads, K and
// V refilled separately as soon as each has been read), rotates its own copy of the queries at
// its entry's query position, and runs the same two MFMA contractions as attn_kernel on 32-key
// tiles with a plain online softmax.  No barrier inside the loop; the eight waves of a
// work-group are eight tiles in flight per CU.  At the end the eight partial results are
// merged through LDS, and the work-groups of one (rows, KV head) are merged by the last one to
// finish: every work-group stores its partial rows past the (per-XCD, mutually non-coherent)
// L2, waits for the acknowledgement and takes a ticket; the holder of the last ticket reads all
// of them, again past the L2, and leaves the counter at zero for the next launch.  Nobody waits
// for anybody and no cache is flushed.
//
// Entries: as in AttnSeq, but every entry carries its own n_splits (pieces) of
// tiles_per_split 32-key tiles and, in split_base, the number of pieces of its group before
// it; the first entry of a group (n_ent > 0) stands for the rows; total_splits = work-groups
// per KV head of the group.
// =========================================================================================
constexpr int kDecodeWaves = kDecodeWavesPerGroup;
constexpr int kDecodeTile = kDecodeTileKeys;  // keys per tile: two pages


// FUSED: the chunk's tokens are not in the cache yet (work-groups of the same launch append
// them meanwhile): the slots from the old end of the sequence on are patched in the wave's
// tile buffer from k_new / v_new -- the keys rotated exactly as the append rotates them, the
// slots past the chunk zeroed -- so whatever the pages hold there, or are just being given,
// does not matter.
template <int D, bool FUSED>
__device__ __forceinline__ void decode_body(const AttnParams &p, const int block) {
    using T = Tile<D>;
    constexpr int KN = kDecodeTile;
    constexpr int KS = D / 16;
    constexpr int DB = D / 32;
    constexpr int ITS = T::ITS;                       // 1 KB loads per page, K and V each
    constexpr int K_BYTES = KN * D * 2, V_BYTES = KN * D * 2;
    constexpr int ML_BYTES = 32 * 8;
    const int TAB_BYTES = p.tab_tokens * (D / 2) * 8;  // table for the longest chunk of the launch
    const int WAVE_BYTES = K_BYTES + V_BYTES + TAB_BYTES + ML_BYTES;
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)smem;

    const int G = p.group, Hq = p.n_q_heads, Hkv = p.n_kv_heads;
    // work-group -> (group of entries, KV head, work-group of that pair): a prefix sum over the
    // entries' work-group counts, one entry per lane (a launch has at most 64 entries here)
    int local = block, s = -1;
    if (p.n_seqs <= 4) {  // a few entries: a scalar walk is the shortest
        for (int e = 0; e < p.n_seqs; ++e) {
            const int here = p.seq[e].n_ent > 0 ? p.seq[e].total_splits * Hkv : 0;
            if (local < here) {
                s = e;
                break;
            }
            local -= here;
        }
        if (s < 0) return;
    } else {
        const int ln = threadIdx.x & 63;
        const int here = ln < p.n_seqs && p.seq[ln].n_ent > 0 ? p.seq[ln].total_splits * Hkv : 0;
        int incl = here;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int up = __shfl_up(incl, off);
            if (ln >= off) incl += up;
        }
        const unsigned long long above = __ballot(incl > local);
        if (above == 0) return;
        s = __ffsll(above) - 1;
        local = __builtin_amdgcn_readfirstlane(local - __shfl(incl - here, s));
        s = __builtin_amdgcn_readfirstlane(s);
    }
    const AttnSeq sq = p.seq[s];
    const int kvh = local % Hkv, wg = local / Hkv;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = lane & 31, h = lane >> 5;
    const int R = sq.n_new * G, C = sq.cache_len;
    unsigned char *wmem = smem + wave * WAVE_BYTES;
    const unsigned wlds = lds0 + wave * WAVE_BYTES;

    // this wave's piece: piece number wg * 8 + wave of the group, counted entry after entry
    // (split_base: pieces of the group before the entry)
    const int piece = wg * kDecodeWaves + wave;
    int ee = s;
    if (sq.n_ent > 1) {
        // lane x looks at entry s + x (a group has at most 64 entries): the entries that start at
        // or before this piece form a prefix of the group
        const int xb = lane < sq.n_ent ? p.seq[s + lane].split_base : 0x7fffffff;
        ee = s + __popcll(__ballot(piece >= xb)) - 1;
    }
    const int split = piece - p.seq[ee].split_base;
    const bool has_piece = split < p.seq[ee].n_splits;
    const int causal = p.seq[ee].causal, k_begin = p.seq[ee].k_begin, tps = p.seq[ee].tiles_per_split;
    const int k_hi = causal ? min(p.seq[ee].k_stop, C + sq.n_new) : p.seq[ee].k_stop;
    const int tile_lo = k_begin / KN + split * tps;
    const int k_lo = max(k_begin, tile_lo * KN);
    const int k_end = min((tile_lo + tps) * KN, k_hi);
    const int n_tiles = has_piece ? max((k_end + KN - 1) / KN - tile_lo, 0) : 0;
    const int q_pos = p.seq[ee].q_pos;

    // rows: lane (j, h) owns packed row j
    const int r = min(j, R - 1);
    const int tok = r / G, g = r - tok * G;
    const int head = kvh * G + g;
    const int klim = causal ? min(C + tok + 1, k_end) : k_end;
    // Loads in the order of their issue (a wave's loads return in order): the small ones first --
    // the frequency this lane fills into the table (64 is a multiple of D/2, so a lane always
    // meets the same one), the block-table entries -- then the queries.
    const double my_rev_freq = p.rev_freq[lane & (D / 2 - 1)];
    // block-table entries of this piece's pages: lane l holds page 2 * tile_lo + l of the
    // sequence (32 tiles per refill), clamped to the last visible page
    const int32_t *bt = p.block_table + (size_t)sq.bt_row * p.max_pages_per_seq;
    const int last_page = max(k_end - 1, 0) / kPage;
    int pid_base = 0;
    int pid_vec = n_tiles > 0 ? bt[min(tile_lo * 2 + lane, last_page)] : 0;
    __builtin_amdgcn_sched_barrier(0);
    bf16x8 Q[KS];
    {
        const bf16 *qrow = (const bf16 *)p.q + ((size_t)(sq.tok_off + tok) * Hq + head) * D;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) Q[ks] = *(const bf16x8 *)(qrow + 16 * ks + 8 * h);
    }
    __builtin_amdgcn_sched_barrier(0);
    // cos / sin for this entry's query position: n_new tokens x D/2 frequencies, spread over
    // the lanes, into the wave's own table (wave-local: no barrier)
    float2 *tab = (float2 *)(wmem + K_BYTES + V_BYTES);
    for (int x = lane; x < sq.n_new * (D / 2); x += 64) {
        const float2 cs = rope_cos_sin(q_pos + x / (D / 2), my_rev_freq);
        tab[x] = make_float2(cs.x * p.q_scale, cs.y * p.q_scale);
    }
    asm volatile("" : "+v"(pid_vec));

    // ---- tile fetch (same LDS layouts as attn_kernel, 2 pages per tile) ----
    const char *k_pool = (const char *)p.k_pool;
    const char *v_pool = (const char *)p.v_pool;
    int k_lane_off[ITS];
#pragma unroll
    for (int it = 0; it < ITS; ++it) {
        const int rr = it * T::ROWS_PER_LOAD + lane / T::CH;
        const int jj = (rr & 3) | ((rr & 4) << 1) | ((rr & 8) >> 1);
        const int gg = D == 128 ? jj : (jj >> 1);
        k_lane_off[it] = rr * (D * 2) + (((lane % T::CH) ^ gg) & (T::CH - 1)) * 16;
    }
    const int v_lane_off = (lane & 31) * (kPage * 2) + (lane >> 5) * 16;
    auto page_of = [&](int rel_page) __attribute__((always_inline)) -> size_t {
        if (__builtin_expect(rel_page - pid_base >= 64, 0)) {
            pid_base += 64;
            pid_vec = bt[min(tile_lo * 2 + pid_base + lane, last_page)];
            asm volatile("" : "+v"(pid_vec));
        }
        const int pid = __builtin_amdgcn_readlane(pid_vec, rel_page - pid_base);
        return ((size_t)clamp_page(pid, p.n_pages) * Hkv + kvh) * (size_t)(kPage * D * 2);
    };
    auto issue_k = [&](int t) __attribute__((always_inline)) {
#pragma unroll
        for (int pg = 0; pg < 2; ++pg) {
            const size_t blk = page_of(2 * t + pg);
#pragma unroll
            for (int it = 0; it < ITS; ++it)
                load_to_lds_16(k_pool + blk, k_lane_off[it], wlds + pg * (kPage * D * 2) + it * 1024);
        }
    };
    auto issue_v = [&](int t) __attribute__((always_inline)) {
#pragma unroll
        for (int pg = 0; pg < 2; ++pg) {
            const size_t blk = page_of(2 * t + pg);
#pragma unroll
            for (int it = 0; it < ITS; ++it)
                load_to_lds_16(v_pool + blk, it * 1024 + v_lane_off, wlds + K_BYTES + pg * (kPage * D * 2) + it * 1024);
        }
    };
    // The chunk's first tokens are fetched when the wave starts (a wave whose piece reaches the
    // old end of the sequence), so that the patches do not wait for memory in mid-loop.
    constexpr int NPRE = 4, VPL = D / 64;  // tokens fetched ahead; value channels per lane
    bf16 pre_k[NPRE][2], pre_v[NPRE][VPL];
    if (FUSED && causal && n_tiles > 0 && k_end > C) {
#pragma unroll
        for (int i = 0; i < NPRE; ++i) {
            const size_t row = ((size_t)(sq.tok_off + min(i, sq.n_new - 1)) * Hkv + kvh) * D;
            pre_k[i][0] = ((const bf16 *)p.k_new)[row + (lane & (D / 2 - 1))];
            pre_k[i][1] = ((const bf16 *)p.k_new)[row + (lane & (D / 2 - 1)) + D / 2];
#pragma unroll
            for (int x = 0; x < VPL; ++x) pre_v[i][x] = ((const bf16 *)p.v_new)[row + lane + 64 * x];
        }
    }
    if (n_tiles > 0) {
        issue_k(0);
        issue_v(0);
    }

    // ---- rotate the queries (table written by this wave above) ----
    {
        const float2 *trow = tab + (size_t)tok * (D / 2) + 8 * h;
#pragma unroll
        for (int ks = 0; ks < KS / 2; ++ks) {
            const bf16x8 lo = Q[ks], hi = Q[ks + KS / 2];
            bf16x8 rlo, rhi;
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                const float2 cs = trow[16 * ks + x];
                const float a = (float)lo[x], b = (float)hi[x];
                rlo[x] = (bf16)(a * cs.x - b * cs.y);
                rhi[x] = (bf16)(b * cs.x + a * cs.y);
            }
            Q[ks] = rlo;
            Q[ks + KS / 2] = rhi;
        }
    }

    f32x16 O[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) O[db][v] = 0.f;
    float m_run = -1.0e30f, l_run = 0.f;

    const int krow = 16 * (j >> 4) + 8 * ((j >> 2) & 1) + 4 * ((j >> 3) & 1) + (j & 3);
    const int gj = D == 128 ? (j & 15) : ((j & 15) >> 1);
    const int v_read_off = K_BYTES + h * 512 + j * 16;
    typedef bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 ones;
    ones[0] = (bf16)1.0f;
    ones[1] = (bf16)1.0f;

    // FUSED: tile tt holds slots at or past the old end C of the sequence.  Keys: the rows of the
    // chunk's tokens are written into the wave's K buffer, rotated as the append rotates them
    // (lane l: channels l and l + D/2); rows past the chunk stay as they are (their scores are
    // masked by assignment).  Values: every slot from C on is rewritten -- the chunk's tokens,
    // zeros behind them (a masked probability is a zero that still multiplies the value) --
    // 8 slots of one channel (one 16-byte word of the buffer) at a time.
    auto patch_k = [&](int tt) __attribute__((always_inline)) {
        const int i_hi = min(sq.n_new, (tt + 1) * KN - C);
        for (int i = max(tt * KN - C, 0); i < i_hi; ++i) {
            const int rr = C + i - tt * KN, r16 = rr & 15;
            const int jj = (r16 & 3) | ((r16 & 4) << 1) | ((r16 & 8) >> 1);
            const int gg = D == 128 ? jj : (jj >> 1);
            if (lane < D / 2) {
                const bf16 *src = (const bf16 *)p.k_new + ((size_t)(sq.tok_off + i) * Hkv + kvh) * D;
                const float2 cs = rope_cos_sin(p.seq[ee].k_pos + i, p.rev_freq[lane]);
                bf16 ka = pre_k[0][0], kb = pre_k[0][1];
                if (i >= NPRE) {
                    ka = src[lane];
                    kb = src[lane + D / 2];
                } else {
#pragma unroll
                    for (int x = 1; x < NPRE; ++x)
                        if (i == x) {
                            ka = pre_k[x][0];
                            kb = pre_k[x][1];
                        }
                }
                const float a = (float)ka, b = (float)kb;
                unsigned char *row = wmem + rr * (D * 2);
                const int e0 = lane, e1 = lane + D / 2;
                bf16 r0, r1;
                rotate_key_pair(a, b, cs, r0, r1);
                *(bf16 *)(row + ((((e0 >> 3) ^ gg) & (T::CH - 1)) * 16) + (e0 & 7) * 2) = r0;
                *(bf16 *)(row + ((((e1 >> 3) ^ gg) & (T::CH - 1)) * 16) + (e1 & 7) * 2) = r1;
            }
        }
    };
    auto patch_v = [&](int tt) __attribute__((always_inline)) {
        const int first = max(C - tt * KN, 0);  // first tile row to rewrite
        for (int w = first >> 3; w < KN / 8; ++w) {  // 8-slot words of the tile
            const int pg = w >> 1, half = w & 1;
#pragma unroll
            for (int cx = 0; cx < VPL; ++cx) {
                const int c = lane + 64 * cx;
                bf16x8 *word = (bf16x8 *)(wmem + K_BYTES + pg * T::V_PAGE_BYTES + (c >> 5) * 1024 + half * 512 +
                                          (c & 31) * 16);
                bf16x8 x = *word;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int rr = w * 8 + e, i = tt * KN + rr - C;
                    if (rr >= first) {
                        bf16 val = (bf16)0.f;
                        if (i < sq.n_new) {
                            if (i >= NPRE) {
                                val = ((const bf16 *)p.v_new)[((size_t)(sq.tok_off + i) * Hkv + kvh) * D + c];
                            } else {
                                val = pre_v[0][cx];
#pragma unroll
                                for (int y = 1; y < NPRE; ++y)
                                    if (i == y) val = pre_v[y][cx];
                            }
                        }
                        x[e] = val;
                    }
                }
                *word = x;
            }
        }
    };

    for (int t = 0; t < n_tiles; ++t) {
        // K of tile t has landed (its V may still be on the way)
        wait_loads<2 * ITS>();
        asm volatile("" ::: "memory");
        if (FUSED && causal && (tile_lo + t + 1) * KN > C) {
            patch_k(tile_lo + t);
            asm volatile("" ::: "memory");
        }
        f32x16 S;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 a = *(const bf16x8 *)(wmem + krow * (D * 2) + (((2 * ks + h) ^ gj) & (T::CH - 1)) * 16);
            if (ks == 0) {
                f32x16 z;
#pragma unroll
                for (int v = 0; v < 16; ++v) z[v] = 0.f;
                S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, Q[ks], z, 0, 0, 0);
            } else {
                S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, Q[ks], S, 0, 0, 0);
            }
        }
        // the K buffer has been read: the next tile's keys can come in behind this tile's V
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (t + 1 < n_tiles) issue_k(t + 1);
        // mask (first / last tiles of the piece, causal limit), online softmax in the log2 domain
        const int tt = tile_lo + t;
        if (tt * KN < k_lo || (tt + 1) * KN > (causal ? min(C + 1, k_end) : k_end)) {
            const int lim = klim - tt * KN - 8 * h, low = k_lo - tt * KN - 8 * h;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int kl = 16 * (v >> 3) + (v & 7);
                if (kl >= lim || kl < low) S[v] = -INFINITY;
            }
        }
        float mx = S[0];
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(mx, S[v]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        bf16x8 P[2];
        float tsum = 0.f;
#pragma unroll
        for (int v = 0; v < 16; v += 2) {
            bf16x2 pe;
            pe[0] = (bf16)__builtin_amdgcn_exp2f(S[v] - m_new);
            pe[1] = (bf16)__builtin_amdgcn_exp2f(S[v + 1] - m_new);
            tsum = __builtin_amdgcn_fdot2_f32_bf16(pe, ones, tsum, false);
            P[v >> 3][v & 7] = pe[0];
            P[v >> 3][(v & 7) + 1] = pe[1];
        }
        l_run = l_run * alpha + tsum;
        if (__any(alpha != 1.0f)) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) O[db][v] *= alpha;
        }
        // V of tile t has landed (the next K may be on the way)
        if (t + 1 < n_tiles)
            wait_loads<2 * ITS>();
        else
            wait_loads<0>();
        asm volatile("" ::: "memory");
        if (FUSED && causal && (tt + 1) * KN > C) {
            patch_v(tt);
            asm volatile("" ::: "memory");
        }
#pragma unroll
        for (int pg = 0; pg < 2; ++pg)
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const bf16x8 a = *(const bf16x8 *)(wmem + v_read_off + pg * T::V_PAGE_BYTES + db * 1024);
                O[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, P[pg], O[db], 0, 0, 0);
            }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (t + 1 < n_tiles) issue_v(t + 1);
    }

    // ---- merge of the eight waves through LDS ----
    // Each wave leaves its unnormalised fp32 output in its own tile buffer, laid out
    // [4-channel group][row][4 floats] so that lanes with consecutive rows are 16 bytes apart
    // when writing; a group takes 33 row slots, not 32, so that the 16 lanes that later read one
    // row's 16 groups do not all hit the same banks (the 16 bytes per group this adds reach into
    // the cos/sin table, which is no longer needed).  (reference, sum) of the rows sit behind
    // the table.
    constexpr int GS = 33;  // row slots per channel group
    {
        const float l_tot = l_run + __shfl_xor(l_run, 32);
        f32x4 *ow = (f32x4 *)wmem;
        if (j < R) {  // only the rows that exist are read back
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    f32x4 o;
#pragma unroll
                    for (int x = 0; x < 4; ++x) o[x] = O[db][4 * a + x];
                    ow[(db * 8 + 2 * a + h) * GS + j] = o;
                }
        }
        if (h == 0) *(float2 *)(wmem + K_BYTES + V_BYTES + TAB_BYTES + j * 8) = make_float2(m_run, l_tot);
    }
    __syncthreads();
    // thread (row, 8-channel slice): D/8 threads per row, 32 rows -> 4 D threads = all of them
    // for D = 128; for D = 64 the upper half idles
    constexpr int LPR = D / 8;
    const int mrow = tid / LPR, sub = tid % LPR;
    const bool merger = mrow < 32 && mrow < R;
    float mm = -1.0e30f, ll = 0.f;
    float acc[8];
#pragma unroll
    for (int x = 0; x < 8; ++x) acc[x] = 0.f;
    if (merger) {
        // every LDS read first (24 of them in flight), then the arithmetic
        float2 ml[kDecodeWaves];
        f32x4 o0[kDecodeWaves], o1[kDecodeWaves];
#pragma unroll
        for (int w = 0; w < kDecodeWaves; ++w) {
            ml[w] = *(const float2 *)(smem + w * WAVE_BYTES + K_BYTES + V_BYTES + TAB_BYTES + mrow * 8);
            const f32x4 *ow = (const f32x4 *)(smem + w * WAVE_BYTES);
            o0[w] = ow[(2 * sub) * GS + mrow];
            o1[w] = ow[(2 * sub + 1) * GS + mrow];
        }
#pragma unroll
        for (int w = 0; w < kDecodeWaves; ++w) mm = fmaxf(mm, ml[w].x);
#pragma unroll
        for (int w = 0; w < kDecodeWaves; ++w) {
            const float wgt = __builtin_amdgcn_exp2f(ml[w].x - mm);
            ll += wgt * ml[w].y;
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                acc[x] += wgt * o0[w][x];
                acc[4 + x] += wgt * o1[w][x];
            }
        }
    }
    // ---- this work-group's result: final output, or a partial for the last work-group ----
    const int mtok = mrow / G, mhead = kvh * G + (mrow - mtok * G);
    const size_t lr = (size_t)mtok * Hq + mhead;
    const bool direct = sq.total_splits == 1;
    if (merger) {
        const float inv = ll > 0.f ? 1.0f / ll : 0.f;
        if (direct) {
            const size_t o_idx = ((size_t)sq.tok_off * Hq + lr) * D + sub * 8;
            if (p.out_f32) {
#pragma unroll
                for (int x = 0; x < 8; x += 4) {
                    f32x4 v;
#pragma unroll
                    for (int c = 0; c < 4; ++c) v[c] = acc[x + c] * inv;
                    *(f32x4 *)((float *)p.out + o_idx + x) = v;
                }
            } else {
                bf16x8 ob;
#pragma unroll
                for (int x = 0; x < 8; ++x) ob[x] = (bf16)(acc[x] * inv);
                *(bf16x8 *)((bf16 *)p.out + o_idx) = ob;
            }
        } else {
            const size_t prow = (size_t)sq.part_off + (size_t)wg * sq.n_new * Hq + lr;
            if (p.out_f32) {
                float *dst = (float *)p.part_o + prow * D + sub * 8;
#pragma unroll
                for (int x = 0; x < 8; x += 2) {
                    union { float f[2]; uint64_t u; } w2;
                    w2.f[0] = acc[x] * inv;
                    w2.f[1] = acc[x + 1] * inv;
                    store_coherent8(dst + x, w2.u);
                }
            } else {
                union { bf16x8 v; uint64_t u[2]; } w8;
#pragma unroll
                for (int x = 0; x < 8; ++x) w8.v[x] = (bf16)(acc[x] * inv);
                bf16 *dst = (bf16 *)p.part_o + prow * D + sub * 8;
                store_coherent8(dst, w8.u[0]);
                store_coherent8(dst + 4, w8.u[1]);
            }
            if (sub == 0) {
                union { float2 v; uint64_t u; } w2;
                w2.v = make_float2(mm, ll);
                store_coherent8(p.part_ml + prow * 2, w2.u);
            }
        }
    }
    if (!direct) {
        wait_loads<0>();  // stores acknowledged
        __syncthreads();
        int *flag = (int *)(smem + kDecodeWaves * WAVE_BYTES);
        if (tid == 0) {
            int *cnt = p.counters + sq.cnt_base + kvh;
            const int ticket = atomicAdd(cnt, 1);
            const int last = ticket == sq.total_splits - 1;
            if (last) atomicExch(cnt, 0);
            *flag = last;
        }
        __syncthreads();
        if (*flag) {  // uniform over the work-group: everybody helps with the merge
            auto row_fn = [&](int rr, size_t &prow0, size_t &o_idx) __attribute__((always_inline)) {
                const int t2 = rr / G, h2 = kvh * G + (rr - t2 * G);
                const size_t lr2 = (size_t)t2 * Hq + h2;
                prow0 = (size_t)sq.part_off + lr2;
                o_idx = ((size_t)sq.tok_off * Hq + lr2) * D;
            };
            float *scratch = (float *)smem;  // the tile buffers are free by now
            if (p.out_f32)
                merge_rows_parallel<D, float, kDecodeWaves * 64>(p.part_o, p.part_ml, (size_t)sq.n_new * Hq,
                                                                 sq.total_splits, R, p.out, true, scratch, row_fn);
            else
                merge_rows_parallel<D, bf16, kDecodeWaves * 64>(p.part_o, p.part_ml, (size_t)sq.n_new * Hq,
                                                                sq.total_splits, R, p.out, false, scratch, row_fn);
        }
    }
}

template <int D>
__global__ __launch_bounds__(kDecodeWaves * 64) void decode_kernel(const AttnParams p) {
    decode_body<D, false>(p, blockIdx.x);
}

// One launch for a whole step of short chunks: work-groups [0, n_attn) attend (reading the
// chunk's own keys and values from the inputs), the others append the chunk to the cache.
// Neither part waits for the other.
template <int D>
__global__ __launch_bounds__(kDecodeWaves * 64) void decode_step_kernel(const AttnParams p, const AppendParams a,
                                                                         const int n_attn) {
    if ((int)blockIdx.x < n_attn) {
        decode_body<D, true>(p, blockIdx.x);
    } else {
        extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
        rope_append_body<D>(a, (int)blockIdx.x - n_attn, (bf16(*)[D + 8]) smem);
    }
}

// =========================================================================================
// Combine: out = sum_s w_s O_s / sum_s w_s with w_s = 2^(m_s - m) l_s, m = max_s m_s, over the
// normalised per-split partials O_s.  D/8 lanes per (token, query head) row, 8 channels each.
// =========================================================================================
template <int D, typename PT>
__global__ __launch_bounds__(kThreads) void combine_kernel(const CombineParams p) {
    constexpr int LPR = D / 8;                 // lanes per row
    constexpr int RPB = kThreads / LPR;        // rows per work-group
    const int sub = threadIdx.x % LPR;
    const int row = blockIdx.x * RPB + threadIdx.x / LPR;
    if (row >= p.n_rows) return;
    int s = 0;
    while (s + 1 < p.n_seqs && row >= p.seq[s + 1].row_begin) ++s;
    const CombineSeq sq = p.seq[s];
    const int Hq = p.n_q_heads;
    const int lr = row - sq.row_begin;  // = token * Hq + head inside the sequence
    merge_row<D, PT>(p.part_o, p.part_ml, (size_t)sq.part_off + lr, (size_t)sq.n_new * Hq, sq.n_splits,
                     p.out, p.out_f32 != 0, ((size_t)sq.tok_off * Hq + lr) * D, sub);
}

// =========================================================================================
// Launchers
// =========================================================================================
hipError_t launch_few_keys(const AttnParams &p, int head_dim, hipStream_t stream) {
    if (p.few_rows <= 0) return hipSuccess;
    const dim3 grid((p.few_rows + kFewRowsPerGroup - 1) / kFewRowsPerGroup), block(kFewRowsPerGroup * 64);
    if (head_dim == 128)
        hipLaunchKernelGGL(few_keys_kernel<128>, grid, block, 0, stream, p);
    else if (head_dim == 64)
        hipLaunchKernelGGL(few_keys_kernel<64>, grid, block, 0, stream, p);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_rope_append(const AppendParams &p, int head_dim, hipStream_t stream) {
    if (p.n_items <= 0) return hipSuccess;
    if (head_dim == 128)
        hipLaunchKernelGGL(rope_append_kernel<128>, dim3(p.n_items), dim3(kThreads), 0, stream, p);
    else if (head_dim == 64)
        hipLaunchKernelGGL(rope_append_kernel<64>, dim3(p.n_items), dim3(kThreads), 0, stream, p);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

// Kernels whose dynamic LDS exceeds 64 KB need the limit raised first: once per kernel and
// device, whichever host thread gets there first (the outcome of that one try is kept).
constexpr int kMaxDevices = 64;
struct LargeLdsOnce {
    std::once_flag once[kMaxDevices];
    hipError_t result[kMaxDevices];
};
static hipError_t allow_large_lds(const void *fn, LargeLdsOnce &st) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::call_once(st.once[dev], [&] {
        st.result[dev] = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    });
    return st.result[dev];
}

// ev_start / ev_stop (both or neither): events the runtime stamps with the begin and the end of
// this very dispatch (not of the stream around it).
template <int D, int QB, bool MULTI, bool HOLES = false>
static hipError_t launch_attn(const AttnParams &p, hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop) {
    const size_t lds = attention_lds_bytes(D, p.tab_tokens, MULTI);
    static LargeLdsOnce large_lds;
    if (lds > 64 * 1024) {
        hipError_t e = allow_large_lds((const void *)attn_kernel<D, QB, MULTI, HOLES>, large_lds);
        if (e != hipSuccess) return e;
    }
    constexpr int NW = kRowsPerWorkgroup / (32 * QB);
    const dim3 grid(p.items_per_xcd * 8 + (p.few_rows + NW - 1) / NW), block(NW * 64);
    if (ev_start)
        hipExtLaunchKernelGGL((attn_kernel<D, QB, MULTI, HOLES>), grid, block, (uint32_t)lds, stream, ev_start, ev_stop, 0, p);
    else
        hipLaunchKernelGGL((attn_kernel<D, QB, MULTI, HOLES>), grid, block, lds, stream, p);
    return hipGetLastError();
}

hipError_t launch_chunk_attention(const AttnParams &p, int head_dim, hipStream_t stream, hipEvent_t ev_start,
                                  hipEvent_t ev_stop) {
    if (p.n_items <= 0 && p.few_rows <= 0) return hipSuccess;
    if (p.hole_width > 0) {  // a pack under the action-isolating mask
        if (p.multi_entry || p.hole_period < kKeyTile) return hipErrorInvalidValue;
        if (head_dim == 128) return launch_attn<128, 1, false, true>(p, stream, ev_start, ev_stop);
        if (head_dim == 64) return launch_attn<64, 1, false, true>(p, stream, ev_start, ev_stop);
        return hipErrorInvalidValue;
    }
    if (head_dim == 128)
        return p.multi_entry ? launch_attn<128, 1, true>(p, stream, ev_start, ev_stop)
                             : launch_attn<128, 1, false>(p, stream, ev_start, ev_stop);
    if (head_dim == 64)
        return p.multi_entry ? launch_attn<64, 1, true>(p, stream, ev_start, ev_stop)
                             : launch_attn<64, 1, false>(p, stream, ev_start, ev_stop);
    return hipErrorInvalidValue;
}

// =========================================================================================
// Page copies between two page pools (offload of cache segments to host memory and reload of
// the ones a sampler selects).  One work-group per page: the K block and the V block of a
// page are page_bytes contiguous bytes each, moved with 16-byte accesses.  Either pool may be
// device memory or pinned host memory the device can address.
// =========================================================================================
__global__ __launch_bounds__(kThreads) void pages_copy_kernel(const PageCopyParams p) {
    const int i = blockIdx.x;
    if (i >= p.n) return;
    const size_t src = (size_t)p.src_page[i] * p.page_bytes, dst = (size_t)p.dst_page[i] * p.page_bytes;
    const int words = p.page_bytes / 16;
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    for (int w = threadIdx.x; w < words; w += kThreads) {
        const u32x4 a = *(const u32x4 *)((const char *)p.src_k + src + (size_t)w * 16);
        const u32x4 b = *(const u32x4 *)((const char *)p.src_v + src + (size_t)w * 16);
        *(u32x4 *)((char *)p.dst_k + dst + (size_t)w * 16) = a;
        *(u32x4 *)((char *)p.dst_v + dst + (size_t)w * 16) = b;
    }
}

hipError_t launch_pages_copy(const PageCopyParams &p, hipStream_t stream) {
    if (p.n <= 0) return hipSuccess;
    hipLaunchKernelGGL(pages_copy_kernel, dim3(p.n), dim3(kThreads), 0, stream, p);
    return hipGetLastError();
}

__global__ void zero_counters_kernel(int *counters, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) counters[i] = 0;
}

// The library's own scratch array: the workspace of the entry point that allocates nothing.
// In host code the array's name is only a handle of the symbol; its device address differs from
// GPU to GPU and comes from hipGetSymbolAddress, asked once per device with that device current.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

hipError_t static_scratch(void **ptr, size_t *bytes) {
    static std::mutex mu;
    static void *dev_ptr[kMaxDevices] = {};
    *ptr = nullptr;
    *bytes = 0;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!dev_ptr[dev]) {
        void *a = nullptr;
        e = hipGetSymbolAddress(&a, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!a) return hipErrorInvalidSymbol;
        dev_ptr[dev] = a;
    }
    *ptr = dev_ptr[dev];
    *bytes = kStaticScratchBytes;
    return hipSuccess;
}

hipError_t launch_zero_counters(int *counters, int n, hipStream_t stream) {
    hipLaunchKernelGGL(zero_counters_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, counters, n);
    return hipGetLastError();
}

hipError_t launch_decode_attention(const AttnParams &p, int head_dim, int n_workgroups, hipStream_t stream,
                                   hipEvent_t ev_start, hipEvent_t ev_stop, const AppendParams *fused) {
    if (n_workgroups <= 0) return hipSuccess;
    const size_t lds = decode_lds_bytes(head_dim, p.tab_tokens);
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    if (head_dim != 128 && head_dim != 64) return hipErrorInvalidValue;
    if (fused) {
        static LargeLdsOnce step_large_lds[2];
        const int si = head_dim == 128 ? 0 : 1;
        const void *sfn =
            head_dim == 128 ? (const void *)decode_step_kernel<128> : (const void *)decode_step_kernel<64>;
        if (lds > 64 * 1024) {
            hipError_t e = allow_large_lds(sfn, step_large_lds[si]);
            if (e != hipSuccess) return e;
        }
        const dim3 sgrid(n_workgroups + fused->n_items), sblock(kDecodeWaves * 64);
        if (ev_start) {
            if (head_dim == 128)
                hipExtLaunchKernelGGL((decode_step_kernel<128>), sgrid, sblock, (uint32_t)lds, stream, ev_start,
                                      ev_stop, 0, p, *fused, n_workgroups);
            else
                hipExtLaunchKernelGGL((decode_step_kernel<64>), sgrid, sblock, (uint32_t)lds, stream, ev_start,
                                      ev_stop, 0, p, *fused, n_workgroups);
        } else if (head_dim == 128) {
            hipLaunchKernelGGL((decode_step_kernel<128>), sgrid, sblock, lds, stream, p, *fused, n_workgroups);
        } else {
            hipLaunchKernelGGL((decode_step_kernel<64>), sgrid, sblock, lds, stream, p, *fused, n_workgroups);
        }
        return hipGetLastError();
    }
    static LargeLdsOnce large_lds[2];
    const int idx = head_dim == 128 ? 0 : 1;
    const void *fn = head_dim == 128 ? (const void *)decode_kernel<128> : (const void *)decode_kernel<64>;
    if (lds > 64 * 1024) {
        hipError_t e = allow_large_lds(fn, large_lds[idx]);
        if (e != hipSuccess) return e;
    }
    const dim3 grid(n_workgroups), block(kDecodeWaves * 64);
    if (ev_start) {
        if (head_dim == 128)
            hipExtLaunchKernelGGL((decode_kernel<128>), grid, block, (uint32_t)lds, stream, ev_start, ev_stop, 0, p);
        else
            hipExtLaunchKernelGGL((decode_kernel<64>), grid, block, (uint32_t)lds, stream, ev_start, ev_stop, 0, p);
    } else if (head_dim == 128) {
        hipLaunchKernelGGL((decode_kernel<128>), grid, block, lds, stream, p);
    } else {
        hipLaunchKernelGGL((decode_kernel<64>), grid, block, lds, stream, p);
    }
    return hipGetLastError();
}

hipError_t launch_combine(const CombineParams &p, int head_dim, hipStream_t stream) {
    if (p.n_rows <= 0) return hipSuccess;
    const int rpb = kThreads / (head_dim / 8);
    const dim3 grid((p.n_rows + rpb - 1) / rpb), block(kThreads);
    if (head_dim == 128 && p.out_f32)
        hipLaunchKernelGGL((combine_kernel<128, float>), grid, block, 0, stream, p);
    else if (head_dim == 128)
        hipLaunchKernelGGL((combine_kernel<128, bf16>), grid, block, 0, stream, p);
    else if (head_dim == 64 && p.out_f32)
        hipLaunchKernelGGL((combine_kernel<64, float>), grid, block, 0, stream, p);
    else if (head_dim == 64)
        hipLaunchKernelGGL((combine_kernel<64, bf16>), grid, block, 0, stream, p);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace evl

// Paged attention for bf16 caches, head_dim 128, 16-position pages, decode form: the layer's
// HBM-bound operator (the paper's memory-bound "decode attention", Section 2), plus the
// device-side work lists shared with the prefill form (kernels_attn_prefill.hip).
//
// A wave serves one token of a single-token sequence against one chunk (up to the handle's
// chunk size, 256 positions by default; a sequence's chunks are of equal size up to rounding) of one kv head, all q heads of that kv head's group at once, so K and V are fetched once per kv
// head.  A page of K is 16 rows of 256 bytes, a page of V is 128 rows (one per head-dim
// index) of 32 bytes; both are loaded straight into MFMA operand layout with fully used
// 64-byte / 32-byte row segments, no LDS.  The group's scores are a skinny but real
// contraction
//     S[16 positions, G heads] = K_page[16, 128] Q^T[128, G]      (4 x mfma 16x16x32)
//     O^T[128, G]           += V_page^T[128, 16] P[16, G]         (8 x mfma 16x16x16)
// whose D layout (lane: head l%16, positions 4*(l/16)+r) is exactly the B layout the second
// product wants, so probabilities never cross lanes.  Doing the same dot products on the
// vector ALUs would need about 28 wave instructions per cached position and kv head, which
// at HBM rate is most of the ALU issue slots of a CU; on the matrix cores it is a few
// percent.  Softmax is online per tile of two pages in the exp2 domain with the running
// max shared by the four lanes of a head; the partial (m, l, o) of the chunk goes to the
// split-KV arrays and attn_combine_kernel merges chunks in order.
#include "common.h"
#include "kernels.h"

namespace dyn {

hipError_t launch_attention_combine(int dtype, bool base2, float *part_o, float *part_ml,
                                    const int32_t *pos_of_token, const int32_t *ct_of_token, void *out, int ld_out,
                                    const AttnShape &sh, int rows, hipStream_t s, int32_t *counter_reset);
int attn_prefill_block_tokens(const AttnShape &sh);
hipError_t launch_attention_prefill(const void *qkv, const int32_t *seq_of_token, const int32_t *pos_of_token,
                                    const int32_t *block_table, const void *k_cache, const void *v_cache, float *part_o,
                                    float *part_ml, const AttnShape &sh, int32_t *plan, long max_items, int max_groups,
                                    hipStream_t s);

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

constexpr int HD = 128, PS = 16, TILE_PAGES = 2;
constexpr int kPersistentGroups = 512;   // two 4-wave workgroups for each of the 256 CUs

// Work lists, built on the device from the positions (contexts differ by 8x inside a batch, so
// a dense token x max_chunks grid would be mostly empty workgroups).  A wave serves a query
// group: tokens of one sequence whose positions fall in the same aligned block of `tg`
// positions, all of them against one pass over the keys.  List 0 holds the tokens that are
// alone in their sequence this step (decode: groups of one, 4 of 16 MFMA columns live), list 1
// the tokens of multi-token sequences (prefill chunks) in query blocks of up to tg1 tokens, against
// chunks of prefill_chunk_positions() positions (1024 unless the block reaches past 8192 keys).
// One entry per (group, chunk) that exists: list[0] = number of entries, entry i =
// (first token row, chunk | tokens << 20) at list[2 + 2 i].
// List 0 is ordered by work, largest first: its entries are bucketed by their size in quarters of
// the largest chunk (kPlanBuckets buckets; with the default chunk of 16 pages a quarter is one
// tile pair of four pages) and inside a bucket they stay in token order, so the eight kv heads of a chunk and the chunks
// of a sequence remain neighbours.  The persistent decode kernel deals the list out by wave index
// in a snake (attn_mfma_kernel): with equal-sized items first and the small ones at the end, the
// waves' totals differ by about one percent instead of six on contexts spread over 1024..8192.
constexpr int kPlanBuckets = 4;

__global__ __launch_bounds__(1024) void attn_plan_kernel(const int32_t *__restrict__ seq_of_token,
                                                         const int32_t *__restrict__ pos_of_token, int rows, int ct,
                                                         int tg1, int32_t *__restrict__ plan0,
                                                         int32_t *__restrict__ plan1, int32_t *__restrict__ ct_of_token) {
    // One workgroup of 16 waves walks the rows 1024 at a time.  A sequence's tokens are adjacent
    // rows with consecutive positions, so a token leads its group iff it starts its sequence or
    // its aligned block, and the group's size comes from a bisection over the look-ahead rows.
    // Entry offsets come from a wave scan plus one LDS step per list (per bucket of list 0).
    constexpr int NL = kPlanBuckets + 1;                    // scanned counters: list 0's buckets, then list 1
    __shared__ int wave_tot[NL][16];
    __shared__ int bucket_total[kPlanBuckets];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int chunk_pages = ct / PS, bucket_pages = max(1, (chunk_pages + kPlanBuckets - 1) / kPlanBuckets);

    // What token row t contributes: which list, how many entries, and for list 0 the buckets of
    // its chunks (all but the last have the sequence's balanced chunk size, the last the rest).
    struct Row { int which, nc, n_tok, b_full, b_last; };
    auto classify = [&](int t) {
        Row r{0, 0, 0, 0, 0};
        const int s = seq_of_token[t], p = pos_of_token[t];
        const bool prev_same = t > 0 && seq_of_token[t - 1] == s, next_same = t + 1 < rows && seq_of_token[t + 1] == s;
        r.which = prev_same || next_same;
        const int tg = r.which ? tg1 : 1;
        if (!prev_same || p % tg == 0) {                     // group leader
            const int cand = tg - p % tg;                    // positions left in the aligned block
            // rows t .. t + n_tok - 1 belong to the sequence: the matches form a prefix of the
            // candidates, found by bisection (a few dependent cache hits instead of tg loads)
            int lo = 1, hi = min(cand, rows - t);            // n_tok lies in [lo, hi]
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (seq_of_token[t + mid - 1] == s) lo = mid;
                else hi = mid - 1;
            }
            r.n_tok = lo;
            const int ctw = r.which ? prefill_chunk_positions((p / tg1 + 1) * tg1) : ct;
            r.nc = (p + r.n_tok - 1 + ctw) / ctw;            // chunks the group's last token reaches
            if (!r.which) {                                  // the decode kernel's own chunking of this sequence
                const int seq_pages = (p + PS) / PS;         // ceil((p + 1) / PS)
                const int cp = (seq_pages + r.nc - 1) / r.nc, last = seq_pages - (r.nc - 1) * cp;
                r.b_full = max(0, kPlanBuckets - (cp + bucket_pages - 1) / bucket_pages);
                r.b_last = max(0, kPlanBuckets - (last + bucket_pages - 1) / bucket_pages);
            }
        }
        return r;
    };

    // pass 1: sizes of list 0's buckets
    if (threadIdx.x < kPlanBuckets) bucket_total[threadIdx.x] = 0;
    __syncthreads();
    Row first_batch{0, 0, 0, 0, 0};                          // the first 1024 rows are classified once (most batches have no more)
    for (int t = threadIdx.x; t < rows; t += 1024) {
        const Row r = classify(t);
        if (t < 1024) first_batch = r;
        if (!r.which && r.nc > 0) {
            if (r.nc > 1) atomicAdd(&bucket_total[r.b_full], r.nc - 1);
            atomicAdd(&bucket_total[r.b_last], 1);
        }
    }
    __syncthreads();
    int base[NL];                                             // next free entry of each bucket / of list 1
    base[0] = 0;
#pragma unroll
    for (int k = 1; k < kPlanBuckets; ++k) base[k] = base[k - 1] + bucket_total[k - 1];
    const int total0 = base[kPlanBuckets - 1] + bucket_total[kPlanBuckets - 1];
    base[kPlanBuckets] = 0;

    // pass 2: entries, in token order inside each bucket
    for (int t0 = 0; t0 < rows; t0 += 1024) {
        const int t = t0 + threadIdx.x;
        Row r{0, 0, 0, 0, 0};
        if (t < rows) {
            r = t0 == 0 ? first_batch : classify(t);
            const int p = pos_of_token[t];
            ct_of_token[t] = r.which ? prefill_chunk_positions((p / tg1 + 1) * tg1) : ct;   // the chunk size this token's partials are indexed by
        }
        int v[NL];                                            // this thread's entries per counter
#pragma unroll
        for (int k = 0; k < NL; ++k) v[k] = 0;
        if (r.which) {
            v[kPlanBuckets] = r.nc;
        } else if (r.nc > 0) {
#pragma unroll
            for (int k = 0; k < kPlanBuckets; ++k) v[k] = (k == r.b_full ? r.nc - 1 : 0) + (k == r.b_last ? 1 : 0);
        }
        int incl[NL];                                         // inclusive wave scans
#pragma unroll
        for (int k = 0; k < NL; ++k) {
            int x = v[k];
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int u = __shfl_up(x, off, 64);
                if (lane >= off) x += u;
            }
            incl[k] = x;
            if (lane == 63) wave_tot[k][wave] = x;
        }
        __syncthreads();
        int start[NL];
#pragma unroll
        for (int k = 0; k < NL; ++k) {
            int pre = 0, tot = 0;
#pragma unroll
            for (int w = 0; w < 16; ++w) {
                if (w < wave) pre += wave_tot[k][w];
                tot += wave_tot[k][w];
            }
            start[k] = base[k] + pre + incl[k] - v[k];
            base[k] += tot;
        }
        if (r.which) {
            for (int c = 0; c < r.nc; ++c) {
                plan1[2 + 2 * (start[kPlanBuckets] + c)] = t;
                plan1[3 + 2 * (start[kPlanBuckets] + c)] = c | (r.n_tok << 20);
            }
        } else if (r.nc > 0) {
            int at_full = 0, at_last = 0;
#pragma unroll
            for (int k = 0; k < kPlanBuckets; ++k) {          // select without indexing the register arrays dynamically
                if (k == r.b_full) at_full = start[k];
                if (k == r.b_last) at_last = start[k] + (r.b_last == r.b_full ? r.nc - 1 : 0);
            }
            for (int c = 0; c + 1 < r.nc; ++c) {
                plan0[2 + 2 * (at_full + c)] = t;
                plan0[3 + 2 * (at_full + c)] = c | (1 << 20);
            }
            plan0[2 + 2 * at_last] = t;
            plan0[3 + 2 * at_last] = (r.nc - 1) | (1 << 20);
        }
        __syncthreads();                                      // wave_tot is reused by the next batch
    }
    if (threadIdx.x == 0) { plan0[0] = total0; plan1[0] = base[kPlanBuckets]; plan1[1] = 0; }   // list sizes; list 1's work counter
}

// Persistent waves: in round k wave w of the launch takes (entry, kv head) pair k * n_waves + w,
// in odd rounds k * n_waves + (n_waves - 1 - w): a snake over a list that is ordered largest first
// (attn_plan_kernel), so a wave that drew the largest item of one round draws the smallest of the next.
// A pair is walked two tiles (four pages) at a time through two register buffers, and when a
// pair runs out of tiles the free buffer is refilled with the first tile of the wave's next
// pair - whose indices were fetched while this pair was being multiplied - so the stream of
// loads never drains at a pair boundary and the three dependent lookups (work list ->
// position / sequence -> block table) are off the critical path.
// NQG = sets of 16 MFMA columns per wave; the decode list uses 1 (eight waves per CU keep HBM
// busy, 4 of the 16 columns live with four q heads per kv head).
struct AttnItem {
    int t, c, n_tok;                  // first token row of the query group, chunk, tokens in the group
    int n_keys, lp_first, seq_pages;  // keys the group's last token attends, first logical page of the chunk, the sequence's pages
    int lp_last, key_end;             // last logical page of the chunk; first position past the chunk (at most n_keys)
    int n_pair;                       // tile pairs to walk
    const int32_t *bt;                // block-table row of the group's sequence
};

template <int NQG>
__global__ __launch_bounds__(256, NQG == 1 ? 2 : 1) void attn_mfma_kernel(const bf16_t *__restrict__ qkv,
                                                           const int32_t *__restrict__ seq_of_token,
                                                           const int32_t *__restrict__ pos_of_token,
                                                           const int32_t *__restrict__ block_table,
                                                           const bf16_t *__restrict__ k_cache,
                                                           const bf16_t *__restrict__ v_cache,
                                                           float *__restrict__ part_o, float *__restrict__ part_ml,
                                                           AttnShape sh, const int32_t *__restrict__ plan) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_items = plan[0] * sh.n_kv;
    const int n_waves = gridDim.x * 4;
    const int G = sh.n_q / sh.n_kv, TG = 16 / G;
    const int lane = threadIdx.x & 63, lr = lane & 15, lq = lane >> 4;
    const int col_tok = lr / G, col_head = lr % G;   // MFMA column lr of set q = (token q * TG + col_tok, q head col_head)
    const float sscale = 1.4426950408889634f / sqrtf((float)HD);   // log2(e) / sqrt(d)

    const int gw = blockIdx.x * 4 + wave;
    int round = 0;
    auto item_at = [&](int k) { return k * n_waves + ((k & 1) ? n_waves - 1 - gw : gw); };
    int item = item_at(0);
    if (item >= n_items) return;

    auto fetch_item = [&](int it, int &g_out) {
        AttnItem m;
        const int g = it % sh.n_kv, e = it / sh.n_kv;
        const int packed = plan[3 + 2 * e];
        m.c = packed & 0xfffff;
        m.n_tok = packed >> 20;
        m.t = plan[2 + 2 * e];
        m.n_keys = pos_of_token[m.t + m.n_tok - 1] + 1;
        m.seq_pages = (m.n_keys + PS - 1) / PS;
        // A sequence of P pages has ceil(P / chunk_pages) chunks, of equal size up to rounding
        // (ceil(P / chunks) pages, the last one the rest) rather than full ones and a short tail:
        // equal work items are what lets a static deal to the waves finish together.  The sizes
        // depend on the sequence's own length only.
        const int n_chunks = (m.seq_pages + sh.chunk_pages - 1) / sh.chunk_pages;
        const int cp = (m.seq_pages + n_chunks - 1) / n_chunks;
        m.lp_first = m.c * cp;
        const int n_pg = min(cp, m.seq_pages - m.lp_first);
        m.lp_last = m.lp_first + n_pg - 1;
        m.key_end = min(m.n_keys, (m.lp_first + n_pg) * PS);
        m.n_pair = (n_pg + 2 * TILE_PAGES - 1) / (2 * TILE_PAGES);          // a trailing odd tile is walked masked
        m.bt = block_table + (size_t)seq_of_token[m.t] * sh.max_pages_per_seq;
        g_out = g;
        return m;
    };

    u32x4 kreg[2][TILE_PAGES][4];
    u32x2 vreg[2][TILE_PAGES][8];
    bf16x8 qb[NQG][4], qn[NQG][4];
    int nk_cur[NQG], nk_nxt[NQG];                  // keys each column attends (0 for a dead column)

    // tile TL of item M into register buffer B; page indices past the chunk's last page
    // are clamped (their scores are masked, the loads hit L2)
#define DYN_ATTN_LOAD(B, M, GG, TL)                                                                               \
    {                                                                                                             \
        _Pragma("unroll") for (int pi = 0; pi < TILE_PAGES; ++pi) {                                               \
            const int lp = min((M).lp_first + (TL) * TILE_PAGES + pi, (M).lp_last);                               \
            const size_t pg = (size_t)(M).bt[lp] * sh.n_kv + (GG);                                                \
            const bf16_t *kp = k_cache + (pg * PS + lr) * HD + 8 * lq;                                            \
            const bf16_t *vp = v_cache + (pg * HD + lr) * PS + 4 * lq;                                            \
            _Pragma("unroll") for (int ks = 0; ks < 4; ++ks)                                                      \
                kreg[B][pi][ks] = *reinterpret_cast<const u32x4 *>(kp + ks * 32);                                 \
            _Pragma("unroll") for (int dt = 0; dt < 8; ++dt)                                                      \
                vreg[B][pi][dt] = *reinterpret_cast<const u32x2 *>(vp + dt * 16 * PS);                            \
        }                                                                                                         \
    }
    // B operands of the score product: column lr of set q = q vector of token t + q*TG + col_tok,
    // head g*G + col_head (zero for columns past the group)
#define DYN_ATTN_LOAD_Q(DST, NK, M, GG)                                                                           \
    _Pragma("unroll") for (int q = 0; q < NQG; ++q) {                                                             \
        const bool live = q * TG + col_tok < (M).n_tok && col_tok < TG;                                           \
        const int tq = (M).t + (live ? q * TG + col_tok : 0);                                                     \
        NK[q] = live ? min(pos_of_token[tq] + 1, (M).key_end) : 0;                                                \
        const bf16_t *qp = qkv + (size_t)tq * ((sh.n_q + 2 * sh.n_kv) * HD) + ((GG) * G + col_head) * HD + 8 * lq; \
        _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) {                                                        \
            u32x4 v = *reinterpret_cast<const u32x4 *>(qp + ks * 32);                                             \
            if (!live) v = u32x4{0u, 0u, 0u, 0u};                                                                 \
            DST[q][ks] = __builtin_bit_cast(bf16x8, v);                                                           \
        }                                                                                                         \
    }
#define DYN_ATTN_COMPUTE(B, TL)                                                                                   \
    _Pragma("unroll") for (int q = 0; q < NQG; ++q) {                                                             \
        f32x4 sv[TILE_PAGES];                                                                                     \
        float mx = -INFINITY;                                                                                     \
        _Pragma("unroll") for (int pi = 0; pi < TILE_PAGES; ++pi) {                                               \
            f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f};                                                                  \
            _Pragma("unroll") for (int ks = 0; ks < 4; ++ks)                                                      \
                s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kreg[B][pi][ks]),          \
                                                            qb[q][ks], s, 0, 0, 0);                               \
            const int jb = (cur.lp_first + (TL) * TILE_PAGES + pi) * PS + 4 * lq;                                 \
            _Pragma("unroll") for (int r = 0; r < 4; ++r) {                                                       \
                s[r] = (jb + r < nk_cur[q]) ? s[r] * sscale : -INFINITY;                                          \
                mx = fmaxf(mx, s[r]);                                                                             \
            }                                                                                                     \
            sv[pi] = s;                                                                                           \
        }                                                                                                         \
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));                                                                   \
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));                                                                   \
        const float m_new = fmaxf(m_run[q], mx);                                                                  \
        const float m_ref = m_new == -INFINITY ? 0.f : m_new;   /* a column with no key yet stays empty */        \
        const float alpha = __builtin_amdgcn_exp2f(m_run[q] - m_ref);                                             \
        m_run[q] = m_new;                                                                                         \
        l_run[q] *= alpha;                                                                                        \
        _Pragma("unroll") for (int dt = 0; dt < 8; ++dt) acc[q][dt] *= alpha;                                     \
        _Pragma("unroll") for (int pi = 0; pi < TILE_PAGES; ++pi) {                                               \
            f32x4 p;                                                                                              \
            _Pragma("unroll") for (int r = 0; r < 4; ++r) p[r] = __builtin_amdgcn_exp2f(sv[pi][r] - m_ref);       \
            const bf16x4 pb = __builtin_convertvector(p, bf16x4);                                                 \
            const u32x2 pw = __builtin_bit_cast(u32x2, pb);                                                       \
            l_run[q] += (__uint_as_float(pw[0] << 16) + __uint_as_float(pw[0] & 0xffff0000u)) +                   \
                        (__uint_as_float(pw[1] << 16) + __uint_as_float(pw[1] & 0xffff0000u));                    \
            const int nvalid = cur.key_end - (cur.lp_first + (TL) * TILE_PAGES + pi) * PS - 4 * lq;               \
            _Pragma("unroll") for (int dt = 0; dt < 8; ++dt) {                                                    \
                u32x2 vv = vreg[B][pi][dt];                                                                       \
                if (nvalid < 4) { /* positions past the group's last: keep stale cache bits out of 0 * x */     \
                    vv[0] &= (nvalid > 0 ? 0x0000ffffu : 0u) | (nvalid > 1 ? 0xffff0000u : 0u);                   \
                    vv[1] &= (nvalid > 2 ? 0x0000ffffu : 0u);                                                     \
                }                                                                                                 \
                acc[q][dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, vv),             \
                                                                       __builtin_bit_cast(s16x4, pb), acc[q][dt], 0, 0, 0); \
            }                                                                                                     \
        }                                                                                                         \
    }

    int g_cur = 0, g_nxt = 0;
    AttnItem cur = fetch_item(item, g_cur);
    DYN_ATTN_LOAD_Q(qb, nk_cur, cur, g_cur)
    DYN_ATTN_LOAD(0, cur, g_cur, 0)
    while (true) {
        const int next_item = item_at(round + 1);
        const bool more = next_item < n_items;
        // the wave's last pair "prefetches" itself again: harmless loads instead of a conditional branch
        AttnItem nxt = fetch_item(more ? next_item : item, g_nxt);
        f32x4 acc[NQG][8];
        float m_run[NQG], l_run[NQG];
#pragma unroll
        for (int q = 0; q < NQG; ++q) {
            m_run[q] = -INFINITY;
            l_run[q] = 0.f;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) acc[q][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }

        for (int pr = 0; pr < cur.n_pair; ++pr) {
            const bool last = pr + 1 == cur.n_pair;
            // buffer 0 holds tile 2 pr (loaded or in flight); scheduling barriers keep each
            // prefetch ahead of the multiply it overlaps
            DYN_ATTN_LOAD(1, cur, g_cur, 2 * pr + 1)
            __builtin_amdgcn_sched_barrier(0);
            DYN_ATTN_COMPUTE(0, 2 * pr)
            __builtin_amdgcn_sched_barrier(0);
            {   // refill buffer 0: this pair's next tile, or tile 0 of the wave's next pair
                const AttnItem src = last ? nxt : cur;
                const int gg = last ? g_nxt : g_cur, tile = last ? 0 : 2 * pr + 2;
                DYN_ATTN_LOAD_Q(qn, nk_nxt, nxt, g_nxt)
                DYN_ATTN_LOAD(0, src, gg, tile)
            }
            __builtin_amdgcn_sched_barrier(0);
            DYN_ATTN_COMPUTE(1, 2 * pr + 1)
            __builtin_amdgcn_sched_barrier(0);
        }

#pragma unroll
        for (int q = 0; q < NQG; ++q) {
            float l = l_run[q];
            l += __shfl_xor(l, 16, 64);
            l += __shfl_xor(l, 32, 64);
            if (nk_cur[q] > cur.lp_first * PS) {                 // the chunk exists for this column's token
                const size_t pidx =
                    ((size_t)(cur.t + q * TG + col_tok) * sh.n_q + g_cur * G + col_head) * sh.max_chunks + cur.c;
#pragma unroll
                for (int dt = 0; dt < 8; ++dt)
                    *reinterpret_cast<f32x4 *>(part_o + pidx * HD + dt * 16 + 4 * lq) = acc[q][dt];
                if (lq == 0) {
                    part_ml[pidx * 2] = m_run[q];
                    part_ml[pidx * 2 + 1] = l;
                }
            }
        }
        if (!more) break;
        item = next_item;
        ++round;
        cur = nxt;
        g_cur = g_nxt;
#pragma unroll
        for (int q = 0; q < NQG; ++q) {
            nk_cur[q] = nk_nxt[q];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) qb[q][ks] = qn[q][ks];
        }
    }
#undef DYN_ATTN_LOAD
#undef DYN_ATTN_LOAD_Q
#undef DYN_ATTN_COMPUTE
}

hipError_t launch_attention_generic(int dtype, const void *qkv, const int32_t *seq_of_token,
                                    const int32_t *pos_of_token, const int32_t *block_table, const void *k_cache,
                                    const void *v_cache, void *out, int ld_out, float *part_o, float *part_ml,
                                    const AttnShape &sh, int rows, hipStream_t s, hipEvent_t mid);

bool attention_mfma_supported(int dtype, const AttnShape &sh) {
    return dtype == 1 && sh.head_dim == HD && sh.page_size == PS && sh.n_q % sh.n_kv == 0 && sh.n_q / sh.n_kv <= 16;
}

hipError_t launch_attention(int dtype, const void *qkv, const int32_t *seq_of_token, const int32_t *pos_of_token,
                            const int32_t *block_table, const void *k_cache, const void *v_cache, void *out, int ld_out,
                            float *part_o, float *part_ml, int32_t *plan, bool any_multi, const AttnShape &sh, int rows,
                            hipStream_t s, hipEvent_t mid, hipEvent_t pre, bool plan_ready) {
    if (rows <= 0) return hipSuccess;
    if (!attention_mfma_supported(dtype, sh))
        return launch_attention_generic(dtype, qkv, seq_of_token, pos_of_token, block_table, k_cache, v_cache, out, ld_out,
                                        part_o, part_ml, sh, rows, s, mid);
    // two work lists per dispatch: single-token sequences, multi-token sequences
    int32_t *plan0 = plan, *plan1 = plan + 2 + 2 * (size_t)rows * sh.max_chunks;
    int32_t *ct_of_token = plan + 4 + 4 * (size_t)rows * sh.max_chunks;
    // The lists depend on the rows' sequences and positions only: the first layer of a forward
    // builds them, the others walk them again (plan_ready).
    if (!plan_ready)
        hipLaunchKernelGGL(attn_plan_kernel, dim3(1), dim3(1024), 0, s, seq_of_token, pos_of_token, rows, sh.chunk_pages * PS,
                           attn_prefill_block_tokens(sh), plan0, plan1, ct_of_token);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && pre) e = hipEventRecord(pre, s);
    if (e != hipSuccess) return e;
    const long max_items = (long)rows * sh.n_kv * sh.max_chunks;
    // every workgroup of a persistent launch has to be resident at once (the work is dealt out by
    // wave index): two per CU of the partition the stream runs on
    const int groups = sh.n_cus > 0 && 2 * sh.n_cus < kPersistentGroups ? 2 * sh.n_cus : kPersistentGroups;
    const int grid = (int)((max_items + 3) / 4 < groups ? (max_items + 3) / 4 : groups);
    hipLaunchKernelGGL(attn_mfma_kernel<1>, dim3(grid), dim3(256), 0, s, (const bf16_t *)qkv, seq_of_token,
                       pos_of_token, block_table, (const bf16_t *)k_cache, (const bf16_t *)v_cache, part_o, part_ml, sh,
                       plan0);
    e = hipGetLastError();
    if (e == hipSuccess && any_multi)
        e = launch_attention_prefill(qkv, seq_of_token, pos_of_token, block_table, k_cache, v_cache, part_o, part_ml, sh,
                                     plan1, max_items, groups, s);
    if (e == hipSuccess && mid) e = hipEventRecord(mid, s);
    if (e != hipSuccess) return e;
    return launch_attention_combine(dtype, true, part_o, part_ml, pos_of_token, ct_of_token, out, ld_out, sh, rows, s, plan1 + 1);
}

}  // namespace dyn

// Causal paged attention for the tokens of multi-token sequences (prefill chunks): the
// compute-bound form of the layer's attention (the paper's compute-bound operator class,
// Section 2), bf16 caches, head_dim 128, 16-position pages.
//
// An 8-wave workgroup serves one query block - up to 8 * 8 tokens of one sequence whose
// positions fall in one aligned block - against one chunk of cached positions (1024, more behind
// a long prefix: prefill_chunk_positions) of one kv head.  K and V tiles of 32 positions (two pages, 16 KB) go from global memory
// straight into an LDS ring with direct loads, once per workgroup, and all eight waves read
// their MFMA operands from there: a key is fetched once per 64 query tokens and q-head
// group, and the waves hold no K/V staging registers.  A wave owns two sets of 16 columns
// (64 accumulator registers): everything fits the 256 vector registers of a wave at two
// waves per SIMD, so one wave's softmax overlaps another's matrix products and no operand
// ever sits in an accumulation register it has to be copied out of.
//   S[32 pos, 32 cols]  = K_tile[32, 128] Q^T[128, 32]       (16 x mfma 16x16x32 per wave)
//   O^T[128, 32 cols]  += V_tile^T[128, 32] P[32, 32]        (16 x mfma 16x16x32 per wave)
// A column is (token, q head of the kv head's group); the D layout of the first product
// (lane: column l % 16, positions 4 (l / 16) + r of a page) is the B layout of the second
// with the k index running over (page 0: 4 positions, page 1: 4 positions), and V's
// position-fastest page layout makes the matching A operand two 8-byte LDS reads.
// K rows are 256 bytes, so their 16-byte columns are XOR-swizzled with the row on the way in
// (the direct load's source address is permuted, its LDS destination cannot be).
// Online softmax in the exp2 domain; the chunk's partial (m, l, o) goes to the split-KV
// arrays and attn_combine_kernel merges a token's chunks in order.
#include "common.h"
#include "kernels.h"

namespace dyn {

namespace {

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

constexpr int HD = 128, PS = 16;
constexpr int kSets = 2;                      // sets of 16 MFMA columns per wave
constexpr int kWaves = 8;                     // waves per workgroup
constexpr int kTP = 4;                         // pages (16 positions each) per K/V tile
constexpr int kRing = 3, kTile = 2 * kTP * 4096;   // LDS ring of K/V tiles: kTP K pages, then kTP V pages, 4 KB each

__device__ __forceinline__ void wait_vm(int n) {   // s_waitcnt vmcnt(n) only
    if (n == 4) __builtin_amdgcn_s_waitcnt(0x0f74);
    else __builtin_amdgcn_s_waitcnt(0x0f70);
}

}  // namespace

__global__ __launch_bounds__(kWaves * 64, 1) void attn_prefill_kernel(const bf16_t *__restrict__ qkv,
                                                              const int32_t *__restrict__ seq_of_token,
                                                              const int32_t *__restrict__ pos_of_token,
                                                              const int32_t *__restrict__ block_table,
                                                              const bf16_t *__restrict__ k_cache,
                                                              const bf16_t *__restrict__ v_cache,
                                                              float *__restrict__ part_o, float *__restrict__ part_ml,
                                                              AttnShape sh, const int32_t *__restrict__ plan, int32_t *__restrict__ counter) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    int32_t *pid = reinterpret_cast<int32_t *>(lds + kRing * kTile);      // physical pages of the chunk
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lr = lane & 15, lq = lane >> 4;
    const int G = sh.n_q / sh.n_kv, TG = 16 / G;                         // tokens per set of 16 columns
    const int col_tok = lr / G, col_head = lr % G;
    const int wave_tok0 = wave * kSets * TG;                             // first token of the block this wave owns
    const float sscale = 1.4426950408889634f / sqrtf((float)HD);
    const int n_items = plan[0] * sh.n_kv;
    const size_t row_elems = (size_t)(sh.n_q + 2 * sh.n_kv) * HD;

    // Work items are claimed from a counter in the list's header (zeroed by the work-list kernel),
    // longest first: the list is in token order, a block's keys grow with its position, so it is
    // walked from the back.  A few hundred claims per launch; which workgroup computes an item
    // does not touch its result.
    int32_t *claim = reinterpret_cast<int32_t *>(lds + kRing * kTile) + kPrefillChunkPagesMax;
    for (;;) {
        __builtin_amdgcn_s_waitcnt(0x0f70);                               // the previous item's stores and trailing tile loads
        __syncthreads();                                                  // everyone has read the previous claim and left the ring
        if (tid == 0) *claim = atomicAdd(counter, 1);
        __syncthreads();
        const int taken = *claim;
        if (taken >= n_items) break;
        const int item = n_items - 1 - taken;
        const int g = item % sh.n_kv, e = item / sh.n_kv;
        const int t0 = plan[2 + 2 * e], packed = plan[3 + 2 * e];
        const int c = packed & 0xfffff, n_tok = packed >> 20;
        const int n_keys = pos_of_token[t0 + n_tok - 1] + 1;             // keys the block's last token attends
        const int seq_pages = (n_keys + PS - 1) / PS;
        const int block_tokens = kWaves * kSets * TG;                     // the aligned position block this item's tokens share
        const int chunk_pages = prefill_chunk_positions((pos_of_token[t0] / block_tokens + 1) * block_tokens) / PS;
        const int lp0 = c * chunk_pages;
        const int n_pg = min(chunk_pages, seq_pages - lp0);
        const int n_tile = (n_pg + kTP - 1) / kTP;
        const int32_t *bt = block_table + (size_t)seq_of_token[t0] * sh.max_pages_per_seq;

        if (tid < chunk_pages) pid[tid] = bt[lp0 + min(tid, n_pg - 1)];

        // this wave's columns: B operands of the score product and the keys each column attends
        bf16x8 qb[kSets][4];
        int nk[kSets];
#pragma unroll
        for (int q = 0; q < kSets; ++q) {
            const int ti = wave_tok0 + q * TG + col_tok;
            const bool live = col_tok < TG && ti < n_tok;
            const int tq = t0 + (live ? ti : 0);
            nk[q] = live ? pos_of_token[tq] + 1 : 0;
            const bf16_t *qp = qkv + (size_t)tq * row_elems + (size_t)(g * G + col_head) * HD + 8 * lq;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                u32x4 v = *reinterpret_cast<const u32x4 *>(qp + ks * 32);
                if (!live) v = u32x4{0u, 0u, 0u, 0u};
                qb[q][ks] = __builtin_bit_cast(bf16x8, v);
            }
        }
        // keys the wave's last live token attends (positions are consecutive within the block)
        const int wave_keys = wave_tok0 < n_tok ? pos_of_token[t0 + min(wave_tok0 + kSets * TG, n_tok) - 1] + 1 : 0;
        // keys its first token attends; columns of dead tokens or heads carry zeros and are never stored
        const int wave_min_keys = wave_tok0 < n_tok ? pos_of_token[t0 + wave_tok0] + 1 : 0;
        __syncthreads();                                                  // pid is visible

        // Wave w copies one 4 KB page of every tile: K pages 0..3 (waves 0..3), V pages 0..3 (waves 4..7).
        const int wpage = wave & (kTP - 1), is_v = wave / kTP;
        auto issue = [&](int tile) {
            const int tcl = min(tile, n_tile - 1);                        // past the end: a harmless reload
            const int pg = pid[min(kTP * tcl + wpage, n_pg - 1)];
            unsigned char *dst = lds + (tile % kRing) * kTile + is_v * (kTP * 4096) + wpage * 4096;
            const size_t page_elems = ((size_t)pg * sh.n_kv + g) * (PS * HD);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bf16_t *src;
                if (is_v) {
                    const int r = j * 32 + (lane >> 1), h = lane & 1;     // V row (head-dim index), 16-byte half in LDS
                    src = v_cache + page_elems + r * PS + ((h ^ ((r >> 2) & 1)) << 3);
                } else {
                    const int r = j * 4 + (lane >> 4), cs = lane & 15;    // K row, 16-byte slot in LDS
                    src = k_cache + page_elems + r * HD + ((cs ^ (r & 7)) << 3);
                }
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                                 (__attribute__((address_space(3))) void *)(dst + j * 1024), 16, 0, 0);
            }
        };

        f32x4 acc[kSets][8], acc_l[kSets];   // O^T tiles; row sums of P (every row of acc_l holds the column's denominator)
        float m_run[kSets];                  // the reference maximum the column's exponentials are taken against (scaled, log2 domain)
#pragma unroll
        for (int q = 0; q < kSets; ++q) {
            m_run[q] = -INFINITY;
            acc_l[q] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) acc[q][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        const bf16x8 ones = __builtin_bit_cast(bf16x8, u32x4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u});
        // V operand: 8 bytes (4 positions) of a 32-byte row.  The row's 16-byte halves are stored
        // swapped when bit 2 of the row is set, which spreads the 16 rows a read touches over
        // twice as many banks as the plain layout.
        const int v_off = lr * 32 + ((((lq >> 1) ^ (lr >> 2)) & 1) << 4) + ((lq & 1) << 3);

        // Operand reads from the ring are assembly with hand-placed waits (common.h): a page's K operands are
        // read while the previous page's score products issue, a V operand group while the previous group's
        // value products issue.  The K operand of k
        // step ks sits in 16-byte column (4 ks + lq) ^ (lr & 7) of row lr: two lane addresses (bit 2 of
        // the column is ks & 1 flipped by bit 2 of the row) and an immediate of 0 or 128 bytes.
        const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds;
        const unsigned k_lane0 = lr * 256 + (((lq ^ (lr & 3)) + 4 * ((lr >> 2) & 1)) << 4);
        const unsigned k_lane1 = lr * 256 + (((lq ^ (lr & 3)) + 4 * (((lr >> 2) & 1) ^ 1)) << 4);

        issue(0);
        issue(1);
        for (int ti = 0; ti < n_tile; ++ti) {
            wait_vm(4);                                                   // tile ti has landed (tile ti + 1 may be in flight)
            __builtin_amdgcn_s_barrier();                                 // everyone's part of it, and everyone is done with tile ti - 1
            issue(ti + 2);
            const int key0 = (lp0 + kTP * ti) * PS;
            if (key0 >= wave_keys) continue;                              // wave-uniform: nothing of this tile is visible to the wave
            const unsigned char *kb = lds + (ti % kRing) * kTile, *vb = kb + kTP * 4096;

            const unsigned tb = lds0 + (unsigned)(ti % kRing) * kTile;
            const unsigned ka0 = tb + k_lane0, ka1 = tb + k_lane1, va = tb + kTP * 4096 + (unsigned)v_off;
            auto read_k = [&](bf16x8 (&kf)[4], auto pi) {
                constexpr int OFF = decltype(pi)::value * 4096;
                kf[0] = lds_read16<OFF>(ka0);
                kf[1] = lds_read16<OFF>(ka1);
                kf[2] = lds_read16<OFF + 128>(ka0);
                kf[3] = lds_read16<OFF + 128>(ka1);
            };
            f32x4 sv[kSets][kTP];                                         // raw scores q . k
            bf16x8 kf[2][4];
            read_k(kf[0], std::integral_constant<int, 0>());
            static_for<0, kTP>([&](auto pi_c) {
                constexpr int pi = decltype(pi_c)::value;
                if constexpr (pi + 1 < kTP) {
                    read_k(kf[(pi + 1) & 1], std::integral_constant<int, pi + 1>());
                    wait_lgkmcnt<4>();                                    // page pi's four operands have arrived
                } else {
                    wait_lgkmcnt<0>();
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = 0; q < kSets; ++q) {
                    f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks) s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[pi & 1][ks], qb[q][ks], s, 0, 0, 0);
                    sv[q][pi] = s;
                }
                __builtin_amdgcn_sched_barrier(0);
            });
            __builtin_amdgcn_sched_barrier(0);
            // Causal mask: only the last tiles of a block have positions that some live column of
            // the wave must not see (wave-uniform test).
            if (key0 + kTP * PS > wave_min_keys) {
#pragma unroll
                for (int q = 0; q < kSets; ++q)
#pragma unroll
                    for (int pi = 0; pi < kTP; ++pi)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            if (key0 + pi * PS + 4 * lq + r >= nk[q]) sv[q][pi][r] = -INFINITY;
            }
            bf16x8 pb[kSets][kTP / 2];                                    // probabilities: one k = 32 operand per pair of pages
            bool rescale = false;
            float alpha[kSets];
#pragma unroll
            for (int q = 0; q < kSets; ++q) {
                float mx = -INFINITY;
#pragma unroll
                for (int pi = 0; pi < kTP; ++pi)
                    mx = fmaxf(mx, fmaxf(fmaxf(sv[q][pi][0], sv[q][pi][1]), fmaxf(sv[q][pi][2], sv[q][pi][3])));
                mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
                mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
                mx *= sscale;
                // The reference maximum follows the true one lazily: it moves only when a score
                // exceeds it by more than 2^8, so exponentials stay below 256 (exact in what
                // follows: the final division by the denominator cancels the reference) and the
                // accumulators are rescaled a few times per block instead of on every tile.
                const bool move = mx > m_run[q] + 8.0f;
                const float m_new = move ? mx : m_run[q];
                const float m_ref = m_new == -INFINITY ? 0.f : m_new;    // a column with no key yet stays empty
                alpha[q] = move ? __builtin_amdgcn_exp2f(m_run[q] - m_ref) : 1.0f;
                rescale |= move;
                m_run[q] = m_new;
#pragma unroll
                for (int pp = 0; pp < kTP / 2; ++pp) {
                    f32x4 p0, p1;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        p0[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[q][2 * pp][r], sscale, -m_ref));
                        p1[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[q][2 * pp + 1][r], sscale, -m_ref));
                    }
                    const u32x2 w0 = __builtin_bit_cast(u32x2, __builtin_convertvector(p0, bf16x4));
                    const u32x2 w1 = __builtin_bit_cast(u32x2, __builtin_convertvector(p1, bf16x4));
                    pb[q][pp] = __builtin_bit_cast(bf16x8, u32x4{w0[0], w0[1], w1[0], w1[1]});
                }
            }
            if (__any(rescale)) {
#pragma unroll
                for (int q = 0; q < kSets; ++q) {
                    acc_l[q] *= alpha[q];
#pragma unroll
                    for (int dt = 0; dt < 8; ++dt) acc[q][dt] *= alpha[q];
                }
            }
            // V operands of output rows 16 dt .. 16 dt + 15, one 8-byte read per page; group 0 is in flight
            // during the denominator's products and the mask arithmetic below
            u32x2 vx[2][kTP];
            auto read_v = [&](u32x2 (&x)[kTP], auto dt_c) {
                static_for<0, kTP>([&](auto pi_c) {
                    x[decltype(pi_c)::value] = lds_read8<decltype(pi_c)::value * 4096 + decltype(dt_c)::value * 512>(va);
                });
            };
            read_v(vx[0], std::integral_constant<int, 0>());
            // the denominator sums the probabilities exactly as the value product sees them (rounded
            // to bf16): one more matrix product, against a block of ones
#pragma unroll
            for (int pp = 0; pp < kTP / 2; ++pp)
#pragma unroll
                for (int q = 0; q < kSets; ++q) acc_l[q] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb[q][pp], acc_l[q], 0, 0, 0);
            // positions past the block's last key (in the chunk's last tile) hold stale cache bits,
            // which must not meet their zero probabilities (0 * NaN): masked out of V
            uint32_t vm[kTP][2];
#pragma unroll
            for (int pi = 0; pi < kTP; ++pi) {
                const int nv = n_keys - key0 - pi * PS - 4 * lq;
                vm[pi][0] = (nv > 0 ? 0x0000ffffu : 0u) | (nv > 1 ? 0xffff0000u : 0u);
                vm[pi][1] = (nv > 2 ? 0x0000ffffu : 0u) | (nv > 3 ? 0xffff0000u : 0u);
            }
            __builtin_amdgcn_sched_barrier(0);
            static_for<0, 8>([&](auto dt_c) {
                constexpr int dt = decltype(dt_c)::value;
                if constexpr (dt + 1 < 8) {
                    read_v(vx[(dt + 1) & 1], std::integral_constant<int, dt + 1>());
                    wait_lgkmcnt<kTP>();                                  // group dt has arrived
                } else {
                    wait_lgkmcnt<0>();
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int pp = 0; pp < kTP / 2; ++pp) {
                    const u32x2 x0 = vx[dt & 1][2 * pp], x1 = vx[dt & 1][2 * pp + 1];
                    const bf16x8 vf = __builtin_bit_cast(bf16x8, u32x4{x0[0] & vm[2 * pp][0], x0[1] & vm[2 * pp][1],
                                                                       x1[0] & vm[2 * pp + 1][0], x1[1] & vm[2 * pp + 1][1]});
#pragma unroll
                    for (int q = 0; q < kSets; ++q)
                        acc[q][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pb[q][pp], acc[q][dt], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            });
        }

#pragma unroll
        for (int q = 0; q < kSets; ++q) {
            if (nk[q] > lp0 * PS) {                                       // the chunk exists for this column's token
                const size_t pidx =
                    ((size_t)(t0 + wave_tok0 + q * TG + col_tok) * sh.n_q + g * G + col_head) * sh.max_chunks + c;
#pragma unroll
                for (int dt = 0; dt < 8; ++dt)
                    *reinterpret_cast<f32x4 *>(part_o + pidx * HD + dt * 16 + 4 * lq) = acc[q][dt];
                if (lq == 0) {
                    part_ml[pidx * 2] = m_run[q];
                    part_ml[pidx * 2 + 1] = acc_l[q][0];
                }
            }
        }
    }
}

int attn_prefill_block_tokens(const AttnShape &sh) { return kWaves * kSets * (16 / (sh.n_q / sh.n_kv)); }

hipError_t launch_attention_prefill(const void *qkv, const int32_t *seq_of_token, const int32_t *pos_of_token,
                                    const int32_t *block_table, const void *k_cache, const void *v_cache, float *part_o,
                                    float *part_ml, const AttnShape &sh, int32_t *plan, long max_items, int max_groups,
                                    hipStream_t s) {
    static_assert(kPrefillChunkPagesMax <= kWaves * 64, "one thread per page id of a chunk");
    const int lds_bytes = kRing * kTile + (kPrefillChunkPagesMax + 4) * (int)sizeof(int32_t);   // ring, page ids of a chunk, the claimed item
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)attn_prefill_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int grid = (int)(max_items < max_groups ? max_items : max_groups);
    hipLaunchKernelGGL(attn_prefill_kernel, dim3(grid), dim3(kWaves * 64), lds_bytes, s, (const bf16_t *)qkv, seq_of_token,
                       pos_of_token, block_table, (const bf16_t *)k_cache, (const bf16_t *)v_cache, part_o, part_ml, sh, plan,
                       plan + 1);
    return hipGetLastError();
}

}  // namespace dyn

// Paged causal attention for bf16 caches, head_dim 128, 16-position pages: the layer's
// HBM-bound operator (the paper's memory-bound "decode attention", Section 2).
//
// One wave owns one (token, kv head, chunk of pages) and serves every q head of that kv
// head's group at once, so K and V are fetched once per kv head.  A page of K is 16 rows
// of 256 bytes, a page of V is 128 rows (one per head-dim index) of 32 bytes; both are
// loaded straight into MFMA operand layout with fully used 64-byte / 32-byte row segments,
// no LDS.  The group's scores are a skinny but real contraction
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

hipError_t launch_attention_combine(int dtype, bool base2, const float *part_o, const float *part_ml,
                                    const int32_t *pos_of_token, void *out, int ld_out, const AttnShape &sh, int rows,
                                    hipStream_t s);

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

constexpr int HD = 128, PS = 16, TILE_PAGES = 2;
constexpr int kPersistentGroups = 256;   // one 8-wave workgroup for each of the 256 CUs

// Work list: one entry per (token, chunk) that really exists, built on the device from the
// positions (contexts differ by 8x inside a batch, so a dense token x max_chunks grid would
// be mostly empty workgroups).  plan[0] = number of entries, entry i at plan[2 + 2 i].
__global__ __launch_bounds__(256) void attn_plan_kernel(const int32_t *__restrict__ pos_of_token, int rows, int ct,
                                                        int32_t *__restrict__ plan) {
    __shared__ int scan[256];
    __shared__ int base;
    if (threadIdx.x == 0) base = 0;
    __syncthreads();
    for (int t0 = 0; t0 < rows; t0 += 256) {
        const int t = t0 + threadIdx.x;
        const int nc = t < rows ? (pos_of_token[t] + ct) / ct : 0;
        scan[threadIdx.x] = nc;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {           // inclusive Hillis-Steele scan
            const int v = threadIdx.x >= off ? scan[threadIdx.x - off] : 0;
            __syncthreads();
            scan[threadIdx.x] += v;
            __syncthreads();
        }
        const int start = base + scan[threadIdx.x] - nc;
        for (int c = 0; c < nc; ++c) {
            plan[2 + 2 * (start + c)] = t;
            plan[3 + 2 * (start + c)] = c;
        }
        __syncthreads();
        if (threadIdx.x == 255) base += scan[255];
        __syncthreads();
    }
    if (threadIdx.x == 0) plan[0] = base;
}

// Persistent workgroups of 8 waves, one per CU.  Workgroup b owns the (entry, kv head) pairs
// b, b + gridDim.x, ...; its waves take them from an LDS counter as they become free, which
// evens out the ragged last chunks.  Which wave computes a pair has no influence on its
// result.
__global__ __launch_bounds__(512, 1) void attn_mfma_kernel(const bf16_t *__restrict__ qkv,
                                                           const int32_t *__restrict__ seq_of_token,
                                                           const int32_t *__restrict__ pos_of_token,
                                                           const int32_t *__restrict__ block_table,
                                                           const bf16_t *__restrict__ k_cache,
                                                           const bf16_t *__restrict__ v_cache,
                                                           float *__restrict__ part_o, float *__restrict__ part_ml,
                                                           AttnShape sh, const int32_t *__restrict__ plan) {
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_items = plan[0] * sh.n_kv;
    const int ct = sh.chunk_pages * PS;
    const int G = sh.n_q / sh.n_kv;
    const int lane = threadIdx.x & 63, lr = lane & 15, lq = lane >> 4;
    const float sscale = 1.4426950408889634f / sqrtf((float)HD);   // log2(e) / sqrt(d)
    (void)wave;
    __shared__ int next_slot;
    if (threadIdx.x == 0) next_slot = 0;
    __syncthreads();
    auto claim = [&]() {
        int v = 0;
        if (lane == 0) v = atomicAdd(&next_slot, 1);
        return blockIdx.x + __builtin_amdgcn_readfirstlane(v) * gridDim.x;
    };
    int item = claim();
  while (item < n_items) {
    const int g = item % sh.n_kv;
    const int t = plan[2 + 2 * (item / sh.n_kv)], c = plan[3 + 2 * (item / sh.n_kv)];
    const int n_keys = pos_of_token[t] + 1;
    const int j0 = c * ct;
    const int seq_pages = (n_keys + PS - 1) / PS;                 // pages this token may read
    const int lp0 = c * sh.chunk_pages;                           // first logical page of the chunk
    const int n_pg = min(sh.chunk_pages, seq_pages - lp0);
    const int n_tiles = (n_pg + TILE_PAGES - 1) / TILE_PAGES;
    const int32_t *bt = block_table + (size_t)seq_of_token[t] * sh.max_pages_per_seq;

    // B operands of the score product: q of head g*G + lr (zero for lr >= G)
    bf16x8 qb[4];
    {
        const bf16_t *q = qkv + (size_t)t * ((sh.n_q + 2 * sh.n_kv) * HD) + (g * G + min(lr, G - 1)) * HD + 8 * lq;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            u32x4 v = *reinterpret_cast<const u32x4 *>(q + ks * 32);
            if (lr >= G) v = u32x4{0u, 0u, 0u, 0u};
            qb[ks] = __builtin_bit_cast(bf16x8, v);
        }
    }

    u32x4 kreg[2][TILE_PAGES][4];
    u32x2 vreg[2][TILE_PAGES][8];
    f32x4 acc[8];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m_run = -INFINITY, l_run = 0.f;

#define DYN_ATTN_LOAD(B, TL)                                                                                      \
    {                                                                                                             \
        _Pragma("unroll") for (int pi = 0; pi < TILE_PAGES; ++pi) {                                               \
            const int lp = min(lp0 + (TL) * TILE_PAGES + pi, seq_pages - 1);                                      \
            const size_t pg = (size_t)bt[lp] * sh.n_kv + g;                                                       \
            const bf16_t *kp = k_cache + (pg * PS + lr) * HD + 8 * lq;                                            \
            const bf16_t *vp = v_cache + (pg * HD + lr) * PS + 4 * lq;                                            \
            _Pragma("unroll") for (int ks = 0; ks < 4; ++ks)                                                      \
                kreg[B][pi][ks] = *reinterpret_cast<const u32x4 *>(kp + ks * 32);                                 \
            _Pragma("unroll") for (int dt = 0; dt < 8; ++dt)                                                      \
                vreg[B][pi][dt] = *reinterpret_cast<const u32x2 *>(vp + dt * 16 * PS);                            \
        }                                                                                                         \
    }

#define DYN_ATTN_COMPUTE(B, TL)                                                                                   \
    {                                                                                                             \
        f32x4 sv[TILE_PAGES];                                                                                     \
        float mx = -INFINITY;                                                                                     \
        _Pragma("unroll") for (int pi = 0; pi < TILE_PAGES; ++pi) {                                               \
            f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f};                                                                  \
            _Pragma("unroll") for (int ks = 0; ks < 4; ++ks)                                                      \
                s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kreg[B][pi][ks]), qb[ks],  \
                                                            s, 0, 0, 0);                                          \
            const int jb = j0 + ((TL) * TILE_PAGES + pi) * PS + 4 * lq;                                           \
            _Pragma("unroll") for (int r = 0; r < 4; ++r) {                                                       \
                s[r] = (jb + r < n_keys) ? s[r] * sscale : -INFINITY;                                             \
                mx = fmaxf(mx, s[r]);                                                                             \
            }                                                                                                     \
            sv[pi] = s;                                                                                           \
        }                                                                                                         \
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));                                                                   \
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));                                                                   \
        const float m_new = fmaxf(m_run, mx);                                                                     \
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);                                                \
        m_run = m_new;                                                                                            \
        l_run *= alpha;                                                                                           \
        _Pragma("unroll") for (int dt = 0; dt < 8; ++dt) acc[dt] *= alpha;                                        \
        _Pragma("unroll") for (int pi = 0; pi < TILE_PAGES; ++pi) {                                               \
            f32x4 p;                                                                                              \
            _Pragma("unroll") for (int r = 0; r < 4; ++r) p[r] = __builtin_amdgcn_exp2f(sv[pi][r] - m_new);       \
            const bf16x4 pb = __builtin_convertvector(p, bf16x4);                                                 \
            const u32x2 pw = __builtin_bit_cast(u32x2, pb);                                                       \
            l_run += (__uint_as_float(pw[0] << 16) + __uint_as_float(pw[0] & 0xffff0000u)) +                      \
                     (__uint_as_float(pw[1] << 16) + __uint_as_float(pw[1] & 0xffff0000u));                       \
            const int nvalid = n_keys - (j0 + ((TL) * TILE_PAGES + pi) * PS) - 4 * lq;                            \
            _Pragma("unroll") for (int dt = 0; dt < 8; ++dt) {                                                    \
                u32x2 vv = vreg[B][pi][dt];                                                                       \
                if (nvalid < 4) { /* positions past the token's own: keep stale cache bits out of 0 * x */      \
                    vv[0] &= (nvalid > 0 ? 0x0000ffffu : 0u) | (nvalid > 1 ? 0xffff0000u : 0u);                   \
                    vv[1] &= (nvalid > 2 ? 0x0000ffffu : 0u);                                                     \
                }                                                                                                 \
                acc[dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, vv),                \
                                                                    __builtin_bit_cast(s16x4, pb), acc[dt], 0, 0, 0); \
            }                                                                                                     \
        }                                                                                                         \
    }

    // Two register buffers; the steady-state loop has no conditional loads, so the compiler
    // counts the loads still in flight exactly and a tile is multiplied while the next one
    // is on its way.
    DYN_ATTN_LOAD(0, 0)
    int tl = 0;
    for (; tl + 2 < n_tiles; tl += 2) {
        // scheduling barriers: keep each prefetch ahead of the multiply it overlaps
        DYN_ATTN_LOAD(1, tl + 1)
        __builtin_amdgcn_sched_barrier(0);
        DYN_ATTN_COMPUTE(0, tl)
        __builtin_amdgcn_sched_barrier(0);
        DYN_ATTN_LOAD(0, tl + 2)
        __builtin_amdgcn_sched_barrier(0);
        DYN_ATTN_COMPUTE(1, tl + 1)
        __builtin_amdgcn_sched_barrier(0);
    }
    if (tl + 2 == n_tiles) {
        DYN_ATTN_LOAD(1, tl + 1)
        __builtin_amdgcn_sched_barrier(0);
        DYN_ATTN_COMPUTE(0, tl)
        DYN_ATTN_COMPUTE(1, tl + 1)
    } else {
        DYN_ATTN_COMPUTE(0, tl)
    }
#undef DYN_ATTN_LOAD
#undef DYN_ATTN_COMPUTE

    l_run += __shfl_xor(l_run, 16, 64);
    l_run += __shfl_xor(l_run, 32, 64);
    if (lr < G) {
        const size_t pidx = ((size_t)t * sh.n_q + g * G + lr) * sh.max_chunks + c;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt)
            *reinterpret_cast<f32x4 *>(part_o + pidx * HD + dt * 16 + 4 * lq) = acc[dt];
        if (lq == 0) {
            part_ml[pidx * 2] = m_run;
            part_ml[pidx * 2 + 1] = l_run;
        }
    }
    item = claim();
  }   // item loop
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
                            float *part_o, float *part_ml, int32_t *plan, const AttnShape &sh, int rows,
                            hipStream_t s, hipEvent_t mid, hipEvent_t pre) {
    if (rows <= 0) return hipSuccess;
    if (!attention_mfma_supported(dtype, sh))
        return launch_attention_generic(dtype, qkv, seq_of_token, pos_of_token, block_table, k_cache, v_cache, out, ld_out,
                                        part_o, part_ml, sh, rows, s, mid);
    hipLaunchKernelGGL(attn_plan_kernel, dim3(1), dim3(256), 0, s, pos_of_token, rows, sh.chunk_pages * PS, plan);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && pre) e = hipEventRecord(pre, s);
    if (e != hipSuccess) return e;
    const long max_items = (long)rows * sh.n_kv * sh.max_chunks;
    const int grid = (int)((max_items + 7) / 8 < kPersistentGroups ? (max_items + 7) / 8 : kPersistentGroups);
    hipLaunchKernelGGL(attn_mfma_kernel, dim3(grid), dim3(512), 0, s, (const bf16_t *)qkv, seq_of_token,
                       pos_of_token, block_table, (const bf16_t *)k_cache, (const bf16_t *)v_cache, part_o, part_ml, sh,
                       plan);
    e = hipGetLastError();
    if (e == hipSuccess && mid) e = hipEventRecord(mid, s);
    if (e != hipSuccess) return e;
    return launch_attention_combine(dtype, true, part_o, part_ml, pos_of_token, out, ld_out, sh, rows, s);
}

}  // namespace dyn

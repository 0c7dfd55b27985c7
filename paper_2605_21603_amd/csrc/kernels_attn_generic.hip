// Paged causal attention, generic path (fp32 storage, or any shape the MFMA kernel does not
// take), and the split-KV combine step shared by both attention kernels.
//
// A token attends cached positions 0..pos of its sequence.  The key range is cut into
// chunks of a fixed number of pages; one wave handles one (token, q head, chunk) and writes
// an un-normalised partial (running max m, sum l, weighted values o).  The combine kernel
// merges a token's partials in chunk order.  Chunk size is a constant of the layer, so the
// arithmetic a row sees does not depend on the batch around it.
#include "common.h"
#include "kernels.h"

namespace dyn {

constexpr int kMaxChunkTokens = 512;

template <typename T>
__global__ __launch_bounds__(64) void attn_generic_kernel(const T *__restrict__ qkv,
                                                          const int32_t *__restrict__ seq_of_token,
                                                          const int32_t *__restrict__ pos_of_token,
                                                          const int32_t *__restrict__ block_table,
                                                          const T *__restrict__ k_cache, const T *__restrict__ v_cache,
                                                          float *__restrict__ part_o, float *__restrict__ part_ml,
                                                          AttnShape sh) {
    const int c = blockIdx.x % sh.max_chunks;
    const int h = (blockIdx.x / sh.max_chunks) % sh.n_q;
    const int t = blockIdx.x / (sh.max_chunks * sh.n_q);
    const int d = sh.head_dim, ps = sh.page_size, ct = sh.chunk_pages * ps;
    const int n_keys = pos_of_token[t] + 1;
    const int j0 = c * ct;
    if (j0 >= n_keys) return;
    const int j1 = min(j0 + ct, n_keys);
    const int g = h / (sh.n_q / sh.n_kv);
    const int lane = threadIdx.x;
    const int32_t *bt = block_table + (size_t)seq_of_token[t] * sh.max_pages_per_seq;

    __shared__ float qs[2 * kMaxHalfDim];
    __shared__ float sc[kMaxChunkTokens];
    const T *q = qkv + (size_t)t * ((sh.n_q + 2 * sh.n_kv) * d) + h * d;
    for (int i = lane; i < d; i += 64) qs[i] = to_f32<T>(q[i]);
    __syncthreads();

    const float scale = 1.0f / sqrtf((float)d);
    float mx = -INFINITY;
    for (int j = j0 + lane; j < j1; j += 64) {
        const T *kr = k_cache + (((size_t)bt[j / ps] * sh.n_kv + g) * ps + j % ps) * d;
        float acc = 0.f;
        for (int i = 0; i < d; ++i) acc += qs[i] * to_f32<T>(kr[i]);
        acc *= scale;
        sc[j - j0] = acc;
        mx = fmaxf(mx, acc);
    }
    mx = wave_max(mx);
    float sum = 0.f;
    for (int j = j0 + lane; j < j1; j += 64) {
        const float p = expf(sc[j - j0] - mx);
        sc[j - j0] = p;
        sum += p;
    }
    sum = wave_sum(sum);
    __syncthreads();
    const size_t pidx = ((size_t)t * sh.n_q + h) * sh.max_chunks + c;
    for (int i = lane; i < d; i += 64) {
        float acc = 0.f;
        for (int j = j0; j < j1; ++j) {
            const T *vr = v_cache + (((size_t)bt[j / ps] * sh.n_kv + g) * d + i) * ps + j % ps;
            acc += sc[j - j0] * to_f32<T>(*vr);
        }
        part_o[pidx * d + i] = acc;
    }
    if (lane == 0) {
        part_ml[pidx * 2] = mx;
        part_ml[pidx * 2 + 1] = sum;
    }
}

// 32 lanes per (token, q head), 8 pairs per 256-thread workgroup; a lane owns 4 consecutive
// head-dim indices.  Partials are merged in chunk order: M = max m_c,
// out = sum_c e(m_c - M) o_c / sum_c e(m_c - M) l_c, where e is exp or exp2 according to the
// domain the producing kernel kept m in.
// A token with more than kMergeSegment chunks (contexts beyond 16384 positions in decode) is
// merged in two levels: first every segment of kMergeSegment chunks into one partial of the same
// (m, l, o) form, stored over the segment's first chunk, then the segments.  Which way a token goes
// depends on its own chunk count only, so its bits do not depend on the batch; the one-level merge
// of a 131072-position context was a 512-step chain on 32 lanes (126 us for one token).
constexpr int kMergeSegment = 64;

template <bool BASE2>
__global__ __launch_bounds__(256) void attn_combine_segments_kernel(float *__restrict__ part_o, float *__restrict__ part_ml,
                                                                    const int32_t *__restrict__ pos_of_token,
                                                                    const int32_t *__restrict__ ct_of_token, AttnShape sh,
                                                                    int n_pairs, int max_segments) {
    const int unit = blockIdx.x * 8 + (threadIdx.x >> 5), sub = threadIdx.x & 31;
    const int pair = unit / max_segments, seg = unit % max_segments;
    if (pair >= n_pairs) return;
    const int t = pair / sh.n_q;
    const int d = sh.head_dim, ct = ct_of_token ? ct_of_token[t] : sh.chunk_pages * sh.page_size;
    const int n_chunks = (pos_of_token[t] + ct) / ct;
    const int c0 = seg * kMergeSegment;
    if (n_chunks <= kMergeSegment || c0 >= n_chunks) return;
    const int n = min(kMergeSegment, n_chunks - c0);
    float *ml = part_ml + ((size_t)pair * sh.max_chunks + c0) * 2;
    float *po = part_o + ((size_t)pair * sh.max_chunks + c0) * d;
    float M = -INFINITY;
    for (int c = sub; c < n; c += 32) M = fmaxf(M, ml[c * 2]);
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1) M = fmaxf(M, __shfl_xor(M, off, 32));
    float L = 0.f;
    f32x4 acc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
    for (int cb = 0; cb < n; cb += 32) {
        const int c = cb + sub;
        float wgt = 0.f, wl = 0.f;
        if (c < n) {
            const float dm = ml[c * 2] - M;
            wgt = BASE2 ? exp2f(dm) : expf(dm);
            wl = wgt * ml[c * 2 + 1];
        }
#pragma unroll
        for (int off = 16; off >= 1; off >>= 1) wl += __shfl_xor(wl, off, 32);
        L += wl;
        const int nb = min(32, n - cb);
        for (int j0 = 0; j0 < nb; j0 += 4) {
            f32x4 v[4][2];
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int i = sub * 4 + q * 128;
                    v[j][q] = (j0 + j < nb && i < d) ? *reinterpret_cast<const f32x4 *>(po + (size_t)(cb + j0 + j) * d + i)
                                                      : f32x4{0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float wj = __shfl(wgt, j0 + j, 32);
#pragma unroll
                for (int q = 0; q < 2; ++q) acc[q] += v[j][q] * wj;
            }
        }
    }
    // every lane has read what it needs of the segment (its own four columns of each chunk, and
    // lane 0 the first chunk's (m, l)): the merged partial replaces the segment's first chunk
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int i = sub * 4 + q * 128;
        if (i < d) *reinterpret_cast<f32x4 *>(po + i) = acc[q];
    }
    if (sub == 0) { ml[0] = M; ml[1] = L; }
}

// Chunks whose partial outputs a half-wave has in flight at once in the final merge (the adds stay in chunk order).
constexpr int kMergeLoads = 8;

template <typename T, bool BASE2>
__global__ __launch_bounds__(256) void attn_combine_kernel(const float *__restrict__ part_o,
                                                           const float *__restrict__ part_ml,
                                                           const int32_t *__restrict__ pos_of_token,
                                                           const int32_t *__restrict__ ct_of_token,
                                                           T *__restrict__ out, int ld_out, AttnShape sh, int n_pairs,
                                                           int32_t *__restrict__ counter_reset) {
    // the query-block kernel that ran before this one has drained its work counter: zero it for the
    // next launch that walks the same work list (the next layer of the forward)
    if (counter_reset && blockIdx.x == 0 && threadIdx.x == 0) *counter_reset = 0;
    const int pair = blockIdx.x * 8 + (threadIdx.x >> 5), sub = threadIdx.x & 31;
    if (pair >= n_pairs) return;
    const int t = pair / sh.n_q;
    const int d = sh.head_dim, ct = ct_of_token ? ct_of_token[t] : sh.chunk_pages * sh.page_size;   // per-token chunk size if given
    const int all_chunks = (pos_of_token[t] + ct) / ct;     // ceil((pos + 1) / ct)
    // beyond kMergeSegment chunks the segments kernel has merged every segment into its first chunk
    const int step = all_chunks > kMergeSegment ? kMergeSegment : 1;
    const int n_chunks = (all_chunks + step - 1) / step;
    const float *ml = part_ml + (size_t)pair * sh.max_chunks * 2;
    const float *po = part_o + (size_t)pair * sh.max_chunks * d;
    float M = -INFINITY;
    for (int c = sub; c < n_chunks; c += 32) M = fmaxf(M, ml[c * step * 2]);
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1) M = fmaxf(M, __shfl_xor(M, off, 32));
    // Lane `sub` weighs chunk cb + sub; the weights travel by shuffle so that the value loads
    // of a block of chunks are independent of one another and can all be in flight together.
    float L = 0.f;
    f32x4 acc[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};   // head_dim <= 256: two float4 per lane
    for (int cb = 0; cb < n_chunks; cb += 32) {
        const int c = cb + sub;
        float wgt = 0.f, wl = 0.f;
        if (c < n_chunks) {
            const float dm = ml[c * step * 2] - M;
            wgt = BASE2 ? exp2f(dm) : expf(dm);
            wl = wgt * ml[c * step * 2 + 1];
        }
#pragma unroll
        for (int off = 16; off >= 1; off >>= 1) wl += __shfl_xor(wl, off, 32);
        L += wl;
        const int nb = min(32, n_chunks - cb);
        for (int j0 = 0; j0 < nb; j0 += kMergeLoads) {
            f32x4 v[kMergeLoads][2];
#pragma unroll
            for (int j = 0; j < kMergeLoads; ++j)
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int i = sub * 4 + q * 128;
                    v[j][q] = (j0 + j < nb && i < d) ? *reinterpret_cast<const f32x4 *>(po + (size_t)(cb + j0 + j) * step * d + i)
                                                      : f32x4{0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
            for (int j = 0; j < kMergeLoads; ++j) {
                const float wj = __shfl(wgt, j0 + j, 32);      // 0 beyond the last chunk
#pragma unroll
                for (int q = 0; q < 2; ++q) acc[q] += v[j][q] * wj;
            }
        }
    }
    const float inv = 1.0f / L;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int i = sub * 4 + q * 128;
        if (i < d) {
            T *o = out + (size_t)t * ld_out + (pair - t * sh.n_q) * d + i;
            if constexpr (sizeof(T) == 2) {            // one 8-byte store (rows and i are 8-byte aligned)
                u32x2 w;
                w[0] = (uint32_t)f2bf(acc[q][0] * inv) | ((uint32_t)f2bf(acc[q][1] * inv) << 16);
                w[1] = (uint32_t)f2bf(acc[q][2] * inv) | ((uint32_t)f2bf(acc[q][3] * inv) << 16);
                *reinterpret_cast<u32x2 *>(o) = w;
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) o[r] = from_f32<T>(acc[q][r] * inv);
            }
        }
    }
}

hipError_t launch_attention_combine(int dtype, bool base2, float *part_o, float *part_ml,
                                    const int32_t *pos_of_token, const int32_t *ct_of_token, void *out, int ld_out,
                                    const AttnShape &sh, int rows, hipStream_t s, int32_t *counter_reset) {
    const int n_pairs = rows * sh.n_q;
    const dim3 grid((n_pairs + 7) / 8), block(256);
    if (sh.max_chunks > kMergeSegment) {       // some token may have that many chunks: first level of the merge
        const int max_segments = (sh.max_chunks + kMergeSegment - 1) / kMergeSegment;
        const dim3 seg_grid((unsigned)(((size_t)n_pairs * max_segments + 7) / 8));
        if (base2) hipLaunchKernelGGL(attn_combine_segments_kernel<true>, seg_grid, block, 0, s, part_o, part_ml, pos_of_token, ct_of_token, sh, n_pairs, max_segments);
        else hipLaunchKernelGGL(attn_combine_segments_kernel<false>, seg_grid, block, 0, s, part_o, part_ml, pos_of_token, ct_of_token, sh, n_pairs, max_segments);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (dtype == 0) {
        if (base2) hipLaunchKernelGGL((attn_combine_kernel<float, true>), grid, block, 0, s, part_o, part_ml, pos_of_token, ct_of_token, (float *)out, ld_out, sh, n_pairs, counter_reset);
        else hipLaunchKernelGGL((attn_combine_kernel<float, false>), grid, block, 0, s, part_o, part_ml, pos_of_token, ct_of_token, (float *)out, ld_out, sh, n_pairs, counter_reset);
    } else {
        if (base2) hipLaunchKernelGGL((attn_combine_kernel<bf16_t, true>), grid, block, 0, s, part_o, part_ml, pos_of_token, ct_of_token, (bf16_t *)out, ld_out, sh, n_pairs, counter_reset);
        else hipLaunchKernelGGL((attn_combine_kernel<bf16_t, false>), grid, block, 0, s, part_o, part_ml, pos_of_token, ct_of_token, (bf16_t *)out, ld_out, sh, n_pairs, counter_reset);
    }
    return hipGetLastError();
}

hipError_t launch_attention_generic(int dtype, const void *qkv, const int32_t *seq_of_token,
                                    const int32_t *pos_of_token, const int32_t *block_table, const void *k_cache,
                                    const void *v_cache, void *out, int ld_out, float *part_o, float *part_ml,
                                    const AttnShape &sh, int rows, hipStream_t s, hipEvent_t mid) {
    if (rows <= 0) return hipSuccess;
    const dim3 grid((unsigned)((size_t)rows * sh.n_q * sh.max_chunks));
    if (dtype == 0)
        hipLaunchKernelGGL(attn_generic_kernel<float>, grid, dim3(64), 0, s, (const float *)qkv, seq_of_token,
                           pos_of_token, block_table, (const float *)k_cache, (const float *)v_cache, part_o, part_ml, sh);
    else
        hipLaunchKernelGGL(attn_generic_kernel<bf16_t>, grid, dim3(64), 0, s, (const bf16_t *)qkv, seq_of_token,
                           pos_of_token, block_table, (const bf16_t *)k_cache, (const bf16_t *)v_cache, part_o, part_ml, sh);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && mid) e = hipEventRecord(mid, s);
    if (e != hipSuccess) return e;
    return launch_attention_combine(dtype, false, part_o, part_ml, pos_of_token, nullptr, out, ld_out, sh, rows, s, nullptr);
}

}  // namespace dyn

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

// One workgroup per (token, q head); thread i < head_dim.  Partials are merged in chunk
// order: M = max m_c, out = sum_c e(m_c - M) o_c / sum_c e(m_c - M) l_c, where e is exp or
// exp2 according to the domain the producing kernel kept m in.
template <typename T, bool BASE2>
__global__ __launch_bounds__(256) void attn_combine_kernel(const float *__restrict__ part_o,
                                                           const float *__restrict__ part_ml,
                                                           const int32_t *__restrict__ pos_of_token,
                                                           T *__restrict__ out, AttnShape sh) {
    const int h = blockIdx.x % sh.n_q, t = blockIdx.x / sh.n_q;
    const int d = sh.head_dim, ct = sh.chunk_pages * sh.page_size;
    const int n_chunks = (pos_of_token[t] + ct) / ct;     // ceil((pos + 1) / ct)
    const size_t base = ((size_t)t * sh.n_q + h) * sh.max_chunks;
    float M = -INFINITY;
    for (int c = 0; c < n_chunks; ++c) M = fmaxf(M, part_ml[(base + c) * 2]);
    float L = 0.f;
    const int i = threadIdx.x;
    float acc = 0.f;
    for (int c = 0; c < n_chunks; ++c) {
        const float dm = part_ml[(base + c) * 2] - M;
        const float w = BASE2 ? exp2f(dm) : expf(dm);
        L += w * part_ml[(base + c) * 2 + 1];
        if (i < d) acc += w * part_o[(base + c) * d + i];
    }
    if (i < d) out[((size_t)t * sh.n_q + h) * d + i] = from_f32<T>(acc / L);
}

hipError_t launch_attention_combine(int dtype, bool base2, const float *part_o, const float *part_ml,
                                    const int32_t *pos_of_token, void *out, const AttnShape &sh, int rows,
                                    hipStream_t s) {
    const dim3 grid(rows * sh.n_q), block(sh.head_dim <= 64 ? 64 : (sh.head_dim <= 128 ? 128 : 256));
    if (dtype == 0) {
        if (base2) hipLaunchKernelGGL((attn_combine_kernel<float, true>), grid, block, 0, s, part_o, part_ml, pos_of_token, (float *)out, sh);
        else hipLaunchKernelGGL((attn_combine_kernel<float, false>), grid, block, 0, s, part_o, part_ml, pos_of_token, (float *)out, sh);
    } else {
        if (base2) hipLaunchKernelGGL((attn_combine_kernel<bf16_t, true>), grid, block, 0, s, part_o, part_ml, pos_of_token, (bf16_t *)out, sh);
        else hipLaunchKernelGGL((attn_combine_kernel<bf16_t, false>), grid, block, 0, s, part_o, part_ml, pos_of_token, (bf16_t *)out, sh);
    }
    return hipGetLastError();
}

hipError_t launch_attention_generic(int dtype, const void *qkv, const int32_t *seq_of_token,
                                    const int32_t *pos_of_token, const int32_t *block_table, const void *k_cache,
                                    const void *v_cache, void *out, float *part_o, float *part_ml,
                                    const AttnShape &sh, int rows, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    const dim3 grid((unsigned)((size_t)rows * sh.n_q * sh.max_chunks));
    if (dtype == 0)
        hipLaunchKernelGGL(attn_generic_kernel<float>, grid, dim3(64), 0, s, (const float *)qkv, seq_of_token,
                           pos_of_token, block_table, (const float *)k_cache, (const float *)v_cache, part_o, part_ml, sh);
    else
        hipLaunchKernelGGL(attn_generic_kernel<bf16_t>, grid, dim3(64), 0, s, (const bf16_t *)qkv, seq_of_token,
                           pos_of_token, block_table, (const bf16_t *)k_cache, (const bf16_t *)v_cache, part_o, part_ml, sh);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_attention_combine(dtype, false, part_o, part_ml, pos_of_token, out, sh, rows, s);
}

}  // namespace dyn

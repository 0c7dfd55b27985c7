// Mixture-of-experts pieces around the grouped projections: router, per-expert row lists,
// weighted combine.  Every token's routing and output depend on that token alone, and every
// sum has a fixed order (experts by router rank, split-K planes ascending), so results do
// not depend on how the batch is cut.
#include "common.h"
#include "kernels.h"

namespace dyn {

constexpr int kMaxExperts = 16;

// One 256-thread workgroup per token.  Every thread takes contiguous 8-element pieces of the
// row, multiplies them with the same pieces of all E router rows (all loads of a piece are
// independent, so they are in flight together), a butterfly and a fixed-order LDS step add the
// slices, thread 0 picks the top_k largest logits (ties to the lower index) and normalises
// exp(logit - max) over the picked ones.
template <typename T>
__global__ __launch_bounds__(256) void route_kernel(const T *__restrict__ h, int ldh, const float *__restrict__ w_router,
                                                    int32_t *__restrict__ sel, float *__restrict__ wgt, int rows,
                                                    int H, int E, int top_k) {
    const int t = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float acc[kMaxExperts];
#pragma unroll
    for (int e = 0; e < kMaxExperts; ++e) acc[e] = 0.f;
    for (int k0 = threadIdx.x * 8; k0 < H; k0 += 256 * 8) {
        float x[8];
        if constexpr (sizeof(T) == 2) {       // one 16-byte load (rows and k0 are 16-byte aligned)
            const u32x4 raw = *reinterpret_cast<const u32x4 *>(h + (size_t)t * ldh + k0);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                x[2 * i] = __uint_as_float(raw[i] << 16);
                x[2 * i + 1] = __uint_as_float(raw[i] & 0xffff0000u);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) x[i] = to_f32<T>(h[(size_t)t * ldh + k0 + i]);
        }
#pragma unroll
        for (int e = 0; e < kMaxExperts; ++e)
            if (e < E) {
                const f32x4 w0 = *reinterpret_cast<const f32x4 *>(w_router + (size_t)e * H + k0);
                const f32x4 w1 = *reinterpret_cast<const f32x4 *>(w_router + (size_t)e * H + k0 + 4);
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[e] = fmaf(x[i], w0[i], acc[e]);
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[e] = fmaf(x[4 + i], w1[i], acc[e]);
            }
    }
    __shared__ float part[4][kMaxExperts];
#pragma unroll
    for (int e = 0; e < kMaxExperts; ++e) {
        const float v = wave_sum(acc[e]);
        if (lane == 0) part[wave][e] = v;
    }
    __syncthreads();
    if (threadIdx.x != 0) return;
    float logit[kMaxExperts];
#pragma unroll
    for (int e = 0; e < kMaxExperts; ++e) logit[e] = ((part[0][e] + part[1][e]) + part[2][e]) + part[3][e];
    // No array is indexed with a run-time value here: that would move it from registers to scratch
    // memory, and this single thread's dependent accesses to it were most of the kernel's time.
    unsigned used = 0;
    float mx = 0.f, denom = 0.f;
    for (int j = 0; j < top_k; ++j) {
        int best = -1;
        float best_val = 0.f;
#pragma unroll
        for (int e = 0; e < kMaxExperts; ++e)
            if (e < E && !((used >> e) & 1u) && (best < 0 || logit[e] > best_val)) { best = e; best_val = logit[e]; }
        used |= 1u << best;
        if (j == 0) mx = best_val;            // picks come in descending order: the first is the maximum
        const float ex = expf(best_val - mx);
        denom += ex;
        sel[(size_t)t * top_k + j] = best;
        wgt[(size_t)t * top_k + j] = ex;
    }
    for (int j = 0; j < top_k; ++j) wgt[(size_t)t * top_k + j] = wgt[(size_t)t * top_k + j] / denom;
}

hipError_t launch_route(int dtype, const void *h, int ldh, const float *w_router, int32_t *sel, float *wgt, int rows,
                        int H, int E, int top_k, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    const dim3 grid(rows);
    if (dtype == 0)
        hipLaunchKernelGGL(route_kernel<float>, grid, dim3(256), 0, s, (const float *)h, ldh, w_router, sel, wgt, rows, H, E, top_k);
    else
        hipLaunchKernelGGL(route_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t *)h, ldh, w_router, sel, wgt, rows, H, E, top_k);
    return hipGetLastError();
}

// One wave per expert scans the dispatch's pairs in ascending order and appends its own.
__global__ void expert_lists_kernel(const int32_t *__restrict__ sel, int n_pairs, int pair_base, int cap,
                                    int32_t *__restrict__ counts, int32_t *__restrict__ lists) {
    const int e = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int count = 0;
    for (int base = 0; base < n_pairs; base += 64) {
        const int p = base + lane;
        const bool mine = p < n_pairs && sel[pair_base + p] == e;
        const unsigned long long mask = __ballot(mine);
        if (mine) lists[(size_t)e * cap + count + __popcll(mask & ((1ull << lane) - 1ull))] = pair_base + p;
        count += __popcll(mask);
    }
    if (lane == 0) counts[e] = count;
}

hipError_t launch_expert_lists(const int32_t *sel, int n_pairs, int pair_base, int E, int cap, int32_t *counts,
                               int32_t *lists, hipStream_t s) {
    if (n_pairs <= 0) return hipSuccess;
    hipLaunchKernelGGL(expert_lists_kernel, dim3(1), dim3(64 * E), 0, s, sel, n_pairs, pair_base, cap, counts, lists);
    return hipGetLastError();
}

// Four outputs per thread.
template <typename T>
__global__ __launch_bounds__(256) void moe_combine_kernel(const float *__restrict__ planes, size_t plane_stride, int S,
                                                          const float *__restrict__ wgt, const T *__restrict__ x2,
                                                          T *__restrict__ y, size_t n_vec, int H, int top_k) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += (size_t)gridDim.x * 256) {
        const size_t t = i / (H / 4), c = (i % (H / 4)) * 4;
        f32x4 m = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int j = 0; j < top_k; ++j) {
            const size_t row = t * top_k + j;
            f32x4 o = *reinterpret_cast<const f32x4 *>(planes + row * H + c);
            for (int p = 1; p < S; ++p) o += *reinterpret_cast<const f32x4 *>(planes + (size_t)p * plane_stride + row * H + c);
            m += o * wgt[row];
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) y[t * H + c + r] = from_f32<T>(to_f32<T>(x2[t * H + c + r]) + m[r]);
    }
}

hipError_t launch_moe_combine(int dtype, const float *planes, size_t plane_stride, int S, const float *wgt,
                              const void *x2, void *y, int rows, int H, int top_k, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    const size_t n_vec = (size_t)rows * H / 4;
    const int blocks = (int)((n_vec + 255) / 256 < 2048 ? (n_vec + 255) / 256 : 2048);
    if (dtype == 0)
        hipLaunchKernelGGL(moe_combine_kernel<float>, dim3(blocks), dim3(256), 0, s, planes, plane_stride, S, wgt,
                           (const float *)x2, (float *)y, n_vec, H, top_k);
    else
        hipLaunchKernelGGL(moe_combine_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, planes, plane_stride, S, wgt,
                           (const bf16_t *)x2, (bf16_t *)y, n_vec, H, top_k);
    return hipGetLastError();
}

}  // namespace dyn

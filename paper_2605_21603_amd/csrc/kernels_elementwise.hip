// RMSNorm, rotary + KV-cache append, SiLU-gate: the memory-bound elementwise operators of
// the layer (the paper's "normalization" class, Section 2).  fp32 arithmetic, storage
// type T.  Every output row depends on its own input row only and is reduced in an order
// fixed by the block shape, so results do not depend on how a batch is split.
#include "common.h"
#include "kernels.h"

namespace dyn {

// ------------------------------------------------------------------ RMSNorm
// One 256-thread workgroup per row.  out = x * g / sqrt(mean(x^2) + eps).
template <typename T>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const T *__restrict__ x, const T *__restrict__ g,
                                                      T *__restrict__ out, int ld_out, int H, float eps) {
    constexpr int V = 16 / sizeof(T);
    typedef T vec_t __attribute__((ext_vector_type(V)));
    const size_t row = blockIdx.x;
    const vec_t *xr = reinterpret_cast<const vec_t *>(x + row * H);
    const vec_t *gr = reinterpret_cast<const vec_t *>(g);
    vec_t *orow = reinterpret_cast<vec_t *>(out + row * ld_out);
    const int nv = H / V;
    float ss = 0.f;
    for (int i = threadIdx.x; i < nv; i += 256) {
        vec_t v = xr[i];
#pragma unroll
        for (int e = 0; e < V; ++e) { float f = to_f32<T>(v[e]); ss += f * f; }
    }
    ss = wave_sum(ss);
    __shared__ float part[4];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float total = ((part[0] + part[1]) + part[2]) + part[3];
    const float r = 1.0f / sqrtf(total / (float)H + eps);
    for (int i = threadIdx.x; i < nv; i += 256) {
        vec_t v = xr[i], gv = gr[i], o;
#pragma unroll
        for (int e = 0; e < V; ++e) o[e] = from_f32<T>(to_f32<T>(v[e]) * r * to_f32<T>(gv[e]));
        orow[i] = o;
    }
}

hipError_t launch_rmsnorm(int dtype, const void *x, const void *g, void *out, int ld_out, int rows, int H, float eps,
                          hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    if (dtype == 0)
        hipLaunchKernelGGL(rmsnorm_kernel<float>, dim3(rows), dim3(256), 0, s, (const float *)x, (const float *)g,
                           (float *)out, ld_out, H, eps);
    else
        hipLaunchKernelGGL(rmsnorm_kernel<bf16_t>, dim3(rows), dim3(256), 0, s, (const bf16_t *)x,
                           (const bf16_t *)g, (bf16_t *)out, ld_out, H, eps);
    return hipGetLastError();
}

// Split-K reduce of a projection fused with the RMSNorm that follows it (bf16): one 256-thread
// workgroup per row sums the row's S fp32 planes in plane order, adds the residual, rounds to
// bf16 (the projection's output Y), and normalises the rounded values exactly as rmsnorm_kernel
// does - same thread-to-column mapping, same order of the sum of squares - so a row has the same
// bits as with gemm_reduce_kernel followed by rmsnorm_kernel.
// (SC = the split factor as a compile-time constant, so that a row's plane loads are all issued
// before the first is added - one workgroup per row has nothing else to hide their latency with;
// 0 = any factor, loop.)
template <int SC>
__global__ __launch_bounds__(256) void gemm_reduce_norm_kernel(const float *__restrict__ P, size_t plane_stride, int S,
                                                               const bf16_t *__restrict__ R, bf16_t *__restrict__ Y,
                                                               const bf16_t *__restrict__ g, bf16_t *__restrict__ out,
                                                               int ld_out, int H, float eps) {
    typedef bf16_t vec_t __attribute__((ext_vector_type(8)));
    constexpr int KEEP = 4;                                 // vectors a thread keeps in registers (H <= 8192); beyond, Y is read back
    const size_t row = blockIdx.x;
    const int nv = H / 8;
    vec_t kept[KEEP];
    float ss = 0.f;
    int n = 0;
    for (int i = threadIdx.x; i < nv; i += 256, ++n) {
        const float *p = P + row * H + (size_t)i * 8;
        f32x4 a, b;
        vec_t rv{};
        if (R) rv = *reinterpret_cast<const vec_t *>(R + row * H + (size_t)i * 8);
        if constexpr (SC > 0) {
            f32x4 pa[SC], pb[SC];
#pragma unroll
            for (int sp = 0; sp < SC; ++sp) {
                pa[sp] = *reinterpret_cast<const f32x4 *>(p + (size_t)sp * plane_stride);
                pb[sp] = *reinterpret_cast<const f32x4 *>(p + (size_t)sp * plane_stride + 4);
            }
            a = pa[0];
            b = pb[0];
#pragma unroll
            for (int sp = 1; sp < SC; ++sp) {
                a[0] += pa[sp][0]; a[1] += pa[sp][1]; a[2] += pa[sp][2]; a[3] += pa[sp][3];
                b[0] += pb[sp][0]; b[1] += pb[sp][1]; b[2] += pb[sp][2]; b[3] += pb[sp][3];
            }
        } else {
            a = *reinterpret_cast<const f32x4 *>(p);
            b = *reinterpret_cast<const f32x4 *>(p + 4);
            for (int sp = 1; sp < S; ++sp) {
                const f32x4 c = *reinterpret_cast<const f32x4 *>(p + (size_t)sp * plane_stride);
                const f32x4 d = *reinterpret_cast<const f32x4 *>(p + (size_t)sp * plane_stride + 4);
                a[0] += c[0]; a[1] += c[1]; a[2] += c[2]; a[3] += c[3];
                b[0] += d[0]; b[1] += d[1]; b[2] += d[2]; b[3] += d[3];
            }
        }
        if (R) {
            a[0] += bf2f(rv[0]); a[1] += bf2f(rv[1]); a[2] += bf2f(rv[2]); a[3] += bf2f(rv[3]);
            b[0] += bf2f(rv[4]); b[1] += bf2f(rv[5]); b[2] += bf2f(rv[6]); b[3] += bf2f(rv[7]);
        }
        vec_t v;
#pragma unroll
        for (int e = 0; e < 4; ++e) { v[e] = f2bf(a[e]); v[e + 4] = f2bf(b[e]); }
        *reinterpret_cast<vec_t *>(Y + row * H + (size_t)i * 8) = v;
        if (n < KEEP) kept[n] = v;
#pragma unroll
        for (int e = 0; e < 8; ++e) { const float f = bf2f(v[e]); ss += f * f; }
    }
    ss = wave_sum(ss);
    __shared__ float part[4];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float total = ((part[0] + part[1]) + part[2]) + part[3];
    const float r = 1.0f / sqrtf(total / (float)H + eps);
    n = 0;
    for (int i = threadIdx.x; i < nv; i += 256, ++n) {
        // beyond the kept vectors a thread reads back what it stored itself
        const vec_t v = n < KEEP ? kept[n] : *reinterpret_cast<const vec_t *>(Y + row * H + (size_t)i * 8);
        const vec_t gv = *reinterpret_cast<const vec_t *>(g + (size_t)i * 8);
        vec_t o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = f2bf(bf2f(v[e]) * r * bf2f(gv[e]));
        *reinterpret_cast<vec_t *>(out + row * ld_out + (size_t)i * 8) = o;
    }
}

hipError_t launch_reduce_norm(const float *P, size_t plane_stride, int S, const void *R, void *Y, const void *g, void *out,
                              int ld_out, int rows, int H, float eps, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
#define DYN_RN(SC) hipLaunchKernelGGL(gemm_reduce_norm_kernel<SC>, dim3(rows), dim3(256), 0, s, P, plane_stride, S, (const bf16_t *)R, \
                                      (bf16_t *)Y, (const bf16_t *)g, (bf16_t *)out, ld_out, H, eps)
    switch (S) {
        case 2: DYN_RN(2); break;
        case 4: DYN_RN(4); break;
        case 8: DYN_RN(8); break;
        default: DYN_RN(0); break;
    }
#undef DYN_RN
    return hipGetLastError();
}

// ------------------------------------------------------------------ rotary + cache append
// One thread per (token, head, pair index i < d/2); heads are the q heads, then the k heads,
// then the v heads (a v "pair" is just two elements to copy).  The angle pos * theta_i is
// formed and reduced to [-pi, pi] in fp64, then sine and cosine are taken in fp32, so the
// rotation is good to fp32 rounding at any position.
template <typename T>
__global__ __launch_bounds__(256) void rope_kv_kernel(T *__restrict__ qkv, const int32_t *__restrict__ seq_of_token,
                                                      const int32_t *__restrict__ pos_of_token,
                                                      const int32_t *__restrict__ block_table,
                                                      T *__restrict__ k_cache, T *__restrict__ v_cache,
                                                      RopeTable tab, AttnShape sh) {
    const int t = blockIdx.x;
    const int d = sh.head_dim, half = d >> 1;
    const int item = blockIdx.y * 256 + threadIdx.x;
    const int hh = item / half, i = item % half;
    if (hh >= sh.n_q + 2 * sh.n_kv) return;
    const int pos = pos_of_token[t];
    T *z = qkv + (size_t)t * ((sh.n_q + 2 * sh.n_kv) * d) + hh * d;
    const float a = to_f32<T>(z[i]), b = to_f32<T>(z[i + half]);
    if (hh >= sh.n_q + sh.n_kv) {                        // v head -> V page [kvh][d][slot]
        const int g = hh - sh.n_q - sh.n_kv;
        const int page = block_table[(size_t)seq_of_token[t] * sh.max_pages_per_seq + pos / sh.page_size];
        T *vp = v_cache + ((size_t)page * sh.n_kv + g) * d * sh.page_size + pos % sh.page_size;
        vp[(size_t)i * sh.page_size] = z[i];
        vp[(size_t)(i + half) * sh.page_size] = z[i + half];
        return;
    }
    const double ang = (double)pos * tab.inv_freq[i];
    const double turns = rint(ang * 0.15915494309189535);              // 1 / (2 pi)
    const float red = (float)fma(-turns, 6.283185307179586, ang);
    float s, c;
    sincosf(red, &s, &c);
    const T lo = from_f32<T>(a * c - b * s), hi = from_f32<T>(b * c + a * s);
    if (hh < sh.n_q) {                                   // q head, in place
        z[i] = lo;
        z[i + half] = hi;
    } else {                                             // k head -> K page [kvh][slot][d]
        const int g = hh - sh.n_q;
        const int page = block_table[(size_t)seq_of_token[t] * sh.max_pages_per_seq + pos / sh.page_size];
        T *kp = k_cache + (((size_t)page * sh.n_kv + g) * sh.page_size + pos % sh.page_size) * d;
        kp[i] = lo;
        kp[i + half] = hi;
    }
}

// Vector form for head dims whose half is a multiple of the 16-byte vector: one workgroup per
// token.  The d/2 angles of the token are reduced and their sine / cosine taken once (not once
// per head) into LDS; then a thread rotates V pair indices of one head with 16-byte loads and
// stores (q in place, k into its cache page), and the v heads are scattered into the
// position-fastest V page element by element.  Same arithmetic per element as the scalar form.
template <typename T>
__global__ __launch_bounds__(256) void rope_kv_vec_kernel(T *__restrict__ qkv, const int32_t *__restrict__ seq_of_token,
                                                          const int32_t *__restrict__ pos_of_token,
                                                          const int32_t *__restrict__ block_table,
                                                          T *__restrict__ k_cache, T *__restrict__ v_cache,
                                                          RopeTable tab, AttnShape sh) {
    constexpr int V = 16 / sizeof(T);
    typedef T vec_t __attribute__((ext_vector_type(V)));
    __shared__ float cs[2][128];                          // cos, sin of the token's angles (head_dim <= 256)
    const int t = blockIdx.x;
    const int d = sh.head_dim, half = d >> 1;
    const int pos = pos_of_token[t];
    for (int i = threadIdx.x; i < half; i += 256) {
        const double ang = (double)pos * tab.inv_freq[i];
        const double turns = rint(ang * 0.15915494309189535);          // 1 / (2 pi)
        const float red = (float)fma(-turns, 6.283185307179586, ang);
        float sn, c;
        sincosf(red, &sn, &c);
        cs[0][i] = c;
        cs[1][i] = sn;
    }
    const int page = block_table[(size_t)seq_of_token[t] * sh.max_pages_per_seq + pos / sh.page_size];
    const int slot = pos % sh.page_size;
    __syncthreads();
    T *row = qkv + (size_t)t * ((sh.n_q + 2 * sh.n_kv) * d);
    const int per_head = half / V, n_rot = (sh.n_q + sh.n_kv) * per_head;
    // a token's units are dealt over gridDim.y workgroups (few tokens: more workgroups than tokens)
    const int first = blockIdx.y * 256 + threadIdx.x, step = gridDim.y * 256;
    for (int u = first; u < n_rot; u += step) {
        const int hh = u / per_head, i0 = (u % per_head) * V;
        T *z = row + hh * d;
        const vec_t a = *reinterpret_cast<const vec_t *>(z + i0), b = *reinterpret_cast<const vec_t *>(z + i0 + half);
        vec_t lo, hi;
#pragma unroll
        for (int e = 0; e < V; ++e) {
            const float c = cs[0][i0 + e], sn = cs[1][i0 + e], fa = to_f32<T>(a[e]), fb = to_f32<T>(b[e]);
            lo[e] = from_f32<T>(fa * c - fb * sn);
            hi[e] = from_f32<T>(fb * c + fa * sn);
        }
        T *dst = hh < sh.n_q ? z : k_cache + (((size_t)page * sh.n_kv + (hh - sh.n_q)) * sh.page_size + slot) * d;
        *reinterpret_cast<vec_t *>(dst + i0) = lo;
        *reinterpret_cast<vec_t *>(dst + i0 + half) = hi;
    }
    const T *vrow = row + (sh.n_q + sh.n_kv) * d;
    for (int u = first; u < sh.n_kv * d; u += step) {                   // v heads -> V page [kvh][d][slot]
        const int g = u / d, i = u % d;
        v_cache[(((size_t)page * sh.n_kv + g) * d + i) * sh.page_size + slot] = vrow[u];
    }
}

// Split-K reduce of the qkv projection fused with rotary + cache append (bf16, the vector form's
// shapes): the a / b halves of a rotation unit are the sums of the S fp32 planes in plane order,
// rounded to bf16 - the values gemm_reduce_kernel would have stored - and from there on the
// arithmetic of rope_kv_vec_kernel, unit for unit.  q' goes to the qkv row, k' and v to the cache
// pages; the unrotated k and v are not stored anywhere (nothing reads them).
template <int SC>
__global__ __launch_bounds__(256) void gemm_reduce_rope_kernel(const float *__restrict__ P, size_t plane_stride, int S,
                                                               bf16_t *__restrict__ qkv, const int32_t *__restrict__ seq_of_token,
                                                               const int32_t *__restrict__ pos_of_token,
                                                               const int32_t *__restrict__ block_table,
                                                               bf16_t *__restrict__ k_cache, bf16_t *__restrict__ v_cache,
                                                               RopeTable tab, AttnShape sh) {
    typedef bf16_t vec_t __attribute__((ext_vector_type(8)));
    constexpr int V = 8;
    __shared__ float cs[2][128];
    const int t = blockIdx.x;
    const int d = sh.head_dim, half = d >> 1;
    const int pos = pos_of_token[t];
    for (int i = threadIdx.x; i < half; i += 256) {
        const double ang = (double)pos * tab.inv_freq[i];
        const double turns = rint(ang * 0.15915494309189535);          // 1 / (2 pi)
        const float red = (float)fma(-turns, 6.283185307179586, ang);
        float sn, c;
        sincosf(red, &sn, &c);
        cs[0][i] = c;
        cs[1][i] = sn;
    }
    const int page = block_table[(size_t)seq_of_token[t] * sh.max_pages_per_seq + pos / sh.page_size];
    const int slot = pos % sh.page_size;
    __syncthreads();
    const int width = (sh.n_q + 2 * sh.n_kv) * d;
    const float *prow = P + (size_t)t * width;
    bf16_t *row = qkv + (size_t)t * width;
    auto summed = [&](int col) {                           // eight consecutive columns of the row, planes added in order, rounded
        const float *p = prow + col;
        f32x4 a, b;
        if constexpr (SC > 0) {                            // all plane loads in flight before the first add
            f32x4 pa[SC], pb[SC];
#pragma unroll
            for (int sp = 0; sp < SC; ++sp) {
                pa[sp] = *reinterpret_cast<const f32x4 *>(p + (size_t)sp * plane_stride);
                pb[sp] = *reinterpret_cast<const f32x4 *>(p + (size_t)sp * plane_stride + 4);
            }
            a = pa[0];
            b = pb[0];
#pragma unroll
            for (int sp = 1; sp < SC; ++sp) {
                a[0] += pa[sp][0]; a[1] += pa[sp][1]; a[2] += pa[sp][2]; a[3] += pa[sp][3];
                b[0] += pb[sp][0]; b[1] += pb[sp][1]; b[2] += pb[sp][2]; b[3] += pb[sp][3];
            }
        } else {
            a = *reinterpret_cast<const f32x4 *>(p);
            b = *reinterpret_cast<const f32x4 *>(p + 4);
            for (int sp = 1; sp < S; ++sp) {
                const f32x4 c = *reinterpret_cast<const f32x4 *>(p + (size_t)sp * plane_stride);
                const f32x4 e = *reinterpret_cast<const f32x4 *>(p + (size_t)sp * plane_stride + 4);
                a[0] += c[0]; a[1] += c[1]; a[2] += c[2]; a[3] += c[3];
                b[0] += e[0]; b[1] += e[1]; b[2] += e[2]; b[3] += e[3];
            }
        }
        vec_t v;
#pragma unroll
        for (int e = 0; e < 4; ++e) { v[e] = f2bf(a[e]); v[e + 4] = f2bf(b[e]); }
        return v;
    };
    const int per_head = half / V, n_rot = (sh.n_q + sh.n_kv) * per_head;
    const int first = blockIdx.y * 256 + threadIdx.x, step = gridDim.y * 256;
    for (int u = first; u < n_rot; u += step) {
        const int hh = u / per_head, i0 = (u % per_head) * V;
        const vec_t a = summed(hh * d + i0), b = summed(hh * d + i0 + half);
        vec_t lo, hi;
#pragma unroll
        for (int e = 0; e < V; ++e) {
            const float c = cs[0][i0 + e], sn = cs[1][i0 + e], fa = bf2f(a[e]), fb = bf2f(b[e]);
            lo[e] = f2bf(fa * c - fb * sn);
            hi[e] = f2bf(fb * c + fa * sn);
        }
        bf16_t *dst = hh < sh.n_q ? row + hh * d : k_cache + (((size_t)page * sh.n_kv + (hh - sh.n_q)) * sh.page_size + slot) * d;
        *reinterpret_cast<vec_t *>(dst + i0) = lo;
        *reinterpret_cast<vec_t *>(dst + i0 + half) = hi;
    }
    const int vbase = (sh.n_q + sh.n_kv) * d;
    for (int u = first; u < sh.n_kv * d / V; u += step) {               // v heads -> V page [kvh][d][slot], eight head-dim indices per thread
        const vec_t v = summed(vbase + u * V);
        const int g = (u * V) / d, i = (u * V) % d;
        bf16_t *vp = v_cache + (((size_t)page * sh.n_kv + g) * d + i) * sh.page_size + slot;
#pragma unroll
        for (int e = 0; e < V; ++e) vp[(size_t)e * sh.page_size] = v[e];
    }
}

bool reduce_rope_supported(int dtype, const AttnShape &sh) { return dtype == 1 && (sh.head_dim / 2) % 8 == 0 && sh.head_dim <= 256; }

hipError_t launch_reduce_rope(const float *P, size_t plane_stride, int S, void *qkv, const int32_t *seq_of_token,
                              const int32_t *pos_of_token, const int32_t *block_table, void *k_cache, void *v_cache,
                              const RopeTable &tab, const AttnShape &sh, int rows, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    const dim3 grid(rows, rows < 512 ? 4 : 1);      // as the unfused kernel: a token's units over four workgroups when tokens are few
#define DYN_RR(SC) hipLaunchKernelGGL(gemm_reduce_rope_kernel<SC>, grid, dim3(256), 0, s, P, plane_stride, S, (bf16_t *)qkv, seq_of_token, \
                                      pos_of_token, block_table, (bf16_t *)k_cache, (bf16_t *)v_cache, tab, sh)
    switch (S) {
        case 2: DYN_RR(2); break;
        case 4: DYN_RR(4); break;
        case 8: DYN_RR(8); break;
        default: DYN_RR(0); break;
    }
#undef DYN_RR
    return hipGetLastError();
}

hipError_t launch_rope_kv(int dtype, void *qkv, const int32_t *seq_of_token, const int32_t *pos_of_token,
                          const int32_t *block_table, void *k_cache, void *v_cache, const RopeTable &tab,
                          const AttnShape &sh, int rows, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    const int vec = dtype == 0 ? 4 : 8;
    if ((sh.head_dim / 2) % vec == 0 && sh.head_dim <= 256) {
        const dim3 grid(rows, rows < 512 ? 4 : 1);
        if (dtype == 0)
            hipLaunchKernelGGL(rope_kv_vec_kernel<float>, grid, dim3(256), 0, s, (float *)qkv, seq_of_token,
                               pos_of_token, block_table, (float *)k_cache, (float *)v_cache, tab, sh);
        else
            hipLaunchKernelGGL(rope_kv_vec_kernel<bf16_t>, grid, dim3(256), 0, s, (bf16_t *)qkv, seq_of_token,
                               pos_of_token, block_table, (bf16_t *)k_cache, (bf16_t *)v_cache, tab, sh);
        return hipGetLastError();
    }
    const int items = (sh.n_q + 2 * sh.n_kv) * (sh.head_dim / 2);
    const dim3 grid(rows, (items + 255) / 256);
    if (dtype == 0)
        hipLaunchKernelGGL(rope_kv_kernel<float>, grid, dim3(256), 0, s, (float *)qkv, seq_of_token,
                           pos_of_token, block_table, (float *)k_cache, (float *)v_cache, tab, sh);
    else
        hipLaunchKernelGGL(rope_kv_kernel<bf16_t>, grid, dim3(256), 0, s, (bf16_t *)qkv, seq_of_token,
                           pos_of_token, block_table, (bf16_t *)k_cache, (bf16_t *)v_cache, tab, sh);
    return hipGetLastError();
}

// ------------------------------------------------------------------ SiLU gate
// out[t, i] = g / (1 + exp(-g)) * u with g = gu[t, i], u = gu[t, I + i].
template <typename T>
__global__ __launch_bounds__(256) void silu_mul_kernel(const T *__restrict__ gu, T *__restrict__ out, int ld_out,
                                                       int I, size_t n_vec) {
    constexpr int V = 16 / sizeof(T);
    typedef T vec_t __attribute__((ext_vector_type(V)));
    const int vec_per_row = I / V;
    for (size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x; idx < n_vec; idx += (size_t)gridDim.x * 256) {
        const size_t t = idx / vec_per_row, c = idx % vec_per_row;
        const vec_t g = *reinterpret_cast<const vec_t *>(gu + t * 2 * I + c * V);
        const vec_t u = *reinterpret_cast<const vec_t *>(gu + t * 2 * I + I + c * V);
        vec_t o;
#pragma unroll
        for (int e = 0; e < V; ++e) {
            const float z = to_f32<T>(g[e]);
            o[e] = from_f32<T>(z / (1.0f + expf(-z)) * to_f32<T>(u[e]));
        }
        *reinterpret_cast<vec_t *>(out + t * ld_out + c * V) = o;
    }
}

hipError_t launch_silu_mul(int dtype, const void *gu, void *out, int ld_out, int rows, int I, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    const int V = dtype == 0 ? 4 : 8;
    const size_t n_vec = (size_t)rows * (I / V);
    const int blocks = (int)((n_vec + 255) / 256 < 4096 ? (n_vec + 255) / 256 : 4096);
    if (dtype == 0)
        hipLaunchKernelGGL(silu_mul_kernel<float>, dim3(blocks), dim3(256), 0, s, (const float *)gu, (float *)out, ld_out,
                           I, n_vec);
    else
        hipLaunchKernelGGL(silu_mul_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, (const bf16_t *)gu,
                           (bf16_t *)out, ld_out, I, n_vec);
    return hipGetLastError();
}

// Read-only streaming probe: every 16-byte word of a buffer is loaded once (a workgroup reads
// 4 KB contiguously per step of a grid-wide stride; eight workgroups per CU keep the loads of
// different steps in flight) and folded into one word per wave so that the loads cannot be
// dropped.  What it reaches is the rate this GPU's memory system delivers to a kernel that does
// nothing else: the practical ceiling next to the datasheet peak.
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4 *__restrict__ p, size_t n_vec, uint32_t *__restrict__ sink) {
    const size_t stride = (size_t)gridDim.x * 256;
    u32x4 acc = u32x4{0u, 0u, 0u, 0u};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += stride) acc ^= p[i];
    uint32_t v = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v ^= __shfl_xor(v, off, 64);
    if ((threadIdx.x & 63) == 0) sink[blockIdx.x * 4 + (threadIdx.x >> 6)] = v;
}

constexpr int kProbeBlocks = 2048;      // eight workgroups for each of the 256 CUs

hipError_t launch_stream_read(const void *buf, size_t bytes, uint32_t *sink, hipStream_t s) {
    hipLaunchKernelGGL(stream_read_kernel, dim3(kProbeBlocks), dim3(256), 0, s, (const u32x4 *)buf, bytes / 16, sink);
    return hipGetLastError();
}

}  // namespace dyn

// Projections: Y[rows, N] = X[rows, K] W[N, K]^T (+ residual).  These are the layer's
// dense contractions (the paper's compute-bound class, Section 2); below roughly 300 rows
// they are in fact bound by streaming W from HBM once, which is what the bf16 kernel is
// shaped for.
//
// Summation order of one output element is a function of (N, K) only: K is cut into
// S = gemm_split_k(N, K) equal chunks, each chunk is accumulated in ascending k by the
// same 16x16x32 MFMA into an fp32 accumulator starting from zero, and the chunk sums are
// added in ascending chunk order, then the residual.  Rows never mix, so a row computed in
// a 64-row micro-batch has the same bits as in the merged batch.
#include "common.h"
#include "kernels.h"

namespace dyn {

// ------------------------------------------------------------------ fp32 (plain FMA) path
// 64x64 output tile per 256-thread workgroup, 4x4 outputs per thread, K staged 16 at a time
// through LDS.  Each output is one fp32 FMA chain in ascending k.
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float *__restrict__ X, const float *__restrict__ W,
                                                       const float *__restrict__ R, float *__restrict__ Y, int M,
                                                       int N, int K) {
    __shared__ float xs[16][64 + 4];
    __shared__ float ws[16][64 + 4];
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        for (int e = threadIdx.x; e < 64 * 16; e += 256) {
            const int r = e / 16, kk = e % 16;
            xs[kk][r] = (m0 + r < M && k0 + kk < K) ? X[(size_t)(m0 + r) * K + k0 + kk] : 0.f;
            ws[kk][r] = (n0 + r < N && k0 + kk < K) ? W[(size_t)(n0 + r) * K + k0 + kk] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = xs[kk][ty * 4 + i]; b[i] = ws[kk][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
            if (m < M && n < N) Y[(size_t)m * N + n] = acc[i][j] + (R ? R[(size_t)m * N + n] : 0.f);
        }
}

// ------------------------------------------------------------------ bf16 MFMA path
// Workgroup = 4 waves, tile = 64 rows of X by 128 rows of W, one K chunk.  Wave w owns 32
// rows of W as two MFMA "A" operands which it loads straight from global memory in operand
// layout (lane l: row l%16, 8 consecutive k at 8*(l/16): 64 contiguous bytes per row and
// instruction), PF stages ahead.  The 64x64 X tile of a stage goes through LDS (rows padded
// to 144 bytes so the four 16-lane groups of a ds_read_b128 hit disjoint banks) and feeds
// the "B" operands of all four waves.  D[i][j]: i = W row (4*(l/16)+r), j = X row (l%16).
constexpr int GN = 128, GM = 64, GK = 64, PF = 3;
constexpr int XROW = GK * 2 + 16;              // bytes per X row in LDS
constexpr int XBUF = GM * XROW;                // bytes per stage buffer

__global__ __launch_bounds__(256, 2) void gemm_bf16_kernel(const bf16_t *__restrict__ X, const bf16_t *__restrict__ W,
                                                           const bf16_t *__restrict__ R, bf16_t *__restrict__ Y,
                                                           float *__restrict__ P, size_t plane_stride, int M, int N,
                                                           int K, int S) {
    __shared__ __attribute__((aligned(16))) unsigned char xl[2 * XBUF];
    const int m_tiles = (M + GM - 1) / GM;
    // Workgroup ids are dealt round-robin to the 8 XCDs.  Tiles that share W rows (the
    // m tiles of one (n tile, chunk)) get ids 8 apart: same XCD, same L2, adjacent in time.
    const int u = blockIdx.x % 8, v = blockIdx.x / 8;
    const int m_tile = v % m_tiles, ns = (v / m_tiles) * 8 + u;
    if (ns >= (N / GN) * S) return;
    const int n_tile = ns / S, sp = ns % S;
    const int Kc = K / S, kbase = sp * Kc, n_stage = Kc / GK;
    const int m0 = m_tile * GM;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lr = lane & 15, lq = lane >> 4;

    const bf16_t *wp[2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
        wp[a] = W + (size_t)(n_tile * GN + wave * 32 + a * 16 + lr) * K + kbase + 8 * lq;
    // X staging: two 16-byte pieces per thread and stage
    const bf16_t *xp[2];
    int xoff[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        const int piece = tid + 256 * p, row = piece >> 3, col = piece & 7;
        const int m = min(m0 + row, M - 1);
        xp[p] = X + (size_t)m * K + kbase + col * 8;
        xoff[p] = row * XROW + col * 16;
    }

    u32x4 wr[PF + 1][2][2];
    u32x4 xr[2][2];
    f32x4 acc[2][4];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

#pragma unroll
    for (int p = 0; p < PF; ++p)
        if (p < n_stage) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int a = 0; a < 2; ++a)
                    wr[p][ks][a] = *reinterpret_cast<const u32x4 *>(wp[a] + p * GK + ks * 32);
        }
#pragma unroll
    for (int p = 0; p < 2; ++p) xr[0][p] = *reinterpret_cast<const u32x4 *>(xp[p]);
    if (n_stage > 1) {
#pragma unroll
        for (int p = 0; p < 2; ++p) xr[1][p] = *reinterpret_cast<const u32x4 *>(xp[p] + GK);
    }
#pragma unroll
    for (int p = 0; p < 2; ++p) *reinterpret_cast<u32x4 *>(xl + xoff[p]) = xr[0][p];
    __syncthreads();

    // One stage: prefetch W for stage st+PF and X for stage st+2, multiply stage st, hand the
    // X tile of stage st+1 to LDS.  J = st mod (PF+1) is a literal so that every register
    // array index is a compile-time constant.
#define DYN_GEMM_STAGE(J)                                                                                         \
    {                                                                                                             \
        const int st = st0 + (J);                                                                                 \
        if (st < n_stage) {                                                                                       \
            if (st + PF < n_stage) {                                                                              \
                _Pragma("unroll") for (int ks = 0; ks < 2; ++ks) _Pragma("unroll") for (int a = 0; a < 2; ++a)    \
                    wr[((J) + PF) % (PF + 1)][ks][a] =                                                            \
                        *reinterpret_cast<const u32x4 *>(wp[a] + (size_t)(st + PF) * GK + ks * 32);               \
            }                                                                                                     \
            if (st + 2 < n_stage) {                                                                               \
                _Pragma("unroll") for (int p = 0; p < 2; ++p)                                                     \
                    xr[(J) % 2][p] = *reinterpret_cast<const u32x4 *>(xp[p] + (size_t)(st + 2) * GK);             \
            }                                                                                                     \
            const unsigned char *xb = xl + ((J) % 2) * XBUF;                                                      \
            _Pragma("unroll") for (int ks = 0; ks < 2; ++ks) {                                                    \
                const bf16x8 a0 = __builtin_bit_cast(bf16x8, wr[(J)][ks][0]);                                     \
                const bf16x8 a1 = __builtin_bit_cast(bf16x8, wr[(J)][ks][1]);                                     \
                _Pragma("unroll") for (int b = 0; b < 4; ++b) {                                                   \
                    const bf16x8 bv =                                                                             \
                        *reinterpret_cast<const bf16x8 *>(xb + (b * 16 + lr) * XROW + ks * 64 + lq * 16);         \
                    acc[0][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, bv, acc[0][b], 0, 0, 0);              \
                    acc[1][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, bv, acc[1][b], 0, 0, 0);              \
                }                                                                                                 \
            }                                                                                                     \
            if (st + 1 < n_stage) {                                                                               \
                unsigned char *xn = xl + (((J) + 1) % 2) * XBUF;                                                  \
                _Pragma("unroll") for (int p = 0; p < 2; ++p)                                                     \
                    *reinterpret_cast<u32x4 *>(xn + xoff[p]) = xr[((J) + 1) % 2][p];                              \
            }                                                                                                     \
            __syncthreads();                                                                                      \
        }                                                                                                         \
    }
    static_assert(PF == 3, "the stage macro is expanded PF + 1 = 4 times below");
    for (int st0 = 0; st0 < n_stage; st0 += PF + 1) {
        DYN_GEMM_STAGE(0)
        DYN_GEMM_STAGE(1)
        DYN_GEMM_STAGE(2)
        DYN_GEMM_STAGE(3)
    }
#undef DYN_GEMM_STAGE

#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int m = m0 + b * 16 + lr;
            const int n = n_tile * GN + wave * 32 + a * 16 + 4 * lq;
            if (m >= M) continue;
            if (S == 1) {
                f32x4 o = acc[a][b];
                if (R) {
                    const uint2 rv = *reinterpret_cast<const uint2 *>(R + (size_t)m * N + n);
                    o[0] += bf2f(rv.x & 0xffff); o[1] += bf2f(rv.x >> 16);
                    o[2] += bf2f(rv.y & 0xffff); o[3] += bf2f(rv.y >> 16);
                }
                uint2 ov;
                ov.x = (uint32_t)f2bf(o[0]) | ((uint32_t)f2bf(o[1]) << 16);
                ov.y = (uint32_t)f2bf(o[2]) | ((uint32_t)f2bf(o[3]) << 16);
                *reinterpret_cast<uint2 *>(Y + (size_t)m * N + n) = ov;
            } else {
                *reinterpret_cast<f32x4 *>(P + (size_t)sp * plane_stride + (size_t)m * N + n) = acc[a][b];
            }
        }
}

// Y = bf16((((P_0 + P_1) + ...) + P_{S-1}) + R), four elements per thread.
__global__ __launch_bounds__(256) void gemm_reduce_kernel(const float *__restrict__ P, size_t plane_stride,
                                                          const bf16_t *__restrict__ R, bf16_t *__restrict__ Y,
                                                          size_t n_vec, int S) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += (size_t)gridDim.x * 256) {
        f32x4 o = *reinterpret_cast<const f32x4 *>(P + i * 4);
        for (int s = 1; s < S; ++s) {
            const f32x4 p = *reinterpret_cast<const f32x4 *>(P + (size_t)s * plane_stride + i * 4);
            o[0] += p[0]; o[1] += p[1]; o[2] += p[2]; o[3] += p[3];
        }
        if (R) {
            const uint2 rv = *reinterpret_cast<const uint2 *>(R + i * 4);
            o[0] += bf2f(rv.x & 0xffff); o[1] += bf2f(rv.x >> 16);
            o[2] += bf2f(rv.y & 0xffff); o[3] += bf2f(rv.y >> 16);
        }
        uint2 ov;
        ov.x = (uint32_t)f2bf(o[0]) | ((uint32_t)f2bf(o[1]) << 16);
        ov.y = (uint32_t)f2bf(o[2]) | ((uint32_t)f2bf(o[3]) << 16);
        *reinterpret_cast<uint2 *>(Y + i * 4) = ov;
    }
}

bool gemm_supported(int dtype, int N, int K) {
    if (dtype == 0) return N > 0 && K > 0;
    return N > 0 && K > 0 && N % GN == 0 && K % GK == 0;
}

int gemm_split_k(int dtype, int N, int K) {
    if (dtype == 0) return 1;
    int S = 1;
    while ((N / GN) * S < 192 && S < 8 && K % (S * 2 * GK) == 0 && K / (S * 2) >= 256) S *= 2;
    return S;
}

hipError_t launch_gemm(int dtype, const void *X, const void *W, const void *R, void *Y, float *partial,
                       size_t plane_stride, int rows, int N, int K, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    if (dtype == 0) {
        hipLaunchKernelGGL(gemm_f32_kernel, dim3((N + 63) / 64, (rows + 63) / 64), dim3(256), 0, s, (const float *)X,
                           (const float *)W, (const float *)R, (float *)Y, rows, N, K);
        return hipGetLastError();
    }
    const int S = gemm_split_k(dtype, N, K);
    const int m_tiles = (rows + GM - 1) / GM;
    const int ns = (N / GN) * S;
    const int grid = ((ns + 7) / 8) * 8 * m_tiles;
    hipLaunchKernelGGL(gemm_bf16_kernel, dim3(grid), dim3(256), 0, s, (const bf16_t *)X, (const bf16_t *)W,
                       (const bf16_t *)R, (bf16_t *)Y, partial, plane_stride, rows, N, K, S);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || S == 1) return e;
    const size_t n_vec = (size_t)rows * N / 4;
    const int blocks = (int)((n_vec + 255) / 256 < 2048 ? (n_vec + 255) / 256 : 2048);
    hipLaunchKernelGGL(gemm_reduce_kernel, dim3(blocks), dim3(256), 0, s, partial, plane_stride, (const bf16_t *)R,
                       (bf16_t *)Y, n_vec, S);
    return hipGetLastError();
}

}  // namespace dyn

// Projections: Y[rows, N] = X[rows, K] W[N, K]^T (+ residual).  These are the layer's
// dense contractions (the paper's compute-bound class, Section 2); below roughly 300 rows
// they are in fact bound by streaming W from HBM once, which is what the bf16 kernel is
// shaped for.
//
// Summation order of one output element is a function of (N, K) only: K is cut into
// S = gemm_split_k(N, K) equal planes, each plane is accumulated in ascending k by the same
// 16x16x32 MFMA into an fp32 accumulator starting from zero, and the plane sums are added
// in ascending plane order, then the residual.  Rows never mix, so a row computed in a
// 64-row micro-batch has the same bits as in the merged batch.
#include <cstdlib>

#include "common.h"
#include "kernels.h"

namespace dyn {

// ------------------------------------------------------------------ fp32 (plain FMA) path
// 64x64 output tile per 256-thread workgroup, 4x4 outputs per thread, K staged 16 at a time
// through LDS.  Each output is one fp32 FMA chain in ascending k.
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float *__restrict__ X, int ldx, const float *__restrict__ W,
                                                       const float *__restrict__ R, float *__restrict__ Y, int M,
                                                       int N, int K, GemmGroups gr) {
    __shared__ float xs[16][64 + 4];
    __shared__ float ws[16][64 + 4];
    const int32_t *list = nullptr;
    if (gr.n_groups) {                                 // blockIdx.z = expert: its rows come from a list
        M = gr.counts[blockIdx.z];
        list = gr.lists + (size_t)blockIdx.z * gr.cap;
        W += (size_t)blockIdx.z * gr.w_stride;
    }
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    if (m0 >= M) return;
    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        for (int e = threadIdx.x; e < 64 * 16; e += 256) {
            const int r = e / 16, kk = e % 16;
            const bool in = m0 + r < M && k0 + kk < K;
            const size_t xrow = in ? (list ? list[m0 + r] / gr.x_div : m0 + r) : 0;
            xs[kk][r] = in ? X[xrow * ldx + k0 + kk] : 0.f;
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
            if (m < M && n < N) {
                const size_t orow = list ? list[m] : m;
                Y[orow * N + n] = acc[i][j] + (R ? R[orow * N + n] : 0.f);
            }
        }
}

// ------------------------------------------------------------------ bf16 MFMA path
// Workgroup = 4 waves on a 128 (W rows) x MT (X rows, 64 or 128) output tile and one K
// plane.  What bounds this kernel below a few hundred rows is not the matrix cores and not
// even HBM alone but the L2 -> CU path: every byte of W must cross it once and the X tile
// crosses it once per W tile, so both operands are fetched exactly once per workgroup with
// fully coalesced 128-byte row segments (8 lanes per row), parked in registers for three
// stages (a stage is 64 k), and handed to the waves through LDS.  LDS rows are padded to
// 144 bytes so the 16-lane groups of a ds_read_b128 in MFMA operand layout (lane l: row
// l%16, 8 consecutive k at 8*(l/16)) touch disjoint banks.  Waves sit 2 x 2 on the tile:
// 64 W rows x MT/2 X rows each.  D[i][j]: i = W row (4*(l/16)+r), j = X row (l%16).
constexpr int BN = 128, BK = 64, ROWB = BK * 2 + 16, RING = 4;
#ifndef DYN_OCC2_TILES
#define DYN_OCC2_TILES 2     // row tiles from which the two-workgroups-per-CU build is used
#endif

// INREG: one workgroup walks all S planes of its tile and adds the plane sums in registers
// (same order, same bits as the plane buffers + gemm_reduce_kernel) - for many-row launches,
// where there are enough tiles to fill the chip without spreading planes over workgroups and
// the fp32 plane traffic would cost more than the weights.
// OCC2: compile for two workgroups per CU (256 VGPRs) - pays when the launch is bound by
// the matrix cores (many row tiles), costs a few spills that hurt when it is bound by memory.
template <int MT, bool INREG, bool OCC2>
__global__ __launch_bounds__(256, OCC2 ? 2 : 1) void gemm_bf16_kernel(const bf16_t *__restrict__ X, int ldx,
                                                        const bf16_t *__restrict__ W, const bf16_t *__restrict__ R,
                                                        bf16_t *__restrict__ Y, float *__restrict__ P,
                                                        size_t plane_stride, int M, int N, int K, int S, GemmGroups gr) {
    constexpr int XP = MT / 32;                     // 16-byte X pieces per thread and stage
    constexpr int NB = MT / 32;                     // B tiles (16 X rows) per wave
    __shared__ __attribute__((aligned(16))) unsigned char lw[2][BN * ROWB];
    __shared__ __attribute__((aligned(16))) unsigned char lx[2][MT * ROWB];
    const int m_tiles = (M + MT - 1) / MT;
    // Workgroup ids are dealt round-robin to the 8 XCDs.  Tiles that share W rows (the
    // m tiles of one (n tile, plane)) get ids 8 apart: same XCD, same L2, adjacent in time.
    const int u = blockIdx.x % 8, v = blockIdx.x / 8;
    const int m_tile = v % m_tiles;
    int ns = (v / m_tiles) * 8 + u;
    const int32_t *list = nullptr;
    const int SG = INREG ? 1 : S;                      // planes spread over the grid
    if (gr.n_groups) {                                 // grouped: (expert, n tile, plane); rows come from the expert's list
        const int per_group = (N / BN) * SG;
        if (ns >= per_group * gr.n_groups) return;
        const int e = ns / per_group;
        ns -= e * per_group;
        M = gr.counts[e];
        if (m_tile * MT >= M) return;
        list = gr.lists + (size_t)e * gr.cap;
        W += (size_t)e * gr.w_stride;
    } else if (ns >= (N / BN) * SG) {
        return;
    }
    const int n_tile = ns / SG, sp = ns % SG;
    const int Kp = K / S, kbase = INREG ? 0 : sp * Kp, n_stage = (INREG ? K : Kp) / BK;
    const int plane_stages = Kp / BK;
    const int n0 = n_tile * BN, m0 = m_tile * MT;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lr = lane & 15, lq = lane >> 4, wn = wave & 1, wm = wave >> 1;

    const int prow = tid >> 3, pcol = tid & 7;      // piece p = tid + 256 u: row prow + 32 u, 16-byte column pcol
    const bf16_t *wg[4], *xg[XP];
#pragma unroll
    for (int q = 0; q < 4; ++q) wg[q] = W + (size_t)(n0 + prow + 32 * q) * K + kbase + pcol * 8;
#pragma unroll
    for (int q = 0; q < XP; ++q) {
        const int mr = min(m0 + prow + 32 * q, M - 1);
        xg[q] = X + (size_t)(list ? list[mr] / gr.x_div : mr) * ldx + kbase + pcol * 8;
    }
    const int loff = prow * ROWB + pcol * 16;

    u32x4 rw[RING][4], rx[RING][XP];
    f32x4 acc[4][NB], total[INREG ? 4 : 1][INREG ? NB : 1];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (INREG) total[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    // a plane ends on a multiple of RING stages: fold its sum into the total, start the next from zero
#define DYN_GEMM_PLANE_END(ST_DONE)                                                                      \
    if (INREG && (ST_DONE) % plane_stages == 0) {                                                        \
        _Pragma("unroll") for (int a = 0; a < 4; ++a) _Pragma("unroll") for (int b = 0; b < NB; ++b) {   \
            total[a][b] += acc[a][b];                                                                    \
            acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};                                                       \
        }                                                                                                \
    }

#define DYN_GEMM_FETCH(SLOT, ST)                                                                         \
    {                                                                                                    \
        _Pragma("unroll") for (int q = 0; q < 4; ++q)                                                    \
            rw[SLOT][q] = *reinterpret_cast<const u32x4 *>(wg[q] + (size_t)(ST) * BK);                   \
        _Pragma("unroll") for (int q = 0; q < XP; ++q)                                                   \
            rx[SLOT][q] = *reinterpret_cast<const u32x4 *>(xg[q] + (size_t)(ST) * BK);                   \
    }
#define DYN_GEMM_PARK(SLOT, BUF)                                                                         \
    {                                                                                                    \
        _Pragma("unroll") for (int q = 0; q < 4; ++q)                                                    \
            *reinterpret_cast<u32x4 *>(&lw[BUF][loff + 32 * q * ROWB]) = rw[SLOT][q];                    \
        _Pragma("unroll") for (int q = 0; q < XP; ++q)                                                   \
            *reinterpret_cast<u32x4 *>(&lx[BUF][loff + 32 * q * ROWB]) = rx[SLOT][q];                    \
    }
#define DYN_GEMM_MMA(BUF)                                                                                \
    _Pragma("unroll") for (int ks = 0; ks < 2; ++ks) {                                                   \
        bf16x8 av[4], bv[NB];                                                                            \
        _Pragma("unroll") for (int a = 0; a < 4; ++a) av[a] = *reinterpret_cast<const bf16x8 *>(         \
            &lw[BUF][(wn * 64 + a * 16 + lr) * ROWB + ks * 64 + lq * 16]);                               \
        _Pragma("unroll") for (int b = 0; b < NB; ++b) bv[b] = *reinterpret_cast<const bf16x8 *>(        \
            &lx[BUF][(wm * (MT / 2) + b * 16 + lr) * ROWB + ks * 64 + lq * 16]);                         \
        _Pragma("unroll") for (int a = 0; a < 4; ++a) _Pragma("unroll") for (int b = 0; b < NB; ++b)     \
            acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[a], bv[b], acc[a][b], 0, 0, 0);       \
    }
    // Stage i: fetch stage i+3 into the ring, multiply stage i out of LDS buffer i%2, park
    // stage i+1 in the other buffer, barrier.  J = i mod 4 is a literal so that every ring
    // index is static; n_stage is a multiple of 4 (gemm_supported / gemm_split_k), and the
    // steady-state loop has no conditional loads so that outstanding loads are counted exactly.
#define DYN_GEMM_STAGE(J, FETCH, PARK)                                                                   \
    {                                                                                                    \
        if (FETCH) DYN_GEMM_FETCH(((J) + 3) % RING, st0 + (J) + 3)                                       \
        DYN_GEMM_MMA((J) % 2)                                                                            \
        if (PARK) DYN_GEMM_PARK(((J) + 1) % RING, ((J) + 1) % 2)                                         \
        __syncthreads();                                                                                 \
    }
    static_assert(RING == 4, "stages are written out four at a time");
    DYN_GEMM_FETCH(0, 0)
    DYN_GEMM_FETCH(1, 1)
    DYN_GEMM_FETCH(2, 2)
    DYN_GEMM_PARK(0, 0)
    __syncthreads();
    int st0 = 0;
    for (; st0 < n_stage - RING; st0 += RING) {
        DYN_GEMM_STAGE(0, true, true)
        DYN_GEMM_STAGE(1, true, true)
        DYN_GEMM_STAGE(2, true, true)
        DYN_GEMM_STAGE(3, true, true)
        DYN_GEMM_PLANE_END(st0 + RING)
    }
    DYN_GEMM_STAGE(0, true, true)
    DYN_GEMM_STAGE(1, false, true)
    DYN_GEMM_STAGE(2, false, true)
    DYN_GEMM_STAGE(3, false, false)
    DYN_GEMM_PLANE_END(st0 + RING)
#undef DYN_GEMM_PLANE_END
#undef DYN_GEMM_STAGE
#undef DYN_GEMM_MMA
#undef DYN_GEMM_PARK
#undef DYN_GEMM_FETCH

#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int m = m0 + wm * (MT / 2) + b * 16 + lr;
            const int n = n0 + wn * 64 + a * 16 + 4 * lq;
            if (m >= M) continue;
            const size_t orow = list ? list[m] : m;
            f32x4 o = INREG ? total[a][b] : acc[a][b];
            if ((S == 1 || INREG) && !gr.force_planes) {
                if (R) {
                    const u32x2 rv = *reinterpret_cast<const u32x2 *>(R + orow * N + n);
                    o[0] += bf2f(rv[0] & 0xffff); o[1] += bf2f(rv[0] >> 16);
                    o[2] += bf2f(rv[1] & 0xffff); o[3] += bf2f(rv[1] >> 16);
                }
                u32x2 ov;
                ov[0] = (uint32_t)f2bf(o[0]) | ((uint32_t)f2bf(o[1]) << 16);
                ov[1] = (uint32_t)f2bf(o[2]) | ((uint32_t)f2bf(o[3]) << 16);
                *reinterpret_cast<u32x2 *>(Y + orow * N + n) = ov;
            } else {
                *reinterpret_cast<f32x4 *>(P + (size_t)sp * plane_stride + orow * N + n) = o;
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
    return N > 0 && K > 0 && N % BN == 0 && K % (BK * RING) == 0;
}

int gemm_split_k(int dtype, int N, int K) {
    if (dtype == 0) return 1;
    // enough workgroups to occupy 256 CUs twice over, chunks of at least 8 k-steps
    static int forced = -1;
    if (forced < 0) { const char *e = getenv("DYN_GEMM_SPLIT"); forced = e ? atoi(e) : 0; }
    const int unit = BK * RING;                       // a plane is a multiple of RING stages
    int S = 1;
    while ((N / BN) * S < 192 && K % (S * 2 * unit) == 0 && K / (S * 2) >= 2 * unit) S *= 2;
    if (forced > 0 && K % (forced * unit) == 0) S = forced;
    return S;
}

hipError_t launch_gemm(int dtype, const void *X, int ldx, const void *W, const void *R, void *Y, float *partial,
                       size_t plane_stride, int rows, int N, int K, hipStream_t s, hipEvent_t mid) {
    if (rows <= 0) return hipSuccess;
    const GemmGroups none{};
    if (dtype == 0) {
        hipLaunchKernelGGL(gemm_f32_kernel, dim3((N + 63) / 64, (rows + 63) / 64), dim3(256), 0, s, (const float *)X, ldx,
                           (const float *)W, (const float *)R, (float *)Y, rows, N, K, none);
        hipError_t e0 = hipGetLastError();
        if (e0 == hipSuccess && mid) e0 = hipEventRecord(mid, s);
        return e0;
    }
    const int S = gemm_split_k(dtype, N, K);
    const int MT = rows <= 64 ? 64 : 128;
    const int m_tiles = (rows + MT - 1) / MT;
    const bool inreg = S > 1 && (N / BN) * m_tiles >= 256;      // enough tiles without spreading the planes
    const int ns = (N / BN) * (inreg ? 1 : S);
    const int grid = ((ns + 7) / 8) * 8 * m_tiles;
#define DYN_GEMM_LAUNCH(...)                                                                                        \
    hipLaunchKernelGGL((gemm_bf16_kernel<__VA_ARGS__>), dim3(grid), dim3(256), 0, s, (const bf16_t *)X, ldx,        \
                       (const bf16_t *)W, (const bf16_t *)R, (bf16_t *)Y, partial, plane_stride, rows, N, K, S, none)
    if (inreg) DYN_GEMM_LAUNCH(128, true, false);
    else if (MT == 64) DYN_GEMM_LAUNCH(64, false, false);
    else if (m_tiles >= DYN_OCC2_TILES) DYN_GEMM_LAUNCH(128, false, true);
    else DYN_GEMM_LAUNCH(128, false, false);
#undef DYN_GEMM_LAUNCH
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && mid) e = hipEventRecord(mid, s);
    if (e != hipSuccess || S == 1 || inreg) return e;
    const size_t n_vec = (size_t)rows * N / 4;
    const int blocks = (int)((n_vec + 255) / 256 < 2048 ? (n_vec + 255) / 256 : 2048);
    hipLaunchKernelGGL(gemm_reduce_kernel, dim3(blocks), dim3(256), 0, s, partial, plane_stride, (const bf16_t *)R,
                       (bf16_t *)Y, n_vec, S);
    return hipGetLastError();
}

// Expert-grouped form: group e multiplies the rows named by its list with its own weight
// matrix W + e * w_stride.  max_rows bounds any group's row count (it sizes the grid; tiles
// past a group's count exit at once).  X, Y and partial are indexed by the lists' row ids (not
// relative to the dispatch); the dispatch's output rows are row0 .. row0 + n_rows - 1.  With
// gr.force_planes the fp32 plane sums go to `partial` for every split factor, including 1, and
// nothing is written to Y.
hipError_t launch_gemm_grouped(int dtype, const void *X, int ldx, const void *W, void *Y, float *partial,
                               size_t plane_stride, const GemmGroups &gr, int max_rows, int row0, int n_rows, int N, int K,
                               hipStream_t s, hipEvent_t mid) {
    if (max_rows <= 0 || gr.n_groups <= 0) return hipSuccess;
    if (dtype == 0) {
        hipLaunchKernelGGL(gemm_f32_kernel, dim3((N + 63) / 64, (max_rows + 63) / 64, gr.n_groups), dim3(256), 0, s,
                           (const float *)X, ldx, (const float *)W, (const float *)nullptr,
                           gr.force_planes ? partial : (float *)Y, max_rows, N, K, gr);
        hipError_t e0 = hipGetLastError();
        if (e0 == hipSuccess && mid) e0 = hipEventRecord(mid, s);
        return e0;
    }
    const int S = gemm_split_k(dtype, N, K);
    const int MT = max_rows <= 64 ? 64 : 128;
    const int m_tiles = (max_rows + MT - 1) / MT;
    const int ns = (N / BN) * S * gr.n_groups;
    const int grid = ((ns + 7) / 8) * 8 * m_tiles;
    if (MT == 64)
        hipLaunchKernelGGL((gemm_bf16_kernel<64, false, false>), dim3(grid), dim3(256), 0, s, (const bf16_t *)X, ldx, (const bf16_t *)W,
                           (const bf16_t *)nullptr, (bf16_t *)Y, partial, plane_stride, max_rows, N, K, S, gr);
    else
        hipLaunchKernelGGL((gemm_bf16_kernel<128, false, false>), dim3(grid), dim3(256), 0, s, (const bf16_t *)X, ldx, (const bf16_t *)W,
                           (const bf16_t *)nullptr, (bf16_t *)Y, partial, plane_stride, max_rows, N, K, S, gr);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && mid) e = hipEventRecord(mid, s);
    if (e != hipSuccess || S == 1 || gr.force_planes) return e;
    // output rows row0 .. row0 + n_rows - 1 are exactly the rows the groups wrote
    const size_t n_vec = (size_t)n_rows * N / 4;
    const int blocks = (int)((n_vec + 255) / 256 < 2048 ? (n_vec + 255) / 256 : 2048);
    hipLaunchKernelGGL(gemm_reduce_kernel, dim3(blocks), dim3(256), 0, s, partial + (size_t)row0 * N, plane_stride,
                       (const bf16_t *)nullptr, (bf16_t *)Y + (size_t)row0 * N, n_vec, S);
    return hipGetLastError();
}

}  // namespace dyn

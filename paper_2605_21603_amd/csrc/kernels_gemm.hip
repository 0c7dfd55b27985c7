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

#include <algorithm>
#include <utility>
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
// Workgroup = NW waves (4 or 8) on a BN (W rows) x MT (X rows) output tile and one K plane (or,
// INREG, all planes in turn).  What bounds this kernel below a few hundred rows is not the matrix
// cores and not even HBM alone but the L2 -> CU path: every byte of W must cross it once and
// the X tile crosses it once per W tile, so both operands are fetched exactly once per
// workgroup, with fully coalesced 128-byte row segments (8 lanes per row), by direct
// global -> LDS loads (no registers in between) into a ring of NS stage buffers (a stage is
// 64 k); NS - 1 stages are in flight while one is multiplied, tracked with exact vmcnt waits
// and one barrier per stage.  A direct load places lane l's 16 bytes at l * 16 of the wave's
// 1 KB window, so rows sit at a 128-byte pitch; bank conflicts of the MFMA-layout reads
// (lane l: row l%16, 8 consecutive k at 8*(l/16)) are avoided by an XOR swizzle of the
// 16-byte column with bits 1..3 of the row, applied to the global column a lane fetches.
// Waves sit 2 (along X rows; 4 on the tall tiles) x NW/2 (along W rows) on the tile.
// D[i][j]: i = W row (4*(l/16)+r), j = X row (l%16).  Which tile a launch uses is gemm_path's
// decision: 128 x 64|128 with a ring of 4 for few rows, 128 x 256|384|512 for 129..512 rows,
// 256 x 256 for many rows without planes, 128 x 128|160 with two workgroups per CU otherwise.
//
// INREG: one workgroup walks all S planes of its tile and adds the plane sums in registers
// (same order, same bits as the plane buffers + gemm_reduce_kernel) - for many-row launches,
// where there are enough tiles to fill the chip without spreading planes over workgroups and
// the fp32 plane traffic would cost more than the weights.
constexpr int BK = 64, ROWB = BK * 2;
constexpr int kRotGroup = 32, kRotStep = 9;   // stage-order rotation of the bf16 kernel
constexpr int kBigBN = 128, kBigMT = 128, kBigNS = 2;   // tile and ring depth of the many-row (matrix-core-bound) regime

__device__ __forceinline__ void wait_vmcnt(int n) {          // s_waitcnt vmcnt(n) only; n folds to a literal <= 63
    // simm16: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14; expcnt 7 and lgkmcnt 15 = no wait
#define DYN_W(N) case N: __builtin_amdgcn_s_waitcnt(0x0f70 | ((N) & 15) | (((N) >> 4) << 14)); break;
    switch (n) {
        DYN_W(0) DYN_W(2) DYN_W(3) DYN_W(4) DYN_W(5) DYN_W(6) DYN_W(7) DYN_W(8) DYN_W(9) DYN_W(12) DYN_W(14) DYN_W(16) DYN_W(18) DYN_W(21) DYN_W(24) DYN_W(27) DYN_W(28) DYN_W(32)
        default: __builtin_amdgcn_s_waitcnt(0x0f70); break;       // unknown count: wait for everything
    }
#undef DYN_W
}

// The MFMA as inline assembly, so that the many-row loop's instruction order is the one written down.
// The compiler neither sees the instruction's latency nor orders anything around it: the caller keeps
// dependent uses of an accumulator far apart and waits before reading it as an ordinary register.
__device__ __forceinline__ void mfma_acc(f32x4 &c, const bf16x8 &a, const bf16x8 &b) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(c) : "v"(a), "v"(b));
}

template <int BN, int MT, bool INREG, int NS, bool GATED, int NW>
__global__ __launch_bounds__(NW * 64, (NW == 4 && (BN + MT) * ROWB * NS <= 72 * 1024) ? 2 : 1) void gemm_bf16_kernel(
    const bf16_t *__restrict__ X, int ldx, const bf16_t *__restrict__ W, const bf16_t *__restrict__ R,
    bf16_t *__restrict__ Y, int ldy, float *__restrict__ P, size_t plane_stride, int M, int N, int K, int S,
    GemmGroups gr) {
    constexpr int ROWS = BN + MT;                   // rows of a stage buffer: W rows, then X rows
    constexpr int WMW = (NW == 8 && BN < MT) ? 4 : 2;   // waves along m
    constexpr int WNW = NW / WMW, RW = BN / WNW;     // waves along n; W rows per wave column
    constexpr int LPS = ROWS / (NW * 8);            // direct loads per thread and stage (8 rows per wave instruction)
    static_assert(ROWS % (NW * 8) == 0, "the stage's rows must divide among the waves' direct loads");
    constexpr int STAGE = ROWS * ROWB;              // bytes; NS of them form the ring
    constexpr int NA = RW / 16, NB = MT / (16 * WMW);       // 16-row operand tiles per wave
    constexpr bool PIPE = MT >= 256;                // the hand-laid-out loop: it pays from 256-row tiles on (128-row tiles: 1-2 % slower with it)
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const int m_tiles = (M + MT - 1) / MT;
    // Workgroup ids are dealt round-robin to the 8 XCDs.  Tiles that share W rows (the
    // m tiles of one (n tile, plane)) get ids 8 apart: same XCD, same L2, adjacent in time.
    const int u = blockIdx.x % 8, v = blockIdx.x / 8;
    int m_tile = v % m_tiles;
    int ns = (v / m_tiles) * 8 + u;
    if (gr.n_groups) {
        // Expert-grouped launches size the grid for the largest possible group, so most tiles
        // past the first m tile are empty.  All first m tiles come first and the mostly empty
        // ones trail the launch (interleaved, every second workgroup was an empty one that
        // still had to wait for a free 128 KB LDS slot, and the launch took twice as long);
        // an m tile keeps the XCD of its n tile.
        const int per_m = gridDim.x / m_tiles;         // a multiple of 8
        m_tile = blockIdx.x / per_m;
        ns = blockIdx.x % per_m;
    }
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
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lr = lane & 15, lq = lane >> 4, wn = wave % WNW, wm = wave / WNW;

    // Direct load j of this wave covers stage rows (j * NW + wave) * 8 .. + 8; lane l fetches
    // row + l / 8, global 16-byte column (l % 8) ^ swizzle(row).
    const bf16_t *src[LPS];
#pragma unroll
    for (int j = 0; j < LPS; ++j) {
        const int row = (j * NW + wave) * 8 + (lane >> 3);
        const int col = (lane & 7) ^ ((row >> 1) & 7);
        if (row < BN) {
            int n = n0 + row;
            if (GATED) {   // stage row = wave half wn, then gate tiles, then up tiles
                const int wn_r = row / RW, in_w = row % RW, up = in_w / (RW / 2);
                n = n_tile * (BN / 2) + wn_r * (RW / 2) + in_w % (RW / 2) + up * (N / 2);
            }
            src[j] = W + (size_t)n * K + kbase + col * 8;
        } else {
            const int mr = min(m0 + row - BN, M - 1);
            src[j] = X + (size_t)(list ? list[mr] / gr.x_div : mr) * ldx + kbase + col * 8;
        }
    }
    // Stage order: the k stages of a plane are visited starting `rot` stages in and wrapping round,
    // with rot a function of the n tile (groups of kRotGroup tiles share one).  Workgroups that run
    // at the same time then read different column offsets of their 8 KB-pitched weight rows, which
    // spreads the requests over the memory channels; tiles of one group keep reading the same X
    // columns together, so X stays shared in L2.  The order depends on (N, K, n tile) only, never
    // on the number of rows, so every schedule adds the same terms in the same order.
    const int rot_group = (GATED ? n_tile * (BN / 2) / 64 : n0 / 128) / kRotGroup;   // by output column, the same for every tile shape
    const int rot = (int)(((unsigned)rot_group * kRotStep) % (unsigned)plane_stages);
    int iss_w = 0, iss_base = 0;                       // next stage to issue: index inside its plane, plane's first stage
    unsigned char *iss_buf = lds;                      // the pending stage's ring buffer and k offset (issue_begin / issue_one)
    int iss_kst = 0;
    auto issue_begin = [&](int st) {                   // stage st goes into ring buffer st % NS; st ascends by one per call
        iss_buf = lds + (st % NS) * STAGE;
        iss_kst = iss_w + rot;
        if (iss_kst >= plane_stages) iss_kst -= plane_stages;
        iss_kst += iss_base;
        if (++iss_w == plane_stages) { iss_w = 0; iss_base += plane_stages; }
    };
    auto issue_one = [&](int j) {                      // direct load j of the stage begun last
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src[j] + (size_t)iss_kst * BK),
                                         (__attribute__((address_space(3))) void *)(iss_buf + (j * NW + wave) * 8 * ROWB),
                                         16, 0, 0);
    };
    auto issue = [&](int st) {                         // all direct loads of stage st
        issue_begin(st);
#pragma unroll
        for (int j = 0; j < LPS; ++j) issue_one(j);
    };

    f32x4 acc[NA][NB], total[INREG ? NA : 1][INREG ? NB : 1];
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (INREG) total[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};
        }

    // operand read offsets inside a stage buffer (bytes), k-step 0; k-step 1 flips column bit 2
    int a_off[NA], b_off[NB];
#pragma unroll
    for (int a = 0; a < NA; ++a) {
        const int row = wn * RW + a * 16 + lr;
        a_off[a] = row * ROWB + ((lq ^ ((row >> 1) & 7)) << 4);
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int row = BN + wm * (MT / WMW) + b * 16 + lr;
        b_off[b] = row * ROWB + ((lq ^ ((row >> 1) & 7)) << 4);
    }

    auto fold_plane = [&](int st) {                    // a plane ends: fold its sum into the total, start from zero
        if (INREG && (st + 1) % plane_stages == 0) {
#pragma unroll
            for (int a = 0; a < NA; ++a)
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    total[a][b] += acc[a][b];
                    acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
        }
    };
    auto wait_stage = [&](int st) {                    // stage st has landed when at most the loads of the stages issued after it are outstanding
        const int ahead = min(NS - 2, n_stage - 1 - st);
        if (ahead >= 4) wait_vmcnt(4 * LPS);
        else if (ahead == 3) wait_vmcnt(3 * LPS);
        else if (ahead == 2) wait_vmcnt(2 * LPS);
        else if (ahead == 1) wait_vmcnt(LPS);
        else wait_vmcnt(0);
    };

    if constexpr (PIPE) {
        // Many rows: the matrix cores are the bound, and what keeps them waiting is everything that comes
        // in bursts - a block of operand reads before a block of MFMAs, all of a stage's direct loads
        // right after the barrier.  So the loop is laid out by hand, as inline assembly that the
        // compiler neither reorders nor waits for.  A stage is four steps, (k half 0 | 1) x (first |
        // second half of the wave's X tiles).  While the MFMAs of a step issue, the operands of the
        // next step are read from LDS, one read every few MFMAs, across the stage boundary too; the
        // direct loads of the stage that refills this stage's buffer are spread over the last step in
        // the same way.  When a step begins, all that is outstanding is what the previous step read,
        // so lgkmcnt(0) opens it (LDS reads return in order; nothing newer is in flight).  An
        // accumulator is used once per step, so dependent MFMAs are never close.  Every accumulator
        // still receives its k halves and stages in ascending order: the same bits as the plain loop.
        constexpr int H0 = (NB + 1) / 2, H1 = NB - H0, TILE = 16 * ROWB;   // X tiles of the first and of the second half
        bf16x8 a_cur[NA], a_nxt[NA], b_lo[H0], b_hi[H1];
        // Operand tile i of a kind sits 16 rows = TILE bytes after tile 0 (the swizzle depends on the
        // row's low four bits only), so one address per (kind, k half) and an immediate offset do.
        const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds;
        const unsigned a_adr[2] = {lds0 + (unsigned)a_off[0], lds0 + (unsigned)(a_off[0] ^ 64)};
        const unsigned b_adr[2] = {lds0 + (unsigned)b_off[0], lds0 + (unsigned)(b_off[0] ^ 64)};
        // The MFMAs of av x bv into accumulator columns b0 .. b0 + hb, with item(0) .. item(n_items - 1)
        // spread evenly between them.
        auto step = [&](const bf16x8 (&av)[NA], const auto &bv, auto b0, auto hb, auto n_items, auto &&item) {
            constexpr int B0 = decltype(b0)::value, M = NA * decltype(hb)::value, T = decltype(n_items)::value;
            static_for<0, M>([&](auto i) {
                constexpr int I = decltype(i)::value;
                mfma_acc(acc[I % NA][B0 + I / NA], av[I % NA], bv[I / NA]);
                static_for<0, T>([&](auto k) {
                    if constexpr (decltype(k)::value * M / T == I) item(k);
                });
            });
        };
        const std::integral_constant<int, 0> c0;
        const std::integral_constant<int, H0> ch0;
        const std::integral_constant<int, H1> ch1;
        // All NS ring buffers are filled before the loop; stage st + NS is issued into the buffer of
        // stage st once every wave has taken its last operands out of it.
#pragma unroll
        for (int d = 0; d < NS; ++d)
            if (d < n_stage) issue(d);
        {
            const int ahead = min(NS - 1, n_stage - 1);
            if (ahead >= 3) wait_vmcnt(3 * LPS);
            else if (ahead == 2) wait_vmcnt(2 * LPS);
            else if (ahead == 1) wait_vmcnt(LPS);
            else wait_vmcnt(0);
        }
        __builtin_amdgcn_s_barrier();
        static_for<0, NA>([&](auto k) { a_cur[decltype(k)::value] = lds_read16<decltype(k)::value * TILE>(a_adr[0]); });
        static_for<0, H0>([&](auto k) { b_lo[decltype(k)::value] = lds_read16<decltype(k)::value * TILE>(b_adr[0]); });
        for (int st = 0; st < n_stage; ++st) {
            const unsigned so = (unsigned)(st % NS) * STAGE;
            const unsigned a1 = a_adr[1] + so, b0 = b_adr[0] + so, b1 = b_adr[1] + so;
            wait_lgkmcnt<0>();
            step(a_cur, b_lo, c0, ch0, ch1, [&](auto k) {
                constexpr int K = decltype(k)::value;
                b_hi[K] = lds_read16<(H0 + K) * TILE>(b0);
            });
            wait_lgkmcnt<0>();
            step(a_cur, b_hi, ch0, ch1, std::integral_constant<int, NA + H0>(), [&](auto k) {
                constexpr int K = decltype(k)::value;
                if constexpr (K < NA) a_nxt[K] = lds_read16<K * TILE>(a1);
                else b_lo[K - NA] = lds_read16<(K - NA) * TILE>(b1);
            });
            wait_lgkmcnt<0>();
            step(a_nxt, b_lo, c0, ch0, ch1, [&](auto k) {
                constexpr int K = decltype(k)::value;
                b_hi[K] = lds_read16<(H0 + K) * TILE>(b1);
            });
            wait_lgkmcnt<0>();                     // this wave has taken its last operands out of stage st's buffer
            // One path for every stage, the last included (a second copy of the step's assembly would
            // give each accumulator two definitions to merge at the loop's head): after the last stage
            // the reads fetch operands nobody uses from the other ring buffer, and nothing is issued.
            wait_stage(st + 1);
            __builtin_amdgcn_s_barrier();          // every wave is done with the buffer and sees stage st + 1
            const unsigned no = (unsigned)((st + 1) % NS) * STAGE;
            const unsigned na = a_adr[0] + no, nb = b_adr[0] + no;
            const bool refill = st + NS < n_stage;
            if (refill) issue_begin(st + NS);
            // reads and direct loads alternate while both last, then the rest of the longer list
            constexpr int R = NA + H0, PAIRS = R < LPS ? R : LPS;
            step(a_nxt, b_hi, ch0, ch1, std::integral_constant<int, R + LPS>(), [&](auto k) {
                constexpr int K = decltype(k)::value;
                constexpr bool is_read = K < 2 * PAIRS ? K % 2 == 0 : R > LPS;
                constexpr int idx = K < 2 * PAIRS ? K / 2 : K - PAIRS;
                if constexpr (is_read) {
                    if constexpr (idx < NA) a_cur[idx] = lds_read16<idx * TILE>(na);
                    else b_lo[idx - NA] = lds_read16<(idx - NA) * TILE>(nb);
                } else {
                    if (refill) issue_one(idx);
                }
            });
            if (INREG && (st + 1) % plane_stages == 0) {
                // the compiler does not know that the assembly's results arrive late: the last MFMAs
                // must have left the pipeline before the accumulators are read as ordinary registers,
                // and the cleared accumulators must be written before the next MFMA reads them
                asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
                fold_plane(st);
                asm volatile("s_nop 7" ::: "memory");
            }
        }
        wait_lgkmcnt<0>();
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    } else {
#pragma unroll
    for (int d = 0; d < NS - 1; ++d)
        if (d < n_stage) issue(d);
    for (int st = 0; st < n_stage; ++st) {
        wait_stage(st);
        // Bare barrier: __syncthreads() would add a fence that drains every outstanding load, which
        // is exactly the prefetch.  The loads of stage st are complete (waited above) and, being
        // direct-to-LDS, visible once complete; the reads of stage st-1 were consumed by MFMAs.
        __builtin_amdgcn_s_barrier();
        if (st + NS - 1 < n_stage) issue(st + NS - 1);
        const unsigned char *buf = lds + (st % NS) * STAGE;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf16x8 av[NA], bv[NB];
#pragma unroll
            for (int a = 0; a < NA; ++a) av[a] = *reinterpret_cast<const bf16x8 *>(buf + (a_off[a] ^ (ks << 6)));
#pragma unroll
            for (int b = 0; b < NB; ++b) bv[b] = *reinterpret_cast<const bf16x8 *>(buf + (b_off[b] ^ (ks << 6)));
#pragma unroll
            for (int a = 0; a < NA; ++a)
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[a], bv[b], acc[a][b], 0, 0, 0);
        }
        fold_plane(st);
    }
    }

    if (GATED) {
#pragma unroll
        for (int a = 0; a < NA / 2; ++a)
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const int m = m0 + wm * (MT / WMW) + b * 16 + lr;
                const int n = n_tile * (BN / 2) + wn * (RW / 2) + a * 16 + 4 * lq;
                if (m >= M) continue;
                const size_t orow = list ? list[m] : m;
                const f32x4 g = acc[a][b], up = acc[a + NA / 2][b];
                float o[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) o[r] = g[r] / (1.0f + expf(-g[r])) * up[r];
                u32x2 ov;
                ov[0] = (uint32_t)f2bf(o[0]) | ((uint32_t)f2bf(o[1]) << 16);
                ov[1] = (uint32_t)f2bf(o[2]) | ((uint32_t)f2bf(o[3]) << 16);
                *reinterpret_cast<u32x2 *>(Y + orow * ldy + n) = ov;
            }
        return;
    }
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int m = m0 + wm * (MT / WMW) + b * 16 + lr;
            const int n = n0 + wn * RW + a * 16 + 4 * lq;
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

template <int BN, int MT, bool INREG, int NS, bool GATED = false, int NW = 4>
hipError_t launch_gemm_bf16(int grid, hipStream_t s, const void *X, int ldx, const void *W, const void *R, void *Y,
                            float *partial, size_t plane_stride, int rows, int N, int K, int S, const GemmGroups &gr,
                            int ldy = 0) {
    constexpr int STAGE = (BN + MT) * ROWB;
    static_assert(NS >= 2 && NS <= 6 && NS * STAGE <= 160 * 1024, "ring does not fit in LDS");
    static bool attr_set = false;                      // above 64 KB of dynamic LDS needs an opt-in, once
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)gemm_bf16_kernel<BN, MT, INREG, NS, GATED, NW>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, NS * STAGE);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((gemm_bf16_kernel<BN, MT, INREG, NS, GATED, NW>), dim3(grid), dim3(NW * 64), NS * STAGE, s,
                       (const bf16_t *)X, ldx, (const bf16_t *)W, (const bf16_t *)R, (bf16_t *)Y, ldy ? ldy : N, partial,
                       plane_stride, rows, N, K, S, gr);
    return hipGetLastError();
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

// Matrix-core probe: the main loop of the 256 x 256-tile kernel above without its indexing - eight
// waves, one workgroup per CU, and per stage and wave 64 MFMAs with 24 operand reads from LDS spread
// between them, one barrier, and eight direct loads (64 KB per workgroup) that refill the other
// stage buffer - on operands that are whatever the caller's buffer holds.  Every workgroup walks a
// 256 KB window of the first 16 MiB of the buffer again and again, so the loads hit L2.  What it
// reaches is what the chip gives a loop of this shape with a schedule that has nothing left to
// improve; it depends on the operands (the chip lowers its clock with the activity of its matrix
// pipes: zeros run a third faster than random values), which is why the caller supplies them.
constexpr size_t kMfmaProbeBytes = (size_t)16 << 20;
__global__ __launch_bounds__(512) void mfma_loop_probe_kernel(const unsigned char *__restrict__ src, int n_stages, float *__restrict__ sink) {
    constexpr int STAGE = 65536;
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int row = (lane & 15) + (wave & 3) * 64;
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)lds;
    const unsigned addr = lds0 + row * 128 + (((lane >> 4) ^ ((row >> 1) & 7)) << 4);       // conflict-free 16-byte reads, as the projections' operand reads
    const unsigned addr1 = addr ^ 64;                  // k half 1: the other half of the 128-byte row
    const unsigned char *gsrc = src + (size_t)(blockIdx.x % 64) * 262144 + wave * 1024 + lane * 16;
    auto load = [&](int st, int j) {        // 1 KB per wave: part j of stage st's 64 KB; offsets stay below 16 MiB and inside the two stage buffers
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gsrc + ((st * 8 + j) & 31) * 8192),
                                         (__attribute__((address_space(3))) void *)(lds + (st & 1) * STAGE + (j * 8 + wave) * 1024), 16, 0, 0);
    };
    f32x4 acc[32];
    bf16x8 fa[2][4], fb[2][8];
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 8; ++j) load(0, j);
    wait_vmcnt(0);
    __builtin_amdgcn_s_barrier();
    static_for<0, 4>([&](auto i) { fa[0][decltype(i)::value] = lds_read16<decltype(i)::value * 2048>(addr); });
    static_for<0, 8>([&](auto i) { fb[0][decltype(i)::value] = lds_read16<16384 + decltype(i)::value * 2048>(addr); });
    for (int st = 0; st < n_stages; ++st) {
        const unsigned so1 = addr1 + (st & 1) * STAGE, sn = addr + ((st + 1) & 1) * STAGE;
        // k half 0: its MFMAs, with the reads of k half 1 and the direct loads of the next stage between them
        wait_lgkmcnt<0>();
        static_for<0, 32>([&](auto i) {
            constexpr int I = decltype(i)::value;
            mfma_acc(acc[I], fa[0][I & 3], fb[0][I >> 2]);
            if constexpr (I % 8 == 1 && I / 8 < 4) fa[1][I / 8] = lds_read16<(I / 8) * 2048>(so1);
            if constexpr (I % 4 == 3) fb[1][I / 4] = lds_read16<16384 + (I / 4) * 2048>(so1);
            if constexpr (I % 4 == 2) load(st + 1, I / 4);
        });
        // k half 1; the next stage's buffer is complete once every wave has waited for its loads and passed the barrier
        wait_lgkmcnt<0>();
        wait_vmcnt(0);
        __builtin_amdgcn_s_barrier();
        static_for<0, 32>([&](auto i) {
            constexpr int I = decltype(i)::value;
            mfma_acc(acc[I], fa[1][I & 3], fb[1][I >> 2]);
            if constexpr (I % 8 == 1 && I / 8 < 4) fa[0][I / 8] = lds_read16<(I / 8) * 2048>(sn);
            if constexpr (I % 4 == 3) fb[0][I / 4] = lds_read16<16384 + (I / 4) * 2048>(sn);
        });
    }
    wait_lgkmcnt<0>();
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    float v = 0.f;
#pragma unroll
    for (int i = 0; i < 32; ++i) v += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    sink[(size_t)blockIdx.x * 512 + tid] = v;        // keeps the products alive
}

size_t mfma_probe_bytes() { return kMfmaProbeBytes; }
double mfma_probe_flops(int n_stages) { return 256.0 * 8 * n_stages * 64 * (16.0 * 16 * 32 * 2); }

hipError_t launch_mfma_probe(const void *buf, int n_stages, float *sink, hipStream_t s) {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)mfma_loop_probe_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * 65536);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(mfma_loop_probe_kernel, dim3(256), dim3(512), 2 * 65536, s, (const unsigned char *)buf, n_stages, sink);
    return hipGetLastError();
}

bool gemm_supported(int dtype, int N, int K) {
    if (dtype == 0) return N > 0 && K > 0;
    return N > 0 && K > 0 && N % 128 == 0 && K % BK == 0;
}

int gemm_split_k(int dtype, int N, int K, int groups) {
    if (dtype == 0) return 1;
    // enough workgroups to occupy 256 CUs twice over, chunks of at least 8 k-steps
    // planes of at least four stages; enough (128-row tile, plane) pairs to occupy the chip
    int S = 1;
    while ((N / 128) * S * std::max(groups, 1) < 192 && K % (S * 2 * BK) == 0 && K / (S * 2) >= 4 * BK * 2) S *= 2;
    return S;
}

namespace {
bool gemm_many_rows(int rows, int N) {      // enough 128 x 128 tiles for the many-row regime
    return N % kBigBN == 0 && (N / kBigBN) * ((rows + kBigMT - 1) / kBigMT) >= 256;
}

// 256 x 256 tiles, eight waves of 64 x 128 each: half the operand bytes moved into LDS per FLOP
// of the 128 x 128 tile.  They pay once there are at
// least two m tiles and enough tiles to fill the chip (2112 x 28672 x 4096: 519 -> 432 us; 512
// rows: 164 -> 121 us; 400 rows: 128 us with a 512-row tall tile, 120 us here).  Not for planes
// folded in registers: the second accumulator set does not fit.
bool gemm_wide_tiles(int rows, int N) { return N % 256 == 0 && rows >= 385 && (N / 256) * ((rows + 255) / 256) >= 192; }

// Tile height of the tall-tile path for a launch of `rows` rows with split factor S (0: another path).
int gemm_tall_rows(int rows, int S, int N, int K) {
    if (rows <= 128 || N % 128) return 0;
    if (rows <= 256) return 256;
    if (S == 1) {
        // Without planes because the n tiles alone fill the chip (gate/up): one tall tile up to 384
        // rows (at 264..320 rows 134-137 us with three 128-row tiles, 108-111 us with one of 384),
        // then the 256 x 256 tile where it applies (400..440 rows: 140-144 us -> 120; a 512-row tall
        // tile took 128).  Without planes because the depth is too short to split: as measured before.
        if (N / 128 < 192) return rows > 320 && rows <= 384 ? 384 : 0;
        return rows <= 384 ? 384 : 0;
    }
    if (rows <= 384) return 384;
    if (rows <= 512) return 512;
    if (rows > 1280) return 0;                  // 1025..1280 rows: two 512-row tiles and a launch for the rest (gemm_path)
    // 513..1024 rows with planes.  Folding planes in registers (the many-row path) wins once it is
    // available, unless its tiles fill only one of the two workgroup slots per CU and the plane
    // traffic is small next to the contraction (S / K small: the down projection; 1024 rows: 212 ->
    // 148 us, while qkv and o stay with the folded path: 79 and 66 us against 99 and 81).
    const bool folded_ok = gemm_many_rows(rows, N);
    const bool half_filled = (N / kBigBN) * ((rows + kBigMT - 1) / kBigMT) < 512;
    if (folded_ok && !(half_filled && K >= 1400 * S)) return 0;
    if (rows > 1024) return folded_ok ? 512 : 0;
    return (rows + 383) / 384 <= (rows + 511) / 512 ? 384 : 512;
}

}  // namespace

GemmPath gemm_path(int dtype, int rows, int N, int K) {
    GemmPath p{};
    p.split = gemm_split_k(dtype, N, K);
    const int S = p.split, nt = N / 128;
    const int tall = gemm_tall_rows(rows, S, N, K);
    if (tall) {
        // 129..512 rows (up to 1024 with planes, see gemm_tall_rows): tall tiles.  Two to four
        // 128-row tiles would move every weight byte into LDS that many times; one tile of 256, 384
        // or 512 rows (eight waves 4 x 2) moves it once: qkv / o / gate-up / down at 256 rows 41 / 34 /
        // 90 / 60 us -> 33 / 28 / 79 / 48 us, o and down at 512 rows 61 / 112 -> 45 / 84 us.  Same planes,
        // same k order, so the same bits.  Without planes the 256 x 256 tile takes over at 385 rows.
        p.kind = GEMM_TALL; p.bn = 128; p.mt = tall;
        // past 1024 rows (the down projection only, see gemm_tall_rows): a third 512-row tile would
        // be a third round of workgroups for at most 256 rows, so those run as a launch of their own
        // (1032 / 1280 rows: 209 / 211 us with planes folded in registers, ~170 this way)
        if (rows > 1024) { p.tail_rows = rows - 1024; rows = 1024; }
        p.workgroups = nt * S * ((rows + tall - 1) / tall);
        p.resident = 256;
        return p;
    }
    // Many-row launches are bound by the matrix cores: enough tiles without spreading planes over
    // workgroups, a shallow ring and two workgroups per CU so that one multiplies while the other
    // waits at its barrier.  Few-row launches are bound by memory: deep ring, one workgroup per CU.
    if (gemm_many_rows(rows, N)) {
        p.folded = S > 1;
        if (S == 1 && gemm_wide_tiles(rows, N)) {
            p.kind = GEMM_WIDE; p.bn = 256; p.mt = 256;
            // 256 tiles run at a time.  When the last m tile alone costs a further round of them,
            // its rows go to a launch of their own on 128-row-wide tiles (one round of N / 128
            // workgroups, shorter than a round here): 520..768 rows of gate/up 208-223 us -> ~180.
            const int m = (rows + 255) / 256, per_m = N / 256;
            if (m >= 3 && (per_m * m + 255) / 256 > (per_m * (m - 1) + 255) / 256) p.tail_rows = rows - 256 * (m - 1);
            p.workgroups = per_m * (p.tail_rows ? m - 1 : m);
            p.resident = 256;
            return p;
        }
        // Tile height: two workgroups fit a CU, so 512 tiles run at a time and the launch takes
        // ceil(tiles / 512) rounds of a duration proportional to the tile height.  A taller
        // tile that saves a round wins (2112 rows x 4096 columns: 544 tiles of 128 rows need
        // two rounds, 448 tiles of 160 rows one).  The summation order of an output element
        // does not depend on the tile height.
        const long cost128 = (long)((nt * ((rows + 127) / 128) + 511) / 512) * 128;
        const long cost160 = (long)((nt * ((rows + 159) / 160) + 511) / 512) * 160;
        p.kind = GEMM_MANY; p.bn = 128; p.mt = cost160 < cost128 ? 160 : 128;
        p.workgroups = nt * ((rows + p.mt - 1) / p.mt);
        p.resident = 512;
        return p;
    }
    p.kind = GEMM_FEW; p.bn = 128; p.mt = rows <= 64 ? 64 : 128;
    p.workgroups = nt * S * ((rows + p.mt - 1) / p.mt);
    p.resident = 256;
    return p;
}

bool gemm_uses_plane_buffer(int dtype, int rows, int N, int K) {
    if (dtype == 0 || rows <= 0) return false;
    const GemmPath p = gemm_path(dtype, rows, N, K);
    return p.split > 1 && !p.folded;
}

namespace {
// The operator that follows the projection, as a kernel of its own on the rows the projection wrote.
hipError_t run_epilogue(int dtype, const GemmEpilogue &ep, void *Y, int rows, int N, hipStream_t s) {
    if (ep.kind == GemmEpilogue::NORM) return launch_rmsnorm(dtype, Y, ep.g, ep.h_out, ep.ld_h, rows, N, ep.eps, s);
    if (ep.kind == GemmEpilogue::ROPE)
        return launch_rope_kv(dtype, Y, ep.seq_of_token, ep.pos_of_token, ep.block_table, ep.k_cache, ep.v_cache, *ep.rope, *ep.shape, rows, s);
    return hipSuccess;
}

GemmEpilogue epilogue_at(const GemmEpilogue &ep, int dtype, int row, int N) {      // the same epilogue for rows starting `row` rows in
    GemmEpilogue e = ep;
    const size_t es = dtype == 0 ? 4 : 2;
    if (e.kind == GemmEpilogue::NORM) e.h_out = (char *)e.h_out + (size_t)row * e.ld_h * es;
    if (e.kind == GemmEpilogue::ROPE) { e.seq_of_token += row; e.pos_of_token += row; }
    (void)N;
    return e;
}
}  // namespace

hipError_t launch_gemm(int dtype, const void *X, int ldx, const void *W, const void *R, void *Y, float *partial,
                       size_t plane_stride, int rows, int N, int K, hipStream_t s, hipEvent_t mid, const GemmEpilogue *ep) {
    if (rows <= 0) return hipSuccess;
    const GemmGroups none{};
    const bool has_ep = ep && ep->kind != GemmEpilogue::NONE;
    if (dtype == 0) {
        hipLaunchKernelGGL(gemm_f32_kernel, dim3((N + 63) / 64, (rows + 63) / 64), dim3(256), 0, s, (const float *)X, ldx,
                           (const float *)W, (const float *)R, (float *)Y, rows, N, K, none);
        hipError_t e0 = hipGetLastError();
        if (e0 == hipSuccess && mid) e0 = hipEventRecord(mid, s);
        if (e0 == hipSuccess && has_ep) e0 = run_epilogue(dtype, *ep, Y, rows, N, s);
        return e0;
    }
    const GemmPath p = gemm_path(dtype, rows, N, K);
    if (p.tail_rows) {         // the last rows in a launch of their own (own tiles, own planes and reduce)
        const int head = rows - p.tail_rows;
        GemmEpilogue tail_ep;
        if (has_ep) tail_ep = epilogue_at(*ep, dtype, head, N);
        hipError_t et = launch_gemm(dtype, (const bf16_t *)X + (size_t)head * ldx, ldx, W, R ? (const bf16_t *)R + (size_t)head * N : nullptr,
                                    (bf16_t *)Y + (size_t)head * N, partial ? partial + (size_t)head * N : nullptr, plane_stride,
                                    p.tail_rows, N, K, s, nullptr, has_ep ? &tail_ep : nullptr);
        if (et != hipSuccess) return et;
        rows = head;
    }
    const int S = p.split, m_tiles = (rows + p.mt - 1) / p.mt;
    // workgroup ids are dealt to the 8 XCDs in turn: (n tile, plane) pairs are padded to a multiple of 8
    const int grid = (((N / p.bn) * (p.folded ? 1 : S) + 7) / 8) * 8 * m_tiles;
#define DYN_GEMM(BN, MT, INREG, NS, NW) \
    launch_gemm_bf16<BN, MT, INREG, NS, false, NW>(grid, s, X, ldx, W, R, Y, partial, plane_stride, rows, N, K, S, none)
    hipError_t e;
    if (p.kind == GEMM_TALL) e = p.mt == 256 ? DYN_GEMM(128, 256, false, 3, 8) : p.mt == 384 ? DYN_GEMM(128, 384, false, 2, 8) : DYN_GEMM(128, 512, false, 2, 8);
    else if (p.kind == GEMM_WIDE) e = DYN_GEMM(256, 256, false, 2, 8);
    else if (p.kind == GEMM_MANY && p.mt == 160) e = p.folded ? DYN_GEMM(kBigBN, 160, true, kBigNS, 4) : DYN_GEMM(kBigBN, 160, false, kBigNS, 4);
    else if (p.kind == GEMM_MANY) e = p.folded ? DYN_GEMM(kBigBN, kBigMT, true, kBigNS, 4) : DYN_GEMM(kBigBN, kBigMT, false, kBigNS, 4);
    else e = p.mt == 64 ? DYN_GEMM(128, 64, false, 4, 8) : DYN_GEMM(128, 128, false, 4, 8);
#undef DYN_GEMM
    if (e == hipSuccess && mid) e = hipEventRecord(mid, s);
    if (e != hipSuccess) return e;
    if (S == 1 || p.folded) return has_ep ? run_epilogue(dtype, *ep, Y, rows, N, s) : hipSuccess;
    // the planes are summed in plane order, with the residual; where an operator follows on the same rows, by its fused form
    if (has_ep && ep->kind == GemmEpilogue::NORM && N % 8 == 0)
        return launch_reduce_norm(partial, plane_stride, S, R, Y, ep->g, ep->h_out, ep->ld_h, rows, N, ep->eps, s);
    if (has_ep && ep->kind == GemmEpilogue::ROPE && !R && reduce_rope_supported(dtype, *ep->shape))
        return launch_reduce_rope(partial, plane_stride, S, Y, ep->seq_of_token, ep->pos_of_token, ep->block_table, ep->k_cache,
                                  ep->v_cache, *ep->rope, *ep->shape, rows, s);
    const size_t n_vec = (size_t)rows * N / 4;
    const int blocks = (int)((n_vec + 255) / 256 < 2048 ? (n_vec + 255) / 256 : 2048);
    hipLaunchKernelGGL(gemm_reduce_kernel, dim3(blocks), dim3(256), 0, s, partial, plane_stride, (const bf16_t *)R,
                       (bf16_t *)Y, n_vec, S);
    e = hipGetLastError();
    if (e == hipSuccess && has_ep) e = run_epilogue(dtype, *ep, Y, rows, N, s);
    return e;
}

namespace {
// Tile of an expert-grouped launch, from the average number of rows per group (the lists' capacity
// holds every row once).  Few rows per expert stream the weights through 128-row tiles; from about
// 100 rows a second 128-row tile per expert would move its weights into LDS again, so the tile
// grows with the rows: one 256-row tall tile up to about 200 rows, 256 x 256 tiles beyond (eight
// experts' gate/up at 512 / 1024 / 2048 tokens: 593 / 989 / 1847 us with 128-row tiles).  The
// grid still covers max_rows per group; tiles past a group's count exit at once.
struct GroupTile { int bn, mt; };
GroupTile gemm_group_tile(const GemmGroups &gr, int max_rows, int N) {
    if (max_rows <= 64) return {128, 64};
    const int avg = gr.cap / (gr.n_groups > 0 ? gr.n_groups : 1);
    if (avg <= 100 || max_rows <= 128) return {128, 128};
    if (avg <= 200 || N % 256) return {128, 256};
    return {256, 256};
}
}  // namespace

bool gemm_gated_supported(int dtype, int N2, int K) { return dtype == 1 && gemm_split_k(dtype, N2, K) == 1; }

// act[rows or listed rows, N2/2] = silu(X Wg^T) * (X Wu^T) with W = [gate rows; up rows] ([N2, K]),
// output row pitch ldy.  Plain (gr.n_groups = 0: X, Y offset to the dispatch) or expert-grouped.
hipError_t launch_gemm_gated(const void *X, int ldx, const void *W, void *Y, int ldy, const GemmGroups &gr, int max_rows,
                             int N2, int K, hipStream_t s, hipEvent_t mid) {
    if (max_rows <= 0) return hipSuccess;
    hipError_t e;
#define DYN_GATED(BN, MT, NS, NW) \
    launch_gemm_bf16<BN, MT, false, NS, true, NW>(grid, s, X, ldx, W, nullptr, Y, nullptr, 0, max_rows, N2, K, 1, gr, ldy)
    if (gr.n_groups) {
        const GroupTile t = gemm_group_tile(gr, max_rows, N2);
        const int grid = ((((N2 / t.bn) * gr.n_groups) + 7) / 8) * 8 * ((max_rows + t.mt - 1) / t.mt);
        e = t.bn == 256 ? DYN_GATED(256, 256, 2, 8) : t.mt == 256 ? DYN_GATED(128, 256, 3, 8) : t.mt == 64 ? DYN_GATED(128, 64, 4, 8) : DYN_GATED(128, 128, 4, 8);
    } else {
        const GemmPath p = gemm_path(1, max_rows, N2, K);          // split factor 1: no planes on any path
        if (p.tail_rows) {     // the last rows in a launch of their own (never a wide one: at most 256 rows)
            const int head = max_rows - p.tail_rows;
            e = launch_gemm_gated((const bf16_t *)X + (size_t)head * ldx, ldx, W, (bf16_t *)Y + (size_t)head * ldy, ldy, gr,
                                  p.tail_rows, N2, K, s, nullptr);
            if (e != hipSuccess) return e;
            max_rows = head;
        }
        const int mt = p.kind == GEMM_MANY ? kBigMT : p.mt;    // the gated many-row kernel has 128-row tiles only
        const int grid = ((N2 / p.bn + 7) / 8) * 8 * ((max_rows + mt - 1) / mt);
        if (p.kind == GEMM_TALL) e = p.mt == 256 ? DYN_GATED(128, 256, 3, 8) : DYN_GATED(128, 384, 2, 8);
        else if (p.kind == GEMM_WIDE) e = DYN_GATED(256, 256, 2, 8);
        else if (p.kind == GEMM_MANY) e = DYN_GATED(kBigBN, kBigMT, kBigNS, 4);
        else e = p.mt == 64 ? DYN_GATED(128, 64, 4, 8) : DYN_GATED(128, 128, 4, 8);
    }
#undef DYN_GATED
    if (e == hipSuccess && mid) e = hipEventRecord(mid, s);
    return e;
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
    const int S = gemm_split_k(dtype, N, K, gr.n_groups);
    GroupTile t = gemm_group_tile(gr, max_rows, N);
    if (S > 1 && t.bn == 256) t = {128, 256};          // the 256 x 256 tile has no planes
    const int m_tiles = (max_rows + t.mt - 1) / t.mt;
    const int ns = (N / t.bn) * S * gr.n_groups;
    const int grid = ((ns + 7) / 8) * 8 * m_tiles;
    hipError_t e;
#define DYN_GROUPED(BN, MT, NS) launch_gemm_bf16<BN, MT, false, NS, false, 8>(grid, s, X, ldx, W, nullptr, Y, partial, plane_stride, max_rows, N, K, S, gr)
    e = t.bn == 256 ? DYN_GROUPED(256, 256, 2) : t.mt == 256 ? DYN_GROUPED(128, 256, 3) : t.mt == 64 ? DYN_GROUPED(128, 64, 4) : DYN_GROUPED(128, 128, 4);
#undef DYN_GROUPED
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

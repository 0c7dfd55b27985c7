// Host-side launch functions of the gfx950 kernels.  Each takes pointers already offset to
// the first token row of the dispatch and the number of rows; none synchronises or
// allocates.  dtype is DYN_F32 (0) or DYN_BF16 (1).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace dyn {

constexpr int kMaxHalfDim = 128;   // rotary tables are passed by value: head_dim <= 256

struct RopeTable {                 // theta_i = base^(-2i/d), i < d/2, computed on the host in fp64
    double inv_freq[kMaxHalfDim];
};

struct AttnShape {
    int n_q, n_kv, head_dim, page_size;
    int max_pages_per_seq;         // block-table row length
    int chunk_pages;               // pages per split-KV chunk (a constant of the layer)
    int max_chunks;                // chunks that fit max_pages_per_seq: stride of the partial arrays
    int n_cus;                     // CUs of the stream's partition (0: whole device); sizes the persistent launch
};

// Expert grouping of a projection (all fields zero: plain GEMM).  Group e has counts[e] rows;
// row i of the group reads X row lists[e * cap + i] / x_div and writes output row
// lists[e * cap + i]; its weights start w_stride elements after the previous group's.
struct GemmGroups {
    const int32_t *counts;
    const int32_t *lists;
    int cap, x_div, n_groups;
    size_t w_stride;
    int force_planes;
};

// Split-K factor of a GEMM with output width N and depth K.  A function of (N, K) alone so
// that a row's summation order never depends on how many rows are in flight.
// Expert-grouped projections multiply `groups` matrices in one launch and need fewer planes each.
int gemm_split_k(int dtype, int N, int K, int groups = 1);
bool gemm_supported(int dtype, int N, int K);
// How launch_gemm runs a plain bf16 projection of `rows` rows (the launcher follows this, and the
// scheduler's cost model prices it).
enum { GEMM_FEW = 0, GEMM_TALL = 1, GEMM_WIDE = 2, GEMM_MANY = 3 };
struct GemmPath {
    int kind;          // GEMM_FEW: 128 x 64|128 tiles, ring of 4; GEMM_TALL: 128 x 256|384|512, eight waves;
                       // GEMM_WIDE: 256 x 256, eight waves; GEMM_MANY: 128 x 128|160, two workgroups per CU
    int bn, mt;        // tile: W rows x X rows
    int split;         // split-K factor S(N, K)
    bool folded;       // planes accumulated one after another in registers: no plane buffer, no reduce kernel
    int workgroups;    // tiles x planes spread over the grid
    int resident;      // workgroups the chip's 256 CUs hold at a time
    int tail_rows;     // this many last rows run as a launch of their own (its path: gemm_path of that many rows);
                       // workgroups counts the first launch only
};
GemmPath gemm_path(int dtype, int rows, int N, int K);
// True if launch_gemm on `rows` rows writes split-K planes to `partial` (false: one plane, or planes folded in registers).
bool gemm_uses_plane_buffer(int dtype, int rows, int N, int K);

// ld_out: elements between output rows (>= H).
hipError_t launch_rmsnorm(int dtype, const void *x, const void *g, void *out, int ld_out, int rows, int H, float eps,
                          hipStream_t s);

// What follows a projection on the same token rows and is applied by the same launch sequence,
// so that its input never makes a round trip through a kernel of its own: the RMSNorm of the
// output rows (after the o and down projections) or rotary + cache append (after the qkv
// projection).  Where the projection's split-K planes are summed by a reduce kernel, that kernel
// applies it (one pass over the planes); otherwise the operator's own kernel runs on the rows the
// projection wrote.  Either way every element sees the same arithmetic in the same order.
struct GemmEpilogue {
    enum { NONE = 0, NORM = 1, ROPE = 2 } kind = NONE;
    // NORM: h_out[row] = RMSNorm(Y[row]) * g, row pitch ld_h
    const void *g = nullptr;
    void *h_out = nullptr;
    int ld_h = 0;
    float eps = 0.f;
    // ROPE: rotary on the q and k heads of the Y rows (q in place), k' and v appended to the cache
    const int32_t *seq_of_token = nullptr, *pos_of_token = nullptr, *block_table = nullptr;
    void *k_cache = nullptr, *v_cache = nullptr;
    const RopeTable *rope = nullptr;
    const AttnShape *shape = nullptr;
};

// Y[rows,N] = X[rows,K] W[N,K]^T (+ R[rows,N]); ldx = elements between rows of X (>= K).  partial: fp32 scratch for split-K planes,
// plane p at partial + p * plane_stride (elements); unused when the split factor is 1.
// If mid is not NULL it is recorded after the contraction kernel, before the split-K reduce.
hipError_t launch_gemm(int dtype, const void *X, int ldx, const void *W, const void *R, void *Y, float *partial,
                       size_t plane_stride, int rows, int N, int K, hipStream_t s, hipEvent_t mid = nullptr,
                       const GemmEpilogue *ep = nullptr);

hipError_t launch_gemm_grouped(int dtype, const void *X, int ldx, const void *W, void *Y, float *partial,
                               size_t plane_stride, const GemmGroups &gr, int max_rows, int row0, int n_rows, int N, int K,
                               hipStream_t s, hipEvent_t mid = nullptr);

// Gate/up projection with the SiLU gate applied in the epilogue (bf16, split factor 1 only):
// Y[row, N2/2] = silu(X Wg^T) * (X Wu^T), row pitch ldy.  gr.n_groups = 0: plain, pointers offset to
// the dispatch's first row, max_rows rows.  Grouped: as launch_gemm_grouped.
bool gemm_gated_supported(int dtype, int N2, int K);
hipError_t launch_gemm_gated(const void *X, int ldx, const void *W, void *Y, int ldy, const GemmGroups &gr, int max_rows,
                             int N2, int K, hipStream_t s, hipEvent_t mid = nullptr);

// MoE router for token rows: logits = h W_r^T in fp32, top_k largest (ties to the lower index),
// softmax over the selected logits.  sel / wgt are [rows, top_k], largest logit first.
hipError_t launch_route(int dtype, const void *h, int ldh, const float *w_router, int32_t *sel, float *wgt, int rows,
                        int H, int E, int top_k, hipStream_t s);

// Per-expert lists of (token, rank) pairs p = t * top_k + j in ascending p, for the rows of one
// dispatch: counts[E], lists[E, cap].  pair_base = first pair id of the dispatch.
hipError_t launch_expert_lists(const int32_t *sel, int n_pairs, int pair_base, int E, int cap, int32_t *counts,
                               int32_t *lists, hipStream_t s);

// y[t] = x2[t] + sum_j wgt[t, j] * (sum_p planes[p][t * top_k + j]) in rank order j, planes in order p.
hipError_t launch_moe_combine(int dtype, const float *planes, size_t plane_stride, int S, const float *wgt,
                              const void *x2, void *y, int rows, int H, int top_k, hipStream_t s);

// Rotary on the q and k heads of qkv rows (in place for q) and cache append of k', v.
hipError_t launch_rope_kv(int dtype, void *qkv, const int32_t *seq_of_token, const int32_t *pos_of_token,
                          const int32_t *block_table, void *k_cache, void *v_cache, const RopeTable &tab,
                          const AttnShape &sh, int rows, hipStream_t s);

// Causal paged attention for token rows; part_o / part_ml are the split-KV partial arrays
// ([rows, n_q, max_chunks, head_dim] and [rows, n_q, max_chunks, 2]); plan is scratch for the
// device-built work lists (2 * (2 + 2 * rows * max_chunks) int32); any_multi: some sequence has more
// than one token in these rows (host knowledge; enables the wide-group launch).
hipError_t launch_attention(int dtype, const void *qkv, const int32_t *seq_of_token, const int32_t *pos_of_token,
                            const int32_t *block_table, const void *k_cache, const void *v_cache, void *out, int ld_out,
                            float *part_o, float *part_ml, int32_t *plan, bool any_multi, const AttnShape &sh,
                            int rows, hipStream_t s, hipEvent_t mid = nullptr,    // mid: recorded between the chunk kernel and the combine
                            hipEvent_t pre = nullptr,   // pre: recorded after the work-list kernel, before the chunk kernel
                            bool plan_ready = false);   // `plan` already holds the lists of these rows (built by an earlier layer's call)

// out[rows, I] = silu(gu[:, :I]) * gu[:, I:]
hipError_t launch_silu_mul(int dtype, const void *gu, void *out, int ld_out, int rows, int I, hipStream_t s);

// The split-K reduce of a projection fused with what follows it (bf16; used by launch_gemm).
hipError_t launch_reduce_norm(const float *P, size_t plane_stride, int S, const void *R, void *Y, const void *g, void *out,
                              int ld_out, int rows, int H, float eps, hipStream_t s);
bool reduce_rope_supported(int dtype, const AttnShape &sh);
hipError_t launch_reduce_rope(const float *P, size_t plane_stride, int S, void *qkv, const int32_t *seq_of_token,
                              const int32_t *pos_of_token, const int32_t *block_table, void *k_cache, void *v_cache,
                              const RopeTable &tab, const AttnShape &sh, int rows, hipStream_t s);

// Measurement aid: reads `bytes` (a multiple of 16, 16-byte aligned) of buf once; sink receives 8192 words.
hipError_t launch_stream_read(const void *buf, size_t bytes, uint32_t *sink, hipStream_t s);
// Matrix-core probe (kernels_gemm.hip): n_stages stages of the wide projection tile's main loop on 256 workgroups,
// operands from the first mfma_probe_bytes() of buf; sink takes 256 x 512 floats.
size_t mfma_probe_bytes();
double mfma_probe_flops(int n_stages);
hipError_t launch_mfma_probe(const void *buf, int n_stages, float *sink, hipStream_t s);

}  // namespace dyn

/*
 * CPU oracle for one transformer decoder layer's forward step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP path is
 * checked against.  It shares no code with the HIP library and must never be called
 * from the product path; only the tests, the smoke check and the benchmark's
 * cpu_baseline leg use it.
 *
 * What it computes.  The paper (Section 2, "Background and Motivation"; Section 3.2.1)
 * treats the decoder layer as a chain of coarse operators - normalisation, GEMMs,
 * decode attention - and defines no arithmetic for them; its method (Section 2.1
 * "Splitting", Section 3.2.2) re-orders those operators over micro-batches and reaches
 * exactly the unsplit result.  The oracle is therefore the textbook pre-norm, gated-MLP
 * decoder layer of the evaluated model families (Section 5.1: Llama-3, Qwen, Mixtral,
 * DeepSeek), computed once over the whole batch, unsplit, in the written order:
 *
 *   h1 = RMSNorm(x; g1)              q,k,v = h1 Wq^T, h1 Wk^T, h1 Wv^T
 *   q',k' = RoPE(q,k; position)      append k', v to the paged cache
 *   o  = softmax(q' K^T / sqrt(d)) V over positions 0..p of the token's sequence
 *   x2 = x + o Wo^T                  h2 = RMSNorm(x2; g2)
 *   y  = x2 + (silu(h2 Wg^T) * (h2 Wu^T)) Wd^T            (dense MLP)
 *   y  = x2 + sum_{e in top-k} w_e MLP_e(h2)               (mixture of experts)
 *
 * Precision: stored tensors are fp32 or bf16; every intermediate is fp64.  The only
 * rounding inside the layer is that appended k', v are rounded to the cache's storage
 * type, because the cache is state the caller sees and attention reads it back.
 *
 * Parallelism: OpenMP over independent rows only, so every result has one fixed
 * summation order regardless of the thread count.
 *
 * Pins (tests/test_oracle_*.py): brute-force attention on gathered contiguous K/V,
 * library scaled-dot-product attention / rms_norm / silu / matmul in fp64, closed forms
 * (RoPE d=2 rotation, SiLU identities, unit RMS), and layer invariants (zero Wo and Wd
 * gives y = x, batch split and sequence permutation leave rows unchanged, identical
 * experts reduce to the dense MLP).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_F32 = 0, ORC_BF16 = 1 };

typedef struct {
    int dtype;
    int hidden, n_q, n_kv, head_dim, inter;
    int n_experts, top_k;
    double eps, rope_base;
    int page_size;
} orc_config;

typedef struct {
    const void *w_qkv, *w_o, *w_gate_up, *w_down, *g_norm1, *g_norm2;
    const float *w_router;
} orc_weights;

static inline double bf16_to_f64(uint16_t v) {
    uint32_t u = (uint32_t)v << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

static inline uint16_t f64_to_bf16(double x) {
    float f = (float)x;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);              /* round to nearest, ties to even */
    return (uint16_t)(u >> 16);
}

static inline double ld(const void *p, size_t i, int dtype) {
    return dtype == ORC_BF16 ? bf16_to_f64(((const uint16_t *)p)[i]) : (double)((const float *)p)[i];
}

static inline void st(void *p, size_t i, int dtype, double v) {
    if (dtype == ORC_BF16) ((uint16_t *)p)[i] = f64_to_bf16(v);
    else ((float *)p)[i] = (float)v;
}

/* Widen a stored tensor to fp64. */
void orc_widen(const void *src, int dtype, size_t n, double *dst) {
    for (size_t i = 0; i < n; ++i) dst[i] = ld(src, i, dtype);
}

/* out[t,i] = x[t,i] g[i] / sqrt(mean_j x[t,j]^2 + eps) */
void orc_rmsnorm(const double *x, const void *g, int dtype, int T, int H, double eps, double *out) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        double ss = 0.0;
        for (int j = 0; j < H; ++j) ss += x[(size_t)t * H + j] * x[(size_t)t * H + j];
        double r = 1.0 / sqrt(ss / H + eps);
        for (int j = 0; j < H; ++j) out[(size_t)t * H + j] = x[(size_t)t * H + j] * r * ld(g, j, dtype);
    }
}

/* out[t,n] = sum_k x[t,k] W[n,k]   (W stored output-major, [N,K]) */
void orc_linear(const double *x, const void *W, int dtype, int T, int K, int N, double *out) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int t = 0; t < T; ++t)
        for (int n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k) acc += x[(size_t)t * K + k] * ld(W, (size_t)n * K + k, dtype);
            out[(size_t)t * N + n] = acc;
        }
}

/* Rotary embedding, rotate-half pairing: for i < d/2, theta_i = base^(-2i/d),
 * (z[i], z[i+d/2]) <- (z[i] cos(p theta_i) - z[i+d/2] sin(p theta_i),
 *                      z[i+d/2] cos(p theta_i) + z[i] sin(p theta_i)).
 * z is [T, n_heads, d] with row stride `stride` doubles between tokens. */
void orc_rope(double *z, size_t stride, const int32_t *pos, int T, int n_heads, int d, double base) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int h = 0; h < n_heads; ++h) {
            double *v = z + (size_t)t * stride + (size_t)h * d;
            for (int i = 0; i < d / 2; ++i) {
                double theta = pow(base, -2.0 * i / d);
                double c = cos(pos[t] * theta), s = sin(pos[t] * theta);
                double a = v[i], b = v[i + d / 2];
                v[i] = a * c - b * s;
                v[i + d / 2] = b * c + a * s;
            }
        }
}

/* Element offsets inside the paged caches.
 * K page: [n_kv][page_size][d];  V page: [n_kv][d][page_size]. */
static inline size_t k_off(const orc_config *c, int page, int kvh, int slot, int i) {
    return (((size_t)page * c->n_kv + kvh) * c->page_size + slot) * c->head_dim + i;
}
static inline size_t v_off(const orc_config *c, int page, int kvh, int slot, int i) {
    return (((size_t)page * c->n_kv + kvh) * c->head_dim + i) * c->page_size + slot;
}

/* Store this step's rotated keys and values at logical position pos of their sequence:
 * physical page block_table[seq][pos / ps], slot pos % ps, rounded to the cache type. */
void orc_cache_append(const orc_config *c, const double *k, const double *v, size_t stride, int T,
                      const int32_t *seq_of_token, const int32_t *pos_of_token,
                      const int32_t *block_table, int max_pages, void *k_cache, void *v_cache) {
    for (int t = 0; t < T; ++t) {
        int p = pos_of_token[t];
        int page = block_table[(size_t)seq_of_token[t] * max_pages + p / c->page_size];
        int slot = p % c->page_size;
        for (int g = 0; g < c->n_kv; ++g)
            for (int i = 0; i < c->head_dim; ++i) {
                st(k_cache, k_off(c, page, g, slot, i), c->dtype, k[(size_t)t * stride + (size_t)g * c->head_dim + i]);
                st(v_cache, v_off(c, page, g, slot, i), c->dtype, v[(size_t)t * stride + (size_t)g * c->head_dim + i]);
            }
    }
}

/* Attention of every token over cached positions 0..pos (inclusive) of its sequence.
 * q is [T, n_q, d] with row stride q_stride; head h reads kv head h / (n_q / n_kv).
 * out is [T, n_q * d].  probs, if not NULL, is [T, n_q, probs_stride] and receives the
 * softmax weights (for tests). */
void orc_attention(const orc_config *c, const double *q, size_t q_stride, int T,
                   const int32_t *seq_of_token, const int32_t *pos_of_token,
                   const int32_t *block_table, int max_pages, const void *k_cache, const void *v_cache,
                   double *out, double *probs, int probs_stride) {
    const int d = c->head_dim, ps = c->page_size, group = c->n_q / c->n_kv;
    const double scale = 1.0 / sqrt((double)d);
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int t = 0; t < T; ++t)
        for (int h = 0; h < c->n_q; ++h) {
            const int n_keys = pos_of_token[t] + 1, g = h / group;
            const int32_t *bt = block_table + (size_t)seq_of_token[t] * max_pages;
            const double *qh = q + (size_t)t * q_stride + (size_t)h * d;
            double *s = (double *)malloc(sizeof(double) * (size_t)n_keys);
            double mx = -INFINITY;
            for (int j = 0; j < n_keys; ++j) {
                double acc = 0.0;
                for (int i = 0; i < d; ++i) acc += qh[i] * ld(k_cache, k_off(c, bt[j / ps], g, j % ps, i), c->dtype);
                s[j] = acc * scale;
                if (s[j] > mx) mx = s[j];
            }
            double denom = 0.0;
            for (int j = 0; j < n_keys; ++j) { s[j] = exp(s[j] - mx); denom += s[j]; }
            for (int j = 0; j < n_keys; ++j) s[j] /= denom;
            double *o = out + ((size_t)t * c->n_q + h) * d;
            for (int i = 0; i < d; ++i) {
                double acc = 0.0;
                for (int j = 0; j < n_keys; ++j) acc += s[j] * ld(v_cache, v_off(c, bt[j / ps], g, j % ps, i), c->dtype);
                o[i] = acc;
            }
            if (probs)
                for (int j = 0; j < n_keys && j < probs_stride; ++j)
                    probs[((size_t)t * c->n_q + h) * probs_stride + j] = s[j];
            free(s);
        }
}

/* out[t,i] = silu(gu[t,i]) * gu[t,I+i],  silu(z) = z / (1 + exp(-z)) */
void orc_silu_mul(const double *gu, int T, int I, double *out) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t)
        for (int i = 0; i < I; ++i) {
            double z = gu[(size_t)t * 2 * I + i];
            out[(size_t)t * I + i] = z / (1.0 + exp(-z)) * gu[(size_t)t * 2 * I + I + i];
        }
}

/* Gated MLP of one weight set: (silu(h Wg^T) * (h Wu^T)) Wd^T */
static void mlp(const double *h, const void *w_gu, const void *w_down, int dtype, int T, int H, int I, double *out) {
    double *gu = (double *)malloc(sizeof(double) * (size_t)T * 2 * I);
    double *a = (double *)malloc(sizeof(double) * (size_t)T * I);
    orc_linear(h, w_gu, dtype, T, H, 2 * I, gu);
    orc_silu_mul(gu, T, I, a);
    orc_linear(a, w_down, dtype, T, I, H, out);
    free(gu);
    free(a);
}

/* Router: logits r = h Wr^T (fp32 weights); the top_k largest logits are selected (ties
 * go to the lower expert index) and their weights are the softmax over the selected
 * logits.  sel [T, top_k] and wgt [T, top_k] are ordered from largest logit down;
 * logits [T, E] may be NULL.  If forced_sel is not NULL the selection is taken from it
 * and only the weights are computed (used where a near tie makes two selections both
 * correct). */
void orc_route(const double *h, const float *w_router, int T, int H, int E, int top_k,
               const int32_t *forced_sel, int32_t *sel, double *wgt, double *logits) {
#pragma omp parallel for schedule(static)
    for (int t = 0; t < T; ++t) {
        double r[256];
        char used[256] = {0};
        for (int e = 0; e < E; ++e) {
            double acc = 0.0;
            for (int k = 0; k < H; ++k) acc += h[(size_t)t * H + k] * (double)w_router[(size_t)e * H + k];
            r[e] = acc;
            if (logits) logits[(size_t)t * E + e] = acc;
        }
        for (int j = 0; j < top_k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e)
                if (!used[e] && (best < 0 || r[e] > r[best])) best = e;
            if (forced_sel) best = forced_sel[(size_t)t * top_k + j];
            used[best] = 1;
            sel[(size_t)t * top_k + j] = best;
        }
        double mx = -INFINITY, denom = 0.0;
        for (int j = 0; j < top_k; ++j) mx = fmax(mx, r[sel[(size_t)t * top_k + j]]);
        for (int j = 0; j < top_k; ++j) denom += exp(r[sel[(size_t)t * top_k + j]] - mx);
        for (int j = 0; j < top_k; ++j) wgt[(size_t)t * top_k + j] = exp(r[sel[(size_t)t * top_k + j]] - mx) / denom;
    }
}

/* out[t] = sum_j wgt[t,j] MLP_{sel[t,j]}(h[t]), experts applied token by token. */
void orc_moe_mlp(const orc_config *c, const double *h, const void *w_gate_up, const void *w_down, int T,
                 const int32_t *sel, const double *wgt, double *out) {
    const int H = c->hidden, I = c->inter;
    const size_t esz = c->dtype == ORC_BF16 ? 2 : 4;
#pragma omp parallel for schedule(dynamic, 1)
    for (int t = 0; t < T; ++t) {
        double *tmp = (double *)malloc(sizeof(double) * (size_t)H);
        double *gu = (double *)malloc(sizeof(double) * (size_t)2 * I);
        double *a = (double *)malloc(sizeof(double) * (size_t)I);
        for (int i = 0; i < H; ++i) out[(size_t)t * H + i] = 0.0;
        for (int j = 0; j < c->top_k; ++j) {
            int e = sel[(size_t)t * c->top_k + j];
            const char *wgu = (const char *)w_gate_up + (size_t)e * 2 * I * H * esz;
            const char *wd = (const char *)w_down + (size_t)e * H * I * esz;
            for (int n = 0; n < 2 * I; ++n) {
                double acc = 0.0;
                for (int k = 0; k < H; ++k) acc += h[(size_t)t * H + k] * ld(wgu, (size_t)n * H + k, c->dtype);
                gu[n] = acc;
            }
            for (int i = 0; i < I; ++i) a[i] = gu[i] / (1.0 + exp(-gu[i])) * gu[I + i];
            for (int n = 0; n < H; ++n) {
                double acc = 0.0;
                for (int k = 0; k < I; ++k) acc += a[k] * ld(wd, (size_t)n * I + k, c->dtype);
                tmp[n] = acc;
            }
            for (int i = 0; i < H; ++i) out[(size_t)t * H + i] += wgt[(size_t)t * c->top_k + j] * tmp[i];
        }
        free(tmp); free(gu); free(a);
    }
}

/* One layer over the whole batch.  x is the input [T, hidden] widened to fp64; y (fp64)
 * receives the output; the caches receive this step's keys and values.  MoE only:
 * sel_out/wgt_out/logits_out (each may be NULL) receive the routing; forced_sel (may be
 * NULL) overrides the expert selection, see orc_route.  Returns 0, or -1 on a bad
 * configuration. */
int orc_layer_forward(const orc_config *c, const orc_weights *w, int T, const double *x,
                      const int32_t *seq_of_token, const int32_t *pos_of_token,
                      const int32_t *block_table, int max_pages, void *k_cache, void *v_cache,
                      double *y, const int32_t *forced_sel, int32_t *sel_out, double *wgt_out, double *logits_out) {
    const int H = c->hidden, d = c->head_dim, I = c->inter;
    if (c->n_q % c->n_kv || d % 2 || T < 0 || (c->n_experts && (c->top_k < 1 || c->top_k > c->n_experts || c->n_experts > 256)))
        return -1;
    const int NQ = c->n_q * d, NKV = c->n_kv * d, NQKV = NQ + 2 * NKV;
    double *h = (double *)malloc(sizeof(double) * (size_t)T * H);
    double *qkv = (double *)malloc(sizeof(double) * (size_t)T * NQKV);
    double *o = (double *)malloc(sizeof(double) * (size_t)T * NQ);
    double *x2 = (double *)malloc(sizeof(double) * (size_t)T * H);
    double *m = (double *)malloc(sizeof(double) * (size_t)T * H);

    orc_rmsnorm(x, w->g_norm1, c->dtype, T, H, c->eps, h);
    orc_linear(h, w->w_qkv, c->dtype, T, H, NQKV, qkv);
    orc_rope(qkv, NQKV, pos_of_token, T, c->n_q, d, c->rope_base);            /* q heads */
    orc_rope(qkv + NQ, NQKV, pos_of_token, T, c->n_kv, d, c->rope_base);      /* k heads */
    orc_cache_append(c, qkv + NQ, qkv + NQ + NKV, NQKV, T, seq_of_token, pos_of_token, block_table, max_pages,
                     k_cache, v_cache);
    orc_attention(c, qkv, NQKV, T, seq_of_token, pos_of_token, block_table, max_pages, k_cache, v_cache, o, NULL, 0);
    orc_linear(o, w->w_o, c->dtype, T, NQ, H, x2);
    for (size_t i = 0; i < (size_t)T * H; ++i) x2[i] += x[i];
    orc_rmsnorm(x2, w->g_norm2, c->dtype, T, H, c->eps, h);
    if (c->n_experts == 0) {
        mlp(h, w->w_gate_up, w->w_down, c->dtype, T, H, I, m);
    } else {
        int32_t *sel = (int32_t *)malloc(sizeof(int32_t) * (size_t)T * c->top_k);
        double *wgt = (double *)malloc(sizeof(double) * (size_t)T * c->top_k);
        orc_route(h, w->w_router, T, H, c->n_experts, c->top_k, forced_sel, sel, wgt, logits_out);
        orc_moe_mlp(c, h, w->w_gate_up, w->w_down, T, sel, wgt, m);
        if (sel_out) memcpy(sel_out, sel, sizeof(int32_t) * (size_t)T * c->top_k);
        if (wgt_out) memcpy(wgt_out, wgt, sizeof(double) * (size_t)T * c->top_k);
        free(sel); free(wgt);
    }
    for (size_t i = 0; i < (size_t)T * H; ++i) y[i] = x2[i] + m[i];
    free(h); free(qkv); free(o); free(x2); free(m);
    return 0;
}

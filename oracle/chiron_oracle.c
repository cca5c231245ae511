/*
 * CPU oracle for one batched decode step of a Llama-style decoder over a paged
 * KV cache: the serving instance's iteration that the paper's local autoscaler
 * sizes (Background: Inference Primer, Continuous Batching, PagedAttention;
 * Local Autoscaler, Alg. 1 observes its latency and throughput).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code with the GPU path and the
 * product never calls it.
 *
 * Numerics: every tensor is float (fp32) at function boundaries; every sum
 * (dot products, mean of squares, softmax denominator, weighted value sum) is
 * accumulated in double in ascending index order, so results do not depend on
 * batch order or on where pages sit in the pool.  Weights and KV storage are
 * either fp32 or bf16 bit patterns (widened exactly); values written into a
 * bf16 pool are rounded to nearest-even.
 *
 * Every function here is pinned by tests/test_oracle_*.py against closed forms,
 * brute force, library routines or hand-worked values; none is "parity unpinned".
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_F32 = 0, ORC_BF16 = 1 };

typedef struct {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
    float rope_base, rms_eps;
    int32_t block_size;
    int32_t wdtype;  /* storage of weights and gains */
    int32_t kvdtype; /* storage of the KV pool */
} orc_config;

typedef struct {
    const void *embed;      /* [vocab, hidden] */
    const void *final_norm; /* [hidden] */
    const void *lm_head;    /* [vocab, hidden] */
    const void *const *attn_norm; /* [n_layers] -> [hidden] */
    const void *const *wq;        /* [n_q*d, hidden]   (out, in) row-major */
    const void *const *wk;        /* [n_kv*d, hidden] */
    const void *const *wv;        /* [n_kv*d, hidden] */
    const void *const *wo;        /* [hidden, n_q*d] */
    const void *const *ffn_norm;  /* [hidden] */
    const void *const *w_gate;    /* [ffn, hidden] */
    const void *const *w_up;      /* [ffn, hidden] */
    const void *const *w_down;    /* [hidden, ffn] */
} orc_weights;

/* ---- storage helpers ---------------------------------------------------- */

static inline float bf16_bits_to_f32(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* round-to-nearest-even to the 8-bit-mantissa format; NaN stays NaN */
uint16_t orc_f32_to_bf16_bits(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

static inline float ld(const void *p, size_t i, int dt) {
    return dt == ORC_BF16 ? bf16_bits_to_f32(((const uint16_t *)p)[i]) : ((const float *)p)[i];
}

static inline void st(void *p, size_t i, int dt, float v) {
    if (dt == ORC_BF16) ((uint16_t *)p)[i] = orc_f32_to_bf16_bits(v);
    else ((float *)p)[i] = v;
}

/* ---- building blocks ---------------------------------------------------- */

/* RMSNorm: out_j = h_j * g_j / sqrt(mean_j(h_j^2) + eps)  (eps inside the root) */
void orc_rmsnorm(const float *h, const void *g, int gdt, int n, float eps, float *out) {
    double ss = 0.0;
    for (int j = 0; j < n; ++j) ss += (double)h[j] * (double)h[j];
    double inv = 1.0 / sqrt(ss / (double)n + (double)eps);
    for (int j = 0; j < n; ++j) out[j] = (float)((double)h[j] * inv * (double)ld(g, j, gdt));
}

/* y[i][n] = sum_k x[i][k] * W[n][k];  W is [N,K] (out,in) row-major */
void orc_linear(const float *x, int rows, const void *W, int wdt, int N, int K, float *y) {
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int i = 0; i < rows; ++i) {
            const float *xi = x + (size_t)i * K;
            double acc = 0.0;
            for (int k = 0; k < K; ++k) acc += (double)xi[k] * (double)ld(W, (size_t)n * K + k, wdt);
            y[(size_t)i * N + n] = (float)acc;
        }
    }
}

/* Rotary embedding, half-split pairing: for j < d/2 the pair (x_j, x_{j+d/2}) is
 * rotated by the angle pos * base^(-2j/d).  x is [n_heads, d], in place. */
void orc_rope(float *x, int n_heads, int d, int pos, float base) {
    int half = d / 2;
    for (int j = 0; j < half; ++j) {
        double inv_freq = pow((double)base, -2.0 * (double)j / (double)d);
        double ang = (double)pos * inv_freq;
        double c = cos(ang), s = sin(ang);
        for (int hd = 0; hd < n_heads; ++hd) {
            float *v = x + (size_t)hd * d;
            double a = v[j], b = v[j + half];
            v[j] = (float)(a * c - b * s);
            v[j + half] = (float)(b * c + a * s);
        }
    }
}

/* slot of token position pos of a sequence whose pages are block_table_row[] */
int64_t orc_slot(const int32_t *block_table_row, int pos, int block_size) {
    return (int64_t)block_table_row[pos / block_size] * block_size + pos % block_size;
}

static inline size_t pool_off(const orc_config *c, int64_t num_slots, int layer, int64_t slot, int kvh) {
    return (((size_t)layer * (size_t)num_slots + (size_t)slot) * (size_t)c->n_kv_heads + (size_t)kvh) *
           (size_t)c->head_dim;
}

/* Write n tokens' K and V of one layer into their slots.
 * k, v: [n, n_kv, d] float; slot = block_table[seq_idx[j]][pos[j]/bs]*bs + pos[j]%bs.
 * slots_out (optional): the slot each token went to. */
void orc_append_kv(const orc_config *c, void *k_pool, void *v_pool, int64_t num_slots, int layer,
                   const float *k, const float *v, const int32_t *block_table, int max_blocks,
                   const int32_t *seq_idx, const int32_t *pos, int n, int64_t *slots_out) {
    int row = c->n_kv_heads * c->head_dim;
    for (int j = 0; j < n; ++j) {
        int64_t slot = orc_slot(block_table + (size_t)seq_idx[j] * max_blocks, pos[j], c->block_size);
        size_t o = pool_off(c, num_slots, layer, slot, 0);
        for (int e = 0; e < row; ++e) {
            st(k_pool, o + e, c->kvdtype, k[(size_t)j * row + e]);
            st(v_pool, o + e, c->kvdtype, v[(size_t)j * row + e]);
        }
        if (slots_out) slots_out[j] = slot;
    }
}

/* Gather the first len tokens of one sequence, one layer, into contiguous
 * [len, n_kv, d] arrays of the pool's storage type (a pure copy). */
void orc_gather_kv(const orc_config *c, const void *k_pool, const void *v_pool, int64_t num_slots, int layer,
                   const int32_t *block_table_row, int len, void *k_out, void *v_out) {
    int row = c->n_kv_heads * c->head_dim;
    size_t es = c->kvdtype == ORC_BF16 ? 2 : 4;
    for (int t = 0; t < len; ++t) {
        int64_t slot = orc_slot(block_table_row, t, c->block_size);
        size_t o = pool_off(c, num_slots, layer, slot, 0);
        memcpy((char *)k_out + (size_t)t * row * es, (const char *)k_pool + o * es, row * es);
        memcpy((char *)v_out + (size_t)t * row * es, (const char *)v_pool + o * es, row * es);
    }
}

/* Page migration (a request evicted to host memory and restored, possibly into other pages): copy the first
 * n_pages pages of a block-table row, every layer, K then V, between the pool and an image laid out as
 * [layer][K|V][page j][block_size][n_kv][d] in the pool's storage type.  to_image != 0: pool -> image. */
void orc_swap(const orc_config *c, void *k_pool, void *v_pool, int64_t num_slots, const int32_t *block_table_row,
              int n_pages, void *image, int to_image) {
    size_t es = c->kvdtype == ORC_BF16 ? 2 : 4;
    size_t page = (size_t)c->block_size * c->n_kv_heads * c->head_dim * es; /* bytes of one page, one layer, K or V */
    for (int l = 0; l < c->n_layers; ++l)
        for (int kv = 0; kv < 2; ++kv)
            for (int j = 0; j < n_pages; ++j) {
                char *pool = (char *)(kv ? v_pool : k_pool) +
                             pool_off(c, num_slots, l, (int64_t)block_table_row[j] * c->block_size, 0) * es;
                char *img = (char *)image + (((size_t)l * 2 + kv) * n_pages + j) * page;
                if (to_image) memcpy(img, pool, page);
                else memcpy(pool, img, page);
            }
}

/* Decode attention of ONE sequence over tokens 0..len-1 of its paged cache:
 * for q head a (KV head a / G): s_t = q_a . K_t / sqrt(d), P = softmax(s),
 * o_a = sum_t P_t V_t.   q: [n_q, d], out: [n_q, d]. */
void orc_paged_attention(const orc_config *c, const void *k_pool, const void *v_pool, int64_t num_slots,
                         int layer, const int32_t *block_table_row, int len, const float *q, float *out) {
    int d = c->head_dim, G = c->n_q_heads / c->n_kv_heads;
    double scale = 1.0 / sqrt((double)d);
    double *s = (double *)malloc(sizeof(double) * (size_t)(len > 0 ? len : 1));
    double *acc = (double *)malloc(sizeof(double) * (size_t)d);
    for (int a = 0; a < c->n_q_heads; ++a) {
        int kvh = a / G;
        const float *qa = q + (size_t)a * d;
        double mx = -INFINITY;
        for (int t = 0; t < len; ++t) {
            size_t o = pool_off(c, num_slots, layer, orc_slot(block_table_row, t, c->block_size), kvh);
            double dot = 0.0;
            for (int e = 0; e < d; ++e) dot += (double)qa[e] * (double)ld(k_pool, o + e, c->kvdtype);
            s[t] = dot * scale;
            if (s[t] > mx) mx = s[t];
        }
        double denom = 0.0;
        for (int t = 0; t < len; ++t) {
            s[t] = exp(s[t] - mx);
            denom += s[t];
        }
        for (int e = 0; e < d; ++e) acc[e] = 0.0;
        for (int t = 0; t < len; ++t) {
            size_t o = pool_off(c, num_slots, layer, orc_slot(block_table_row, t, c->block_size), kvh);
            double p = s[t] / denom;
            for (int e = 0; e < d; ++e) acc[e] += p * (double)ld(v_pool, o + e, c->kvdtype);
        }
        for (int e = 0; e < d; ++e) out[(size_t)a * d + e] = (float)acc[e];
    }
    free(s);
    free(acc);
}

/* SwiGLU: act_j = silu(g_j) * u_j, silu(z) = z / (1 + exp(-z)) */
void orc_swiglu(const float *g, const float *u, int n, float *act) {
    for (int j = 0; j < n; ++j) {
        double z = g[j];
        act[j] = (float)(z / (1.0 + exp(-z)) * (double)u[j]);
    }
}

/* ---- the whole step ----------------------------------------------------- */

/* One decode step for `batch` sequences.  Sequence i feeds tokens[i] at position
 * p = seq_lens[i] (tokens already cached), writes that token's K (after RoPE) and
 * V of every layer into slot(i, p), attends over positions 0..p inclusive, and
 * yields logits[i][0..vocab).  seq_lens is not modified.
 * slots_out (optional) [batch]: the slot written for each sequence.
 * Returns 0, or -1 on allocation failure. */
int orc_decode_step(const orc_config *c, const orc_weights *w, void *k_pool, void *v_pool, int64_t num_slots,
                    const int32_t *block_table, int max_blocks, const int32_t *seq_lens, const int32_t *tokens,
                    int batch, float *logits, int64_t *slots_out) {
    int H = c->hidden, d = c->head_dim, nq = c->n_q_heads, nkv = c->n_kv_heads, F = c->ffn;
    int qn = nq * d, kn = nkv * d;
    size_t B = (size_t)batch;
    float *h = (float *)malloc(sizeof(float) * B * H);
    float *x = (float *)malloc(sizeof(float) * B * H);
    float *q = (float *)malloc(sizeof(float) * B * qn);
    float *k = (float *)malloc(sizeof(float) * B * kn);
    float *v = (float *)malloc(sizeof(float) * B * kn);
    float *o = (float *)malloc(sizeof(float) * B * qn);
    float *t = (float *)malloc(sizeof(float) * B * H);
    float *g = (float *)malloc(sizeof(float) * B * F);
    float *u = (float *)malloc(sizeof(float) * B * F);
    int32_t *idx = (int32_t *)malloc(sizeof(int32_t) * (B ? B : 1));
    if (!h || !x || !q || !k || !v || !o || !t || !g || !u || !idx) return -1;

    for (int i = 0; i < batch; ++i) {
        idx[i] = i;
        for (int j = 0; j < H; ++j) h[(size_t)i * H + j] = ld(w->embed, (size_t)tokens[i] * H + j, c->wdtype);
    }
    for (int l = 0; l < c->n_layers; ++l) {
        for (int i = 0; i < batch; ++i)
            orc_rmsnorm(h + (size_t)i * H, w->attn_norm[l], c->wdtype, H, c->rms_eps, x + (size_t)i * H);
        orc_linear(x, batch, w->wq[l], c->wdtype, qn, H, q);
        orc_linear(x, batch, w->wk[l], c->wdtype, kn, H, k);
        orc_linear(x, batch, w->wv[l], c->wdtype, kn, H, v);
        for (int i = 0; i < batch; ++i) {
            orc_rope(q + (size_t)i * qn, nq, d, seq_lens[i], c->rope_base);
            orc_rope(k + (size_t)i * kn, nkv, d, seq_lens[i], c->rope_base);
        }
        orc_append_kv(c, k_pool, v_pool, num_slots, l, k, v, block_table, max_blocks, idx, seq_lens, batch,
                      l == 0 ? slots_out : NULL);
#pragma omp parallel for schedule(dynamic, 1)
        for (int i = 0; i < batch; ++i)
            orc_paged_attention(c, k_pool, v_pool, num_slots, l, block_table + (size_t)i * max_blocks,
                                seq_lens[i] + 1, q + (size_t)i * qn, o + (size_t)i * qn);
        orc_linear(o, batch, w->wo[l], c->wdtype, H, qn, t);
        for (size_t e = 0; e < B * H; ++e) h[e] += t[e];
        for (int i = 0; i < batch; ++i)
            orc_rmsnorm(h + (size_t)i * H, w->ffn_norm[l], c->wdtype, H, c->rms_eps, x + (size_t)i * H);
        orc_linear(x, batch, w->w_gate[l], c->wdtype, F, H, g);
        orc_linear(x, batch, w->w_up[l], c->wdtype, F, H, u);
        orc_swiglu(g, u, batch * F, g);
        orc_linear(g, batch, w->w_down[l], c->wdtype, H, F, t);
        for (size_t e = 0; e < B * H; ++e) h[e] += t[e];
    }
    for (int i = 0; i < batch; ++i)
        orc_rmsnorm(h + (size_t)i * H, w->final_norm, c->wdtype, H, c->rms_eps, x + (size_t)i * H);
    orc_linear(x, batch, w->lm_head, c->wdtype, c->vocab, H, logits);

    free(h); free(x); free(q); free(k); free(v); free(o); free(t); free(g); free(u); free(idx);
    return 0;
}

/* Multi-token step: request i feeds q_len tokens at positions seq_lens[i] .. seq_lens[i]+q_len-1; token t
 * attends causally over positions 0 .. seq_lens[i]+t; all q_len tokens' K/V are written.  Written out as
 * what it means: the q_len tokens are taken one after the other, each as an ordinary single-token step of
 * the whole batch at the next position (the cache then holds exactly the earlier tokens of the block).
 * tokens [batch][q_len], logits [batch][q_len][vocab]. */
int orc_decode_step_multi(const orc_config *c, const orc_weights *w, void *k_pool, void *v_pool, int64_t num_slots,
                          const int32_t *block_table, int max_blocks, const int32_t *seq_lens, const int32_t *tokens,
                          int batch, int q_len, float *logits) {
    int32_t *lens = (int32_t *)malloc(sizeof(int32_t) * (size_t)(batch ? batch : 1));
    int32_t *tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)(batch ? batch : 1));
    float *lg = (float *)malloc(sizeof(float) * (size_t)(batch ? batch : 1) * c->vocab);
    if (!lens || !tok || !lg) return -1;
    for (int t = 0; t < q_len; ++t) {
        for (int i = 0; i < batch; ++i) {
            lens[i] = seq_lens[i] + t;
            tok[i] = tokens[(size_t)i * q_len + t];
        }
        if (orc_decode_step(c, w, k_pool, v_pool, num_slots, block_table, max_blocks, lens, tok, batch, lg, NULL)) return -1;
        for (int i = 0; i < batch; ++i)
            memcpy(logits + ((size_t)i * q_len + t) * c->vocab, lg + (size_t)i * c->vocab, sizeof(float) * c->vocab);
    }
    free(lens); free(tok); free(lg);
    return 0;
}

/* ---- local autoscaler --------------------------------------------------------------------- */

/* One pass of the batch-size autoscaling loop (Local Autoscaler, Alg. 1), in the paper's notation:
 * latency-based backpressure LBP = ITL / ITL SLO, throughput-based backpressure TBP =
 * Throughput_prev / Throughput_curr, local backpressure = max of the two; below one the maximum
 * batch size grows to alpha * (1 / backpressure) * MBS + (1 - alpha) * MBS, otherwise it is halved.
 * Readings where the paper is silent (the same as the library documents): no previous throughput
 * -> TBP = 0; no current observation -> unchanged; zero backpressure -> the limit; nearest integer,
 * clamped to [1, limit].  Returns the new maximum batch size; *lb_out receives the backpressure
 * (-1 if the tick was skipped). */
int orc_autoscale_step(double itl, double itl_slo, double thr_prev, double thr_curr, double alpha, int limit, int mbs,
                       double *lb_out) {
    double LBP, TBP, LB, next;
    if (lb_out) *lb_out = -1.0;
    if (!(itl > 0.0) || !(thr_curr > 0.0)) return mbs;
    LBP = itl / itl_slo;
    TBP = thr_prev > 0.0 ? thr_prev / thr_curr : 0.0;
    LB = fmax(LBP, TBP);
    if (lb_out) *lb_out = LB;
    if (LB < 1.0) {
        if (LB > 0.0) next = alpha * (1.0 / LB) * (double)mbs + (1.0 - alpha) * (double)mbs;
        else next = (double)limit;
    } else {
        next = (double)mbs / 2.0;
    }
    next = floor(next + 0.5);
    if (next < 1.0) next = 1.0;
    if (next > (double)limit) next = (double)limit;
    return (int)next;
}

/* threads the parallel loops above will use (reported beside timings) */
int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

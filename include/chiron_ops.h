/*
 * chiron_ops.h: the individual kernels of the decode step, exported so that each can be
 * checked against the plain definition and timed on its own.  chiron_decode_step (chiron.h)
 * is the product call; these run exactly the kernels it runs.
 *
 * Same conventions as chiron.h: int32 status return, dev/host pointers, `stream` is a
 * hipStream_t as void*, calls enqueue and do not synchronise.  Activations are fp32,
 * weights/gains/cache are bf16 bit patterns.
 */
#ifndef CHIRON_OPS_H
#define CHIRON_OPS_H

#include <stdint.h>

#include "chiron.h"

#ifdef __cplusplus
extern "C" {
#endif

/* out[r][j] = h[r][j] * gain[j] / sqrt(mean_j(h[r][j]^2) + eps); h, out dev fp32 [rows, n]; gain dev bf16 [n]. */
int32_t chiron_op_rmsnorm(const float *h, const void *gain, int32_t rows, int32_t n, float eps, float *out,
                          void *stream);

/* A weight matrix repacked into matrix-core tile order (library-owned device copy). */
typedef struct chiron_linear chiron_linear;
/* w dev bf16 [N, K] (out, in) row-major; any N >= 1 (padded to 32 inside), K a multiple of 16. */
int32_t chiron_linear_create(const void *w, int32_t N, int32_t K, void *stream, chiron_linear **out);
int32_t chiron_linear_destroy(chiron_linear *l);

/* y[M,N] = x[M,K] * W^T (accumulate == 0) or y += x * W^T (accumulate != 0, the residual add).
 * x, y dev fp32 row-major.  x is split into two bf16 terms, products accumulate in fp32. */
int32_t chiron_op_linear(const chiron_linear *l, const float *x, int32_t M, float *y, int32_t accumulate,
                         void *stream);

/* The fused gate/up matrix of a feed-forward block: w_gate, w_up dev bf16 [F, K] each, row-major, F and K multiples
 * of 16.  The library's copy interleaves the two so that gate column j and up column j are produced by one wave; it
 * goes with the two SwiGLU entry points below only (chiron_op_linear refuses it). */
int32_t chiron_linear_create_gate_up(const void *w_gate, const void *w_up, int32_t F, int32_t K, void *stream,
                                     chiron_linear **out);

/* SwiGLU fused into the gate/up projection's epilogue:
 *     act[m][j] = silu(gate[m][j]) * up[m][j],  gate = x * Wg^T,  up = x * Wu^T,  silu(z) = z / (1 + exp(-z)).
 * x dev fp32 [M, K]; act dev fp32 [M, F], caller-owned. */
int32_t chiron_op_gate_up_swiglu(const chiron_linear *gate_up, const float *x, int32_t M, float *act, void *stream);

/* The feed-forward block as the decode step runs it, two launches:  y (+)= act * Wd^T  with act as above.
 * down is a plain chiron_linear over Wd [N, F].  The intermediate never leaves the library: fp32 rows with few rows,
 * and from the row count of the linear_big_min_m knob on the two bf16 terms of act in the tile order that the down
 * projection copies straight into LDS.  x dev fp32 [M, K]; y dev fp32 [M, N]. */
int32_t chiron_op_swiglu_ffn(const chiron_linear *gate_up, const chiron_linear *down, const float *x, int32_t M,
                             float *y, int32_t accumulate, void *stream);

/* Rotary embedding in place: x dev fp32 [rows, n_heads, d]; row r is rotated for position pos[r]
 * (pairs (j, j+d/2), angle pos*base^(-2j/d), angles evaluated in fp64). */
int32_t chiron_op_rope(float *x, int32_t rows, int32_t n_heads, int32_t d, const int32_t *pos, float base,
                       void *stream);

/* chiron_op_rope for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): same arguments, same kernels, bit-identical result, but the cos/sin
 * table the two kernels share lives in a fixed 1 MiB device array inside the library (one per GPU, held until the
 * process ends) instead of a stream-ordered allocation.  The call itself allocates nothing.  Limit: rows * d <=
 * 262144 (e.g. 2048 rows at head_dim 128); beyond it CHIRON_ERR_SHAPE and nothing is launched.  All calls on one
 * GPU share the array: calls that overlap there (different streams or threads) race; calls on one stream do not. */
int32_t chiron_op_rope_noalloc(float *x, int32_t rows, int32_t n_heads, int32_t d, const int32_t *pos, float base,
                               void *stream);

/* Paged GQA decode attention of one layer: for request i and query head a (KV head a / G)
 *     out[i][a] = softmax_t(q[i][a] . K_t / sqrt(d)) . V_t   over positions t < ctx_lens[i]
 * of the request's paged cache.  q, out dev fp32 [batch, n_q_heads*head_dim]; ctx_lens dev
 * int32 [batch], each >= 1.  Uses the model's attention workspace (split-K partials). */
int32_t chiron_op_paged_attention(chiron_model *m, const chiron_kvpool *p, int32_t layer, const float *q,
                                  const int32_t *block_table, const int32_t *ctx_lens, int32_t batch, float *out,
                                  void *stream);

/* Performance knobs of the kernels, process-wide (0 restores the built-in heuristic where one exists):
 *   linear_nf (1|2|4), linear_mt (1|2|3|4), linear_xcd_remap (0|1), linear_ksplit, linear_target_blocks,
 *   linear_big_min_m (rows from which the gate/up projection hands the down projection tiled bf16 terms; <0 never),
 *   linear_big_all (1: from that row count on every other projection's input is split into such terms first),
 *   linear_ks (4|8|16: k-steps per chunk, the depth of the weight ring),
 *   attn_grid, attn_target_waves, attn_chunk_pages.
 * They change launch shapes only, never results beyond summation order. Unknown keys are an error. */
int32_t chiron_set_tuning(const char *key, int32_t value);

#ifdef __cplusplus
}
#endif
#endif /* CHIRON_OPS_H */

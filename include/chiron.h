/*
 * chiron.h: C ABI of the serving instance's batched iteration on one MI355X.
 *
 * The paper (Hierarchical Autoscaling for LLM Serving with Chiron) treats a
 * serving instance as the unit its autoscalers size: an LLM serving system plus
 * a model (Definitions: "LLM Serving Instance") that runs continuous batching
 * over a paged KV cache (Background: Inference Primer, Continuous Batching,
 * PagedAttention).  The local autoscaler (Local Autoscaler, Alg. 1) picks the
 * instance's maximum batch size from the inter-token latency and throughput
 * that this iteration exhibits.  This library is that iteration: one decode
 * step of a Llama-style decoder for a batch of requests with per-request
 * context lengths, and the latency/throughput profile over batch sizes.
 *
 * Conventions
 *  - All functions return CHIRON_OK (0) or a negative chiron_status; the text of
 *    the last error on the calling thread is chiron_last_error().  Nothing
 *    throws across this boundary.
 *  - "dev" pointers are device (HBM) addresses on the current HIP device, "host"
 *    pointers are ordinary host memory.  `stream` is a hipStream_t passed as
 *    void* (NULL = the default stream).  Calls only enqueue work on `stream`
 *    and do not synchronise it, except where stated.
 *  - Storage type of weights and of the KV pool is bf16 (raw 16-bit patterns).
 *    Activations inside the step are fp32 split into two bf16 terms for the
 *    matrix cores; logits are fp32.
 *  - Matrices are (out_features, in_features) row-major: y = x * W^T.
 *  - There is no CPU fallback: every entry point that computes needs the GPU.
 */
#ifndef CHIRON_H
#define CHIRON_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CHIRON_OK = 0,
    CHIRON_ERR_INVALID_ARG = -1,     /* null pointer, negative size, bad enum              */
    CHIRON_ERR_SHAPE = -2,           /* model shape the kernels do not support             */
    CHIRON_ERR_BATCH_TOO_LARGE = -3, /* batch > config.max_batch                           */
    CHIRON_ERR_BLOCK_TABLE = -4,     /* a needed page id is -1/out of range, or aliased    */
    CHIRON_ERR_OOM = -5,             /* device or host allocation failed / pool too small  */
    CHIRON_ERR_HIP = -6,             /* a HIP runtime call failed                          */
    CHIRON_ERR_TOKEN = -7            /* token id outside [0, vocab)                        */
} chiron_status;

enum { CHIRON_BF16 = 1 };

typedef struct chiron_model chiron_model;   /* opaque, library-owned; destroy with chiron_model_destroy */
typedef struct chiron_kvpool chiron_kvpool; /* opaque descriptor over CALLER-owned device memory        */

/* Shape of the decoder (Evaluation: Llama 3.1 8B / 70B are the served models; any
 * Llama-style shape with head_dim 64 or 128, hidden/ffn multiples of 16 works). */
typedef struct {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab;
    float rope_base; /* rotary base; pairs (j, j+head_dim/2) turn by pos*base^(-2j/head_dim) */
    float rms_eps;   /* added to the mean square inside the root                          */
    int32_t dtype;   /* CHIRON_BF16                                                        */
    int32_t max_batch;          /* largest batch any later call may pass                   */
    int32_t max_blocks_per_seq; /* row length of every block table passed later            */
} chiron_model_config;

/* One decoder layer's parameters, dev pointers to bf16, read during the load call only. */
typedef struct {
    const void *attn_norm; /* [hidden]                    */
    const void *wq;        /* [n_q_heads*head_dim, hidden] */
    const void *wk;        /* [n_kv_heads*head_dim, hidden]*/
    const void *wv;        /* [n_kv_heads*head_dim, hidden]*/
    const void *wo;        /* [hidden, n_q_heads*head_dim] */
    const void *ffn_norm;  /* [hidden]                    */
    const void *w_gate;    /* [ffn, hidden]               */
    const void *w_up;      /* [ffn, hidden]               */
    const void *w_down;    /* [hidden, ffn]               */
} chiron_layer_weights;

/* ---- model ---------------------------------------------------------------------------------- */

/* Allocates the model's packed weight buffers and step workspace on the current device
 * (hipMalloc; sized from cfg, max_batch and max_blocks_per_seq).  Weights are loaded
 * afterwards, layer by layer, so the caller never needs more than one layer of its own
 * copies resident.  *out is NULL on failure. */
int32_t chiron_model_create(const chiron_model_config *cfg, chiron_model **out);

/* Repack one layer (fused QKV and gate/up, matrix-core tile order) into the model's own
 * buffers.  Enqueued on `stream`; the caller's buffers may be freed once the stream has
 * passed this point. */
int32_t chiron_model_load_layer(chiron_model *m, int32_t layer, const chiron_layer_weights *w, void *stream);

/* Embedding table [vocab, hidden], final norm gain [hidden], LM head [vocab, hidden]; dev bf16. */
int32_t chiron_model_load_head(chiron_model *m, const void *embed, const void *final_norm, const void *lm_head,
                               void *stream);

/* Frees everything the model owns.  The caller must have synchronised streams using it. */
int32_t chiron_model_destroy(chiron_model *m);

/* ---- paged KV pool (PagedAttention: the cache is managed in fixed-size pages) ---------------- */

/* Bytes of pool memory one page (block_size tokens, all layers, K and V) occupies. */
int64_t chiron_kv_block_bytes(const chiron_model *m, int32_t block_size);

/* Describe `bytes` of caller-owned device memory at dev_mem (256-byte aligned) as a pool of
 * *num_blocks_out pages of block_size (must be 16) tokens.  The physical layout inside
 * dev_mem is private to the library; the logical contract is
 *     slot(seq, pos) = block_table[seq][pos / block_size] * block_size + pos % block_size
 * and is observable through chiron_append_kv / chiron_gather_kv.  Memory is not cleared. */
int32_t chiron_kv_pool_create(const chiron_model *m, void *dev_mem, uint64_t bytes, int32_t block_size,
                              chiron_kvpool **out, int32_t *num_blocks_out);
int32_t chiron_kv_pool_destroy(chiron_kvpool *p); /* does not free dev_mem */

/* Write n tokens' K and V of one layer into their slots (K is stored as given: for a real
 * prefill that means after the rotary embedding).
 *   k, v         dev bf16 [n, n_kv_heads, head_dim]
 *   block_table  dev int32 [*, max_blocks_per_seq]
 *   seq_idx, pos dev int32 [n]: token j belongs to row seq_idx[j] at position pos[j]
 * Distinct tokens must map to distinct slots. n == 0 is a no-op. */
int32_t chiron_append_kv(chiron_kvpool *p, int32_t layer, const void *k, const void *v, const int32_t *block_table,
                         int32_t max_blocks_per_seq, const int32_t *seq_idx, const int32_t *pos, int64_t n,
                         void *stream);

/* Logical read-back: copy positions 0..len-1 of one sequence, one layer, into contiguous
 * dev bf16 [len, n_kv_heads, head_dim] arrays (pure copies, bit-exact).
 *   block_table_row  dev int32 [max_blocks_per_seq] */
int32_t chiron_gather_kv(const chiron_kvpool *p, int32_t layer, const int32_t *block_table_row, int32_t len,
                         void *k_out, void *v_out, void *stream);

/* Eviction support (Design: a mixed instance evicts a batch request when an interactive one arrives, and
 * saves its KV cache by migrating it to CPU memory so that it can restart fast).
 * chiron_kv_swap_out copies the first n_pages pages of one request (every layer, K and V) into `image`;
 * chiron_kv_swap_in copies an image back into the pages listed in block_table_row, which may be other pages
 * than the ones it came from.  `image` is n_pages * chiron_kv_block_bytes() bytes of device-accessible memory:
 * device memory or pinned host memory (hipHostMalloc), 16-byte aligned; its byte layout is private and only
 * meaningful to swap_in on a pool of the same model shape.  Pure copies: a request swapped out and back in
 * gathers bit-identically.   block_table_row: dev int32 [>= n_pages]. */
int32_t chiron_kv_swap_out(const chiron_kvpool *p, const int32_t *block_table_row, int32_t n_pages, void *image,
                           void *stream);
int32_t chiron_kv_swap_in(chiron_kvpool *p, const int32_t *block_table_row, int32_t n_pages, const void *image,
                          void *stream);

/* ---- the iteration --------------------------------------------------------------------------- */

/* One decode step for `batch` running requests (Continuous Batching: the batch and its
 * per-request context lengths change between iterations, so they are arguments).
 *   block_table dev int32 [batch, max_blocks_per_seq], -1 = unused entry
 *   seq_lens    dev int32 [batch]: tokens ALREADY cached for each request
 *   tokens      dev int32 [batch]: the token each request feeds this step
 *   logits      dev fp32 [batch, vocab], caller-owned
 * For request i the step embeds tokens[i] at position p = seq_lens[i], writes its K (after
 * the rotary embedding) and V of every layer into slot(i, p) (that page must already be
 * in block_table[i]; pages may be shared read-only between requests but the written page
 * must be unique), attends over positions 0..p, and writes logits[i].  seq_lens is not
 * modified: the running queue and its lengths belong to the caller's scheduler.
 * Device-resident index arrays are NOT range-checked here (see chiron_validate_step_inputs).
 * batch == 0 is a no-op; batch > max_batch is CHIRON_ERR_BATCH_TOO_LARGE.
 * Calls on one model must not overlap (they share the model's workspace).
 * The call only enqueues kernels on `stream`: no allocation, no memory-set or copy node, no host synchronisation
 * (outside chiron_kernel_timing_begin/end).  It can therefore be recorded into a HIP graph; a replay reads the index
 * arrays and writes logits at the addresses recorded, with whatever they hold then. */
int32_t chiron_decode_step(chiron_model *m, chiron_kvpool *p, const int32_t *block_table, const int32_t *seq_lens,
                           const int32_t *tokens, int32_t batch, float *logits, void *stream);

/* Multi-token step (Evaluation setup: speculative decoding, where the served model verifies several drafted
 * tokens per iteration; Local Autoscaler: chunked prefill is named as another per-instance option): request i
 * feeds q_len tokens tokens[i][0..q_len) at positions seq_lens[i] .. seq_lens[i]+q_len-1.  Token t attends
 * causally over positions 0..seq_lens[i]+t, the K/V of all q_len tokens are written (their pages must be in
 * the block table), and logits[i][t] are the next-token logits after token t.
 *   tokens dev int32 [batch, q_len];  logits dev fp32 [batch, q_len, vocab];  batch*q_len <= max_batch.
 * q_len == 1 is chiron_decode_step.  The projections run over batch*q_len rows.  In attention as many tokens of
 * a request as fit the kernel's 16 operand columns (16 / query heads per KV head: 4 at the 8B geometry, 2 at
 * 70B's) share one pass over its pages; longer blocks take ceil(q_len / that many) passes. */
int32_t chiron_decode_step_multi(chiron_model *m, chiron_kvpool *p, const int32_t *block_table, const int32_t *seq_lens,
                                 const int32_t *tokens, int32_t batch, int32_t q_len, float *logits, void *stream);

/* Debug aid: copies the index arrays to the host (synchronises `stream`) and checks every
 * entry the step would use: page ids in range, written pages unique, token ids in vocab,
 * lengths within max_blocks_per_seq pages. */
int32_t chiron_validate_step_inputs(const chiron_model *m, const chiron_kvpool *p, const int32_t *block_table,
                                    const int32_t *seq_lens, const int32_t *tokens, int32_t batch, void *stream);

/* The same checks on HOST copies of the arrays (no GPU needed). */
int32_t chiron_check_step_inputs_host(const chiron_model_config *cfg, int32_t num_blocks, int32_t block_size,
                                      const int32_t *block_table, const int32_t *seq_lens, const int32_t *tokens,
                                      int32_t batch);

/* The two checks above for the inputs of chiron_decode_step_multi: tokens holds [batch, q_len] ids, every page that
 * holds one of the positions seq_lens[i] .. seq_lens[i]+q_len-1 counts as written, batch*q_len <= max_batch. */
int32_t chiron_validate_step_inputs_multi(const chiron_model *m, const chiron_kvpool *p, const int32_t *block_table,
                                          const int32_t *seq_lens, const int32_t *tokens, int32_t batch, int32_t q_len,
                                          void *stream);
int32_t chiron_check_step_inputs_host_multi(const chiron_model_config *cfg, int32_t num_blocks, int32_t block_size,
                                            const int32_t *block_table, const int32_t *seq_lens, const int32_t *tokens,
                                            int32_t batch, int32_t q_len);

/* One point of the curve the local autoscaler walks (Local Autoscaler: LBP is observed
 * ITL over the ITL SLO, TBP is previous over current throughput). */
typedef struct {
    int32_t batch;
    double lat_ms_median, lat_ms_p99, lat_ms_mean;
    double tokens_per_s; /* batch / median latency */
} chiron_profile_point;

/* For every batch size b in batch_sizes (host, n_sizes entries, each <= max_batch and <=
 * the rows of the supplied arrays) run `warmup` untimed and `iters` timed decode steps
 * over the first b rows, each timed with HIP events on `stream`, and fill out[k] (host).
 * Steps rewrite the same slots each iteration, so the cache is left as after one step.
 * Synchronises `stream`. */
int32_t chiron_step_latency_profile(chiron_model *m, chiron_kvpool *p, const int32_t *block_table,
                                    const int32_t *seq_lens, const int32_t *tokens, const int32_t *batch_sizes,
                                    int32_t n_sizes, int32_t warmup, int32_t iters, float *logits_scratch,
                                    void *stream, chiron_profile_point *out);

/* ---- local autoscaler (Local Autoscaler: Local Backpressure, Batch Size Autoscaling, Alg. 1) ---------------
 *
 * One update of an instance's maximum batch size from what the iteration exhibited since the last update:
 *     LBP = itl / itl_slo                      (latency-based backpressure)
 *     TBP = tput_prev / tput_curr              (throughput-based backpressure)
 *     LB  = max(LBP, TBP)                      (local backpressure)
 *     LB <  1:  MBS <- alpha * (1/LB) * MBS + (1 - alpha) * MBS     (EWMA-weighted proportional growth)
 *     LB >= 1:  MBS <- MBS / 2
 * itl_slo is the smallest ITL SLO among the requests running on the instance; the paper uses alpha = 0.5 and
 * runs the update on every change of the running queue.  Where the paper is silent: tput_prev <= 0 (no previous
 * observation) makes TBP 0; tput_curr <= 0 or itl <= 0 (nothing observed) leaves *max_batch unchanged; LB == 0
 * grows straight to the limit; the result is rounded to the nearest integer and clamped to [1, batch_limit].
 * Host only (plain arithmetic, no device work).  *backpressure_out (optional) receives LB, or -1 when the tick
 * was skipped. */
int32_t chiron_local_autoscale_step(double itl, double itl_slo, double tput_prev, double tput_curr, double alpha,
                                    int32_t batch_limit, int32_t *max_batch, double *backpressure_out);

/* Measurement aid: between _begin and _end every kernel that chiron_decode_step[_multi] launches for this
 * model from the calling thread carries a start and a stop event of its own (hipExtLaunchKernelGGL): they read
 * the begin and end timestamps of the dispatch, the same ones a profiler's kernel trace reports, and add nothing
 * to the stream between kernels.  _end synchronises `stream` and returns, per kernel class, the summed kernel
 * time and the number of launches since _begin.  (The QKV, O, gate/up, down and LM-head projections are
 * instances of one kernel; a projection of many rows that first splits its input counts as one launch and its
 * time is the sum of its two kernels.) */
enum {
    CHIRON_K_QKV = 0, CHIRON_K_O, CHIRON_K_GATEUP, CHIRON_K_DOWN, CHIRON_K_LMHEAD, CHIRON_K_ATTN, CHIRON_K_ATTN_MERGE,
    CHIRON_K_RMSNORM, CHIRON_K_ROPE_APPEND, CHIRON_K_OTHER, CHIRON_K_COUNT
};
typedef struct {
    double ms;
    int64_t launches;
} chiron_kernel_time;
int32_t chiron_kernel_timing_begin(chiron_model *m);
int32_t chiron_kernel_timing_end(chiron_model *m, void *stream, chiron_kernel_time *out /* host [CHIRON_K_COUNT] */);

/* Text of the last failure on this thread ("" if none). */
const char *chiron_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CHIRON_H */

// Internal declarations shared by the host API and the kernel launchers.
// gfx950 only (wave64, MFMA bf16 32x32x16 / 16x16x32 / 16x16x16).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <vector>

#include "../../include/chiron.h"
#include "../../include/chiron_ops.h"

namespace chiron {

constexpr int kBlockSize = 16;  // tokens per KV page
constexpr int kNumCU = 256;

// ---- error plumbing -----------------------------------------------------------------------------
int32_t fail(int32_t code, const char* fmt, ...);
#define CHIRON_HIP(expr)                                                                      \
    do {                                                                                      \
        hipError_t _e = (expr);                                                               \
        if (_e != hipSuccess)                                                                 \
            return ::chiron::fail(CHIRON_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(_e)); \
    } while (0)

// ---- kernel launches, optionally timed -------------------------------------------------------------
// While a timing scope is open on the calling thread (chiron_kernel_timing_begin .. end), every launch carries a
// start and a stop event of its own (hipExtLaunchKernelGGL): they read the dispatch's begin and end timestamps, the
// same ones a profiler's kernel trace shows, and put nothing between the kernels.  Otherwise a plain launch.
struct TimedLaunch {
    int cls;      // chiron_kernel_class
    bool first;   // first kernel of a step's launch (a launch may consist of two kernels)
    hipEvent_t a, b;
};
struct TimingScope {
    std::vector<TimedLaunch>* sink = nullptr;
    int cls = 0;
    bool first = true;
};
TimingScope*& timing_scope();  // thread-local; null when no scope is open

template <typename... P, typename... A>
inline void launch(void (*kernel)(P...), dim3 grid, dim3 block, hipStream_t st, A... args) {
    TimingScope* ts = timing_scope();
    hipEvent_t a = nullptr, b = nullptr;
    if (ts && hipEventCreate(&a) == hipSuccess && hipEventCreate(&b) == hipSuccess) {
        hipExtLaunchKernelGGL(kernel, grid, block, 0, st, a, b, 0, static_cast<P>(args)...);
        ts->sink->push_back(TimedLaunch{ts->cls, ts->first, a, b});
        ts->first = false;
        return;
    }
    if (a) (void)hipEventDestroy(a);
    kernel<<<grid, block, 0, st>>>(static_cast<P>(args)...);
}

// ---- packed linear layer --------------------------------------------------------------------------
// Weight W [N,K] (out,in) is stored as 32-row tiles, each tile as K/8 groups of [32 rows][8 k] bf16:
//   packed[((n/32)*(Kpad/8) + k/8)*256 + (n%32)*8 + k%8] = W[n][k]
// so one 32x16 MFMA operand fragment (two adjacent k-groups) is 1 KiB of contiguous memory.  N is padded to a
// multiple of 32 and K to a multiple of 256 with zeros, so the kernel's loads need no bounds checks.
struct Linear {
    uint16_t* w = nullptr;  // device, packed and zero-padded
    int N = 0, K = 0, Npad = 0, Kpad = 0;
    size_t tstride = 0;  // elements from one 32-row tile to the next (32*Kpad; padding it was measured to change nothing)
    bool owned = false;
};

// PRO_PACKED: the input is already split into its two bf16 terms and tiled (see linear_big.hip)
enum Prologue { PRO_NONE = 0, PRO_PACKED = 2 };
// What a projection does with its result.  EPI_SLICES is chosen inside launch_linear when it slices K.  The SwiGLU
// epilogues belong to a fused gate/up matrix packed with launch_pack_rows(..., interleave): the output has N/2 columns,
// out[m][j] = silu(gate[m][j]) * up[m][j], as fp32 rows (EPI_SWIGLU) or as the two bf16 terms in the tile order that
// PRO_PACKED reads (EPI_SWIGLU_PACKED: y is the base of the hi terms, ldy the padded K of the consuming projection).
enum Epilogue { EPI_STORE = 0, EPI_ADD = 1, EPI_SLICES = 2, EPI_SWIGLU = 3, EPI_SWIGLU_PACKED = 4 };

// Performance knobs (0 = built-in heuristic); see chiron_set_tuning.
struct Tuning {
    int linear_nf = 0;              // 32-column tiles per wave (1 or 2)
    int linear_mt = 0;              // 32-row tiles per workgroup (1, 2, 3 or 4)
    int linear_xcd_remap = 1;       // deal logical workgroup ids XCD by XCD (M-tiles of one weight tile share an L2)
    int linear_ksplit = 0;          // forced number of K-slices
    int linear_target_blocks = 256; // K is sliced until the grid has about this many workgroups
    int linear_big_min_m = 0;       // rows from which the down projection's input is written as tiled bf16 terms (0 = built-in, <0 = never)
    int linear_ks = 0;              // k-steps of 16 per chunk (depth of the weight ring): 4, 8 or 16
    int linear_big_all = 0;         // 1: pre-split every projection's input from that row count on, not only the down projection's
    int attn_grid = 0;              // workgroups of the persistent attention grid
    int attn_target_waves = 0;      // work items aimed for when one round of the grid cannot hold the list (0 = 4 rounds)
    int attn_chunk_pages = 0;       // forced pages per item
};
Tuning& tuning();

// C[M,N] = A[M,K] * W^T.  A is fp32 with row stride lda (PRO_NONE), or the tiled bf16 terms of it (PRO_PACKED: hi terms
// at A, lo terms linear_big_split_elems(M, L.Kpad) bf16 values further).
// If the launch slices K (only when `part` is given; at most max_split slices), slice s stores its partial product
// at part[s][M][N] and *ksplit_out = number of slices: the caller's consumer adds them up.  Otherwise the result
// goes to y as `epilogue` (EPI_STORE, EPI_ADD, or a SwiGLU epilogue, which never slices) says and *ksplit_out = 1.
// `asplit` (optional) is a workspace of 2 * linear_big_split_elems(M, L.Kpad) bf16 values: with it and the
// linear_big_all knob, launches of many rows first store the two bf16 terms of A there (launch_linear_big).
int32_t launch_linear(const Linear& L, const float* A, int lda, int M, float* y, int ldy, int epilogue, int prologue,
                      float* part, int max_split, int* ksplit_out, uint16_t* asplit, hipStream_t st);
int32_t launch_linear_big(const Linear& L, const float* A, int lda, int M, float* y, int ldy, int epilogue,
                          float* part, int max_split, int* ksplit_out, uint16_t* asplit, hipStream_t st);
size_t linear_big_split_elems(int M, int Kpad);
int linear_big_min_rows(const Linear& L);
int linear_max_split();
int32_t launch_reduce_partials(const float* part, int ks, int64_t n, float* y, int accumulate, hipStream_t st);
// interleave: 0 = source row r becomes packed row row_offset + r; 1 / 2 = the source is the gate / up half of a fused
// gate/up matrix, whose 32-row tiles hold 16 gate and the 16 up columns of the same indices (rows % 16 == 0)
int32_t launch_pack_rows(const uint16_t* src, int rows, int K, size_t tstride, uint16_t* dst_packed, int row_offset,
                         hipStream_t st, int interleave = 0);

// ---- elementwise / indexing kernels ---------------------------------------------------------------
int32_t launch_embed(const uint16_t* table, const int32_t* tokens, int batch, int H, float* h, hipStream_t st);
// out = rmsnorm(h) * gain.  With ks > 0 the row first absorbs the K-slices of the projection that feeds the
// residual stream: h += sum_s part[s] (h is rewritten), then the norm is taken.
int32_t launch_rmsnorm(float* h, const float* part, int ks, const uint16_t* gain, int rows, int n, float eps, float* out,
                       hipStream_t st);
// cos/sin of pos[i]*base^(-2j/d), j < d/2, evaluated in fp64 and stored as fp32 [rows, d/2] each
int32_t launch_rope_table(const int32_t* pos, int rows, int d, float base, float* cos_t, float* sin_t, hipStream_t st);
// rotate x [rows, n_heads, d] (row stride ldx floats) in place with the table
int32_t launch_rope(float* x, int ldx, int n_heads, int d, const float* cos_t, const float* sin_t, int rows,
                    hipStream_t st);

struct PoolDesc {
    uint16_t* base = nullptr;
    int64_t layer_stride = 0;  // elements
    int num_blocks = 0, n_kv = 0, d = 0, n_layers = 0;
};
// K tile of one (page, kv head): [d/8][16 tok][8];  V tile: [d/32][4 tok-groups][16][2][4 tok]  (see kernels)
int32_t launch_append_kv(const PoolDesc& p, int layer, const uint16_t* k, const uint16_t* v, const int32_t* bt,
                         int max_blocks, const int32_t* seq_idx, const int32_t* pos, int64_t n, hipStream_t st);
int32_t launch_gather_kv(const PoolDesc& p, int layer, const int32_t* bt_row, int len, uint16_t* k_out, uint16_t* v_out,
                         hipStream_t st);
// multi-token step: row (i,t) of the expanded batch gets request i's block-table row and length seq_lens[i] + t
int32_t launch_expand_rows(const int32_t* bt, const int32_t* seq_lens, int batch, int q_len, int max_blocks, int32_t* bt_out,
                           int32_t* lens_out, hipStream_t st);
// page migration: image = [page j][layer][kv head][K tile | V tile]; to_image != 0 copies pool -> image
int32_t launch_swap(const PoolDesc& p, const int32_t* bt_row, int n_pages, uint16_t* image, int to_image, hipStream_t st);
// decode-step variant: the fused qkv row [rows, (nq+2nkv)*d] is the sum of ks slices qkv[s] (slice stride
// rows*ld); q and k are rotated in fp32; q goes to q_out [rows, nq*d]; k, v are rounded to bf16 and written at
// slot(i, seq_lens[i]).
int32_t launch_rope_append(const PoolDesc& p, int layer, const float* qkv, int ks, int n_q, const float* cos_t,
                           const float* sin_t, const int32_t* bt, int max_blocks, const int32_t* seq_lens, int batch,
                           float* q_out, hipStream_t st);

// ---- paged attention ------------------------------------------------------------------------------
struct AttnWorkspace {
    int32_t* plan = nullptr;     // [0]=n_items, [1]=chunk_pages; then per-seq and per-item tables, ticket counters (see attention.hip)
    float* part_o = nullptr;     // [items*n_kv][tg*G][d], items*tg <= cap_items
    float* part_ml = nullptr;    // [items*n_kv][tg*G][2]
    int cap_items = 0, max_batch = 0;
};
int64_t attn_plan_ints(int max_batch, int cap_items);
// How the q_len new tokens of a request map onto passes of the attention kernel.  The kernel has 16 operand columns:
// a pass serves tg tokens x G query heads of one KV head (tg*G <= 16) while reading the request's pages once, so a
// request is attended in ng = ceil(q_len / tg) passes ("token groups"); group g holds tokens g*tg .. and attends
// len(i, g) = seq_lens[i] + bias0 + g*tg + (tokens in g) positions, token t of the request seeing positions
// <= seq_lens[i] + bias0 + t.  q and out hold rows request*q_len + token.  q_len = 1: one group, len = seq_lens + bias0 + 1.
struct AttnShape {
    int q_len = 1, tg = 1, ng = 1, bias0 = 0;
};
// len_bias: what to add to seq_lens[i] for the number of positions the LAST new token attends (q_len when all new
// tokens are appended and seq_lens counts only the older ones; 0 when seq_lens is already the attended length)
AttnShape attn_shape(int G, int q_len, int len_bias);
// (bt: the block table the attention launches of this plan will use; the plan copies each item's first page ids)
int32_t launch_attn_plan(const AttnWorkspace& ws, const int32_t* seq_lens, const int32_t* bt, int max_blocks, const AttnShape& sh,
                         int batch, int n_kv, hipStream_t st);
// launch_attn_main leaves the plan's ticket counters used; launch_attn_merge, which must follow it on the same stream
// before the next launch_attn_main, puts them back to 0.
int32_t launch_attn_main(const AttnWorkspace& ws, const PoolDesc& p, int layer, const float* q, int ldq, int n_q,
                         const int32_t* bt, int max_blocks, const int32_t* seq_lens, const AttnShape& sh, int batch,
                         hipStream_t st);
int32_t launch_attn_merge(const AttnWorkspace& ws, const PoolDesc& p, int n_q, const AttnShape& sh, int batch, float* out,
                          int ldo, hipStream_t st);

}  // namespace chiron

struct chiron_linear {
    chiron::Linear L;
    bool gate_up = false;  // rows are the interleaved [gate | up] of a feed-forward block
};

struct chiron_kvpool {
    chiron::PoolDesc d;
    int block_size = 16;
};

struct chiron_model {
    chiron_model_config cfg;
    int device = 0;
    // packed weights
    chiron::Linear *qkv = nullptr, *wo = nullptr, *gu = nullptr, *down = nullptr;  // [n_layers]
    chiron::Linear lm;
    uint16_t *attn_norm = nullptr, *ffn_norm = nullptr, *final_norm = nullptr;  // [n_layers*H], [H]
    uint16_t* embed = nullptr;
    // step workspace, sized for max_batch
    float *h = nullptr, *x = nullptr, *qkvb = nullptr, *qb = nullptr, *attn = nullptr, *gub = nullptr;
    int32_t *x_bt = nullptr, *x_lens = nullptr;  // expanded index arrays of the multi-token step
    float* part = nullptr;  // K-slice workspace of the projections: [max_split][max_batch][max(qkv width, hidden)]
    uint16_t* asplit = nullptr;  // hi and lo bf16 terms of a projection's input in tile order (large batches only)
    float *cos_t = nullptr, *sin_t = nullptr;
    chiron::AttnWorkspace aws;
    // optional per-kernel event timing of decode steps
    bool timing = false;
    std::vector<chiron::TimedLaunch> timed;
};

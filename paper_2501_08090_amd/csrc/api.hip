// Host side of the C ABI (include/chiron.h, include/chiron_ops.h): handles, argument checks,
// weight loading, and the sequence of kernel launches that makes one decode step.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <unordered_set>
#include <vector>

#include "chiron_internal.h"

namespace chiron {

static thread_local char g_err[512] = "";

TimingScope*& timing_scope() {
    static thread_local TimingScope* scope = nullptr;
    return scope;
}

int32_t fail(int32_t code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

// smallest max_batch for which the model carries the workspace of the large-batch projection kernel
static constexpr int kBigWorkspaceMinBatch = 96;

static int32_t dev_alloc(void** p, size_t bytes) {
    *p = nullptr;
    hipError_t e = hipMalloc(p, bytes ? bytes : 256);
    if (e != hipSuccess) {
        *p = nullptr;
        (void)hipGetLastError();
        return fail(CHIRON_ERR_OOM, "hipMalloc of %zu bytes failed: %s", bytes, hipGetErrorString(e));
    }
    return CHIRON_OK;
}

static int32_t linear_alloc(Linear& L, int N, int K) {
    L.N = N;
    L.K = K;
    L.Npad = (N + 31) / 32 * 32;
    L.Kpad = (K + 255) / 256 * 256;  // whole chunks of the deepest weight ring (16 k-steps of 16)
    L.owned = true;
    L.tstride = (size_t)32 * L.Kpad;
    const size_t bytes = (size_t)(L.Npad / 32) * L.tstride * 2;
    int32_t rc = dev_alloc((void**)&L.w, bytes);
    if (rc) return rc;
    if (L.Npad != N || L.Kpad != K) {
        // the packing kernels run on the caller's stream, which need not be ordered after the null stream's memset
        CHIRON_HIP(hipMemset(L.w, 0, bytes));
        CHIRON_HIP(hipStreamSynchronize(nullptr));
    }
    return CHIRON_OK;
}

static void linear_free(Linear& L) {
    if (L.owned && L.w) (void)hipFree(L.w);
    L.w = nullptr;
}

static int32_t check_config(const chiron_model_config* c) {
    if (!c) return fail(CHIRON_ERR_INVALID_ARG, "config is null");
    if (c->dtype != CHIRON_BF16) return fail(CHIRON_ERR_INVALID_ARG, "dtype %d: only CHIRON_BF16 is supported", c->dtype);
    if (c->n_layers < 1 || c->hidden < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->ffn < 1 || c->vocab < 1 ||
        c->max_batch < 1 || c->max_blocks_per_seq < 1)
        return fail(CHIRON_ERR_INVALID_ARG, "config has a non-positive size");
    if (c->head_dim != 64 && c->head_dim != 128) return fail(CHIRON_ERR_SHAPE, "head_dim %d: must be 64 or 128", c->head_dim);
    if (c->n_q_heads % c->n_kv_heads != 0) return fail(CHIRON_ERR_SHAPE, "n_q_heads must be a multiple of n_kv_heads");
    int G = c->n_q_heads / c->n_kv_heads;
    if (G != 1 && G != 2 && G != 4 && G != 8 && G != 16) return fail(CHIRON_ERR_SHAPE, "query heads per KV head %d: must be 1,2,4,8,16", G);
    if (c->hidden % 16 != 0 || c->ffn % 16 != 0) return fail(CHIRON_ERR_SHAPE, "hidden and ffn must be multiples of 16");
    if (c->hidden > 16384) return fail(CHIRON_ERR_SHAPE, "hidden %d: at most 16384", c->hidden);
    if (!(c->rope_base > 1.0f) || !(c->rms_eps >= 0.0f)) return fail(CHIRON_ERR_INVALID_ARG, "rope_base must be > 1 and rms_eps >= 0");
    return CHIRON_OK;
}

}  // namespace chiron

using namespace chiron;

extern "C" {

const char* chiron_last_error(void) { return g_err; }

// ---- model ---------------------------------------------------------------------------------------------
int32_t chiron_model_destroy(chiron_model* m) {
    if (!m) return CHIRON_OK;
    for (int l = 0; l < m->cfg.n_layers; ++l) {
        if (m->qkv) linear_free(m->qkv[l]);
        if (m->wo) linear_free(m->wo[l]);
        if (m->gu) linear_free(m->gu[l]);
        if (m->down) linear_free(m->down[l]);
    }
    delete[] m->qkv; delete[] m->wo; delete[] m->gu; delete[] m->down;
    for (auto& t : m->timed) {
        (void)hipEventDestroy(t.a);
        (void)hipEventDestroy(t.b);
    }
    linear_free(m->lm);
    void* bufs[] = {m->attn_norm, m->ffn_norm, m->final_norm, m->embed, m->h, m->x, m->qkvb, m->qb, m->part, m->asplit, m->x_bt, m->x_lens, m->attn, m->gub,
                    m->cos_t, m->sin_t, m->aws.plan, m->aws.part_o, m->aws.part_ml};
    for (void* b : bufs)
        if (b) (void)hipFree(b);
    delete m;
    return CHIRON_OK;
}

int32_t chiron_model_create(const chiron_model_config* cfg, chiron_model** out) {
    if (!out) return fail(CHIRON_ERR_INVALID_ARG, "out is null");
    *out = nullptr;
    int32_t rc = check_config(cfg);
    if (rc) return rc;
    chiron_model* m = new (std::nothrow) chiron_model();
    if (!m) return fail(CHIRON_ERR_OOM, "host allocation failed");
    m->cfg = *cfg;
    const int L = cfg->n_layers, H = cfg->hidden, d = cfg->head_dim, F = cfg->ffn;
    const int qn = cfg->n_q_heads * d, kn = cfg->n_kv_heads * d, B = cfg->max_batch;
    if (hipGetDevice(&m->device) != hipSuccess) {
        delete m;
        return fail(CHIRON_ERR_HIP, "no HIP device is available");
    }
    m->qkv = new (std::nothrow) Linear[L]; m->wo = new (std::nothrow) Linear[L];
    m->gu = new (std::nothrow) Linear[L]; m->down = new (std::nothrow) Linear[L];
#define TRY(expr)                     \
    do {                              \
        rc = (expr);                  \
        if (rc) {                     \
            chiron_model_destroy(m);  \
            return rc;                \
        }                             \
    } while (0)
    if (!m->qkv || !m->wo || !m->gu || !m->down) TRY(fail(CHIRON_ERR_OOM, "host allocation failed"));
    for (int l = 0; l < L; ++l) {
        TRY(linear_alloc(m->qkv[l], qn + 2 * kn, H));
        TRY(linear_alloc(m->wo[l], H, qn));
        TRY(linear_alloc(m->gu[l], 2 * F, H));
        TRY(linear_alloc(m->down[l], H, F));
    }
    TRY(linear_alloc(m->lm, cfg->vocab, H));
    TRY(dev_alloc((void**)&m->attn_norm, (size_t)L * H * 2));
    TRY(dev_alloc((void**)&m->ffn_norm, (size_t)L * H * 2));
    TRY(dev_alloc((void**)&m->final_norm, (size_t)H * 2));
    TRY(dev_alloc((void**)&m->embed, (size_t)cfg->vocab * H * 2));
    TRY(dev_alloc((void**)&m->h, (size_t)B * H * 4));
    TRY(dev_alloc((void**)&m->x, (size_t)B * H * 4));
    TRY(dev_alloc((void**)&m->qkvb, (size_t)B * (qn + 2 * kn) * 4));
    TRY(dev_alloc((void**)&m->qb, (size_t)B * qn * 4));
    TRY(dev_alloc((void**)&m->part, (size_t)linear_max_split() * B * std::max(qn + 2 * kn, H) * 4));
    if (B >= kBigWorkspaceMinBatch) {
        const size_t kmax = (size_t)(std::max(std::max(F, H), qn) + 255) / 256 * 256;
        const size_t bytes = 2 * linear_big_split_elems(B, (int)kmax) * 2;
        TRY(dev_alloc((void**)&m->asplit, bytes));
        // the gate/up epilogue writes the columns below F only: what the down projection reads of its K padding is 0
        if (hipMemset(m->asplit, 0, bytes) != hipSuccess || hipDeviceSynchronize() != hipSuccess)
            TRY(fail(CHIRON_ERR_HIP, "clearing the activation workspace failed"));
    }
    TRY(dev_alloc((void**)&m->x_bt, (size_t)B * cfg->max_blocks_per_seq * 4));
    TRY(dev_alloc((void**)&m->x_lens, (size_t)B * 4));
    TRY(dev_alloc((void**)&m->attn, (size_t)B * qn * 4));
    TRY(dev_alloc((void**)&m->gub, (size_t)B * F * 4));  // silu(gate) * up, fp32 rows
    TRY(dev_alloc((void**)&m->cos_t, (size_t)B * (d / 2) * 4));
    TRY(dev_alloc((void**)&m->sin_t, (size_t)B * (d / 2) * 4));
    // attention work list: room for a few items per wave slot plus one ragged tail per request
    m->aws.max_batch = B;
    m->aws.cap_items = 8192 + 2 * B;
    TRY(dev_alloc((void**)&m->aws.plan, (size_t)attn_plan_ints(B, m->aws.cap_items) * 4));
    TRY(dev_alloc((void**)&m->aws.part_o, (size_t)m->aws.cap_items * cfg->n_q_heads * d * 4));
    TRY(dev_alloc((void**)&m->aws.part_ml, (size_t)m->aws.cap_items * cfg->n_q_heads * 2 * 4));
#undef TRY
    *out = m;
    return CHIRON_OK;
}

int32_t chiron_model_load_layer(chiron_model* m, int32_t layer, const chiron_layer_weights* w, void* stream) {
    if (!m || !w) return fail(CHIRON_ERR_INVALID_ARG, "model or weights is null");
    if (layer < 0 || layer >= m->cfg.n_layers) return fail(CHIRON_ERR_INVALID_ARG, "layer %d out of range", layer);
    if (!w->attn_norm || !w->wq || !w->wk || !w->wv || !w->wo || !w->ffn_norm || !w->w_gate || !w->w_up || !w->w_down)
        return fail(CHIRON_ERR_INVALID_ARG, "a layer weight pointer is null");
    hipStream_t st = (hipStream_t)stream;
    const chiron_model_config& c = m->cfg;
    const int H = c.hidden, d = c.head_dim, F = c.ffn, qn = c.n_q_heads * d, kn = c.n_kv_heads * d;
    int32_t rc;
    // fused QKV: rows [q | k | v]; fused gate/up: 16 gate and the 16 up columns of the same indices per 32-row tile
    if ((rc = launch_pack_rows((const uint16_t*)w->wq, qn, H, m->qkv[layer].tstride, m->qkv[layer].w, 0, st))) return rc;
    if ((rc = launch_pack_rows((const uint16_t*)w->wk, kn, H, m->qkv[layer].tstride, m->qkv[layer].w, qn, st))) return rc;
    if ((rc = launch_pack_rows((const uint16_t*)w->wv, kn, H, m->qkv[layer].tstride, m->qkv[layer].w, qn + kn, st))) return rc;
    if ((rc = launch_pack_rows((const uint16_t*)w->wo, H, qn, m->wo[layer].tstride, m->wo[layer].w, 0, st))) return rc;
    if ((rc = launch_pack_rows((const uint16_t*)w->w_gate, F, H, m->gu[layer].tstride, m->gu[layer].w, 0, st, 1))) return rc;
    if ((rc = launch_pack_rows((const uint16_t*)w->w_up, F, H, m->gu[layer].tstride, m->gu[layer].w, 0, st, 2))) return rc;
    if ((rc = launch_pack_rows((const uint16_t*)w->w_down, H, F, m->down[layer].tstride, m->down[layer].w, 0, st))) return rc;
    CHIRON_HIP(hipMemcpyAsync(m->attn_norm + (size_t)layer * H, w->attn_norm, (size_t)H * 2, hipMemcpyDeviceToDevice, st));
    CHIRON_HIP(hipMemcpyAsync(m->ffn_norm + (size_t)layer * H, w->ffn_norm, (size_t)H * 2, hipMemcpyDeviceToDevice, st));
    return CHIRON_OK;
}

int32_t chiron_model_load_head(chiron_model* m, const void* embed, const void* final_norm, const void* lm_head,
                               void* stream) {
    if (!m || !embed || !final_norm || !lm_head) return fail(CHIRON_ERR_INVALID_ARG, "model or a weight pointer is null");
    hipStream_t st = (hipStream_t)stream;
    const chiron_model_config& c = m->cfg;
    CHIRON_HIP(hipMemcpyAsync(m->embed, embed, (size_t)c.vocab * c.hidden * 2, hipMemcpyDeviceToDevice, st));
    CHIRON_HIP(hipMemcpyAsync(m->final_norm, final_norm, (size_t)c.hidden * 2, hipMemcpyDeviceToDevice, st));
    return launch_pack_rows((const uint16_t*)lm_head, c.vocab, c.hidden, m->lm.tstride, m->lm.w, 0, st);
}

// ---- KV pool -------------------------------------------------------------------------------------------
int64_t chiron_kv_block_bytes(const chiron_model* m, int32_t block_size) {
    if (!m || block_size != kBlockSize) return 0;
    return (int64_t)m->cfg.n_layers * m->cfg.n_kv_heads * 2 * block_size * m->cfg.head_dim * 2;
}

int32_t chiron_kv_pool_create(const chiron_model* m, void* dev_mem, uint64_t bytes, int32_t block_size,
                              chiron_kvpool** out, int32_t* num_blocks_out) {
    if (!out) return fail(CHIRON_ERR_INVALID_ARG, "out is null");
    *out = nullptr;
    if (!m || !dev_mem) return fail(CHIRON_ERR_INVALID_ARG, "model or dev_mem is null");
    if (block_size != kBlockSize) return fail(CHIRON_ERR_INVALID_ARG, "block_size %d: must be 16", block_size);
    if ((uintptr_t)dev_mem & 255) return fail(CHIRON_ERR_INVALID_ARG, "dev_mem must be 256-byte aligned");
    uint64_t per_block = (uint64_t)chiron_kv_block_bytes(m, block_size);
    uint64_t nb = bytes / per_block;
    if (nb < 1) return fail(CHIRON_ERR_OOM, "pool of %llu bytes holds no page (one page is %llu bytes)",
                            (unsigned long long)bytes, (unsigned long long)per_block);
    if (nb > 0x7fffffffull / kBlockSize) nb = 0x7fffffffull / kBlockSize;
    chiron_kvpool* p = new (std::nothrow) chiron_kvpool();
    if (!p) return fail(CHIRON_ERR_OOM, "host allocation failed");
    p->block_size = block_size;
    p->d.base = (uint16_t*)dev_mem;
    p->d.num_blocks = (int)nb;
    p->d.n_kv = m->cfg.n_kv_heads;
    p->d.d = m->cfg.head_dim;
    p->d.n_layers = m->cfg.n_layers;
    p->d.layer_stride = (int64_t)nb * m->cfg.n_kv_heads * 2 * kBlockSize * m->cfg.head_dim;
    *out = p;
    if (num_blocks_out) *num_blocks_out = (int32_t)nb;
    return CHIRON_OK;
}

int32_t chiron_kv_pool_destroy(chiron_kvpool* p) {
    delete p;
    return CHIRON_OK;
}

int32_t chiron_append_kv(chiron_kvpool* p, int32_t layer, const void* k, const void* v, const int32_t* block_table,
                         int32_t max_blocks_per_seq, const int32_t* seq_idx, const int32_t* pos, int64_t n,
                         void* stream) {
    if (!p) return fail(CHIRON_ERR_INVALID_ARG, "pool is null");
    if (n < 0) return fail(CHIRON_ERR_INVALID_ARG, "n is negative");
    if (n == 0) return CHIRON_OK;
    if (layer < 0 || layer >= p->d.n_layers) return fail(CHIRON_ERR_INVALID_ARG, "layer %d out of range", layer);
    if (!k || !v || !block_table || !seq_idx || !pos) return fail(CHIRON_ERR_INVALID_ARG, "a pointer argument is null");
    if (max_blocks_per_seq < 1) return fail(CHIRON_ERR_INVALID_ARG, "max_blocks_per_seq must be positive");
    return launch_append_kv(p->d, layer, (const uint16_t*)k, (const uint16_t*)v, block_table, max_blocks_per_seq, seq_idx,
                            pos, n, (hipStream_t)stream);
}

int32_t chiron_gather_kv(const chiron_kvpool* p, int32_t layer, const int32_t* block_table_row, int32_t len, void* k_out,
                         void* v_out, void* stream) {
    if (!p) return fail(CHIRON_ERR_INVALID_ARG, "pool is null");
    if (len < 0) return fail(CHIRON_ERR_INVALID_ARG, "len is negative");
    if (len == 0) return CHIRON_OK;
    if (layer < 0 || layer >= p->d.n_layers) return fail(CHIRON_ERR_INVALID_ARG, "layer %d out of range", layer);
    if (!block_table_row || !k_out || !v_out) return fail(CHIRON_ERR_INVALID_ARG, "a pointer argument is null");
    return launch_gather_kv(p->d, layer, block_table_row, len, (uint16_t*)k_out, (uint16_t*)v_out, (hipStream_t)stream);
}

static int32_t swap_common(const chiron_kvpool* p, const int32_t* row, int32_t n_pages, const void* image, int to_image,
                           void* stream) {
    if (!p) return fail(CHIRON_ERR_INVALID_ARG, "pool is null");
    if (n_pages < 0) return fail(CHIRON_ERR_INVALID_ARG, "n_pages is negative");
    if (n_pages == 0) return CHIRON_OK;
    if (!row || !image) return fail(CHIRON_ERR_INVALID_ARG, "a pointer argument is null");
    if ((uintptr_t)image & 15) return fail(CHIRON_ERR_INVALID_ARG, "image must be 16-byte aligned");
    return launch_swap(p->d, row, n_pages, (uint16_t*)const_cast<void*>(image), to_image, (hipStream_t)stream);
}

int32_t chiron_kv_swap_out(const chiron_kvpool* p, const int32_t* block_table_row, int32_t n_pages, void* image,
                           void* stream) {
    return swap_common(p, block_table_row, n_pages, image, 1, stream);
}

int32_t chiron_kv_swap_in(chiron_kvpool* p, const int32_t* block_table_row, int32_t n_pages, const void* image,
                          void* stream) {
    return swap_common(p, block_table_row, n_pages, image, 0, stream);
}

// ---- the step ------------------------------------------------------------------------------------------
static int32_t check_step_args(const chiron_model* m, const chiron_kvpool* p, const int32_t* block_table,
                               const int32_t* seq_lens, const int32_t* tokens, int32_t batch) {
    if (!m || !p) return fail(CHIRON_ERR_INVALID_ARG, "model or pool is null");
    if (batch < 0) return fail(CHIRON_ERR_INVALID_ARG, "batch is negative");
    if (batch > m->cfg.max_batch) return fail(CHIRON_ERR_BATCH_TOO_LARGE, "batch %d exceeds max_batch %d", batch, m->cfg.max_batch);
    if (batch > 0 && (!block_table || !seq_lens || !tokens)) return fail(CHIRON_ERR_INVALID_ARG, "an index array is null");
    if (p->d.n_kv != m->cfg.n_kv_heads || p->d.d != m->cfg.head_dim || p->d.n_layers != m->cfg.n_layers)
        return fail(CHIRON_ERR_INVALID_ARG, "pool was created for a different model shape");
    return CHIRON_OK;
}

// whether the feed-forward block's intermediate takes the tiled two-term form (needs the workspace for it)
static bool ffn_packed(const Linear& down, int M, const uint16_t* asplit) { return asplit && M >= linear_big_min_rows(down); }

// One pass of the model over B rows.  Row r carries token tokens[r] at position seq_lens[r] of the request whose
// pages block_table row r lists.  With q_len == 1 a row is a request.  With q_len > 1 rows r = i*q_len + t are the
// new tokens of request i (expanded index arrays), and attention runs per request over (req_bt, req_lens, B/q_len):
// a pass over a request's pages serves as many of its q_len tokens as fit the attention kernel's operand columns.
static int32_t step_rows(chiron_model* m, chiron_kvpool* p, const int32_t* block_table, const int32_t* seq_lens,
                         const int32_t* tokens, int32_t B, const int32_t* req_bt, const int32_t* req_lens, int32_t q_len,
                         float* logits, hipStream_t st) {
    const AttnShape ash = attn_shape(m->cfg.n_q_heads / m->cfg.n_kv_heads, q_len, q_len);
    int32_t rc;
    const chiron_model_config& c = m->cfg;
    const int H = c.hidden, d = c.head_dim, F = c.ffn, qn = c.n_q_heads * d, kn = c.n_kv_heads * d;
    const int n_req = B / q_len;
    const int mb = c.max_blocks_per_seq;
    // while kernel timing is on, the kernels of each launch carry their own start/stop events (see launch())
    TimingScope scope;
    scope.sink = &m->timed;
    struct ScopeGuard {
        bool on;
        explicit ScopeGuard(TimingScope* s) : on(s != nullptr) { if (on) timing_scope() = s; }
        ~ScopeGuard() { if (on) timing_scope() = nullptr; }
    } guard(m->timing ? &scope : nullptr);
#define STEP(cls_, expr)              \
    do {                              \
        scope.cls = (cls_);           \
        scope.first = true;           \
        if ((rc = (expr))) return rc; \
    } while (0)
    const int msplit = linear_max_split();
    int ks_res = 0, ks_qkv = 1;  // K-slices waiting in m->part for the residual stream / of the QKV projection
    STEP(CHIRON_K_OTHER, launch_embed(m->embed, tokens, B, H, m->h, st));
    STEP(CHIRON_K_OTHER, launch_rope_table(seq_lens, B, d, c.rope_base, m->cos_t, m->sin_t, st));
    STEP(CHIRON_K_OTHER, launch_attn_plan(m->aws, req_lens, req_bt, mb, ash, n_req, c.n_kv_heads, st));
    for (int l = 0; l < c.n_layers; ++l) {
        // h += (slices of the previous down projection); x = norm(h)
        STEP(CHIRON_K_RMSNORM, launch_rmsnorm(m->h, m->part, ks_res, m->attn_norm + (size_t)l * H, B, H, c.rms_eps, m->x, st));
        STEP(CHIRON_K_QKV, launch_linear(m->qkv[l], m->x, H, B, m->qkvb, qn + 2 * kn, 0, PRO_NONE, m->part, msplit, &ks_qkv, m->asplit, st));
        STEP(CHIRON_K_ROPE_APPEND,
             launch_rope_append(p->d, l, ks_qkv > 1 ? m->part : m->qkvb, ks_qkv, c.n_q_heads, m->cos_t, m->sin_t, block_table,
                                mb, seq_lens, B, m->qb, st));
        STEP(CHIRON_K_ATTN, launch_attn_main(m->aws, p->d, l, m->qb, qn, c.n_q_heads, req_bt, mb, req_lens, ash, n_req, st));
        STEP(CHIRON_K_ATTN_MERGE, launch_attn_merge(m->aws, p->d, c.n_q_heads, ash, n_req, m->attn, qn, st));
        STEP(CHIRON_K_O, launch_linear(m->wo[l], m->attn, qn, B, m->h, H, 1, PRO_NONE, m->part, msplit, &ks_res, m->asplit, st));
        if (ks_res == 1) ks_res = 0;  // written straight into h
        STEP(CHIRON_K_RMSNORM, launch_rmsnorm(m->h, m->part, ks_res, m->ffn_norm + (size_t)l * H, B, H, c.rms_eps, m->x, st));
        // a = silu(x Wg) * (x Wu) leaves the gate/up projection as fp32 rows, or, with many rows, as the tiled bf16 terms
        // that the down projection copies straight into LDS
        if (ffn_packed(m->down[l], B, m->asplit)) {
            STEP(CHIRON_K_GATEUP, launch_linear(m->gu[l], m->x, H, B, reinterpret_cast<float*>(m->asplit), m->down[l].Kpad, EPI_SWIGLU_PACKED,
                                                PRO_NONE, nullptr, 1, nullptr, nullptr, st));
            STEP(CHIRON_K_DOWN, launch_linear(m->down[l], reinterpret_cast<const float*>(m->asplit), 0, B, m->h, H, EPI_ADD, PRO_PACKED,
                                              m->part, msplit, &ks_res, nullptr, st));
        } else {
            STEP(CHIRON_K_GATEUP, launch_linear(m->gu[l], m->x, H, B, m->gub, F, EPI_SWIGLU, PRO_NONE, nullptr, 1, nullptr, m->asplit, st));
            STEP(CHIRON_K_DOWN, launch_linear(m->down[l], m->gub, F, B, m->h, H, EPI_ADD, PRO_NONE, m->part, msplit, &ks_res, m->asplit, st));
        }
        if (ks_res == 1) ks_res = 0;
    }
    STEP(CHIRON_K_RMSNORM, launch_rmsnorm(m->h, m->part, ks_res, m->final_norm, B, H, c.rms_eps, m->x, st));
    STEP(CHIRON_K_LMHEAD, launch_linear(m->lm, m->x, H, B, logits, c.vocab, 0, PRO_NONE, nullptr, 1, nullptr, m->asplit, st));
#undef STEP
    return CHIRON_OK;
}

int32_t chiron_decode_step(chiron_model* m, chiron_kvpool* p, const int32_t* block_table, const int32_t* seq_lens,
                           const int32_t* tokens, int32_t batch, float* logits, void* stream) {
    int32_t rc = check_step_args(m, p, block_table, seq_lens, tokens, batch);
    if (rc) return rc;
    if (batch == 0) return CHIRON_OK;
    if (!logits) return fail(CHIRON_ERR_INVALID_ARG, "logits is null");
    return step_rows(m, p, block_table, seq_lens, tokens, batch, block_table, seq_lens, 1, logits, (hipStream_t)stream);
}

int32_t chiron_decode_step_multi(chiron_model* m, chiron_kvpool* p, const int32_t* block_table, const int32_t* seq_lens,
                                 const int32_t* tokens, int32_t batch, int32_t q_len, float* logits, void* stream) {
    if (q_len < 1) return fail(CHIRON_ERR_INVALID_ARG, "q_len must be at least 1");
    if (q_len == 1) return chiron_decode_step(m, p, block_table, seq_lens, tokens, batch, logits, stream);
    if (batch < 0) return fail(CHIRON_ERR_INVALID_ARG, "batch is negative");
    if (!m) return fail(CHIRON_ERR_INVALID_ARG, "model or pool is null");
    if ((int64_t)batch * q_len > m->cfg.max_batch)
        return fail(CHIRON_ERR_BATCH_TOO_LARGE, "batch*q_len = %lld exceeds max_batch %d", (long long)batch * q_len, m->cfg.max_batch);
    int32_t rc = check_step_args(m, p, block_table, seq_lens, tokens, batch);
    if (rc) return rc;
    if (batch == 0) return CHIRON_OK;
    // rows (i, t) share request i's pages; row t sees the K/V that rows t' <= t append in the same layer, because
    // every layer appends all rows before its attention starts
    if (!logits) return fail(CHIRON_ERR_INVALID_ARG, "logits is null");
    rc = launch_expand_rows(block_table, seq_lens, batch, q_len, m->cfg.max_blocks_per_seq, m->x_bt, m->x_lens,
                            (hipStream_t)stream);
    if (rc) return rc;
    // attention runs per request: its pages are read once per group of as many tokens as fit the 16 operand columns
    return step_rows(m, p, m->x_bt, m->x_lens, tokens, batch * q_len, block_table, seq_lens, q_len, logits, (hipStream_t)stream);
}

static int32_t check_inputs_host(const chiron_model_config* cfg, int32_t num_blocks, int32_t block_size,
                                 const int32_t* block_table, const int32_t* seq_lens, const int32_t* tokens, int32_t batch,
                                 int32_t q_len) {
    if (!cfg) return fail(CHIRON_ERR_INVALID_ARG, "config is null");
    if (batch < 0) return fail(CHIRON_ERR_INVALID_ARG, "batch is negative");
    if (q_len < 1) return fail(CHIRON_ERR_INVALID_ARG, "q_len must be at least 1");
    if ((int64_t)batch * q_len > cfg->max_batch)
        return fail(CHIRON_ERR_BATCH_TOO_LARGE, "batch*q_len = %lld exceeds max_batch %d", (long long)batch * q_len, cfg->max_batch);
    if (block_size != kBlockSize) return fail(CHIRON_ERR_INVALID_ARG, "block_size %d: must be 16", block_size);
    if (batch > 0 && (!block_table || !seq_lens || !tokens)) return fail(CHIRON_ERR_INVALID_ARG, "an index array is null");
    std::unordered_set<int32_t> written;
    for (int i = 0; i < batch; ++i) {
        for (int t = 0; t < q_len; ++t) {
            const int32_t tok = tokens[(size_t)i * q_len + t];
            if (tok < 0 || tok >= cfg->vocab)
                return fail(CHIRON_ERR_TOKEN, "tokens[%d] = %d is outside [0, %d)", i * q_len + t, tok, cfg->vocab);
        }
        if (seq_lens[i] < 0) return fail(CHIRON_ERR_INVALID_ARG, "seq_lens[%d] = %d is negative", i, seq_lens[i]);
        int64_t need = ((int64_t)seq_lens[i] + q_len + block_size - 1) / block_size;
        if (need > cfg->max_blocks_per_seq)
            return fail(CHIRON_ERR_BLOCK_TABLE, "request %d needs %lld pages, block table rows hold %d", i, (long long)need,
                        cfg->max_blocks_per_seq);
        const int32_t* row = block_table + (size_t)i * cfg->max_blocks_per_seq;
        for (int64_t b = 0; b < need; ++b)
            if (row[b] < 0 || row[b] >= num_blocks)
                return fail(CHIRON_ERR_BLOCK_TABLE, "block_table[%d][%lld] = %d is not a page of the pool (%d pages)", i,
                            (long long)b, row[b], num_blocks);
        // the pages that hold positions seq_lens[i] .. seq_lens[i]+q_len-1 are written
        for (int64_t b = seq_lens[i] / block_size; b < need; ++b)
            if (!written.insert(row[b]).second)
                return fail(CHIRON_ERR_BLOCK_TABLE, "page %d is written by more than one request (request %d)", row[b], i);
    }
    // a page that one request writes must not be read by another (shared pages are read-only)
    for (int i = 0; i < batch; ++i) {
        const int32_t* row = block_table + (size_t)i * cfg->max_blocks_per_seq;
        int64_t wi = seq_lens[i] / block_size;
        for (int64_t b = 0; b < wi; ++b)
            if (written.count(row[b]))
                return fail(CHIRON_ERR_BLOCK_TABLE, "page %d is read by request %d and written by another", row[b], i);
    }
    return CHIRON_OK;
}

int32_t chiron_check_step_inputs_host(const chiron_model_config* cfg, int32_t num_blocks, int32_t block_size,
                                      const int32_t* block_table, const int32_t* seq_lens, const int32_t* tokens,
                                      int32_t batch) {
    return check_inputs_host(cfg, num_blocks, block_size, block_table, seq_lens, tokens, batch, 1);
}

int32_t chiron_check_step_inputs_host_multi(const chiron_model_config* cfg, int32_t num_blocks, int32_t block_size,
                                            const int32_t* block_table, const int32_t* seq_lens, const int32_t* tokens,
                                            int32_t batch, int32_t q_len) {
    return check_inputs_host(cfg, num_blocks, block_size, block_table, seq_lens, tokens, batch, q_len);
}

static int32_t validate_on_device(const chiron_model* m, const chiron_kvpool* p, const int32_t* block_table,
                                  const int32_t* seq_lens, const int32_t* tokens, int32_t batch, int32_t q_len, void* stream) {
    if (q_len < 1) return fail(CHIRON_ERR_INVALID_ARG, "q_len must be at least 1");
    int32_t rc = check_step_args(m, p, block_table, seq_lens, tokens, batch);
    if (rc) return rc;
    if (batch == 0) return CHIRON_OK;
    hipStream_t st = (hipStream_t)stream;
    const int mb = m->cfg.max_blocks_per_seq;
    std::vector<int32_t> bt((size_t)batch * mb), sl(batch), tk((size_t)batch * q_len);
    CHIRON_HIP(hipMemcpyAsync(bt.data(), block_table, bt.size() * 4, hipMemcpyDeviceToHost, st));
    CHIRON_HIP(hipMemcpyAsync(sl.data(), seq_lens, sl.size() * 4, hipMemcpyDeviceToHost, st));
    CHIRON_HIP(hipMemcpyAsync(tk.data(), tokens, tk.size() * 4, hipMemcpyDeviceToHost, st));
    CHIRON_HIP(hipStreamSynchronize(st));
    return check_inputs_host(&m->cfg, p->d.num_blocks, p->block_size, bt.data(), sl.data(), tk.data(), batch, q_len);
}

int32_t chiron_validate_step_inputs(const chiron_model* m, const chiron_kvpool* p, const int32_t* block_table,
                                    const int32_t* seq_lens, const int32_t* tokens, int32_t batch, void* stream) {
    return validate_on_device(m, p, block_table, seq_lens, tokens, batch, 1, stream);
}

int32_t chiron_validate_step_inputs_multi(const chiron_model* m, const chiron_kvpool* p, const int32_t* block_table,
                                          const int32_t* seq_lens, const int32_t* tokens, int32_t batch, int32_t q_len,
                                          void* stream) {
    return validate_on_device(m, p, block_table, seq_lens, tokens, batch, q_len, stream);
}

int32_t chiron_step_latency_profile(chiron_model* m, chiron_kvpool* p, const int32_t* block_table,
                                    const int32_t* seq_lens, const int32_t* tokens, const int32_t* batch_sizes,
                                    int32_t n_sizes, int32_t warmup, int32_t iters, float* logits_scratch, void* stream,
                                    chiron_profile_point* out) {
    if (!batch_sizes || !out) return fail(CHIRON_ERR_INVALID_ARG, "batch_sizes or out is null");
    if (n_sizes < 0 || warmup < 0 || iters < 1) return fail(CHIRON_ERR_INVALID_ARG, "n_sizes/warmup must be >= 0 and iters >= 1");
    hipStream_t st = (hipStream_t)stream;
    for (int k = 0; k < n_sizes; ++k) {
        int b = batch_sizes[k];
        if (b < 1) return fail(CHIRON_ERR_INVALID_ARG, "batch_sizes[%d] = %d must be positive", k, b);
        int32_t rc = check_step_args(m, p, block_table, seq_lens, tokens, b);
        if (rc) return rc;
    }
    std::vector<hipEvent_t> ev((size_t)iters + 1, nullptr);
    int32_t rc = CHIRON_OK;
    for (auto& e : ev)
        if (rc == CHIRON_OK && hipEventCreate(&e) != hipSuccess) rc = fail(CHIRON_ERR_HIP, "profile: cannot create an event");
    for (int k = 0; k < n_sizes && rc == CHIRON_OK; ++k) {
        int b = batch_sizes[k];
        for (int w = 0; w < warmup && rc == CHIRON_OK; ++w)
            rc = chiron_decode_step(m, p, block_table, seq_lens, tokens, b, logits_scratch, stream);
        if (rc) break;
        hipError_t e = hipEventRecord(ev[0], st);
        for (int it = 0; it < iters && rc == CHIRON_OK && e == hipSuccess; ++it) {
            rc = chiron_decode_step(m, p, block_table, seq_lens, tokens, b, logits_scratch, stream);
            e = hipEventRecord(ev[it + 1], st);
        }
        if (rc == CHIRON_OK && e == hipSuccess) e = hipStreamSynchronize(st);
        if (rc == CHIRON_OK && e != hipSuccess) rc = fail(CHIRON_ERR_HIP, "profile: %s", hipGetErrorString(e));
        if (rc) break;
        std::vector<double> ms(iters);
        double sum = 0;
        for (int it = 0; it < iters; ++it) {
            float t = 0.f;
            (void)hipEventElapsedTime(&t, ev[it], ev[it + 1]);
            ms[it] = t;
            sum += t;
        }
        std::sort(ms.begin(), ms.end());
        out[k].batch = b;
        out[k].lat_ms_median = (iters % 2) ? ms[iters / 2] : 0.5 * (ms[iters / 2 - 1] + ms[iters / 2]);
        int i99 = (int)std::min<double>(iters - 1, std::ceil(0.99 * iters) - 1);
        out[k].lat_ms_p99 = ms[i99 < 0 ? 0 : i99];
        out[k].lat_ms_mean = sum / iters;
        out[k].tokens_per_s = b / (out[k].lat_ms_median * 1e-3);
    }
    for (auto& e : ev)
        if (e) (void)hipEventDestroy(e);
    return rc;
}

// ---- single kernels ------------------------------------------------------------------------------------
int32_t chiron_op_rmsnorm(const float* h, const void* gain, int32_t rows, int32_t n, float eps, float* out, void* stream) {
    if (rows < 0 || n < 1) return fail(CHIRON_ERR_INVALID_ARG, "rmsnorm: bad sizes");
    if (rows == 0) return CHIRON_OK;
    if (!h || !gain || !out) return fail(CHIRON_ERR_INVALID_ARG, "rmsnorm: a pointer is null");
    return launch_rmsnorm(const_cast<float*>(h), nullptr, 0, (const uint16_t*)gain, rows, n, eps, out, (hipStream_t)stream);
}

int32_t chiron_linear_create(const void* w, int32_t N, int32_t K, void* stream, chiron_linear** out) {
    if (!out) return fail(CHIRON_ERR_INVALID_ARG, "out is null");
    *out = nullptr;
    if (!w || N < 1 || K < 1) return fail(CHIRON_ERR_INVALID_ARG, "linear: null weight or non-positive size");
    if (K % 16 != 0) return fail(CHIRON_ERR_SHAPE, "linear: K=%d must be a multiple of 16", K);
    chiron_linear* l = new (std::nothrow) chiron_linear();
    if (!l) return fail(CHIRON_ERR_OOM, "host allocation failed");
    int32_t rc = linear_alloc(l->L, N, K);
    if (!rc) rc = launch_pack_rows((const uint16_t*)w, N, K, l->L.tstride, l->L.w, 0, (hipStream_t)stream);
    if (rc) {
        linear_free(l->L);
        delete l;
        return rc;
    }
    *out = l;
    return CHIRON_OK;
}

int32_t chiron_linear_create_gate_up(const void* w_gate, const void* w_up, int32_t F, int32_t K, void* stream, chiron_linear** out) {
    if (!out) return fail(CHIRON_ERR_INVALID_ARG, "out is null");
    *out = nullptr;
    if (!w_gate || !w_up || F < 1 || K < 1) return fail(CHIRON_ERR_INVALID_ARG, "gate/up: null weight or non-positive size");
    if (K % 16 != 0 || F % 16 != 0) return fail(CHIRON_ERR_SHAPE, "gate/up: K=%d and F=%d must be multiples of 16", K, F);
    chiron_linear* l = new (std::nothrow) chiron_linear();
    if (!l) return fail(CHIRON_ERR_OOM, "host allocation failed");
    l->gate_up = true;
    int32_t rc = linear_alloc(l->L, 2 * F, K);
    if (!rc) rc = launch_pack_rows((const uint16_t*)w_gate, F, K, l->L.tstride, l->L.w, 0, (hipStream_t)stream, 1);
    if (!rc) rc = launch_pack_rows((const uint16_t*)w_up, F, K, l->L.tstride, l->L.w, 0, (hipStream_t)stream, 2);
    if (rc) {
        linear_free(l->L);
        delete l;
        return rc;
    }
    *out = l;
    return CHIRON_OK;
}

int32_t chiron_linear_destroy(chiron_linear* l) {
    if (l) {
        linear_free(l->L);
        delete l;
    }
    return CHIRON_OK;
}

// the projection as the decode step launches it (K sliced into a workspace when the grid would otherwise be
// too small), followed by the plain sum of the slices that the step's consumers do on the fly
static int32_t op_linear_common(const Linear& L, const float* x, int lda, int M, float* y, int accumulate, int prologue,
                                hipStream_t st) {
    float* part = nullptr;
    const int msplit = linear_max_split();
    // wide outputs (LM head, gate/up) have enough column tiles on their own and are never sliced in the step
    const bool may_split = L.N <= 16384;
    if (may_split) CHIRON_HIP(hipMallocAsync((void**)&part, (size_t)msplit * M * L.N * sizeof(float), st));
    uint16_t* asplit = nullptr;
    if (prologue == PRO_NONE && tuning().linear_big_all && M >= linear_big_min_rows(L))
        CHIRON_HIP(hipMallocAsync((void**)&asplit, 2 * linear_big_split_elems(M, L.Kpad) * 2, st));
    int ks = 1;
    int32_t rc = launch_linear(L, x, lda, M, y, L.N, accumulate ? EPI_ADD : EPI_STORE, prologue, part, msplit, &ks, asplit, st);
    if (asplit) (void)hipFreeAsync(asplit, st);
    if (!rc && ks > 1) rc = launch_reduce_partials(part, ks, (int64_t)M * L.N, y, accumulate, st);
    if (part) (void)hipFreeAsync(part, st);
    return rc;
}

int32_t chiron_op_linear(const chiron_linear* l, const float* x, int32_t M, float* y, int32_t accumulate, void* stream) {
    if (!l) return fail(CHIRON_ERR_INVALID_ARG, "linear is null");
    if (M < 0) return fail(CHIRON_ERR_INVALID_ARG, "M is negative");
    if (M == 0) return CHIRON_OK;
    if (!x || !y) return fail(CHIRON_ERR_INVALID_ARG, "linear: a pointer is null");
    if (l->gate_up) return fail(CHIRON_ERR_INVALID_ARG, "linear: a fused gate/up matrix goes with the SwiGLU entry points only");
    return op_linear_common(l->L, x, l->L.K, M, y, accumulate, PRO_NONE, (hipStream_t)stream);
}

int32_t chiron_op_gate_up_swiglu(const chiron_linear* gate_up, const float* x, int32_t M, float* act, void* stream) {
    if (!gate_up) return fail(CHIRON_ERR_INVALID_ARG, "linear is null");
    if (M < 0) return fail(CHIRON_ERR_INVALID_ARG, "M is negative");
    if (M == 0) return CHIRON_OK;
    if (!x || !act) return fail(CHIRON_ERR_INVALID_ARG, "gate_up_swiglu: a pointer is null");
    if (!gate_up->gate_up) return fail(CHIRON_ERR_INVALID_ARG, "gate_up_swiglu: the matrix was not created as a fused gate/up matrix");
    const Linear& L = gate_up->L;
    return launch_linear(L, x, L.K, M, act, L.N / 2, EPI_SWIGLU, PRO_NONE, nullptr, 1, nullptr, nullptr, (hipStream_t)stream);
}

int32_t chiron_op_swiglu_ffn(const chiron_linear* gate_up, const chiron_linear* down, const float* x, int32_t M, float* y,
                             int32_t accumulate, void* stream) {
    if (!gate_up || !down) return fail(CHIRON_ERR_INVALID_ARG, "linear is null");
    if (M < 0) return fail(CHIRON_ERR_INVALID_ARG, "M is negative");
    if (M == 0) return CHIRON_OK;
    if (!x || !y) return fail(CHIRON_ERR_INVALID_ARG, "swiglu_ffn: a pointer is null");
    if (!gate_up->gate_up || down->gate_up) return fail(CHIRON_ERR_INVALID_ARG, "swiglu_ffn: wants a fused gate/up matrix and a plain one");
    const Linear &G = gate_up->L, &D = down->L;
    const int F = G.N / 2;
    if (D.K != F) return fail(CHIRON_ERR_SHAPE, "swiglu_ffn: gate/up has %d columns, the down projection %d inputs", F, D.K);
    hipStream_t st = (hipStream_t)stream;
    // the intermediate in the form the decode step gives it at this row count
    const bool packed = M >= linear_big_min_rows(D);
    const size_t bytes = packed ? 2 * linear_big_split_elems(M, D.Kpad) * 2 : (size_t)M * F * 4;
    void* act = nullptr;
    CHIRON_HIP(hipMallocAsync(&act, bytes, st));
    int32_t rc = CHIRON_OK;
    if (packed) {
        if (hipMemsetAsync(act, 0, bytes, st) != hipSuccess) rc = fail(CHIRON_ERR_HIP, "clearing the activation workspace failed");
        if (!rc) rc = launch_linear(G, x, G.K, M, (float*)act, D.Kpad, EPI_SWIGLU_PACKED, PRO_NONE, nullptr, 1, nullptr, nullptr, st);
        if (!rc) rc = op_linear_common(D, (const float*)act, 0, M, y, accumulate, PRO_PACKED, st);
    } else {
        rc = launch_linear(G, x, G.K, M, (float*)act, F, EPI_SWIGLU, PRO_NONE, nullptr, 1, nullptr, nullptr, st);
        if (!rc) rc = op_linear_common(D, (const float*)act, F, M, y, accumulate, PRO_NONE, st);
    }
    (void)hipFreeAsync(act, st);
    return rc;
}

int32_t chiron_op_rope(float* x, int32_t rows, int32_t n_heads, int32_t d, const int32_t* pos, float base, void* stream) {
    if (rows < 0 || n_heads < 1 || d < 2 || (d & 1)) return fail(CHIRON_ERR_INVALID_ARG, "rope: bad sizes");
    if (rows == 0) return CHIRON_OK;
    if (!x || !pos) return fail(CHIRON_ERR_INVALID_ARG, "rope: a pointer is null");
    hipStream_t st = (hipStream_t)stream;
    float* tab = nullptr;
    size_t n = (size_t)rows * (d / 2);
    CHIRON_HIP(hipMallocAsync((void**)&tab, 2 * n * sizeof(float), st));
    int32_t rc = launch_rope_table(pos, rows, d, base, tab, tab + n, st);
    if (!rc) rc = launch_rope(x, n_heads * d, n_heads, d, tab, tab + n, rows, st);
    (void)hipFreeAsync(tab, st);
    return rc;
}

// ---- the rotary embedding for callers that cannot allocate ---------------------------------------------------
// Same kernels as chiron_op_rope; the cos/sin table they pass between them lives in a file-scope device array
// instead of a hipMallocAsync block.  `scratch` names the array for the device compiler only: host code never passes
// the name to a kernel or a copy but the address that hipGetSymbolAddress reports, looked up once per device (each
// device holds its own copy of the array at its own address).
static constexpr size_t kRopeScratchFloats = (size_t)1 << 18;  // 1 MiB: cos and sin of rows * d/2 angles each
static __device__ __align__(256) float scratch[kRopeScratchFloats];
static constexpr int kMaxDevices = 64;
static float* g_scratch_addr[kMaxDevices];  // per device, null until looked up
static std::mutex g_scratch_mutex;

static int32_t rope_scratch(float** out) {
    int dev = -1;
    CHIRON_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(CHIRON_ERR_HIP, "rope_noalloc: device index %d is out of range", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_addr[dev]) {
        void* p = nullptr;
        CHIRON_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(CHIRON_ERR_HIP, "rope_noalloc: the scratch array has no address on device %d", dev);
        g_scratch_addr[dev] = (float*)p;
    }
    *out = g_scratch_addr[dev];
    return CHIRON_OK;
}

int32_t chiron_op_rope_noalloc(float* x, int32_t rows, int32_t n_heads, int32_t d, const int32_t* pos, float base,
                               void* stream) {
    if (rows < 0 || n_heads < 1 || d < 2 || (d & 1)) return fail(CHIRON_ERR_INVALID_ARG, "rope: bad sizes");
    if (rows == 0) return CHIRON_OK;
    if (!x || !pos) return fail(CHIRON_ERR_INVALID_ARG, "rope: a pointer is null");
    const size_t n = (size_t)rows * (d / 2);
    if (2 * n > kRopeScratchFloats)
        return fail(CHIRON_ERR_SHAPE, "rope_noalloc: rows*d = %zu exceeds the fixed table of %zu values (use chiron_op_rope)",
                    2 * n, kRopeScratchFloats);
    float* tab = nullptr;
    int32_t rc = rope_scratch(&tab);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    // the table kernel writes every entry the rotation reads (rows * d/2 of each half): nothing to clear
    rc = launch_rope_table(pos, rows, d, base, tab, tab + n, st);
    if (!rc) rc = launch_rope(x, n_heads * d, n_heads, d, tab, tab + n, rows, st);
    return rc;
}

int32_t chiron_op_paged_attention(chiron_model* m, const chiron_kvpool* p, int32_t layer, const float* q,
                                  const int32_t* block_table, const int32_t* ctx_lens, int32_t batch, float* out,
                                  void* stream) {
    if (!m || !p) return fail(CHIRON_ERR_INVALID_ARG, "model or pool is null");
    if (batch < 0) return fail(CHIRON_ERR_INVALID_ARG, "batch is negative");
    if (batch > m->cfg.max_batch) return fail(CHIRON_ERR_BATCH_TOO_LARGE, "batch %d exceeds max_batch %d", batch, m->cfg.max_batch);
    if (batch == 0) return CHIRON_OK;
    if (layer < 0 || layer >= p->d.n_layers) return fail(CHIRON_ERR_INVALID_ARG, "layer %d out of range", layer);
    if (!q || !block_table || !ctx_lens || !out) return fail(CHIRON_ERR_INVALID_ARG, "attention: a pointer is null");
    hipStream_t st = (hipStream_t)stream;
    const int qn = m->cfg.n_q_heads * m->cfg.head_dim;
    const AttnShape sh = attn_shape(m->cfg.n_q_heads / m->cfg.n_kv_heads, 1, 0);
    int32_t rc = launch_attn_plan(m->aws, ctx_lens, block_table, m->cfg.max_blocks_per_seq, sh, batch, m->cfg.n_kv_heads, st);
    if (rc) return rc;
    rc = launch_attn_main(m->aws, p->d, layer, q, qn, m->cfg.n_q_heads, block_table, m->cfg.max_blocks_per_seq, ctx_lens, sh,
                          batch, st);
    if (rc) return rc;
    return launch_attn_merge(m->aws, p->d, m->cfg.n_q_heads, sh, batch, out, qn, st);
}

int32_t chiron_local_autoscale_step(double itl, double itl_slo, double tput_prev, double tput_curr, double alpha,
                                    int32_t batch_limit, int32_t* max_batch, double* backpressure_out) {
    if (!max_batch) return fail(CHIRON_ERR_INVALID_ARG, "max_batch is null");
    if (!(itl_slo > 0.0) || !(alpha >= 0.0 && alpha <= 1.0) || batch_limit < 1 || *max_batch < 1)
        return fail(CHIRON_ERR_INVALID_ARG, "autoscale: need itl_slo > 0, 0 <= alpha <= 1, batch_limit >= 1, max_batch >= 1");
    if (backpressure_out) *backpressure_out = -1.0;
    if (!(itl > 0.0) || !(tput_curr > 0.0)) return CHIRON_OK;  // nothing was observed: keep the batch size
    const double lbp = itl / itl_slo;
    const double tbp = tput_prev > 0.0 ? tput_prev / tput_curr : 0.0;
    const double lb = lbp > tbp ? lbp : tbp;
    double mbs = (double)*max_batch;
    if (lb < 1.0) mbs = lb > 0.0 ? alpha * (1.0 / lb) * mbs + (1.0 - alpha) * mbs : (double)batch_limit;
    else mbs = mbs / 2.0;
    double r = std::floor(mbs + 0.5);
    if (r < 1.0) r = 1.0;
    if (r > (double)batch_limit) r = (double)batch_limit;
    *max_batch = (int32_t)r;
    if (backpressure_out) *backpressure_out = lb;
    return CHIRON_OK;
}

int32_t chiron_set_tuning(const char* key, int32_t value) {
    if (!key) return fail(CHIRON_ERR_INVALID_ARG, "key is null");
    Tuning& t = tuning();
    // allowed values per key: a value outside them would size a grid for a tile shape that is not built
    struct { const char* k; int* p; int lo, hi; unsigned mask; } tab[] = {  // value in [lo, hi]; if mask: bit `value` set
        {"linear_nf", &t.linear_nf, 0, 4, 0x17u},         {"linear_mt", &t.linear_mt, 0, 4, 0u},
        {"linear_xcd_remap", &t.linear_xcd_remap, 0, 1, 0u}, {"linear_ksplit", &t.linear_ksplit, 0, 16, 0u},
        {"linear_target_blocks", &t.linear_target_blocks, 1, 1 << 20, 0u},
        {"linear_big_min_m", &t.linear_big_min_m, -1, 1 << 30, 0u}, {"linear_big_all", &t.linear_big_all, 0, 1, 0u},
        {"linear_ks", &t.linear_ks, 0, 16, 0x10111u},        {"attn_grid", &t.attn_grid, 0, 1 << 16, 0u},
        {"attn_target_waves", &t.attn_target_waves, 0, 1 << 24, 0u}, {"attn_chunk_pages", &t.attn_chunk_pages, 0, 1 << 20, 0u}};
    for (auto& e : tab)
        if (!strcmp(e.k, key)) {
            if (value < e.lo || value > e.hi || (e.mask && !((e.mask >> value) & 1u)))
                return fail(CHIRON_ERR_INVALID_ARG, "tuning key '%s': value %d is not allowed", key, value);
            *e.p = value;
            return CHIRON_OK;
        }
    return fail(CHIRON_ERR_INVALID_ARG, "unknown tuning key '%s'", key);
}

int32_t chiron_kernel_timing_begin(chiron_model* m) {
    if (!m) return fail(CHIRON_ERR_INVALID_ARG, "model is null");
    for (auto& t : m->timed) {
        (void)hipEventDestroy(t.a);
        (void)hipEventDestroy(t.b);
    }
    m->timed.clear();
    m->timing = true;
    return CHIRON_OK;
}

int32_t chiron_kernel_timing_end(chiron_model* m, void* stream, chiron_kernel_time* out) {
    if (!m || !out) return fail(CHIRON_ERR_INVALID_ARG, "model or out is null");
    m->timing = false;
    for (int k = 0; k < CHIRON_K_COUNT; ++k) {
        out[k].ms = 0.0;
        out[k].launches = 0;
    }
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    for (auto& t : m->timed) {
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, t.a, t.b);
        out[t.cls].ms += ms;
        out[t.cls].launches += t.first ? 1 : 0;
        (void)hipEventDestroy(t.a);
        (void)hipEventDestroy(t.b);
    }
    m->timed.clear();
    if (e != hipSuccess) return fail(CHIRON_ERR_HIP, "kernel timing: %s", hipGetErrorString(e));
    return CHIRON_OK;
}

}  // extern "C"

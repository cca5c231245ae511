// Paged GQA decode attention, split over the context ("split-K") with a wavefront-level online
// softmax.  gfx950, wave64.
//
// One wave owns one work item: (request, KV head, run of consecutive pages).  It streams the
// K and V tiles of its pages from HBM straight into matrix-core operand registers (the pool's
// tile orders make each fragment a contiguous 1 KiB read), computes the 16-token x G-head score
// tile with v_mfma_f32_16x16x32_bf16, keeps the running max / sum per head in registers, and
// accumulates P*V with v_mfma_f32_16x16x16_bf16 (the score tile's register layout is exactly the
// operand layout that instruction wants, so P never leaves registers).  q and P enter the matrix
// cores as two bf16 terms each.  Items write (max, sum, unnormalised output); a second kernel
// merges the items of a request.
//
// The work list is built on the device from seq_lens (the host never sees the lengths), and the
// attention grid is persistent: a wave starts on the item of its own index and then draws the
// index of each further item from a ticket counter, one item ahead, so that waves whose items
// were short (the ragged last run of a request) take more of them.  There are eight counters,
// each on a cache line of its own and each serving every eighth item and every eighth workgroup
// (one counter takes about 50 M draws a second, too few for lists of small items).  Tickets only
// grow and the list has a fixed length in memory, so every wave terminates.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <type_traits>

#include "chiron_internal.h"
#include "device_util.h"

namespace chiron {

// plan buffer layout (int32): [0] n_items, [1] chunk_pages, [2..3] unused,
// [4, 4+max_batch) first item of pass v, [.., +max_batch) number of items of pass v,
// then item_seq[cap_items] (the pass), item_pg0[cap_items].  A pass v = request * ng + token group (AttnShape).
// Last, 32-byte aligned, one record of 8 ints per item: {pass, first page, attended length, the ids of the item's
// first four pages (past its end: its last page), 0}: everything a wave needs before its first tile load, in one
// scalar load instead of a chain of four dependent ones (the block table does not differ between layers).
// After the records, kTicketQueues ticket counters kTicketStride ints apart, all 0 between attention launches.
__host__ __device__ inline int64_t plan_rec_offset(int max_batch, int cap_items) {
    return (4 + 2 * (int64_t)max_batch + 2 * (int64_t)cap_items + 7) / 8 * 8;
}
constexpr int kTicketQueues = 8, kTicketStride = 64;
__host__ __device__ inline int64_t plan_ticket_offset(int max_batch, int cap_items) {
    return (plan_rec_offset(max_batch, cap_items) + 8 * (int64_t)cap_items + kTicketStride - 1) / kTicketStride * kTicketStride;
}
int64_t attn_plan_ints(int max_batch, int cap_items) { return plan_ticket_offset(max_batch, cap_items) + kTicketQueues * kTicketStride; }

AttnShape attn_shape(int G, int q_len, int len_bias) {
    AttnShape sh;
    sh.q_len = q_len;
    sh.tg = std::min(q_len, std::max(1, 16 / G));
    sh.ng = (q_len + sh.tg - 1) / sh.tg;
    sh.bias0 = len_bias - q_len;
    return sh;
}

// positions attended by pass v (its last token's view)
__device__ __forceinline__ int pass_len(const int32_t* __restrict__ seq_lens, const AttnShape& sh, int v) {
    const int i = v / sh.ng, g = v - i * sh.ng;
    return seq_lens[i] + sh.bias0 + g * sh.tg + min(sh.tg, sh.q_len - g * sh.tg);
}

constexpr int kPlanThreads = 1024;

__global__ __launch_bounds__(kPlanThreads) void attn_plan_kernel(int32_t* __restrict__ plan, int max_batch, int cap_items,
                                                                 const int32_t* __restrict__ seq_lens, AttnShape sh,
                                                                 int batch, int n_kv, int slots, int target_waves, int force_cp, int item_limit,
                                                                 const int32_t* __restrict__ bt, int max_blocks) {
    batch *= sh.ng;  // passes
    __shared__ int scan[kPlanThreads];
    int32_t* seq_item0 = plan + 4;
    int32_t* seq_nch = plan + 4 + max_batch;
    int32_t* item_seq = plan + 4 + 2 * max_batch;
    int32_t* item_pg0 = item_seq + cap_items;
    const int tid = threadIdx.x;
    if (tid < kTicketQueues) plan[plan_ticket_offset(max_batch, cap_items) + tid * kTicketStride] = 0;
    const int per = (batch + kPlanThreads - 1) / kPlanThreads;  // requests per thread, contiguous
    const int i0 = tid * per, i1 = min(batch, i0 + per);

    // block-wide sums over the requests (every thread gets the total)
    auto block_sum = [&](int v) {
        __syncthreads();
        scan[tid] = v;
        __syncthreads();
        for (int o = kPlanThreads / 2; o > 0; o >>= 1) {
            if (tid < o) scan[tid] += scan[tid + o];
            __syncthreads();
        }
        return scan[0];
    };
    auto count_items = [&](int cp) {
        int n = 0;
        for (int i = i0; i < i1; ++i) n += ((pass_len(seq_lens, sh, i) + kBlockSize - 1) / kBlockSize + cp - 1) / cp;
        return block_sum(n);
    };
    int pages = 0;
    for (int i = i0; i < i1; ++i) pages += (pass_len(seq_lens, sh, i) + kBlockSize - 1) / kBlockSize;
    const int total = block_sum(pages);

    // Pages per item.  A wave takes items w, w + slots, ...: if the list is only a little longer than the number of
    // wave slots, a few waves run a second item alone, at latency-bound speed, after everyone else has finished.
    // So: when one round can hold everything, take the smallest item size that fits one round (all items stream
    // concurrently); otherwise make the items small enough for at least four rounds, where a ragged last round
    // costs little, but not so small that the per-item partial result weighs against the bytes the item reads.
    int cp;
    if ((int64_t)count_items(64) * n_kv <= slots) {
        int lo = 2, hi = 64;
        while (lo < hi) {  // uniform over the workgroup: every thread sees the same counts
            const int mid = (lo + hi) / 2;
            if ((int64_t)count_items(mid) * n_kv <= slots) hi = mid;
            else lo = mid + 1;
        }
        cp = lo;
    } else {
        cp = 64;
        while (cp > 8 && (int64_t)(total / cp) * n_kv < target_waves) cp >>= 1;
    }
    while (cp < (1 << 24) && total / cp + batch > item_limit) cp <<= 1;  // the host has checked that batch < item_limit
    if (force_cp > 0 && total / force_cp + batch <= item_limit) cp = force_cp;
    __syncthreads();

    // exclusive scan of items per request
    int items = 0;
    for (int i = i0; i < i1; ++i) {
        int np = (pass_len(seq_lens, sh, i) + kBlockSize - 1) / kBlockSize;
        items += (np + cp - 1) / cp;
    }
    scan[tid] = items;
    __syncthreads();
    for (int o = 1; o < kPlanThreads; o <<= 1) {
        int v = tid >= o ? scan[tid - o] : 0;
        __syncthreads();
        scan[tid] += v;
        __syncthreads();
    }
    int off = scan[tid] - items;
    for (int i = i0; i < i1; ++i) {
        int np = (pass_len(seq_lens, sh, i) + kBlockSize - 1) / kBlockSize;
        int nch = (np + cp - 1) / cp;
        seq_item0[i] = off;
        seq_nch[i] = nch;
        const int len = pass_len(seq_lens, sh, i);
        const int32_t* btrow = bt + (size_t)(i / sh.ng) * max_blocks;
        for (int ch = 0; ch < nch; ++ch) {
            item_seq[off + ch] = i;
            item_pg0[off + ch] = ch * cp;
            int32_t* rec = plan + plan_rec_offset(max_batch, cap_items) + 8 * (int64_t)(off + ch);
            const int pg1 = min(ch * cp + cp, np);
            rec[0] = i;
            rec[1] = ch * cp;
            rec[2] = len;
            for (int u = 0; u < 4; ++u) rec[3 + u] = btrow[min(ch * cp + u, pg1 - 1)];
            rec[7] = 0;
        }
        off += nch;
    }
    if (tid == kPlanThreads - 1) {
        plan[0] = scan[tid];
        plan[1] = cp;
    }
}

int32_t launch_attn_plan(const AttnWorkspace& ws, const int32_t* seq_lens, const int32_t* bt, int max_blocks, const AttnShape& sh,
                         int batch, int n_kv, hipStream_t st) {
    const Tuning& t = tuning();
    if ((int64_t)batch * sh.ng > ws.max_batch) return fail(CHIRON_ERR_BATCH_TOO_LARGE, "attention: %d requests x %d token groups exceed the workspace", batch, sh.ng);
    const int slots = 4 * (t.attn_grid > 0 ? t.attn_grid : kNumCU * 2);  // waves of the persistent attention grid
    if ((int64_t)batch * sh.ng >= ws.cap_items / sh.tg)
        return fail(CHIRON_ERR_BATCH_TOO_LARGE, "attention: %d passes do not fit a work list of %d items", batch * sh.ng, ws.cap_items / sh.tg);
    launch(attn_plan_kernel, dim3(1), dim3(kPlanThreads), st, ws.plan, ws.max_batch, ws.cap_items, seq_lens, sh, batch, n_kv, slots,
                                                  t.attn_target_waves > 0 ? t.attn_target_waves : 4 * slots, t.attn_chunk_pages,
                                                  ws.cap_items / sh.tg,  // a partial result holds tg tokens' heads
                                                  bt, max_blocks);
    CHIRON_HIP(hipGetLastError());
    return CHIRON_OK;
}

// ---- the attention kernel ---------------------------------------------------------------------------
// MULTI: every request brings q_len new tokens (rows i*q_len .. of q), all already appended.  A pass serves one token
// group of tv <= tg tokens: operand column t*G + h is query head h of the group's token t, which sees positions
// < len - (tv-1) + t of the pass's len; the request's pages are read once per pass (G*tg <= 16 columns).
template <int D, int G, bool MULTI>
__global__ __launch_bounds__(256, 2) void paged_attn_kernel(PoolDesc p, int layer, const float* __restrict__ q, int ldq, AttnShape sh,
                                                         const int32_t* __restrict__ bt, int max_blocks,
                                                         const int32_t* __restrict__ seq_lens,
                                                         const int32_t* __restrict__ plan, int32_t* __restrict__ tickets,
                                                         int max_batch, int cap_items,
                                                         float* __restrict__ part_o, float* __restrict__ part_ml,
                                                         float scale_log2e) {
    constexpr int KSTEPS = D / 32;  // 16x16x32 MFMAs per score tile; also 16-byte V fragments per page
    constexpr int NPG = 2;          // pages per pipeline stage
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_waves = gridDim.x * 4;
    const int n_kv = p.n_kv;
    const int n_work = plan[0] * n_kv;
    const int cp = plan[1];
    const int head = lane & 15, lg = lane >> 4;
    const int pcols = MULTI ? G * sh.tg : G;         // columns of a partial result
    const int tq = MULTI ? head / G : 0, hq = MULTI ? head % G : head;
    const size_t tile_elems = (size_t)16 * D;

    // item metadata (pass, first page, length, first page ids) comes in one record, fetched one item ahead.  The first
    // record is read without waiting for the item count (any record of the list is readable memory; a wave past the
    // end of the list discards it).
    const int32_t* recs = plan + plan_rec_offset(max_batch, cap_items);
    int w = blockIdx.x * 4 + wave;
    int v_nx, pg0_nx, len_nx, b0_nx, b1_nx, b2_nx, b3_nx;
    auto fetch_rec = [&](int item) {
        const int32_t* r = recs + 8 * (size_t)min(item, cap_items - 1);
        v_nx = __builtin_amdgcn_readfirstlane(r[0]);
        pg0_nx = __builtin_amdgcn_readfirstlane(r[1]);
        len_nx = __builtin_amdgcn_readfirstlane(r[2]);
        b0_nx = __builtin_amdgcn_readfirstlane(r[3]);
        b1_nx = __builtin_amdgcn_readfirstlane(r[4]);
        b2_nx = __builtin_amdgcn_readfirstlane(r[5]);
        b3_nx = __builtin_amdgcn_readfirstlane(r[6]);
    };
    fetch_rec(w / n_kv);
    const bool draw = n_work > n_waves;  // one round holds everything: no second item for anybody
    // queue j hands out the indices n_waves + j, n_waves + j + nq, ... to the workgroups j, j + nq, ...
    const int nq = gridDim.x >= kTicketQueues ? kTicketQueues : 1, qj = blockIdx.x % nq;
    int32_t* ticket = tickets + qj * kTicketStride;
    while (w < n_work) {
        const int it = w / n_kv, c = w - it * n_kv;
        const int pg0 = pg0_nx, len = len_nx;
        const int first_ids[4] = {b0_nx, b1_nx, b2_nx, b3_nx};
        const int i = MULTI ? v_nx / sh.ng : v_nx, g = MULTI ? v_nx - i * sh.ng : 0;
        const int tv = MULTI ? min(sh.tg, sh.q_len - g * sh.tg) : 1;  // tokens of this pass
        const int cols = G * tv;                                       // live operand columns
        const int npages = (len + kBlockSize - 1) / kBlockSize;
        const int pg1 = min(pg0 + cp, npages);
        const int32_t* btrow = bt + (size_t)i * max_blocks;
        const uint16_t* lbase = p.base + (size_t)layer * (size_t)p.layer_stride;

        floatx4 o[D / 16];
#pragma unroll
        for (int t = 0; t < D / 16; ++t) o[t] = floatx4{0.f, 0.f, 0.f, 0.f};
        float m_run = -INFINITY, l_run = 0.f;
        uint4 qh[KSTEPS], ql[KSTEPS];  // filled below, after the first tile loads have been issued

        uint4 kc[NPG][KSTEPS], vc[NPG][KSTEPS], kn[NPG][KSTEPS], vn[NPG][KSTEPS];
        // page ids are fetched one stage ahead of the tiles they address (scalar loads)
        int blk_next[NPG];
        auto fetch_ids = [&](int pg) {
#pragma unroll
            for (int u = 0; u < NPG; ++u) blk_next[u] = btrow[min(pg + u, pg1 - 1)];  // past the end: the last page, masked
        };
        auto load_group = [&](uint4 (&kk)[NPG][KSTEPS], uint4 (&vv)[NPG][KSTEPS]) {
#pragma unroll
            for (int u = 0; u < NPG; ++u) {
                int blk = __builtin_amdgcn_readfirstlane(blk_next[u]);
                const uint16_t* tile = lbase + ((size_t)blk * n_kv + c) * (2 * tile_elems);
#pragma unroll
                for (int s = 0; s < KSTEPS; ++s) {
                    kk[u][s] = load_stream_16(tile + (size_t)(s * 64 + lane) * 8);
                    vv[u][s] = load_stream_16(tile + tile_elems + (size_t)(s * 64 + lane) * 8);
                }
            }
        };
        // one pipeline stage: scores, online-softmax update, P*V.  TAIL stages may hold slots past the
        // sequence end or a page past the item's end; inner stages are full and need no masks.
        auto compute = [&](int pg, auto tail_tag) {
            constexpr bool TAIL = decltype(tail_tag)::value;
            floatx4 s[NPG];
            float mx = -INFINITY;
#pragma unroll
            for (int u = 0; u < NPG; ++u) {
                s[u] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int k = 0; k < KSTEPS; ++k) {
                    bf16x8 a = *reinterpret_cast<bf16x8*>(&kc[u][k]);
                    s[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, *reinterpret_cast<bf16x8*>(&qh[k]), s[u], 0, 0, 0);
                    s[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, *reinterpret_cast<bf16x8*>(&ql[k]), s[u], 0, 0, 0);
                }
                if (TAIL) {
                    const int len_eff = (pg + u < pg1) ? len : 0;
                    const int len_col = MULTI ? min(len_eff, len - (tv - 1) + tq) : len_eff;  // causal among the new tokens
                    const int tok0 = (pg + u) * 16 + lg * 4;
#pragma unroll
                    for (int r = 0; r < 4; ++r) s[u][r] = (tok0 + r < len_col) ? s[u][r] : -INFINITY;
                    // slots past the end may hold any bits (NaN included): clear their V so that 0 * V stays 0
                    int valid = len_eff - tok0;
                    uint32_t m01 = (valid > 0 ? 0x0000ffffu : 0u) | (valid > 1 ? 0xffff0000u : 0u);
                    uint32_t m23 = (valid > 2 ? 0x0000ffffu : 0u) | (valid > 3 ? 0xffff0000u : 0u);
#pragma unroll
                    for (int k = 0; k < KSTEPS; ++k) {
                        vc[u][k].x &= m01; vc[u][k].y &= m23; vc[u][k].z &= m01; vc[u][k].w &= m23;
                    }
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) mx = fmaxf(mx, s[u][r]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run, mx);
            // a column can have nothing visible yet (an item that starts among the new tokens): keep the exponents finite
            const float m_use = MULTI ? fmaxf(m_new, -1e30f) : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int t = 0; t < D / 16; ++t) o[t] *= alpha;
#pragma unroll
            for (int u = 0; u < NPG; ++u) {
                float pr[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    pr[r] = __builtin_amdgcn_exp2f(s[u][r] - m_use);
                    l_run += pr[r];
                }
                uint2 ph, pl;
                split2(pr[0], pr[1], ph.x, pl.x);
                split2(pr[2], pr[3], ph.y, pl.y);
                short4v bh = *reinterpret_cast<short4v*>(&ph), bl = *reinterpret_cast<short4v*>(&pl);
#pragma unroll
                for (int k = 0; k < KSTEPS; ++k) {
                    uint2 v0 = make_uint2(vc[u][k].x, vc[u][k].y), v1 = make_uint2(vc[u][k].z, vc[u][k].w);
                    short4v a0 = *reinterpret_cast<short4v*>(&v0), a1 = *reinterpret_cast<short4v*>(&v1);
                    o[2 * k] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a0, bh, o[2 * k], 0, 0, 0);
                    o[2 * k + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a1, bh, o[2 * k + 1], 0, 0, 0);
                    o[2 * k] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a0, bl, o[2 * k], 0, 0, 0);
                    o[2 * k + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a1, bl, o[2 * k + 1], 0, 0, 0);
                }
            }
        };

        // The steady loop has no divergent branch and a fixed order of loads (next stage's tiles first, then
        // this stage's arithmetic), so exactly one stage of loads stays in flight behind the one in use.
        static_assert(NPG == 2, "the item record carries the ids of two stages of two pages");
        blk_next[0] = first_ids[0];
        blk_next[1] = first_ids[1];
        load_group(kc, vc);   // the first tiles are on their way before anything else of the item is touched
        blk_next[0] = first_ids[2];
        blk_next[1] = first_ids[3];
        // the next item's index: drawn now, read after the q loads below have returned (memory operations return in
        // order, so by then the draw costs no wait of its own)
        int drawn = 0;
        if (draw && lane == 0) drawn = atomicAdd(ticket, 1);
        __builtin_amdgcn_sched_barrier(0);
        // q fragments: operand column = head, 8 consecutive dims per lane group; scaled by log2(e)/sqrt(d)
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) {
            if (head < cols) {
                const float* qp = q + (size_t)(MULTI ? i * sh.q_len + g * sh.tg + tq : i) * ldq + (size_t)(c * G + hq) * D + s * 32 + lg * 8;
                float4 a = *reinterpret_cast<const float4*>(qp), b = *reinterpret_cast<const float4*>(qp + 4);
                split2(a.x * scale_log2e, a.y * scale_log2e, qh[s].x, ql[s].x);
                split2(a.z * scale_log2e, a.w * scale_log2e, qh[s].y, ql[s].y);
                split2(b.x * scale_log2e, b.y * scale_log2e, qh[s].z, ql[s].z);
                split2(b.z * scale_log2e, b.w * scale_log2e, qh[s].w, ql[s].w);
            } else {
                qh[s] = ql[s] = make_uint4(0, 0, 0, 0);
            }
        }
        const int w_next = draw ? n_waves + __builtin_amdgcn_readfirstlane(drawn) * nq + qj : n_work;
        fetch_rec(w_next / n_kv);  // next item's record, needed only after this item is done
        int pg = pg0;
        for (; pg + NPG < pg1; pg += NPG) {
            load_group(kn, vn);
            fetch_ids(pg + 2 * NPG);
            __builtin_amdgcn_sched_barrier(0);
            compute(pg, std::integral_constant<bool, MULTI>{});  // the new tokens' masks can reach into the stage before the last
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < NPG; ++u)
#pragma unroll
                for (int k = 0; k < KSTEPS; ++k) {
                    kc[u][k] = kn[u][k];
                    vc[u][k] = vn[u][k];
                }
        }
        compute(pg, std::true_type{});

        // each lane group summed its own tokens; combine the four groups
        l_run += __shfl_xor(l_run, 16);
        l_run += __shfl_xor(l_run, 32);
        if (head < cols) {
            const size_t slot = (size_t)w * pcols + head;
            if (lg == 0) {
                part_ml[slot * 2] = MULTI ? fmaxf(m_run, -1e30f) : m_run;
                part_ml[slot * 2 + 1] = l_run;
            }
#pragma unroll
            for (int t = 0; t < D / 16; ++t)
                *reinterpret_cast<float4*>(part_o + slot * D + t * 16 + lg * 4) = make_float4(o[t][0], o[t][1], o[t][2], o[t][3]);
        }
        w = w_next;
    }
}

// merge the items of one (request, query head): out = sum_j 2^(m_j - M) o_j / sum_j 2^(m_j - M) l_j.
// 256 threads = 8 item slices x 32 lanes of float4 (D = 128) or 16 slices x 16 lanes (D = 64); slice k takes
// items k, k+S, ...; the slices are combined through LDS in a fixed order.
template <int D>
__global__ __launch_bounds__(256) void attn_reduce_kernel(const int32_t* __restrict__ plan, int32_t* __restrict__ tickets,
                                                          int max_batch, int n_kv, int G, AttnShape sh,
                                                          const float* __restrict__ part_o,
                                                          const float* __restrict__ part_ml, float* __restrict__ out,
                                                          int ldo) {
    constexpr int LANES = D / 4, S = 256 / LANES;
    __shared__ float4 s_num[S][LANES];
    __shared__ float s_den[S], s_max[S];
    // row = request * q_len + token; the token's pass v = request * ng + token / tg; a partial result holds G*tg
    // columns per (item, kv head), column = (token % tg) * G + head
    const int row = blockIdx.x, t = row % sh.q_len, v = row / sh.q_len * sh.ng + t / sh.tg;
    const int a = blockIdx.y, c = a / G, j = (t % sh.tg) * G + a % G, GT = G * sh.tg;
    const int sl = threadIdx.x / LANES, ln = threadIdx.x % LANES;
    const int item0 = plan[4 + v], nch = plan[4 + max_batch + v];
    // the attention kernel before this one has drained: its ticket counters go back to 0 for the next one
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < kTicketQueues) tickets[threadIdx.x * kTicketStride] = 0;
    // each slice folds its items with a running maximum, two items' loads in flight at a time
    float M = -INFINITY, den = 0.f;
    float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
    auto fold = [&](float m, float l, float4 o) {
        float Mn = fmaxf(M, m);
        float a0 = __builtin_amdgcn_exp2f(M - Mn), b0 = __builtin_amdgcn_exp2f(m - Mn);
        den = den * a0 + l * b0;
        num.x = num.x * a0 + o.x * b0; num.y = num.y * a0 + o.y * b0;
        num.z = num.z * a0 + o.z * b0; num.w = num.w * a0 + o.w * b0;
        M = Mn;
    };
    int ch = sl;
    for (; ch + S < nch; ch += 2 * S) {
        size_t s0 = ((size_t)(item0 + ch) * n_kv + c) * GT + j, s1 = ((size_t)(item0 + ch + S) * n_kv + c) * GT + j;
        float2 ml0 = *reinterpret_cast<const float2*>(part_ml + s0 * 2), ml1 = *reinterpret_cast<const float2*>(part_ml + s1 * 2);
        float4 o0 = *reinterpret_cast<const float4*>(part_o + s0 * D + ln * 4);
        float4 o1 = *reinterpret_cast<const float4*>(part_o + s1 * D + ln * 4);
        fold(ml0.x, ml0.y, o0);
        fold(ml1.x, ml1.y, o1);
    }
    if (ch < nch) {
        size_t s0 = ((size_t)(item0 + ch) * n_kv + c) * GT + j;
        float2 ml0 = *reinterpret_cast<const float2*>(part_ml + s0 * 2);
        fold(ml0.x, ml0.y, *reinterpret_cast<const float4*>(part_o + s0 * D + ln * 4));
    }
    s_num[sl][ln] = num;
    if (ln == 0) {
        s_den[sl] = den;
        s_max[sl] = M;
    }
    __syncthreads();
    if (sl == 0) {
        float Mt = -INFINITY;
        for (int k = 0; k < S; ++k) Mt = fmaxf(Mt, s_max[k]);
        float dsum = 0.f;
        float4 n4 = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int k = 0; k < S; ++k) {
            float wk = __builtin_amdgcn_exp2f(s_max[k] - Mt);  // empty slices carry max -inf: weight 0
            dsum += wk * s_den[k];
            float4 t = s_num[k][ln];
            n4.x += wk * t.x; n4.y += wk * t.y; n4.z += wk * t.z; n4.w += wk * t.w;
        }
        float inv = 1.0f / dsum;
        *reinterpret_cast<float4*>(out + (size_t)row * ldo + (size_t)a * D + ln * 4) =
            make_float4(n4.x * inv, n4.y * inv, n4.z * inv, n4.w * inv);
    }
}

template <int D>
static int32_t launch_attn_d(int G, dim3 grid, hipStream_t st, const PoolDesc& p, int layer, const float* q, int ldq,
                             const AttnShape& sh, const int32_t* bt, int max_blocks, const int32_t* seq_lens,
                             const AttnWorkspace& ws, float scale) {
    int32_t* tickets = ws.plan + plan_ticket_offset(ws.max_batch, ws.cap_items);
#define CHIRON_ATTN(G_)                                                                                              \
    do {                                                                                                             \
        if (sh.q_len > 1)                                                                                            \
            launch(paged_attn_kernel<D, G_, true>, dim3(grid), dim3(256), st, p, layer, q, ldq, sh, bt, max_blocks, seq_lens,     \
                                                                 ws.plan, tickets, ws.max_batch, ws.cap_items, ws.part_o,     \
                                                                 ws.part_ml, scale);                                 \
        else                                                                                                         \
            launch(paged_attn_kernel<D, G_, false>, dim3(grid), dim3(256), st, p, layer, q, ldq, sh, bt, max_blocks, seq_lens,    \
                                                                  ws.plan, tickets, ws.max_batch, ws.cap_items, ws.part_o,    \
                                                                  ws.part_ml, scale);                                \
    } while (0)
    switch (G) {
        case 1: CHIRON_ATTN(1); break;
        case 2: CHIRON_ATTN(2); break;
        case 4: CHIRON_ATTN(4); break;
        case 8: CHIRON_ATTN(8); break;
        case 16: CHIRON_ATTN(16); break;
        default: return fail(CHIRON_ERR_SHAPE, "attention: query heads per KV head must be 1, 2, 4, 8 or 16 (got %d)", G);
    }
#undef CHIRON_ATTN
    return CHIRON_OK;
}

int32_t launch_attn_main(const AttnWorkspace& ws, const PoolDesc& p, int layer, const float* q, int ldq, int n_q,
                         const int32_t* bt, int max_blocks, const int32_t* seq_lens, const AttnShape& sh, int batch,
                         hipStream_t st) {
    if (batch == 0) return CHIRON_OK;
    const int G = n_q / p.n_kv;
    if (sh.q_len < 1 || sh.tg < 1 || G * sh.tg > 16 || sh.ng != (sh.q_len + sh.tg - 1) / sh.tg)
        return fail(CHIRON_ERR_INVALID_ARG, "attention: %d tokens in groups of %d x %d heads per KV head do not fit 16 operand columns",
                    sh.q_len, sh.tg, G);
    const float scale = (float)(1.4426950408889634 / std::sqrt((double)p.d));
    const Tuning& t = tuning();
    dim3 grid(t.attn_grid > 0 ? t.attn_grid : kNumCU * 2);
    int32_t rc;
    if (p.d == 128) rc = launch_attn_d<128>(G, grid, st, p, layer, q, ldq, sh, bt, max_blocks, seq_lens, ws, scale);
    else if (p.d == 64) rc = launch_attn_d<64>(G, grid, st, p, layer, q, ldq, sh, bt, max_blocks, seq_lens, ws, scale);
    else return fail(CHIRON_ERR_SHAPE, "attention: head_dim must be 64 or 128 (got %d)", p.d);
    if (rc) return rc;
    CHIRON_HIP(hipGetLastError());
    return CHIRON_OK;
}

int32_t launch_attn_merge(const AttnWorkspace& ws, const PoolDesc& p, int n_q, const AttnShape& sh, int batch, float* out,
                          int ldo, hipStream_t st) {
    if (batch == 0) return CHIRON_OK;
    const int G = n_q / p.n_kv;
    dim3 rgrid(batch * sh.q_len, n_q);
    int32_t* tickets = ws.plan + plan_ticket_offset(ws.max_batch, ws.cap_items);
    if (p.d == 128) launch(attn_reduce_kernel<128>, dim3(rgrid), dim3(256), st, ws.plan, tickets, ws.max_batch, p.n_kv, G, sh, ws.part_o, ws.part_ml, out, ldo);
    else launch(attn_reduce_kernel<64>, dim3(rgrid), dim3(256), st, ws.plan, tickets, ws.max_batch, p.n_kv, G, sh, ws.part_o, ws.part_ml, out, ldo);
    CHIRON_HIP(hipGetLastError());
    return CHIRON_OK;
}

}  // namespace chiron

// Projections of the decode step: y[M,N] (+)= A[M,K] * W^T with bf16 weights streamed from HBM
// straight into matrix-core operand registers, and fp32 activations staged through LDS as two
// bf16 terms (hi + lo).  gfx950, wave64, v_mfma_f32_32x32x16_bf16.
//
// Work split: a workgroup of 4 waves owns 4*NF tiles of 32 output columns (one wave = NF tiles),
// one M-tile of 32*MT rows and one slice of K.  Weights are read exactly once per M-tile; the
// activation chunk of the current K-slice is shared by the 4 waves through LDS.  With more than
// one K-slice each slice stores its partial product in a workspace [slice][M][N]; the kernel that
// consumes the projection (residual add + RMSNorm, or RoPE) sums the slices while it reads them,
// in a fixed order, so results are reproducible run to run.
//
// PRO_PACKED (large batches, see linear_big.hip): the activations arrive already split into their two bf16
// terms in tile order and are copied global -> LDS directly, without staging registers or conversion work.
//
// The gate/up projection of the feed-forward block ends in SwiGLU: its weights are packed so that every 32-column
// tile holds 16 gate columns and the 16 up columns of the same indices (gate_up_packed_row below), which puts
// gate[m][j] and up[m][j] into the two halves of one wave, and the epilogue writes silu(gate) * up, either as fp32
// rows or already split into bf16 terms in the tile order that PRO_PACKED reads.  The down projection then is a plain
// projection over half the bytes, and nothing evaluates exp() more than once per element.
#include <climits>
#include <cstdlib>

#include "chiron_internal.h"
#include "device_util.h"

namespace chiron {

// ---- weight repacking -------------------------------------------------------------------------------
// Packed row of gate (kind 0) or up (kind 1) column j in the fused gate/up matrix.  Row i of a 32-row tile lands in
// accumulator register r of the lanes of half h with i = 8*(r/4) + 4*h + r%4: the gate column 16*tile + r goes to
// half 0, register r, the up column of the same index to half 1, register r.
__host__ __device__ inline int gate_up_packed_row(int j, int kind) {
    return 32 * (j / 16) + 8 * ((j % 16) / 4) + 4 * kind + j % 4;
}

// interleave: 0 = rows go to row_offset + r; 1 / 2 = r is a gate / up column of a fused gate/up matrix
__global__ __launch_bounds__(256) void pack_rows_kernel(const uint16_t* __restrict__ src, int rows, int K, size_t tstride,
                                                        uint16_t* __restrict__ dst, int row_offset, int interleave) {
    int kgroups = K / 8;
    int64_t total = (int64_t)rows * kgroups;
    for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
        int r = (int)(t / kgroups), kg = (int)(t % kgroups);
        int n = interleave ? gate_up_packed_row(r, interleave - 1) : r + row_offset;
        uint4 v = *reinterpret_cast<const uint4*>(src + (size_t)r * K + (size_t)kg * 8);
        *reinterpret_cast<uint4*>(dst + (size_t)(n / 32) * tstride + (size_t)kg * 256 + (size_t)(n % 32) * 8) = v;
    }
}

int32_t launch_pack_rows(const uint16_t* src, int rows, int K, size_t tstride, uint16_t* dst_packed, int row_offset,
                         hipStream_t st, int interleave) {
    if (rows == 0) return CHIRON_OK;
    if (interleave && rows % 16 != 0) return fail(CHIRON_ERR_SHAPE, "gate/up packing: %d columns are not a multiple of 16", rows);
    int64_t total = (int64_t)rows * (K / 8);
    int blocks = (int)((total + 255) / 256 < 8192 ? (total + 255) / 256 : 8192);
    launch(pack_rows_kernel, dim3(blocks), dim3(256), st, src, rows, K, tstride, dst_packed, row_offset, interleave);
    CHIRON_HIP(hipGetLastError());
    return CHIRON_OK;
}

// ---- the kernel ------------------------------------------------------------------------------------------
// Pipeline per workgroup: weights sit in a ring of KS*NF register fragments per wave; as soon as the MFMAs of
// k-step s have been issued, slot s is reloaded with the same k-step of the NEXT chunk, so about one chunk of
// weight loads (KS*NF KiB per wave) is always in flight.  Activations are double-buffered in LDS: while chunk c
// is consumed, chunk c+1 is written to the other buffer and chunk c+2 is on its way from L2 into registers;
// one barrier per chunk.
// WNT: weight loads carry the non-temporal hint (every weight is read once: a single M-tile).  With several M-tiles
// the same weights are read once per M-tile through the L2, and the hint makes those re-reads slower (measured on the
// 8B gate/up shape at 2048 rows: the weight stream alone 268 us with the hint, 194 us without).
template <int MT, int NF, int KS, int PRO, bool WNT = true>
__global__ __launch_bounds__(256, (MT * NF <= 8 && !(MT == 4 && PRO != PRO_NONE) ? 2 : 1)) void linear_kernel(const uint16_t* __restrict__ Wp, size_t tstride, int Npad, int Nreal, int K, int Kpad,
                                                     const float* __restrict__ A, int lda, int M,
                                                     float* __restrict__ Y, int ldy, int chunks_per_split,
                                                     int mode, size_t part_stride, int gx, int gy, int gz, int remap) {
    constexpr int MROWS = 32 * MT;
    constexpr int RS = MROWS + 1;      // LDS row stride in 16-byte units (+1 breaks the power-of-two stride)
    constexpr int KG = 2 * KS;         // 8-wide k-groups per chunk
    constexpr int KC = 16 * KS;        // k per chunk
    constexpr int TASKS = MROWS * KG;  // 8-float staging tasks per chunk
    static_assert(TASKS % 256 == 0, "staging assumes whole passes of the workgroup");
    constexpr int TPT = TASKS / 256;
    // activation loads and staging spread over the k-steps of a chunk (see below; measured on one device against the
    // bunched form: gate/up at 64 rows 50.3 against 53.6 us, at 192 rows 101 against 109 us).  The widest tile keeps
    // them bunched: it has no registers left for the first chunk's separate staging set.
    constexpr bool SPREAD = PRO != PRO_PACKED && MT * NF <= 8 && TPT <= KS;

    __shared__ uint4 lds_hi[2][KG * RS];
    __shared__ uint4 lds_lo[2][KG * RS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // Workgroups are dealt to the 8 XCDs round-robin.  The 1-D grid is re-read so that consecutive logical ids
    // sit on ONE XCD, and the M-tile index varies fastest: the workgroups that stream the same weight tiles for
    // different rows then share that XCD's L2 instead of each pulling the tile from HBM.
    const int total = gx * gy * gz;
    const int per_xcd = (total + 7) / 8;
    const int logical = remap ? (blockIdx.x % 8) * per_xcd + blockIdx.x / 8 : blockIdx.x;
    if (logical >= total) return;  // grid is padded to a multiple of 8 (uniform over the workgroup)
    const int bz = logical % gz, bx = (logical / gz) % gx, by = logical / (gz * gx);
    const int m0 = bz * MROWS;
    const int tile0 = (bx * 4 + wave) * NF;  // first 32-column tile of this wave
    const int chunks_total = (K + KC - 1) / KC;
    const int c_begin = by * chunks_per_split;
    int c_end = c_begin + chunks_per_split;
    if (c_end > chunks_total) c_end = chunks_total;

    floatx16 acc[NF][MT];
#pragma unroll
    for (int f = 0; f < NF; ++f)
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[f][t][r] = 0.f;

    uint4 w[KS][NF];
    float4 areg[TPT][2];  // fp32 staging registers (unused with PRO_PACKED, whose input goes straight into LDS)
    // PRO_PACKED: A points at the hi terms in 32-row x 8-k tile order, the lo terms follow them
    const int mtiles_all = (M + 31) / 32;
    const float4* Ahi = reinterpret_cast<const float4*>(A);
    const float4* Alo = Ahi + (size_t)mtiles_all * 32 * (Kpad / 8);

    // The loop body holds no divergent branch: every load is unconditional on a clamped address (the packed
    // weights are zero-padded in K to a whole chunk, out-of-range activation rows/columns are zeroed by a
    // select), so the compiler can count outstanding loads exactly and never drains the queue.
    const int kgroups = Kpad / 8;
    const uint16_t* wp[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) {
        int tile = min(tile0 + f, Npad / 32 - 1);  // a wave past the last tile recomputes it; its stores are masked
        wp[f] = Wp + (size_t)tile * tstride + (lane >> 5) * 256 + (lane & 31) * 8;
    }
    auto load_w = [&](int c, int s) {
        size_t off = (size_t)(c * KC + s * 16) * 32;
#pragma unroll
        // non-temporal: a step reads every weight once, and what the weights do not displace stays cached for the
        // activations and the K/V pages (same-device A/B on the whole step: -7 % at 1 request, -1.5 % at 64..2048)
        for (int f = 0; f < NF; ++f)
            w[s][f] = WNT ? load_stream_16(wp[f] + off) : *reinterpret_cast<const uint4*>(wp[f] + off);
    };
    // staging task i of a chunk: 8 consecutive k of one row, thread tid + 256*i
    auto load_task = [&](int c, int i, float4 (&ar)[2]) {
        int task = tid + i * 256;
        int kg = task % KG, m = task / KG;
        int k = c * KC + kg * 8;
        const float* p = A + (size_t)min(m0 + m, M - 1) * lda + min(k, K - 8);
        ar[0] = *reinterpret_cast<const float4*>(p);
        ar[1] = *reinterpret_cast<const float4*>(p + 4);
    };
    auto stage_task = [&](int c, int i, int buf, const float4 (&ar)[2]) {
        int task = tid + i * 256;
        int kg = task % KG, m = task / KG;
        const bool ok = (m0 + m < M) && (c * KC + kg * 8 < K);
        float v[8] = {ar[0].x, ar[0].y, ar[0].z, ar[0].w, ar[1].x, ar[1].y, ar[1].z, ar[1].w};
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = ok ? v[e] : 0.f;
        uint4 hi, lo;
        split2(v[0], v[1], hi.x, lo.x);
        split2(v[2], v[3], hi.y, lo.y);
        split2(v[4], v[5], hi.z, lo.z);
        split2(v[6], v[7], hi.w, lo.w);
        lds_hi[buf][kg * RS + m] = hi;
        lds_lo[buf][kg * RS + m] = lo;
    };
    auto load_a = [&](int c) {
#pragma unroll
        for (int i = 0; i < TPT; ++i) load_task(c, i, areg[i]);
    };
    auto stage_a = [&](int c, int buf) {
#pragma unroll
        for (int i = 0; i < TPT; ++i) stage_task(c, i, buf, areg[i]);
    };
    // PRO_PACKED: chunk c of the pre-split activations goes HBM/L2 -> LDS directly (16 bytes per lane, a wave
    // fills 64 consecutive rows of one k-group), no registers and no LDS store instructions in between
    constexpr int JOBS = KG * (MROWS / 64) * 2;  // (k-group, 64-row half, hi|lo) per chunk, dealt to the 4 waves
    static_assert(PRO != PRO_PACKED || (MROWS % 64 == 0 && JOBS % 4 == 0), "packed input needs 64-row halves");
    constexpr int WJOBS = PRO == PRO_PACKED ? JOBS / 4 : 1;
    // per job: this lane's source at chunk 0 (it advances by one chunk of k-groups per chunk) and the wave-uniform
    // LDS byte address of the job's destination in either buffer
    const float4* dma_src[WJOBS];
    uint32_t dma_dst[WJOBS];  // in buffer 0; buffer 1 lies KG*RS pieces further in both arrays
    if (PRO == PRO_PACKED) {
#pragma unroll
        for (int j = 0; j < WJOBS; ++j) {
            const int job = wave + 4 * j;
            const int lo = job & 1, half = (job >> 1) % (MROWS / 64), kg = (job >> 1) / (MROWS / 64);
            const int m = half * 64 + lane;
            const size_t idx = ((size_t)min(bz * MT + m / 32, mtiles_all - 1) * kgroups + kg) * 32 + (m & 31);
            dma_src[j] = (lo ? Alo : Ahi) + idx;
            dma_dst[j] = __builtin_amdgcn_readfirstlane(lds_address((lo ? lds_lo[0] : lds_hi[0]) + kg * RS + half * 64));
        }
    }
    auto dma_a = [&](int c, int buf) {
#pragma unroll
        for (int j = 0; j < WJOBS; ++j)
            global_to_lds_16(dma_src[j] + (size_t)c * (KG * 32), dma_dst[j] + (uint32_t)buf * (uint32_t)(KG * RS * sizeof(uint4)));
    };
    // LDS fragments of one k-step: hi and lo terms of the MT row tiles
    struct Frags {
        bf16x8 h[MT], l[MT];
    };
    auto read_frags = [&](int buf, int s, Frags& fr) {
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            int idx = (s * 2 + (lane >> 5)) * RS + t * 32 + (lane & 31);
            uint4 h = lds_hi[buf][idx], l = lds_lo[buf][idx];
            fr.h[t] = *reinterpret_cast<bf16x8*>(&h);
            fr.l[t] = *reinterpret_cast<bf16x8*>(&l);
        }
    };
    auto mma_frags = [&](int s, const Frags& fr) {
        // hi terms of every accumulator first, then the lo terms: consecutive MFMAs never chain on one accumulator
#pragma unroll
        for (int f = 0; f < NF; ++f)
#pragma unroll
            for (int t = 0; t < MT; ++t)
                acc[f][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&w[s][f]), fr.h[t], acc[f][t], 0, 0, 0);
#pragma unroll
        for (int f = 0; f < NF; ++f)
#pragma unroll
            for (int t = 0; t < MT; ++t)
                acc[f][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<bf16x8*>(&w[s][f]), fr.l[t], acc[f][t], 0, 0, 0);
    };
    // Up to 96 rows a workgroup has one wave per SIMD and few MFMAs per k-step, so the chain "fragments arrive from
    // LDS -> MFMAs -> reload the weight slot" paces the weight stream.  There the fragments of k-step s+1 are read while
    // the MFMAs of k-step s run (two register sets); only a chunk's first k-step waits for LDS.  (Measured on the 8B
    // gate/up shape at 64 rows with the LDS reads taken out: 5.5 of 55 us.)  The 128-row tiles have enough MFMAs per
    // k-step to cover the reads and no registers to spare.
    constexpr bool PIPE = MT < 4;
    Frags fr[PIPE ? 2 : 1];
    auto mma_step = [&](int buf, int s) {
        if constexpr (PIPE) {
            if (s == 0) read_frags(buf, 0, fr[0]);
            if (s + 1 < KS) read_frags(buf, s + 1, fr[(s + 1) & 1]);
            mma_frags(s, fr[s & 1]);
        } else {
            read_frags(buf, s, fr[0]);
            mma_frags(s, fr[0]);
        }
    };

    // Order of memory operations (kept in place by the scheduling fences): per iteration the KS weight reloads
    // come first, the activation loads last, in the prologue likewise, so at every use the number of younger
    // loads in flight is the same on the loop's entry edge and on its back edge.
    if (PRO == PRO_PACKED) {
        if (c_begin < c_end) {  // uniform over the workgroup
            const int c_last = c_end - 1;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                load_w(c_begin, s);
                __builtin_amdgcn_sched_barrier(0);  // same issue order as in the loop: k-step 0 is the oldest
            }
            dma_a(c_begin, 0);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            lds_barrier();
            int buf = 0;
            for (int c = c_begin; c < c_last; ++c) {
                // start the copy of chunk c+1 into the idle buffer (last read before the barrier that ended the
                // previous round), multiply chunk c out of the other one while refilling the weight ring
                dma_a(c + 1, buf ^ 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int s = 0; s < KS; ++s) {
                    mma_step(buf, s);
                    load_w(c + 1, s);
                    __builtin_amdgcn_sched_barrier(0);
                }
                // the KS*NF weight loads just issued are younger than the activation copy: let them fly
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(KS * NF) : "memory");
                lds_barrier();
                buf ^= 1;
            }
#pragma unroll
            for (int s = 0; s < KS; ++s) mma_step(buf, s);
        }
    } else if (SPREAD) {
        // Activation traffic spread over the chunk: the loads of a task's next-but-one chunk are issued, and the task's
        // next chunk is converted and written to LDS, right after one particular k-step's weight reload instead of all
        // together before the barrier.  A burst of activation loads keeps the CU's address unit busy (1 KiB per load
        // instruction at 64 bytes per cycle, four waves at once) exactly when the next chunk's weight reloads want to
        // go out, and in a latency-bound weight stream every delayed request is lost time.
        if (c_begin < c_end) {  // uniform over the workgroup
            const int c_last = c_end - 1;
            // first chunk through a register set of its own, issued before everything else; the ring and the second
            // chunk's tasks follow in the loop's order, so that the wait counts of entry and back edge agree.  (Two
            // chunks or more and a single chunk are separate paths: in one path the compiler moves the second chunk's
            // loads, which only the loop uses, behind the barrier and out of that order.)
            float4 a0[TPT][2];
#pragma unroll
            for (int i = 0; i < TPT; ++i) load_task(c_begin, i, a0[i]);
            __builtin_amdgcn_sched_barrier(0);
            if (c_begin < c_last) {
#pragma unroll
                for (int s = 0; s < KS; ++s) {
                    load_w(c_begin, s);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int i = 0; i < TPT; ++i)
                        if (i * KS / TPT == s) {
                            load_task(c_begin + 1, i, areg[i]);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                }
#pragma unroll
                for (int i = 0; i < TPT; ++i) stage_task(c_begin, i, 0, a0[i]);
                lds_barrier();
                int buf = 0, c = c_begin;
                do {
#pragma unroll
                    for (int s = 0; s < KS; ++s) {
                        mma_step(buf, s);
                        load_w(c + 1, s);
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int i = 0; i < TPT; ++i)
                            if (i * KS / TPT == s) {
                                stage_task(c + 1, i, buf ^ 1, areg[i]);
                                __builtin_amdgcn_sched_barrier(0);
                                load_task(min(c + 2, c_last), i, areg[i]);
                                __builtin_amdgcn_sched_barrier(0);
                            }
                    }
                    lds_barrier();
                    buf ^= 1;
                } while (++c < c_last);
#pragma unroll
                for (int s = 0; s < KS; ++s) mma_step(buf, s);
            } else {
#pragma unroll
                for (int s = 0; s < KS; ++s) load_w(c_begin, s);
#pragma unroll
                for (int i = 0; i < TPT; ++i) stage_task(c_begin, i, 0, a0[i]);
                lds_barrier();
#pragma unroll
                for (int s = 0; s < KS; ++s) mma_step(0, s);
            }
        }
    } else
    if (c_begin < c_end) {   // uniform over the workgroup
        const int c_last = c_end - 1;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            load_w(c_begin, s);
            __builtin_amdgcn_sched_barrier(0);  // same issue order as in the loop: k-step 0 is the oldest
        }
        load_a(c_begin);
        stage_a(c_begin, 0);
        load_a(min(c_begin + 1, c_last));
        lds_barrier();
        int buf = 0;
        for (int c = c_begin; c < c_last; ++c) {
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                mma_step(buf, s);
                load_w(c + 1, s);  // slot s is free again: fetch the same k-step of the next chunk
                __builtin_amdgcn_sched_barrier(0);
            }
            stage_a(c + 1, buf ^ 1);
            __builtin_amdgcn_sched_barrier(0);
            load_a(min(c + 2, c_last));
            __builtin_amdgcn_sched_barrier(0);
            lds_barrier();
            buf ^= 1;
        }
#pragma unroll
        for (int s = 0; s < KS; ++s) mma_step(buf, s);
    }

    // D[i][j]: lane holds column j = lane%32 (an activation row m) and rows i = 8*(r/4) + 4*(lane/32) + r%4
    // (output columns n) for r = 0..15.
    if (mode >= EPI_SWIGLU) {
        // Fused gate/up: in tile T the lanes of half 0 hold gate[m][16T + r], those of half 1 up[m][16T + r].  The halves
        // swap eight values each, after which half h owns the columns 16T + 8h .. + 7 of row m.
        const int half = lane >> 5;
#pragma unroll
        for (int f = 0; f < NF; ++f) {
            const int tile = tile0 + f;
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float mine_g = acc[f][t][e], mine_u = acc[f][t][8 + e];  // half 0: gate e, (gate 8+e); half 1: (up e), up 8+e
                    const float got = __shfl_xor(half ? mine_g : mine_u, 32);       // half 0 receives up e, half 1 gate 8+e
                    const float g = half ? got : mine_g, u = half ? mine_u : got;
                    v[e] = g / (1.0f + __expf(-g)) * u;
                }
                const int m = m0 + t * 32 + (lane & 31);
                if (m >= M || tile >= Npad / 32) continue;
                if (mode == EPI_SWIGLU) {
                    float* dst = Y + (size_t)m * ldy + tile * 16 + half * 8;
                    *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
                    *reinterpret_cast<float4*>(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
                } else {
                    // the two bf16 terms in 32-row x 8-k tile order (ldy = k-groups of the consumer, part_stride = distance
                    // from the hi to the lo terms in 16-byte units)
                    uint4 hi, lo;
                    split2(v[0], v[1], hi.x, lo.x);
                    split2(v[2], v[3], hi.y, lo.y);
                    split2(v[4], v[5], hi.z, lo.z);
                    split2(v[6], v[7], hi.w, lo.w);
                    uint4* dst = reinterpret_cast<uint4*>(Y) + ((size_t)(m / 32) * ldy + (size_t)(2 * tile + half)) * 32 + (m & 31);
                    dst[0] = hi;
                    dst[part_stride] = lo;
                }
            }
        }
        return;
    }
#pragma unroll
    for (int f = 0; f < NF; ++f) {
        int nb = (tile0 + f) * 32 + (lane >> 5) * 4;
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            int m = m0 + t * 32 + (lane & 31);
            if (m >= M) continue;
            // EPI_STORE: y = acc;  EPI_ADD: y += acc (this workgroup is the only writer);  EPI_SLICES: slice `by` of the workspace
            float* yrow = Y + (mode == EPI_SLICES ? (size_t)by * part_stride : (size_t)0) + (size_t)m * ldy;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                int n = nb + q * 8;
                if (n + 3 < Nreal && (ldy & 3) == 0) {
                    float4 v = make_float4(acc[f][t][q * 4], acc[f][t][q * 4 + 1], acc[f][t][q * 4 + 2], acc[f][t][q * 4 + 3]);
                    float4* dst = reinterpret_cast<float4*>(yrow + n);
                    if (mode == EPI_ADD) {
                        float4 o = *dst;
                        v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
                    }
                    *dst = v;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (n + e < Nreal) {
                            float v = acc[f][t][q * 4 + e];
                            yrow[n + e] = mode == EPI_ADD ? yrow[n + e] + v : v;
                        }
                }
            }
        }
    }
}

// sum of K-slices: y (+)= sum_s part[s]  (used by the single-kernel entry points; inside the decode step the
// consumers of a projection do this sum themselves)
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ part, int ks, size_t stride,
                                                              int64_t n, float* __restrict__ y, int accumulate) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
        float v = accumulate ? y[i] : 0.f;
        for (int s = 0; s < ks; ++s) v += part[(size_t)s * stride + i];
        y[i] = v;
    }
}

int32_t launch_reduce_partials(const float* part, int ks, int64_t n, float* y, int accumulate, hipStream_t st) {
    int blocks = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
    launch(reduce_partials_kernel, dim3(blocks), dim3(256), st, part, ks, (size_t)n, n, y, accumulate);
    CHIRON_HIP(hipGetLastError());
    return CHIRON_OK;
}

Tuning& tuning() {
    static Tuning t;
    return t;
}

template <int MT, int NF, int PRO, int KS = 4, bool WNT = true>
static void launch_cfg(int nblocks, hipStream_t st, const Linear& L, const float* A, int lda, int M, float* y, int ldy,
                       int cps, int mode, size_t part_stride, int gx, int gy, int gz) {
    launch(linear_kernel<MT, NF, KS, PRO, WNT>, dim3(nblocks), dim3(256), st, L.w, L.tstride, L.Npad, L.N, L.K, L.Kpad, A, lda, M, y, ldy, cps, mode,
                                                           part_stride, gx, gy, gz, tuning().linear_xcd_remap);
}

int linear_max_split() { return 16; }

// Rows from which the down projection is faster on the tiled two-term form of its input (128-row tiles, copied straight
// into LDS) than on fp32 rows (64- and 96-row tiles, split on the way into LDS); the gate/up epilogue writes whichever
// is asked for.  Measured inside the step, gate/up + down per layer: at K = 14336 (N = 4096) fp32 rows win up to 320
// rows (160 rows: 138 against 155 us), the two are level at 384..512, the tiled form wins from 768 (533 against 556 us);
// at K = 28672 (N = 8192) fp32 rows win at 96 rows (92 against 100 us), the tiled form at 128 (102 against 108 us).
static int big_min_rows_default(const Linear& L) { return L.K >= 16384 ? 97 : 513; }

int linear_big_min_rows(const Linear& L) {
    const int v = tuning().linear_big_min_m;
    return v == 0 ? big_min_rows_default(L) : (v < 0 ? INT32_MAX : v);
}

int32_t launch_linear(const Linear& L, const float* A, int lda, int M, float* y, int ldy, int epilogue, int prologue,
                      float* part, int max_split, int* ksplit_out, uint16_t* asplit, hipStream_t st) {
    if (ksplit_out) *ksplit_out = 1;
    if (M == 0) return CHIRON_OK;
    if (epilogue != EPI_STORE && epilogue != EPI_ADD && epilogue != EPI_SWIGLU && epilogue != EPI_SWIGLU_PACKED)
        return fail(CHIRON_ERR_INVALID_ARG, "linear: unknown epilogue %d", epilogue);
    if (epilogue >= EPI_SWIGLU) {
        // gate and up of one column must meet in one workgroup with the whole sum over K
        if (part) return fail(CHIRON_ERR_INVALID_ARG, "linear: the SwiGLU epilogue cannot slice K");
        if (L.N % 32 != 0) return fail(CHIRON_ERR_SHAPE, "linear: a fused gate/up matrix has a multiple of 32 rows (got %d)", L.N);
        if (ldy % (epilogue == EPI_SWIGLU ? 4 : 8) != 0 || ((uintptr_t)y & 15))
            return fail(CHIRON_ERR_INVALID_ARG, "linear: SwiGLU output rows must be 16-byte aligned");
    }
    if (asplit && prologue != PRO_PACKED && M >= linear_big_min_rows(L) && tuning().linear_big_all)
        return launch_linear_big(L, A, lda, M, y, ldy, epilogue, part, max_split, ksplit_out, asplit, st);
    if (L.K % 16 != 0 || L.K < 16) return fail(CHIRON_ERR_SHAPE, "linear: K=%d must be a positive multiple of 16", L.K);
    if (prologue != PRO_PACKED && (lda % 4 != 0 || ((uintptr_t)A & 15)))
        return fail(CHIRON_ERR_INVALID_ARG, "linear: input rows must be 16-byte aligned");
    const Tuning& tn = tuning();
    // Tile shape.  Up to 64 rows the kernel is HBM-bound: 32- or 64-row tiles; one column tile per wave when K can
    // be sliced (twice the workgroups along N, so half the K-slices for the consumer to add up) or when that is
    // what it takes to give every CU a workgroup, else two.  With many rows it is matrix-core bound and the
    // 128-row x 4-tile wave shape wins (fewer LDS reads and staging per MFMA, at one wave per SIMD): always from
    // 384 rows, and earlier when 128-row tiles pad the rows no further than 64-row tiles do, from 96 rows for a
    // very wide output (the LM head), 224 rows at K >= 8192 (measured on the 8B and 70B shapes).
    const int tiles_n = L.Npad / 32;
    const int pad64 = (M + 63) / 64 * 64, pad128 = (M + 127) / 128 * 128;
    const int thr128 = tiles_n >= 2048 ? 96 : (L.K >= 8192 ? 224 : 384);
    // (outputs narrower than 256 column tiles keep the 64-row shape at any row count: measured 8-12 % faster)
    const bool big = tiles_n >= 256 && (M >= 384 || (pad128 == pad64 && M >= thr128));
    // 65..96 rows take one 96-row tile: with 64-row tiles the second M-tile would stream every weight again for a
    // handful of rows (a step of 17 % in the whole decode step's latency between batch 64 and 65).  Likewise above
    // 128 rows wherever 96-row tiles pad the rows no further than 64-row tiles do (129..192, 257..288, 321..384:
    // a third fewer passes over the weights; measured 10-20 % on the gate/up and O projections).
    const int pad96 = (M + 95) / 96 * 96;
    int mt = tn.linear_mt ? tn.linear_mt : (big ? 4 : (M > 64 && pad96 <= pad64 ? 3 : (M > 32 ? 2 : 1)));
    int tiles = L.Npad / 32;
    int gz = (M + 32 * mt - 1) / (32 * mt);
    // Column tiles per wave.  A projection that cannot slice K takes the smallest count that fits the grid into one
    // round of the chip (224 workgroups for a 57344-wide gate/up with two tiles: 190 against 260 us at 65 rows; 251 for
    // the LM head with four: 169 against 192 us at 64 rows), two if none does.  A sliced one takes one tile up to 64
    // rows and two above, and more where the K-slices that fill the grid still hold twelve chunks or more (hidden
    // size 8192: QKV 34 against 39 us at 64 rows with two tiles, 50 against 56 us at 128 rows with four): wider
    // workgroups re-read the activations less often, but short slices are mostly ramp.
    int nf;
    if (tn.linear_nf) nf = tn.linear_nf;
    else if (big && tiles >= 256) nf = 4;
    else if (tiles < 64) nf = 1;
    else if (!part) {
        const int max_nf = mt == 3 ? 2 : 4;
        nf = 1;
        while (nf < max_nf && ((tiles + 4 * nf - 1) / (4 * nf)) * gz > kNumCU) nf *= 2;
        if (((tiles + 4 * nf - 1) / (4 * nf)) * gz > kNumCU) nf = 2;
    } else {
        nf = M <= 64 ? 1 : 2;
        const int max_nf = mt == 3 ? 2 : 4;
        const int chunks64 = (L.K + 63) / 64;
        for (int c = max_nf; c > nf; c /= 2) {
            const int g = ((tiles + 4 * c - 1) / (4 * c)) * gz;
            const int ks = g >= kNumCU ? 1 : (kNumCU / g < max_split ? kNumCU / g : max_split);
            if (chunks64 / ks >= 12 && g * ks >= kNumCU * 3 / 4) {  // (and the sliced grid still covers the chip)
                nf = c;
                break;
            }
        }
    }
    if (prologue == PRO_PACKED) {  // only the large-batch shapes are built for pre-split input
        mt = 4;
        // four column tiles per wave unless K-slicing cannot make up for the smaller grid (one 128-row tile of a
        // 4096-wide output: 8 workgroup columns x 16 slices = half the chip; 58 against 45 us)
        const int gx4 = (tiles + 15) / 16, gz4 = (M + 127) / 128;
        const bool fills = !part || (int64_t)gx4 * gz4 * max_split >= 200;
        nf = tn.linear_nf ? (tn.linear_nf == 4 ? 4 : 2) : (tiles >= 128 && fills ? 4 : 2);
    }
    if (nf == 4 && mt == 1) mt = 2;
    if (nf == 4 && mt == 3) mt = 4;  // four column tiles per wave are built for 64- and 128-row tiles only
    gz = (M + 32 * mt - 1) / (32 * mt);  // mt may have changed above
    int gx = (tiles + 4 * nf - 1) / (4 * nf);
    // an unsliced projection whose 64-row tiles give a few workgroups more than two per CU takes 96-row tiles if those
    // fit (gate/up at 289..320 rows: 560 workgroups 190 us, 448 workgroups 167 us)
    if (!tn.linear_mt && !part && mt == 2 && prologue == PRO_NONE && nf <= 2 && gx * gz > 2 * kNumCU && gx * gz <= 3 * kNumCU &&
        gx * ((M + 95) / 96) <= 2 * kNumCU) {
        mt = 3;
        gz = (M + 95) / 96;
    }
    // A projection that cannot slice K (no workspace) runs one workgroup per CU; a ring of 8 k-steps then keeps twice
    // the weight bytes in flight per wave, which measured 9 % faster on the gate/up shape at 64 rows.
    const bool ks8 = (mt == 2 || (mt == 3 && nf == 1)) && nf <= 2 && prologue != PRO_PACKED &&
                     (tn.linear_ks == 8 || (tn.linear_ks == 0 && nf == 1 && !part && prologue == PRO_NONE));
    // Up to 32 rows a wave has two MFMAs per k-step and its weight stream is bound by the bytes it keeps in flight over
    // the load latency: the unsliced one-tile-per-wave shape takes a ring of 16 k-steps (16 KiB per wave; measured on the
    // 8B gate/up shape: 37.3 against 40.0 us at one row, 39.8 against 41.4 us at 32 rows; no gain at 64 rows)
    const bool ks16 = mt == 1 && nf == 1 && prologue == PRO_NONE && L.Kpad % 256 == 0 &&
                      (tn.linear_ks == 16 || (tn.linear_ks == 0 && !part));
    const int KC = ks16 ? 256 : (ks8 ? 128 : 64);
    int chunks = (L.K + KC - 1) / KC;
    int ksplit = tn.linear_ksplit ? tn.linear_ksplit : (tn.linear_target_blocks + gx * gz - 1) / (gx * gz);
    // never a few workgroups more than one per CU: the CUs that get a second one take twice as long (264 workgroups
    // of the one-per-CU shape took 141 us where 240 take 100; the QKV projection at 64 rows 20.7 us with 288
    // workgroups, 16.2 us with 240)
    // (except that two slices on two workgroups per CU beat one slice on fewer workgroups than CUs, for the shapes
    // that fit two on a CU: 384 workgroups 65 us, 192 workgroups 73 us; but 192 with two slices 40 us, 288 with
    // three 46 us)
    const bool one_per_cu = mt * nf > 8 || (mt == 4 && prologue != PRO_NONE);
    if (!tn.linear_ksplit && gx * gz * ksplit > kNumCU && gx * gz <= kNumCU) {
        const int fl = kNumCU / (gx * gz);
        if (one_per_cu || fl >= 2) ksplit = fl;
    }
    if (ksplit > chunks / 2) ksplit = chunks / 2;
    if (ksplit > max_split) ksplit = max_split;
    if (!part) ksplit = 1;
    if (ksplit < 1) ksplit = 1;
    int cps = (chunks + ksplit - 1) / ksplit;
    ksplit = (chunks + cps - 1) / cps;  // no empty slices
    int mode = ksplit > 1 ? EPI_SLICES : epilogue;
    float* dst = ksplit > 1 ? part : y;
    int ldd = ksplit > 1 ? L.N : ldy;
    size_t part_stride = (size_t)M * L.N;
    if (epilogue == EPI_SWIGLU_PACKED) {  // ldy: the consumer's padded K
        ldd = ldy / 8;
        part_stride = linear_big_split_elems(M, ldy) / 8;
    }
    int nblocks = (gx * ksplit * gz + 7) / 8 * 8;
#define CHIRON_LAUNCH(MT_, NF_) launch_cfg<MT_, NF_, PRO_NONE>(nblocks, st, L, A, lda, M, dst, ldd, cps, mode, part_stride, gx, ksplit, gz)
    if (ks16) {
        launch_cfg<1, 1, PRO_NONE, 16>(nblocks, st, L, A, lda, M, dst, ldd, cps, mode, part_stride, gx, ksplit, gz);
    } else if (ks8 && mt == 3) {
        launch_cfg<3, 1, PRO_NONE, 8>(nblocks, st, L, A, lda, M, dst, ldd, cps, mode, part_stride, gx, ksplit, gz);
    } else if (ks8) {
        if (nf == 1) launch_cfg<2, 1, PRO_NONE, 8>(nblocks, st, L, A, lda, M, dst, ldd, cps, mode, part_stride, gx, ksplit, gz);
        else launch_cfg<2, 2, PRO_NONE, 8>(nblocks, st, L, A, lda, M, dst, ldd, cps, mode, part_stride, gx, ksplit, gz);
    } else if (prologue == PRO_PACKED) {
        // several M-tiles re-read the weights through the L2: no streaming hint then
        if (nf == 4 && gz > 1) launch_cfg<4, 4, PRO_PACKED, 4, false>(nblocks, st, L, A, lda, M, dst, ldd, cps, mode, part_stride, gx, ksplit, gz);
        else if (nf == 4) launch_cfg<4, 4, PRO_PACKED>(nblocks, st, L, A, lda, M, dst, ldd, cps, mode, part_stride, gx, ksplit, gz);
        else if (gz > 1) launch_cfg<4, 2, PRO_PACKED, 4, false>(nblocks, st, L, A, lda, M, dst, ldd, cps, mode, part_stride, gx, ksplit, gz);
        else launch_cfg<4, 2, PRO_PACKED>(nblocks, st, L, A, lda, M, dst, ldd, cps, mode, part_stride, gx, ksplit, gz);
    } else if (nf == 4) {
        if (mt == 4 && gz > 1) launch_cfg<4, 4, PRO_NONE, 4, false>(nblocks, st, L, A, lda, M, dst, ldd, cps, mode, part_stride, gx, ksplit, gz);
        else if (mt == 4) launch_cfg<4, 4, PRO_NONE>(nblocks, st, L, A, lda, M, dst, ldd, cps, mode, part_stride, gx, ksplit, gz);
        else launch_cfg<2, 4, PRO_NONE>(nblocks, st, L, A, lda, M, dst, ldd, cps, mode, part_stride, gx, ksplit, gz);
    } else if (mt == 1 && nf == 1) CHIRON_LAUNCH(1, 1);
    else if (mt == 1) CHIRON_LAUNCH(1, 2);
    else if (mt == 2 && nf == 1) CHIRON_LAUNCH(2, 1);
    else if (mt == 2) CHIRON_LAUNCH(2, 2);
    else if (mt == 3 && nf == 1) CHIRON_LAUNCH(3, 1);
    else if (mt == 3) CHIRON_LAUNCH(3, 2);
    else if (nf == 1) CHIRON_LAUNCH(4, 1);
    else CHIRON_LAUNCH(4, 2);
#undef CHIRON_LAUNCH
    CHIRON_HIP(hipGetLastError());
    if (ksplit_out) *ksplit_out = ksplit;
    return CHIRON_OK;
}

}  // namespace chiron

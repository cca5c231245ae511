// Projections of the decode step: y[M,N] (+)= A[M,K] * W^T with bf16 weights streamed from HBM
// straight into matrix-core operand registers, and fp32 activations staged through LDS as two
// bf16 terms (hi + lo).  gfx950, wave64, v_mfma_f32_32x32x16_bf16.
//
// Work split: a workgroup of 4 waves owns 4*NF tiles of 32 output columns (one wave = NF tiles),
// one M-tile of 32*MT rows and one slice of K.  Weights are read exactly once per M-tile; the
// activation chunk of the current K-slice is shared by the 4 waves through LDS.  With more than
// one K-slice the partial sums are combined with fp32 atomics in the output.
#include <cstdlib>

#include "chiron_internal.h"
#include "device_util.h"

namespace chiron {

// ---- weight repacking -------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void pack_rows_kernel(const uint16_t* __restrict__ src, int rows, int K,
                                                        uint16_t* __restrict__ dst, int row_offset) {
    int kgroups = K / 8;
    int64_t total = (int64_t)rows * kgroups;
    for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
        int r = (int)(t / kgroups), kg = (int)(t % kgroups);
        int n = r + row_offset;
        uint4 v = *reinterpret_cast<const uint4*>(src + (size_t)r * K + (size_t)kg * 8);
        *reinterpret_cast<uint4*>(dst + ((size_t)(n / 32) * kgroups + kg) * 256 + (size_t)(n % 32) * 8) = v;
    }
}

int32_t launch_pack_rows(const uint16_t* src, int rows, int K, uint16_t* dst_packed, int row_offset, hipStream_t st) {
    if (rows == 0) return CHIRON_OK;
    int64_t total = (int64_t)rows * (K / 8);
    int blocks = (int)((total + 255) / 256 < 8192 ? (total + 255) / 256 : 8192);
    pack_rows_kernel<<<blocks, 256, 0, st>>>(src, rows, K, dst_packed, row_offset);
    CHIRON_HIP(hipGetLastError());
    return CHIRON_OK;
}

// ---- the kernel ------------------------------------------------------------------------------------------
template <int MT, int NF, int KS, int PRO>
__global__ __launch_bounds__(256) void linear_kernel(const uint16_t* __restrict__ Wp, int Npad, int Nreal, int K,
                                                     const float* __restrict__ A, int lda, int M,
                                                     float* __restrict__ Y, int ldy, int chunks_per_split,
                                                     int use_atomic) {
    constexpr int MROWS = 32 * MT;
    constexpr int RS = MROWS + 1;      // LDS row stride in 16-byte units (+1 breaks the power-of-two stride)
    constexpr int KG = 2 * KS;         // 8-wide k-groups per chunk
    constexpr int KC = 16 * KS;        // k per chunk
    constexpr int TASKS = MROWS * KG;  // 8-float staging tasks per chunk
    constexpr int TPT = (TASKS + 255) / 256;

    __shared__ uint4 lds_hi[KG * RS];
    __shared__ uint4 lds_lo[KG * RS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m0 = blockIdx.z * MROWS;
    const int tile0 = (blockIdx.x * 4 + wave) * NF;  // first 32-column tile of this wave
    const int kgroups = K / 8;
    const int chunks_total = (K + KC - 1) / KC;
    const int c_begin = blockIdx.y * chunks_per_split;
    int c_end = c_begin + chunks_per_split;
    if (c_end > chunks_total) c_end = chunks_total;

    floatx16 acc[NF][MT];
#pragma unroll
    for (int f = 0; f < NF; ++f)
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[f][t][r] = 0.f;

    uint4 wnext[KS][NF];
    float4 areg[TPT][2];
    float4 ureg[PRO == PRO_SWIGLU ? TPT : 1][2];

    auto load_w = [&](int c) {
        int kbase = c * KC;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            int kk = kbase + s * 16;
#pragma unroll
            for (int f = 0; f < NF; ++f) {
                int tile = tile0 + f;
                if (kk < K && tile * 32 < Npad) {
                    const uint16_t* p = Wp + ((size_t)tile * kgroups + (kk >> 3) + (lane >> 5)) * 256 + (lane & 31) * 8;
                    wnext[s][f] = *reinterpret_cast<const uint4*>(p);
                } else {
                    wnext[s][f] = make_uint4(0, 0, 0, 0);
                }
            }
        }
    };
    auto load_a = [&](int c) {
        int kbase = c * KC;
#pragma unroll
        for (int i = 0; i < TPT; ++i) {
            int task = tid + i * 256;
            int kg = task % KG, m = task / KG;
            int k = kbase + kg * 8;
            bool ok = (TASKS % 256 == 0 || task < TASKS) && (m0 + m < M) && (k < K);
            if (ok) {
                const float* p = A + (size_t)(m0 + m) * lda + k;
                areg[i][0] = *reinterpret_cast<const float4*>(p);
                areg[i][1] = *reinterpret_cast<const float4*>(p + 4);
                if (PRO == PRO_SWIGLU) {
                    ureg[i][0] = *reinterpret_cast<const float4*>(p + K);
                    ureg[i][1] = *reinterpret_cast<const float4*>(p + K + 4);
                }
            } else {
                areg[i][0] = areg[i][1] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (PRO == PRO_SWIGLU) ureg[i][0] = ureg[i][1] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
    };
    auto stage_a = [&]() {
#pragma unroll
        for (int i = 0; i < TPT; ++i) {
            int task = tid + i * 256;
            if (TASKS % 256 != 0 && task >= TASKS) continue;
            int kg = task % KG, m = task / KG;
            float v[8] = {areg[i][0].x, areg[i][0].y, areg[i][0].z, areg[i][0].w,
                          areg[i][1].x, areg[i][1].y, areg[i][1].z, areg[i][1].w};
            if (PRO == PRO_SWIGLU) {
                float u[8] = {ureg[i][0].x, ureg[i][0].y, ureg[i][0].z, ureg[i][0].w,
                              ureg[i][1].x, ureg[i][1].y, ureg[i][1].z, ureg[i][1].w};
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = v[e] / (1.0f + __expf(-v[e])) * u[e];
            }
            uint4 hi, lo;
            split2(v[0], v[1], hi.x, lo.x);
            split2(v[2], v[3], hi.y, lo.y);
            split2(v[4], v[5], hi.z, lo.z);
            split2(v[6], v[7], hi.w, lo.w);
            lds_hi[kg * RS + m] = hi;
            lds_lo[kg * RS + m] = lo;
        }
    };

    if (c_begin < c_end) {
        load_w(c_begin);
        load_a(c_begin);
    }
    for (int c = c_begin; c < c_end; ++c) {
        uint4 wcur[KS][NF];
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int f = 0; f < NF; ++f) wcur[s][f] = wnext[s][f];
        lds_barrier();  // every wave has finished reading the previous chunk
        stage_a();
        lds_barrier();
        if (c + 1 < c_end) {
            load_w(c + 1);
            load_a(c + 1);
        }
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            bf16x8 ah[MT], al[MT];
#pragma unroll
            for (int t = 0; t < MT; ++t) {
                int idx = (s * 2 + (lane >> 5)) * RS + t * 32 + (lane & 31);
                uint4 h = lds_hi[idx], l = lds_lo[idx];
                ah[t] = *reinterpret_cast<bf16x8*>(&h);
                al[t] = *reinterpret_cast<bf16x8*>(&l);
            }
#pragma unroll
            for (int f = 0; f < NF; ++f) {
                bf16x8 w = *reinterpret_cast<bf16x8*>(&wcur[s][f]);
#pragma unroll
                for (int t = 0; t < MT; ++t) {
                    acc[f][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w, ah[t], acc[f][t], 0, 0, 0);
                    acc[f][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w, al[t], acc[f][t], 0, 0, 0);
                }
            }
        }
    }

    // D[i][j]: lane holds column j = lane%32 (an activation row m) and rows i = 8*(r/4) + 4*(lane/32) + r%4
    // (output columns n) for r = 0..15.
#pragma unroll
    for (int f = 0; f < NF; ++f) {
        int nb = (tile0 + f) * 32 + (lane >> 5) * 4;
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            int m = m0 + t * 32 + (lane & 31);
            if (m >= M) continue;
            float* yrow = Y + (size_t)m * ldy;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                int n = nb + q * 8;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (n + e < Nreal) {
                        float v = acc[f][t][q * 4 + e];
                        if (use_atomic) atomicAdd(yrow + n + e, v);
                        else yrow[n + e] = v;
                    }
                }
            }
        }
    }
}

struct LinearTuning {
    int ksplit = 0;   // 0 = heuristic
    int nf = 0;
    int target_blocks = 512;
};
static LinearTuning tuning() {
    static LinearTuning t = [] {
        LinearTuning x;
        if (const char* e = getenv("CHIRON_LINEAR_KSPLIT")) x.ksplit = atoi(e);
        if (const char* e = getenv("CHIRON_LINEAR_NF")) x.nf = atoi(e);
        if (const char* e = getenv("CHIRON_LINEAR_BLOCKS")) x.target_blocks = atoi(e);
        return x;
    }();
    return t;
}

template <int MT, int NF, int PRO>
static void launch_cfg(dim3 grid, hipStream_t st, const Linear& L, const float* A, int lda, int M, float* y, int ldy,
                       int cps, int use_atomic) {
    linear_kernel<MT, NF, 4, PRO><<<grid, 256, 0, st>>>(L.w, L.Npad, L.N, L.K, A, lda, M, y, ldy, cps, use_atomic);
}

int32_t launch_linear(const Linear& L, const float* A, int lda, int M, float* y, int ldy, int accumulate, int prologue,
                      hipStream_t st) {
    if (M == 0) return CHIRON_OK;
    if (L.K % 16 != 0) return fail(CHIRON_ERR_SHAPE, "linear: K=%d must be a multiple of 16", L.K);
    if (lda % 4 != 0 || ((uintptr_t)A & 15)) return fail(CHIRON_ERR_INVALID_ARG, "linear: input rows must be 16-byte aligned");
    LinearTuning tn = tuning();
    constexpr int KS = 4, KC = 16 * KS;
    int mt = M > 32 ? 2 : 1;
    int tiles = L.Npad / 32;
    int nf = tn.nf ? tn.nf : (tiles >= 64 ? 2 : 1);
    // (MT=2, NF=1, SwiGLU) is not instantiated: hipcc 7.2 crashes in code generation on that one combination
    if (mt == 2 && prologue == PRO_SWIGLU) nf = 2;
    int gx = (tiles + 4 * nf - 1) / (4 * nf);
    int gz = (M + 32 * mt - 1) / (32 * mt);
    int chunks = (L.K + KC - 1) / KC;
    int ksplit = tn.ksplit ? tn.ksplit : (tn.target_blocks + gx * gz - 1) / (gx * gz);
    if (ksplit > chunks / 2) ksplit = chunks / 2;
    if (ksplit < 1) ksplit = 1;
    int cps = (chunks + ksplit - 1) / ksplit;
    ksplit = (chunks + cps - 1) / cps;  // no empty slices
    int use_atomic = (ksplit > 1 || accumulate) ? 1 : 0;
    if (ksplit > 1 && !accumulate) {
        // partial sums are added into y, so it has to start from zero
        if (ldy == L.N) {
            int32_t rc = launch_fill_zero(y, (int64_t)M * L.N, st);
            if (rc) return rc;
        } else {
            for (int m = 0; m < M; ++m) {
                int32_t rc = launch_fill_zero(y + (size_t)m * ldy, L.N, st);
                if (rc) return rc;
            }
        }
    }
    dim3 grid(gx, ksplit, gz);
#define CHIRON_LAUNCH(MT_, NF_)                                                                                   \
    do {                                                                                                           \
        if (prologue == PRO_SWIGLU) launch_cfg<MT_, NF_, PRO_SWIGLU>(grid, st, L, A, lda, M, y, ldy, cps, use_atomic); \
        else launch_cfg<MT_, NF_, PRO_NONE>(grid, st, L, A, lda, M, y, ldy, cps, use_atomic);                      \
    } while (0)
    if (mt == 1 && nf == 1) CHIRON_LAUNCH(1, 1);
    else if (mt == 1) CHIRON_LAUNCH(1, 2);
    else if (nf == 1) launch_cfg<2, 1, PRO_NONE>(grid, st, L, A, lda, M, y, ldy, cps, use_atomic);
    else CHIRON_LAUNCH(2, 2);
#undef CHIRON_LAUNCH
    CHIRON_HIP(hipGetLastError());
    return CHIRON_OK;
}

}  // namespace chiron

// Projections at large row counts (hundreds of requests per step): there the product is bound by the matrix
// cores, not by the weight stream, and the projection kernel is fastest when its activations arrive as their two
// bf16 terms in the same 32-row x 8-k tile order as the packed weights: it copies those pieces straight from global
// memory into LDS (no conversion work, no staging registers).  The down projection gets its input in that form from
// the gate/up projection's epilogue; split_pack_kernel produces it from fp32 rows for any other projection (a knob,
// off by default: the extra pass costs more than it saves there).
#include "chiron_internal.h"
#include "device_util.h"

namespace chiron {

__global__ __launch_bounds__(256) void split_pack_kernel(const float* __restrict__ A, int lda, int M, int K, int Kpad,
                                                         uint16_t* __restrict__ Ah, uint16_t* __restrict__ Al) {
    const int kgroups = Kpad / 8;
    const int r = threadIdx.x & 31, kgl = threadIdx.x >> 5;
    const int mtile = blockIdx.y;
    const int m = mtile * 32 + r;
    for (int kg = blockIdx.x * 8 + kgl; kg < kgroups; kg += gridDim.x * 8) {
        const int k = kg * 8;
        const bool ok = m < M && k < K;  // rows past M and the K padding are stored as zeros
        const float* p = A + (size_t)min(m, M - 1) * lda + min(k, K - 8);
        float4 a0 = *reinterpret_cast<const float4*>(p), a1 = *reinterpret_cast<const float4*>(p + 4);
        float v[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = ok ? v[e] : 0.f;
        uint4 hi, lo;
        split2(v[0], v[1], hi.x, lo.x);
        split2(v[2], v[3], hi.y, lo.y);
        split2(v[4], v[5], hi.z, lo.z);
        split2(v[6], v[7], hi.w, lo.w);
        size_t idx = ((size_t)mtile * kgroups + kg) * 256 + (size_t)r * 8;
        *reinterpret_cast<uint4*>(Ah + idx) = hi;
        *reinterpret_cast<uint4*>(Al + idx) = lo;
    }
}

size_t linear_big_split_elems(int M, int Kpad) { return (size_t)((M + 31) / 32) * 32 * Kpad; }

int32_t launch_linear_big(const Linear& L, const float* A, int lda, int M, float* y, int ldy, int epilogue,
                          float* part, int max_split, int* ksplit_out, uint16_t* asplit, hipStream_t st) {
    if (ksplit_out) *ksplit_out = 1;
    if (M == 0) return CHIRON_OK;
    if (L.K % 16 != 0 || L.K < 16) return fail(CHIRON_ERR_SHAPE, "linear: K=%d must be a positive multiple of 16", L.K);
    if (lda % 4 != 0 || ((uintptr_t)A & 15)) return fail(CHIRON_ERR_INVALID_ARG, "linear: input rows must be 16-byte aligned");
    if (!asplit) return fail(CHIRON_ERR_INVALID_ARG, "linear: no workspace for the split activations");
    uint16_t* ah = asplit;
    uint16_t* al = asplit + linear_big_split_elems(M, L.Kpad);
    const int mtiles = (M + 31) / 32, kgroups = L.Kpad / 8;
    {
        dim3 grid((unsigned)((kgroups / 8 < 64) ? (kgroups + 7) / 8 : 64), (unsigned)mtiles);
        launch(split_pack_kernel, dim3(grid), dim3(256), st, A, lda, M, L.K, L.Kpad, ah, al);
        CHIRON_HIP(hipGetLastError());
    }
    return launch_linear(L, reinterpret_cast<const float*>(ah), 0, M, y, ldy, epilogue, PRO_PACKED, part, max_split, ksplit_out,
                         nullptr, st);
}

}  // namespace chiron

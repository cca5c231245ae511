// Bandwidth-bound kernels of the decode step: embedding gather, RMSNorm, rotary embedding,
// KV append / gather (the slot contract), and small utilities.  gfx950, wave64.
#include "chiron_internal.h"
#include "device_util.h"

namespace chiron {

// ---- embedding gather: h[i] = E[tokens[i]] widened to fp32 --------------------------------------------
__global__ __launch_bounds__(256) void embed_kernel(const uint16_t* __restrict__ table,
                                                    const int32_t* __restrict__ tokens, int H,
                                                    float* __restrict__ h) {
    int i = blockIdx.x;
    const uint16_t* row = table + (size_t)tokens[i] * H;
    float* out = h + (size_t)i * H;
    for (int j = threadIdx.x * 8; j < H; j += 256 * 8) {
        uint4 v = *reinterpret_cast<const uint4*>(row + j);
        float4 a, b;
        a.x = bf16_lo(v.x); a.y = bf16_hi(v.x); a.z = bf16_lo(v.y); a.w = bf16_hi(v.y);
        b.x = bf16_lo(v.z); b.y = bf16_hi(v.z); b.z = bf16_lo(v.w); b.w = bf16_hi(v.w);
        *reinterpret_cast<float4*>(out + j) = a;
        *reinterpret_cast<float4*>(out + j + 4) = b;
    }
}

int32_t launch_embed(const uint16_t* table, const int32_t* tokens, int batch, int H, float* h, hipStream_t st) {
    if (batch == 0) return CHIRON_OK;
    embed_kernel<<<batch, 256, 0, st>>>(table, tokens, H, h);
    CHIRON_HIP(hipGetLastError());
    return CHIRON_OK;
}

// ---- RMSNorm: one workgroup per row, row held in registers, wavefront + LDS reduction -------------------
template <int VPT>  // float4 vectors per thread; covers n <= 256*4*VPT
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* __restrict__ h, const uint16_t* __restrict__ gain,
                                                      int n, float eps, float* __restrict__ out) {
    __shared__ float red[4];
    const float* row = h + (size_t)blockIdx.x * n;
    float* orow = out + (size_t)blockIdx.x * n;
    float4 v[VPT];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        int j = (i * 256 + threadIdx.x) * 4;
        if (j < n) {
            v[i] = *reinterpret_cast<const float4*>(row + j);
            ss += v[i].x * v[i].x + v[i].y * v[i].y + v[i].z * v[i].z + v[i].w * v[i].w;
        }
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = red[0] + red[1] + red[2] + red[3];
    float inv = 1.0f / sqrtf(tot / (float)n + eps);
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        int j = (i * 256 + threadIdx.x) * 4;
        if (j < n) {
            uint2 g = *reinterpret_cast<const uint2*>(gain + j);
            float4 o;
            o.x = v[i].x * inv * bf16_lo(g.x);
            o.y = v[i].y * inv * bf16_hi(g.x);
            o.z = v[i].z * inv * bf16_lo(g.y);
            o.w = v[i].w * inv * bf16_hi(g.y);
            *reinterpret_cast<float4*>(orow + j) = o;
        }
    }
}

int32_t launch_rmsnorm(const float* h, const uint16_t* gain, int rows, int n, float eps, float* out, hipStream_t st) {
    if (rows == 0) return CHIRON_OK;
    if (n % 4 != 0 || n > 256 * 4 * 16) return fail(CHIRON_ERR_SHAPE, "rmsnorm: n=%d must be a multiple of 4, <= 16384", n);
    if (n <= 1024) rmsnorm_kernel<1><<<rows, 256, 0, st>>>(h, gain, n, eps, out);
    else if (n <= 4096) rmsnorm_kernel<4><<<rows, 256, 0, st>>>(h, gain, n, eps, out);
    else if (n <= 8192) rmsnorm_kernel<8><<<rows, 256, 0, st>>>(h, gain, n, eps, out);
    else rmsnorm_kernel<16><<<rows, 256, 0, st>>>(h, gain, n, eps, out);
    CHIRON_HIP(hipGetLastError());
    return CHIRON_OK;
}

// ---- zero fill (used instead of memset so that it can live inside captured graphs) ---------------------
__global__ __launch_bounds__(256) void fill_zero_kernel(float4* __restrict__ p, int64_t n4, float* tail_base, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t j = i; j < n4; j += stride) p[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < n - n4 * 4) tail_base[n4 * 4 + i] = 0.f;
}

int32_t launch_fill_zero(float* p, int64_t n, hipStream_t st) {
    if (n <= 0) return CHIRON_OK;
    int64_t n4 = n / 4;
    int blocks = (int)((n4 + 255) / 256);
    if (blocks < 1) blocks = 1;
    if (blocks > 2048) blocks = 2048;
    fill_zero_kernel<<<blocks, 256, 0, st>>>(reinterpret_cast<float4*>(p), n4, p, n);
    CHIRON_HIP(hipGetLastError());
    return CHIRON_OK;
}

// ---- rotary table: fp64 angle and trigonometry, once per step -------------------------------------------
__global__ void rope_table_kernel(const int32_t* __restrict__ pos, int rows, int d, float base, int pos_bias,
                                  float* __restrict__ cos_t, float* __restrict__ sin_t) {
    int half = d / 2;
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= rows * half) return;
    int r = idx / half, j = idx % half;
    double inv_freq = pow((double)base, -2.0 * (double)j / (double)d);
    double ang = (double)(pos[r] + pos_bias) * inv_freq;
    double s, c;
    sincos(ang, &s, &c);
    cos_t[idx] = (float)c;
    sin_t[idx] = (float)s;
}

int32_t launch_rope_table(const int32_t* pos, int rows, int d, float base, float* cos_t, float* sin_t, hipStream_t st) {
    if (rows == 0) return CHIRON_OK;
    int n = rows * (d / 2);
    rope_table_kernel<<<(n + 255) / 256, 256, 0, st>>>(pos, rows, d, base, 0, cos_t, sin_t);
    CHIRON_HIP(hipGetLastError());
    return CHIRON_OK;
}

__global__ __launch_bounds__(256) void rope_kernel(float* __restrict__ x, int ldx, int n_heads, int d,
                                                   const float* __restrict__ cos_t, const float* __restrict__ sin_t) {
    int r = blockIdx.x, half = d / 2;
    float* row = x + (size_t)r * ldx;
    for (int e = threadIdx.x; e < n_heads * half; e += 256) {
        int hd = e / half, j = e % half;
        float c = cos_t[r * half + j], s = sin_t[r * half + j];
        float a = row[hd * d + j], b = row[hd * d + j + half];
        row[hd * d + j] = a * c - b * s;
        row[hd * d + j + half] = b * c + a * s;
    }
}

int32_t launch_rope(float* x, int ldx, int n_heads, int d, const float* cos_t, const float* sin_t, int rows,
                    hipStream_t st) {
    if (rows == 0) return CHIRON_OK;
    rope_kernel<<<rows, 256, 0, st>>>(x, ldx, n_heads, d, cos_t, sin_t);
    CHIRON_HIP(hipGetLastError());
    return CHIRON_OK;
}

// ---- KV pool addressing -----------------------------------------------------------------------------------
// Pool memory: [layer][block][kv head][K tile | V tile], each tile 16*d bf16.
//   K tile: element (tok t, dim e) at ((e/8)*16 + t)*8 + e%8               -> rows of 8 dims, token-major groups
//   V tile: element (tok t, dim e) at ((((e/32)*4 + t/4)*16 + e%16)*2 + (e%32)/16)*4 + t%4   -> token-minor
// Both orders make every matrix-core operand fragment of the attention kernel a contiguous 1 KiB read.
__device__ __forceinline__ size_t tile_base(const PoolDesc& p, int layer, int block, int kvh) {
    return (size_t)layer * (size_t)p.layer_stride + ((size_t)block * p.n_kv + kvh) * (size_t)(2 * 16 * p.d);
}
__device__ __forceinline__ int k_off(int t, int e) { return ((e >> 3) * 16 + t) * 8 + (e & 7); }
__device__ __forceinline__ int v_off(int t, int e) {
    return (((((e >> 5) * 4 + (t >> 2)) * 16 + (e & 15)) * 2 + ((e & 31) >> 4)) * 4) + (t & 3);
}

__global__ __launch_bounds__(256) void append_kv_kernel(PoolDesc p, int layer, const uint16_t* __restrict__ k,
                                                        const uint16_t* __restrict__ v, const int32_t* __restrict__ bt,
                                                        int max_blocks, const int32_t* __restrict__ seq_idx,
                                                        const int32_t* __restrict__ pos, int64_t n) {
    int row = p.n_kv * p.d;
    for (int64_t j = blockIdx.x; j < n; j += gridDim.x) {
        int ps = pos[j];
        int block = bt[(size_t)seq_idx[j] * max_blocks + ps / kBlockSize];
        int t = ps % kBlockSize;
        for (int e = threadIdx.x; e < row; e += 256) {
            int kvh = e / p.d, dd = e % p.d;
            size_t tb = tile_base(p, layer, block, kvh);
            p.base[tb + k_off(t, dd)] = k[j * row + e];
            p.base[tb + 16 * p.d + v_off(t, dd)] = v[j * row + e];
        }
    }
}

int32_t launch_append_kv(const PoolDesc& p, int layer, const uint16_t* k, const uint16_t* v, const int32_t* bt,
                         int max_blocks, const int32_t* seq_idx, const int32_t* pos, int64_t n, hipStream_t st) {
    if (n == 0) return CHIRON_OK;
    int blocks = (int)(n < 65536 ? n : 65536);
    append_kv_kernel<<<blocks, 256, 0, st>>>(p, layer, k, v, bt, max_blocks, seq_idx, pos, n);
    CHIRON_HIP(hipGetLastError());
    return CHIRON_OK;
}

__global__ __launch_bounds__(256) void gather_kv_kernel(PoolDesc p, int layer, const int32_t* __restrict__ bt_row,
                                                        int len, uint16_t* __restrict__ k_out,
                                                        uint16_t* __restrict__ v_out) {
    int row = p.n_kv * p.d;
    for (int tk = blockIdx.x; tk < len; tk += gridDim.x) {
        int block = bt_row[tk / kBlockSize];
        int t = tk % kBlockSize;
        for (int e = threadIdx.x; e < row; e += 256) {
            int kvh = e / p.d, dd = e % p.d;
            size_t tb = tile_base(p, layer, block, kvh);
            k_out[(size_t)tk * row + e] = p.base[tb + k_off(t, dd)];
            v_out[(size_t)tk * row + e] = p.base[tb + 16 * p.d + v_off(t, dd)];
        }
    }
}

int32_t launch_gather_kv(const PoolDesc& p, int layer, const int32_t* bt_row, int len, uint16_t* k_out, uint16_t* v_out,
                         hipStream_t st) {
    if (len == 0) return CHIRON_OK;
    gather_kv_kernel<<<len < 65536 ? len : 65536, 256, 0, st>>>(p, layer, bt_row, len, k_out, v_out);
    CHIRON_HIP(hipGetLastError());
    return CHIRON_OK;
}

// ---- decode step: rotate q and k, round k and v to bf16, write them at slot(i, seq_lens[i]) ----------------
__global__ __launch_bounds__(256) void rope_append_kernel(PoolDesc p, int layer, float* __restrict__ qkv, int n_q,
                                                          const float* __restrict__ cos_t,
                                                          const float* __restrict__ sin_t,
                                                          const int32_t* __restrict__ bt, int max_blocks,
                                                          const int32_t* __restrict__ seq_lens) {
    int i = blockIdx.x, d = p.d, half = d / 2;
    int ld = (n_q + 2 * p.n_kv) * d;
    float* row = qkv + (size_t)i * ld;
    int ps = seq_lens[i];
    int block = bt[(size_t)i * max_blocks + ps / kBlockSize];
    int t = ps % kBlockSize;
    const float* ct = cos_t + (size_t)i * half;
    const float* sn = sin_t + (size_t)i * half;
    // q heads then k heads: rotate pairs (j, j+half)
    for (int e = threadIdx.x; e < (n_q + p.n_kv) * half; e += 256) {
        int hd = e / half, j = e % half;
        float c = ct[j], s = sn[j];
        float a = row[hd * d + j], b = row[hd * d + j + half];
        float ra = a * c - b * s, rb = b * c + a * s;
        if (hd < n_q) {
            row[hd * d + j] = ra;
            row[hd * d + j + half] = rb;
        } else {
            int kvh = hd - n_q;
            size_t tb = tile_base(p, layer, block, kvh);
            p.base[tb + k_off(t, j)] = f32_to_bf16_rne(ra);
            p.base[tb + k_off(t, j + half)] = f32_to_bf16_rne(rb);
        }
    }
    const float* vrow = row + (n_q + p.n_kv) * d;
    for (int e = threadIdx.x; e < p.n_kv * d; e += 256) {
        int kvh = e / d, dd = e % d;
        size_t tb = tile_base(p, layer, block, kvh);
        p.base[tb + 16 * d + v_off(t, dd)] = f32_to_bf16_rne(vrow[e]);
    }
}

int32_t launch_rope_append(const PoolDesc& p, int layer, float* qkv, int n_q, const float* cos_t, const float* sin_t,
                           const int32_t* bt, int max_blocks, const int32_t* seq_lens, int batch, hipStream_t st) {
    if (batch == 0) return CHIRON_OK;
    rope_append_kernel<<<batch, 256, 0, st>>>(p, layer, qkv, n_q, cos_t, sin_t, bt, max_blocks, seq_lens);
    CHIRON_HIP(hipGetLastError());
    return CHIRON_OK;
}

}  // namespace chiron

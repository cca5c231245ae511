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
    launch(embed_kernel, dim3(batch), dim3(256), st, table, tokens, H, h);
    CHIRON_HIP(hipGetLastError());
    return CHIRON_OK;
}

// ---- RMSNorm: one workgroup per row, row held in registers, wavefront + LDS reduction -------------------
// Also the place where a K-sliced projection into the residual stream is summed: h += sum_s part[s].  The
// slice loads of a thread are independent, so they are issued four at a time.
template <int THREADS, int VPT>  // float4 vectors per thread; covers n <= THREADS*4*VPT
__global__ __launch_bounds__(THREADS) void rmsnorm_kernel(float* __restrict__ h, const float* __restrict__ part, int ks,
                                                          size_t part_stride, const uint16_t* __restrict__ gain, int n,
                                                          float eps, float* __restrict__ out) {
    __shared__ float red[THREADS / 64];
    float* row = h + (size_t)blockIdx.x * n;
    const float* prow = part + (size_t)blockIdx.x * n;
    float* orow = out + (size_t)blockIdx.x * n;
    float4 v[VPT];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        int j = (i * THREADS + threadIdx.x) * 4;
        if (j < n) {
            v[i] = *reinterpret_cast<const float4*>(row + j);
            if (ks > 0) {
                int s = 0;
                for (; s + 4 <= ks; s += 4) {
                    float4 t[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) t[u] = *reinterpret_cast<const float4*>(prow + (size_t)(s + u) * part_stride + j);
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        v[i].x += t[u].x; v[i].y += t[u].y; v[i].z += t[u].z; v[i].w += t[u].w;
                    }
                }
                for (; s < ks; ++s) {
                    float4 t = *reinterpret_cast<const float4*>(prow + (size_t)s * part_stride + j);
                    v[i].x += t.x; v[i].y += t.y; v[i].z += t.z; v[i].w += t.w;
                }
                *reinterpret_cast<float4*>(row + j) = v[i];
            }
            ss += v[i].x * v[i].x + v[i].y * v[i].y + v[i].z * v[i].z + v[i].w * v[i].w;
        }
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int k = 0; k < THREADS / 64; ++k) tot += red[k];
    float inv = 1.0f / sqrtf(tot / (float)n + eps);
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        int j = (i * THREADS + threadIdx.x) * 4;
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

int32_t launch_rmsnorm(float* h, const float* part, int ks, const uint16_t* gain, int rows, int n, float eps, float* out,
                       hipStream_t st) {
    if (rows == 0) return CHIRON_OK;
    if (n % 4 != 0 || n > 16384) return fail(CHIRON_ERR_SHAPE, "rmsnorm: n=%d must be a multiple of 4, <= 16384", n);
    size_t ps = (size_t)rows * n;
    if (n <= 1024) launch(rmsnorm_kernel<256, 1>, dim3(rows), dim3(256), st, h, part, ks, ps, gain, n, eps, out);
    else if (n <= 4096) launch(rmsnorm_kernel<1024, 1>, dim3(rows), dim3(1024), st, h, part, ks, ps, gain, n, eps, out);
    else if (n <= 8192) launch(rmsnorm_kernel<1024, 2>, dim3(rows), dim3(1024), st, h, part, ks, ps, gain, n, eps, out);
    else launch(rmsnorm_kernel<1024, 4>, dim3(rows), dim3(1024), st, h, part, ks, ps, gain, n, eps, out);
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
    launch(rope_table_kernel, dim3((n + 255) / 256), dim3(256), st, pos, rows, d, base, 0, cos_t, sin_t);
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
    launch(rope_kernel, dim3(rows), dim3(256), st, x, ldx, n_heads, d, cos_t, sin_t);
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
    launch(append_kv_kernel, dim3(blocks), dim3(256), st, p, layer, k, v, bt, max_blocks, seq_idx, pos, n);
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
    launch(gather_kv_kernel, dim3(len < 65536 ? len : 65536), dim3(256), st, p, layer, bt_row, len, k_out, v_out);
    CHIRON_HIP(hipGetLastError());
    return CHIRON_OK;
}

// ---- multi-token step: expand [batch] requests x q_len tokens into batch*q_len rows ----------------------
__global__ __launch_bounds__(256) void expand_rows_kernel(const int32_t* __restrict__ bt, const int32_t* __restrict__ seq_lens,
                                                          int q_len, int max_blocks, int32_t* __restrict__ bt_out,
                                                          int32_t* __restrict__ lens_out) {
    const int r = blockIdx.x, i = r / q_len, t = r % q_len;
    for (int e = threadIdx.x; e < max_blocks; e += 256) bt_out[(size_t)r * max_blocks + e] = bt[(size_t)i * max_blocks + e];
    if (threadIdx.x == 0) lens_out[r] = seq_lens[i] + t;
}

int32_t launch_expand_rows(const int32_t* bt, const int32_t* seq_lens, int batch, int q_len, int max_blocks, int32_t* bt_out,
                           int32_t* lens_out, hipStream_t st) {
    if (batch * q_len == 0) return CHIRON_OK;
    launch(expand_rows_kernel, dim3(batch * q_len), dim3(256), st, bt, seq_lens, q_len, max_blocks, bt_out, lens_out);
    CHIRON_HIP(hipGetLastError());
    return CHIRON_OK;
}

// ---- page migration (eviction to host memory and back): one workgroup per (page, layer), 16-byte copies ------
__global__ __launch_bounds__(256) void swap_kernel(PoolDesc p, const int32_t* __restrict__ bt_row, uint16_t* image,
                                                   int to_image) {
    const int j = blockIdx.x, layer = blockIdx.y;
    const size_t page_elems = (size_t)p.n_kv * 2 * 16 * p.d;
    uint4* pool = reinterpret_cast<uint4*>(p.base + (size_t)layer * (size_t)p.layer_stride + (size_t)bt_row[j] * page_elems);
    uint4* img = reinterpret_cast<uint4*>(image + ((size_t)j * p.n_layers + layer) * page_elems);
    const int n16 = (int)(page_elems / 8);
    for (int e = threadIdx.x; e < n16; e += 256) {
        if (to_image) img[e] = pool[e];
        else pool[e] = img[e];
    }
}

int32_t launch_swap(const PoolDesc& p, const int32_t* bt_row, int n_pages, uint16_t* image, int to_image, hipStream_t st) {
    if (n_pages == 0) return CHIRON_OK;
    launch(swap_kernel, dim3(dim3(n_pages, p.n_layers)), dim3(256), st, p, bt_row, image, to_image);
    CHIRON_HIP(hipGetLastError());
    return CHIRON_OK;
}

// ---- decode step: sum the K-slices of the QKV projection, rotate q and k, round k and v to bf16, write them
// at slot(i, seq_lens[i]).  One wave per (request, head): lane j owns dims j, j+64, ... of the head. ------------
__global__ __launch_bounds__(64) void rope_append_kernel(PoolDesc p, int layer, const float* __restrict__ qkv, int ks,
                                                         size_t slice_stride, int n_q,
                                                         const float* __restrict__ cos_t,
                                                         const float* __restrict__ sin_t,
                                                         const int32_t* __restrict__ bt, int max_blocks,
                                                         const int32_t* __restrict__ seq_lens,
                                                         float* __restrict__ q_out) {
    const int i = blockIdx.x, hd = blockIdx.y, d = p.d, half = d / 2;
    const int ld = (n_q + 2 * p.n_kv) * d;
    const float* row = qkv + (size_t)i * ld + (size_t)hd * d;
    // sum over the K-slices, four independent loads in flight at a time, slices added in ascending order
    auto val = [&](int e) {
        const float* q = row + e;
        float v = 0.f;
        int s = 0;
        for (; s + 4 <= ks; s += 4) {
            float t0 = q[(size_t)s * slice_stride], t1 = q[(size_t)(s + 1) * slice_stride];
            float t2 = q[(size_t)(s + 2) * slice_stride], t3 = q[(size_t)(s + 3) * slice_stride];
            v += t0; v += t1; v += t2; v += t3;
        }
        for (; s < ks; ++s) v += q[(size_t)s * slice_stride];
        return v;
    };
    const int ps = seq_lens[i];
    const int block = bt[(size_t)i * max_blocks + ps / kBlockSize];
    const int t = ps % kBlockSize;
    if (hd < n_q + p.n_kv) {
        for (int j = threadIdx.x; j < half; j += 64) {
            float c = cos_t[(size_t)i * half + j], s = sin_t[(size_t)i * half + j];
            float a = val(j), b = val(j + half);
            float ra = a * c - b * s, rb = b * c + a * s;
            if (hd < n_q) {
                float* qrow = q_out + (size_t)i * n_q * d + (size_t)hd * d;
                qrow[j] = ra;
                qrow[j + half] = rb;
            } else {
                size_t tb = tile_base(p, layer, block, hd - n_q);
                p.base[tb + k_off(t, j)] = f32_to_bf16_rne(ra);
                p.base[tb + k_off(t, j + half)] = f32_to_bf16_rne(rb);
            }
        }
    } else {
        size_t tb = tile_base(p, layer, block, hd - n_q - p.n_kv);
        for (int e = threadIdx.x; e < d; e += 64) p.base[tb + 16 * d + v_off(t, e)] = f32_to_bf16_rne(val(e));
    }
}

int32_t launch_rope_append(const PoolDesc& p, int layer, const float* qkv, int ks, int n_q, const float* cos_t,
                           const float* sin_t, const int32_t* bt, int max_blocks, const int32_t* seq_lens, int batch,
                           float* q_out, hipStream_t st) {
    if (batch == 0) return CHIRON_OK;
    size_t stride = (size_t)batch * (n_q + 2 * p.n_kv) * p.d;
    dim3 grid(batch, n_q + 2 * p.n_kv);
    launch(rope_append_kernel, dim3(grid), dim3(64), st, p, layer, qkv, ks, stride, n_q, cos_t, sin_t, bt, max_blocks, seq_lens, q_out);
    CHIRON_HIP(hipGetLastError());
    return CHIRON_OK;
}

}  // namespace chiron

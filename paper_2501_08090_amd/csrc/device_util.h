// Device-side helpers: bf16 widening/rounding, the two-term bf16 split of fp32 activations,
// wavefront reductions, LDS-only barrier.  gfx950 (wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace chiron {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// two bf16 packed in a 32-bit word: low half first in memory
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// round-to-nearest-even pair conversion (v_cvt_pk_bf16_f32); first argument lands in the low half
__device__ __forceinline__ uint32_t pack_bf16_rne(float a, float b) {
    floatx2 x = {a, b};
    bf16x2 h = __builtin_convertvector(x, bf16x2);
    return *reinterpret_cast<uint32_t*>(&h);
}
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float a) { return (uint16_t)(pack_bf16_rne(a, 0.f) & 0xffffu); }

// x ~= hi + lo with hi = bf16(x), lo = bf16(x - hi): 16 significant bits instead of 8, so that
// rounding the activations costs ~2^-17 relative instead of 2^-9 while the products still run
// on the bf16 matrix cores (two MFMAs per weight fragment).
__device__ __forceinline__ void split2(float a, float b, uint32_t& hi, uint32_t& lo) {
    hi = pack_bf16_rne(a, b);
    lo = pack_bf16_rne(a - bf16_lo(hi), b - bf16_hi(hi));
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// Workgroup barrier that waits for this wave's LDS traffic only: global loads already in
// flight (weight prefetch) stay in flight across it.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// 16-byte load of data that is read exactly once (K/V tiles, weights when a single workgroup row streams them):
// the non-temporal hint keeps such streams from displacing the L2's working set and measured 8-12 % more
// streaming bandwidth than plain loads (7.0 against 6.3 TB/s at 512 workgroups).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream_16(const void* p) {
    u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// 16 bytes per lane straight from global memory into LDS: lane l's piece lands at lds_addr + 16*l (lds_addr is
// the wave-uniform byte address inside the workgroup's LDS).  Written as assembly on purpose: the compiler makes
// every later LDS read wait for all outstanding copies of this kind, which would undo the overlap; the caller
// waits itself (s_waitcnt vmcnt, then a barrier) before anyone reads the destination.
__device__ __forceinline__ void global_to_lds_16(const void* g, uint32_t lds_addr) {
    const uint32_t base = __builtin_amdgcn_readfirstlane(lds_addr);  // the "s" constraint alone does not move a VGPR value
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(base), "v"(g) : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_address(const void* p) {
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void*)p;
}

}  // namespace chiron

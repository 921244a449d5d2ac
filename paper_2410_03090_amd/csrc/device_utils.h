// Device helpers shared by the kernel files: element loads for the two storage types and
// wavefront-level reductions.  gfx950 only (64-wide wavefronts).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <stdint.h>

namespace uncomp {

typedef uint16_t bf16_bits;   // storage of one bf16 element

__device__ __forceinline__ float bf16_to_f32(bf16_bits v) {
    return __uint_as_float(((uint32_t)v) << 16);
}

// Loads 8 consecutive elements starting at p (16-byte aligned for bf16, 32-byte for
// fp32 by the interface's stride rules) and widens them to fp32.
__device__ __forceinline__ void load8(const bf16_bits* p, float out[8]) {
    uint4 raw = *reinterpret_cast<const uint4*>(p);
    uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        out[2 * i] = __uint_as_float(w[i] << 16);
        out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}
__device__ __forceinline__ void load8(const float* p, float out[8]) {
    float4 a = *reinterpret_cast<const float4*>(p);
    float4 b = *reinterpret_cast<const float4*>(p + 4);
    out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
    out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
}

// Operand / accumulator vectors of v_mfma_f32_16x16x32_bf16.  Lane l holds: A row l%16 (or
// B column l%16), k = 8*(l/16) .. +8; accumulator column l%16, rows 4*(l/16) .. +4.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// Lane layout: four rows of 16 lanes.  For four registers X, Y, Z, W returns, in lane row
// 0 / 1 / 2 / 3, the sum over all four rows of X / Z / Y / W (per lane%16).
// v_permlane32_swap(a,b) -> ([a.lo32, b.lo32], [a.hi32, b.hi32]);
// v_permlane16_swap(a,b) -> ([a.r0, b.r0, a.r2, b.r2], [a.r1, b.r1, a.r3, b.r3]).
__device__ __forceinline__ float reduce4_over_rows(float x, float y, float z, float w) {
    auto s1 = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(y), false, false);
    auto s2 = __builtin_amdgcn_permlane32_swap(__float_as_uint(z), __float_as_uint(w), false, false);
    const float t1 = __uint_as_float(s1[0]) + __uint_as_float(s1[1]);
    const float t2 = __uint_as_float(s2[0]) + __uint_as_float(s2[1]);
    auto s3 = __builtin_amdgcn_permlane16_swap(__float_as_uint(t1), __float_as_uint(t2), false, false);
    return __uint_as_float(s3[0]) + __uint_as_float(s3[1]);
}

// float -> uint32 whose unsigned order equals the float order (negative values included; -0.0 and +0.0
// get the same key).  The selection kernels rank scores by this key.
__device__ __forceinline__ uint32_t order_key(float f) {
    uint32_t u = __float_as_uint(f + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

}  // namespace uncomp

// Small device helpers shared by the gfx950 kernel files: exact widening of the 16-bit storage
// formats, the single final rounding, the keep-predicate of the sparsification function.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rsparse {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));

constexpr int F16 = 0, BF16 = 1, F32 = 2;
constexpr int kUnroll = 8;       // rows in flight per wave in the streaming loop

__device__ __forceinline__ float as_f(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u(float f) { return __builtin_bit_cast(uint32_t, f); }

// Exact widening of eight packed 16-bit values (element 0 in the low half of word 0).
template <int DT>
__device__ __forceinline__ void unpack8(const u32x4 v, float (&f)[8])
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (DT == F16) {
            const uint32_t word = v[i];      // bit_cast needs a scalar copy, not a vector-element lvalue
            h2 p = __builtin_bit_cast(h2, word);
            f[2 * i] = (float)p[0];          // v_cvt_f32_f16 keeps fp16 subnormals
            f[2 * i + 1] = (float)p[1];
        } else {
            f[2 * i] = as_f(v[i] << 16);
            f[2 * i + 1] = as_f(v[i] & 0xffff0000u);
        }
    }
}

// One round-to-nearest-even from the fp32 accumulator to the output type.
__device__ __forceinline__ uint16_t to_bf16(float f)
{
    uint32_t u = as_u(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ uint16_t to_f16(float f)
{
    _Float16 h = (_Float16)f;
    return __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ void store_out(void *Y, size_t i, float v, int out_dtype)
{
    if (out_dtype == F32) ((float *)Y)[i] = v;
    else if (out_dtype == F16) ((uint16_t *)Y)[i] = to_f16(v);
    else ((uint16_t *)Y)[i] = to_bf16(v);
}

// Keep-predicate of the sparsification function: |x| >= t (mode 0) or |x| > t (mode 1).
// NaN compares false and is never kept.
__device__ __forceinline__ bool keep(float x, float tau, int mode)
{
    float a = __builtin_fabsf(x);
    return mode == 0 ? (a >= tau) : (a > tau);
}

template <bool NT>
__device__ __forceinline__ u32x4 ldg16(const uint16_t *p)
{
    const u32x4 *q = reinterpret_cast<const u32x4 *>(p);
    return NT ? __builtin_nontemporal_load(q) : *q;
}

__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ float uniform(float v) { return as_f(__builtin_amdgcn_readfirstlane(as_u(v))); }

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

}  // namespace
}  // namespace rsparse

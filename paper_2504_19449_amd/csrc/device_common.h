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

// SiLU of the gated MLP input (Sec. 3.1), as a fixed fp32 recipe so that the 16-bit product and with it
// the kept-channel sets do not depend on a math library: x = max(-g, -86), n = rint(x log2 e),
// r = x - n ln2 (two-constant reduction, fused multiply-adds), exp(r) by its degree-7 Taylor
// polynomial, e = exp(r) 2^n by exponent addition, silu = g / (1 + e).  Every step is one correctly
// rounded fp32 operation; contraction is off so that no step is merged with its neighbour.
__device__ __forceinline__ float silu32(float g)
{
#pragma clang fp contract(off)
    if (g != g) return g;
    if (!(g >= -87.0f)) return -0.0f;
    float x = -g;
    if (x < -86.0f) x = -86.0f;
    const float n = __builtin_rintf(x * 1.44269504f);
    float r = __builtin_fmaf(-n, 0.693145752f, x);
    r = __builtin_fmaf(-n, 1.42860677e-6f, r);
    float p = 1.98412698e-4f;
    p = __builtin_fmaf(p, r, 1.38888889e-3f);
    p = __builtin_fmaf(p, r, 8.33333333e-3f);
    p = __builtin_fmaf(p, r, 4.16666667e-2f);
    p = __builtin_fmaf(p, r, 1.66666667e-1f);
    p = __builtin_fmaf(p, r, 0.5f);
    p = __builtin_fmaf(p, r, 1.0f);
    p = __builtin_fmaf(p, r, 1.0f);
    const float e = as_f(as_u(p) + ((uint32_t)(int32_t)n << 23));
    const float d = 1.0f + e;
    return __fdiv_rn(g, d);
}

// One element of the gated input: round16(silu(g) * u), 16-bit patterns in and out.
template <int DT>
__device__ __forceinline__ uint16_t gated1(uint16_t g, uint16_t u)
{
    const float gf = DT == F16 ? (float)__builtin_bit_cast(_Float16, g) : as_f((uint32_t)g << 16);
    const float uf = DT == F16 ? (float)__builtin_bit_cast(_Float16, u) : as_f((uint32_t)u << 16);
    float h = silu32(gf) * uf;
    // The product is rounded to fp32 first and to 16 bits second, on purpose: without this barrier the
    // compiler merges the multiply and the fp16 conversion into one mixed-precision instruction with a
    // single rounding (and loses the sign of a zero product).
    __asm__ volatile("" : "+v"(h));
    return DT == F16 ? to_f16(h) : to_bf16(h);
}

// Eight consecutive input values: X[off..off+8), or, with a gate operand, round16(silu(G) * X).
template <int DT>
__device__ __forceinline__ u32x4 load_x8(const uint16_t *X, const uint16_t *G, size_t off)
{
    const u32x4 xu = *reinterpret_cast<const u32x4 *>(X + off);
    if (!G) return xu;
    const u32x4 xg = *reinterpret_cast<const u32x4 *>(G + off);
    u32x4 o;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint32_t gw = xg[i], uw = xu[i];
        o[i] = (uint32_t)gated1<DT>((uint16_t)gw, (uint16_t)uw) |
               ((uint32_t)gated1<DT>((uint16_t)(gw >> 16), (uint16_t)(uw >> 16)) << 16);
    }
    return o;
}
// Exact widening of one stored 16-bit value.
template <int DT>
__device__ __forceinline__ float widen16(uint16_t h)
{
    return DT == F16 ? (float)__builtin_bit_cast(_Float16, h) : as_f((uint32_t)h << 16);
}

// Keep-predicate of the sparsification function (see KeepRule).  NaN compares false and is never kept.
__device__ __forceinline__ bool keep(float x, int c, const KeepRule &r, bool sgn)
{
    const float v = sgn ? x : __builtin_fabsf(x);
    return (v >= r.ge) | ((v == r.eq) & (c <= r.cut));
}
// The same for rules known to be a plain threshold on the magnitude (no `eq` part, not signed).
__device__ __forceinline__ bool keep_threshold(float x, const KeepRule &r) { return __builtin_fabsf(x) >= r.ge; }
// The rule of token b of the call: the layer's threshold, or the token's own fixed-count rule.
__device__ __forceinline__ KeepRule rule_of(const LayerView &L, int b)
{
    KeepRule r;
    if (L.rules) {
        r.ge = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, L.rules[b].ge)));
        r.eq = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, L.rules[b].eq)));
        r.cut = __builtin_amdgcn_readfirstlane(L.rules[b].cut);
    } else {
        r.ge = L.tau_ge;
        r.eq = __builtin_nanf("");
        r.cut = -1;
    }
    r.pad = 0;
    return r;
}
__device__ __forceinline__ float bias_at(const LayerView &L, int o) { return L.bias ? L.bias[o] : 0.f; }

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

// Device-side helpers: bf16 <-> f32, typed loads/stores, the epilogue interpreter.
#pragma once
#include "kernels.h"

namespace rl {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// round to nearest, ties to even; finite inputs (NaN maps to a quiet NaN)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ float round_bf16(float f) { return bf16_bits_to_f32(f32_to_bf16_bits(f)); }

__device__ __forceinline__ float load_as_f32(const void *p, int dtype, int64_t i)
{
    if (dtype == DT_BF16) return bf16_bits_to_f32(((const uint16_t *)p)[i]);
    return ((const float *)p)[i];
}

__device__ __forceinline__ void store_from_f32(void *p, int dtype, int64_t i, float v)
{
    if (dtype == DT_BF16) ((uint16_t *)p)[i] = (uint16_t)f32_to_bf16_bits(v);
    else ((float *)p)[i] = v;
}

__device__ __forceinline__ float sigmoidf_(float x) { return 1.0f / (1.0f + __expf(-x)); }

// tanh through one exponential; exact limits for large |x|, odd symmetry kept
__device__ __forceinline__ float tanhf_(float x)
{
    float ax = fabsf(x);
    float e = __expf(-2.0f * ax);
    float t = (1.0f - e) / (1.0f + e);
    // for tiny |x| the quotient loses relative accuracy; tanh x = x - x^3/3 + ...
    if (ax < 0.02f) t = ax * (1.0f - ax * ax * (1.0f / 3.0f));
    return copysignf(t, x);
}

// One step of the epilogue chain on one element.
//   idx : flat offset of the element in the group's output tensor (operands
//         of the group's shape share its layout)
//   ch  : channel index for E_BIAS
__device__ __forceinline__ float epi_step(const Epilogue &e, int s, float v, int64_t idx, int ch)
{
    const int a = e.arg[s];
    switch (e.op[s]) {
    case E_BIAS: return v + load_as_f32(e.ptr[a], e.ptr_dtype[a], ch);
    case E_ADD: return v + load_as_f32(e.ptr[a], e.ptr_dtype[a], idx);
    case E_SUB: return v - load_as_f32(e.ptr[a], e.ptr_dtype[a], idx);
    case E_RSUB: return load_as_f32(e.ptr[a], e.ptr_dtype[a], idx) - v;
    case E_MUL: return v * load_as_f32(e.ptr[a], e.ptr_dtype[a], idx);
    case E_DIV: return v / load_as_f32(e.ptr[a], e.ptr_dtype[a], idx);
    case E_RDIV: return load_as_f32(e.ptr[a], e.ptr_dtype[a], idx) / v;
    case E_NEG: return -v;
    case E_SQ: return v * v;
    case E_RELU: return v > 0.0f ? v : 0.0f;
    case E_SIGMOID: return sigmoidf_(v);
    case E_TANH: return tanhf_(v);
    case E_ADD_VV: return v + v;
    case E_SUB_VV: return v - v;
    case E_DIV_VV: return v / v;
    case E_ROUND_BF16: return round_bf16(v);
    default: return v;
    }
}

}  // namespace rl

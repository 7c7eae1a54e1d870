// Device-side helpers: bf16 <-> f32, typed loads/stores, the epilogue interpreter.
#pragma once
#include "kernels.h"

namespace rl {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// Lanes of one wave exchanging data through LDS without a workgroup barrier: the LDS executes a
// wave's instructions in order, so no hardware wait is needed, but the compiler must not move or
// reuse LDS accesses across the exchange point (to it, what other lanes wrote is invisible).
__device__ __forceinline__ void wave_lds_exchange()
{
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    asm volatile("" ::: "memory");
#endif
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// round to nearest, ties to even; finite inputs (NaN maps to a quiet NaN)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// two floats to a packed pair of bf16 (low half = a), round to nearest even, by the hardware
// conversion of gfx950 (v_cvt_pk_bf16_f32)
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b)
{
#if defined(__HIP_DEVICE_COMPILE__)
    f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
#else
    return 0;
#endif
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

// 1 / v by the hardware reciprocal (1 ulp), in place of a correctly rounded division's ten instructions: the gate
// math of a recurrent cell is five of these per hidden unit
__device__ __forceinline__ float rcp_(float v)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_rcpf(v);
#else
    return 1.0f / v;
#endif
}

__device__ __forceinline__ float sigmoidf_(float x) { return rcp_(1.0f + __expf(-x)); }

// tanh through one exponential; exact limits for large |x|, odd symmetry kept
__device__ __forceinline__ float tanhf_(float x)
{
    float ax = fabsf(x);
    float e = __expf(-2.0f * ax);
    float t = (1.0f - e) * rcp_(1.0f + e);
    // for tiny |x| the quotient loses relative accuracy; tanh x = x - x^3/3 + ...
    if (ax < 0.02f) t = ax * (1.0f - ax * ax * (1.0f / 3.0f));
    return copysignf(t, x);
}

// operand-free steps
__device__ __forceinline__ float unary_step(int op, float v)
{
    switch (op) {
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

// Table lookups with compile-time indices only: the tables live in the kernel-argument segment,
// and a run-time index would turn every lookup into a dependent memory load.
__device__ __forceinline__ int epi_op(const Epilogue &e, int s)
{
    uint32_t w = e.opw[0];
#pragma unroll
    for (int i = 1; i < RL_EPI_MAX_OPS / 4; ++i) w = (i == (s >> 2)) ? e.opw[i] : w;
    return (int)((w >> (8 * (s & 3))) & 0xffu);
}
__device__ __forceinline__ int epi_arg(const Epilogue &e, int s)
{
    uint32_t w = e.argw[0];
#pragma unroll
    for (int i = 1; i < RL_EPI_MAX_OPS / 4; ++i) w = (i == (s >> 2)) ? e.argw[i] : w;
    return (int)((w >> (8 * (s & 3))) & 0xffu);
}
__device__ __forceinline__ const void *epi_ptr(const Epilogue &e, int a)
{
    const void *r = e.ptr[0];
#pragma unroll
    for (int i = 1; i < RL_EPI_MAX_PTRS; ++i) r = (i == a) ? e.ptr[i] : r;
    return r;
}
__device__ __forceinline__ int epi_ptr_dtype(const Epilogue &e, int a) { return (int)((e.dtw >> (4 * a)) & 0xfu); }

// One step of the epilogue chain on one element.
//   idx : flat offset of the element in the group's output tensor (operands
//         of the group's shape share its layout)
//   ch  : channel index for E_BIAS
__device__ __forceinline__ float epi_step(const Epilogue &e, int s, float v, int64_t idx, int ch)
{
    const int a = epi_arg(e, s);
    const int op = epi_op(e, s);
    if (op <= E_RDIV) {
        const void *ptr = epi_ptr(e, a);
        const int dt = epi_ptr_dtype(e, a);
        const float o = load_as_f32(ptr, dt, op == E_BIAS ? (int64_t)ch : idx);
        switch (op) {
        case E_BIAS: case E_ADD: return v + o;
        case E_SUB: return v - o;
        case E_RSUB: return o - v;
        case E_MUL: return v * o;
        case E_DIV: return v / o;
        default: return o / v;   // E_RDIV
        }
    }
    return unary_step(op, v);
}


// ---- 8-element vector forms (one 16-byte access for bf16, two for f32) -----
__device__ __forceinline__ void load8(const void *p, int dtype, int64_t i, float v[8])
{
    if (dtype == DT_BF16) {
        u32x4 r = *(const u32x4 *)((const uint16_t *)p + i);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v[2 * k] = __uint_as_float(r[k] << 16);
            v[2 * k + 1] = __uint_as_float(r[k] & 0xffff0000u);
        }
    } else {
        f32x4 a = *(const f32x4 *)((const float *)p + i);
        f32x4 b = *(const f32x4 *)((const float *)p + i + 4);
#pragma unroll
        for (int k = 0; k < 4; ++k) { v[k] = a[k]; v[4 + k] = b[k]; }
    }
}

__device__ __forceinline__ void store8(void *p, int dtype, int64_t i, const float v[8])
{
    if (dtype == DT_BF16) {
        u32x4 r;
#pragma unroll
        for (int k = 0; k < 4; ++k) r[k] = pack_bf16x2(v[2 * k], v[2 * k + 1]);
        *(u32x4 *)((uint16_t *)p + i) = r;
    } else {
        f32x4 a, b;
#pragma unroll
        for (int k = 0; k < 4; ++k) { a[k] = v[k]; b[k] = v[4 + k]; }
        *(f32x4 *)((float *)p + i) = a;
        *(f32x4 *)((float *)p + i + 4) = b;
    }
}

// Streaming forms (nontemporal: the data is not expected to be re-read from cache soon), for tensors
// far larger than the caches.
__device__ __forceinline__ void load8_nt(const void *p, int dtype, int64_t i, float v[8])
{
    if (dtype == DT_BF16) {
        u32x4 r = __builtin_nontemporal_load((const u32x4 *)((const uint16_t *)p + i));
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v[2 * k] = __uint_as_float(r[k] << 16);
            v[2 * k + 1] = __uint_as_float(r[k] & 0xffff0000u);
        }
    } else {
        f32x4 a = __builtin_nontemporal_load((const f32x4 *)((const float *)p + i));
        f32x4 b = __builtin_nontemporal_load((const f32x4 *)((const float *)p + i + 4));
#pragma unroll
        for (int k = 0; k < 4; ++k) { v[k] = a[k]; v[4 + k] = b[k]; }
    }
}

__device__ __forceinline__ void store8_nt(void *p, int dtype, int64_t i, const float v[8])
{
    if (dtype == DT_BF16) {
        u32x4 r;
#pragma unroll
        for (int k = 0; k < 4; ++k) r[k] = pack_bf16x2(v[2 * k], v[2 * k + 1]);
        __builtin_nontemporal_store(r, (u32x4 *)((uint16_t *)p + i));
    } else {
        f32x4 a, b;
#pragma unroll
        for (int k = 0; k < 4; ++k) { a[k] = v[k]; b[k] = v[4 + k]; }
        __builtin_nontemporal_store(a, (f32x4 *)((float *)p + i));
        __builtin_nontemporal_store(b, (f32x4 *)((float *)p + i + 4));
    }
}

__device__ __forceinline__ float binop(int op, float v, float t)
{
    switch (op) {
    case E_ADD: return v + t;
    case E_SUB: return v - t;
    case E_RSUB: return t - v;
    case E_MUL: return v * t;
    case E_DIV: return v / t;
    default: return t / v;   // E_RDIV
    }
}


// The whole chain on 8 consecutive elements.
//   idx0  : flat offset of the first element in the output tensor (full-shape
//           operands share the output's layout)
//   ci0   : flat index used to derive channels: channel of element k is
//           ((ci0 + k) / ch_inner) % ch_count
//   ch_hint: >= 0 when the caller already knows the one channel all 8 elements share (8 | ch_inner)
//   nt    : full-shape operands are read with streaming loads
__device__ __forceinline__ void chain8(const Epilogue &e, float v[8], int64_t idx0, int64_t ci0, int64_t ch_inner, int ch_count,
                                       int ch_hint = -1, bool nt = false)
{
    for (int s = 0; s < e.n_ops; ++s) {
        const int op = epi_op(e, s), a = epi_arg(e, s);
        const void *optr = epi_ptr(e, a);
        const int odt = epi_ptr_dtype(e, a);
        if (op == E_BIAS) {
            if (ch_inner == 1 && (ch_count & 7) == 0) {
                int ch = (int)(ci0 % ch_count);
                float b[8];
                load8(optr, odt, ch, b);
#pragma unroll
                for (int k = 0; k < 8; ++k) v[k] += b[k];
            } else if ((ch_inner & 7) == 0) {
                int ch = ch_hint >= 0 ? ch_hint : (int)((ci0 / ch_inner) % ch_count);
                float b = load_as_f32(optr, odt, ch);
#pragma unroll
                for (int k = 0; k < 8; ++k) v[k] += b;
            } else {
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    int ch = (int)(((ci0 + k) / ch_inner) % ch_count);
                    v[k] += load_as_f32(optr, odt, ch);
                }
            }
        } else if (op >= E_ADD && op <= E_RDIV) {
            float tt[8];
            if (nt) load8_nt(optr, odt, idx0, tt);
            else load8(optr, odt, idx0, tt);
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = binop(op, v[k], tt[k]);
        } else if (op == E_RELU) {
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = v[k] > 0.0f ? v[k] : 0.0f;
        } else {
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = unary_step(op, v[k]);
        }
    }
}

}  // namespace rl

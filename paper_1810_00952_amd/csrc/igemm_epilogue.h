// Epilogue of the contraction kernels: 32 rows of fp32 accumulators staged in
// LDS (row stride LDC floats) are turned into output rows, 8 consecutive
// channels per thread, with the group's injective chain applied in between.
//
// A thread keeps the same 8 channels for every row it touches, so a leading
// bias_add is loaded once, and the one full-shape operand most chains have
// (the residual) is fetched one 32-row pass ahead: global-load latency is paid
// once per tile instead of once per dependent step.  Chains of another form
// take the generic path (operands loaded where the chain needs them).
#pragma once
#include "device_utils.h"

namespace rl {

// The chain's form is classified on the host (Epilogue::simple, has_bias, t_op, rest_ops and the
// resolved bias_ptr / t_ptr), so the kernels read fixed kernel-argument fields here.
// One thread's operand vectors for one 32-row pass (raw 16 or 32 bytes each).
template <int NV> struct OperandRegs { u32x4 lo[NV], hi[NV]; };

template <int BN>
struct TileEpilogue {
    static constexpr int VPR = BN / 8;            // 8-channel vectors per row
    static constexpr int SWEEP = 256 / VPR;       // rows covered by the 256 threads at once
    static constexpr int NV = 32 / SWEEP;         // vectors per thread per 32-row pass

    // issue the loads of the full-shape operand for the rows of one pass
    static __device__ __forceinline__ void prefetch(const IgemmParams &p, int t, int mq, int n0,
                                                    OperandRegs<NV> &r)
    {
        const int cv = t % VPR, r0 = t / VPR;
        const int n = n0 + cv * 8;
        const void *ptr = p.epi.t_ptr;
        const bool f32 = p.epi.t_dtype == DT_F32;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int m = mq + r0 + SWEEP * i;
            r.lo[i] = u32x4{0u, 0u, 0u, 0u};
            r.hi[i] = u32x4{0u, 0u, 0u, 0u};
            if (p.epi.t_op >= 0 && m < p.M && n < p.N) {
                const int64_t off = (int64_t)m * p.ys_p + n;
                if (f32) {
                    r.lo[i] = *(const u32x4 *)((const float *)ptr + off);
                    r.hi[i] = *(const u32x4 *)((const float *)ptr + off + 4);
                } else {
                    r.lo[i] = *(const u32x4 *)((const uint16_t *)ptr + off);
                }
            }
        }
    }

    static __device__ __forceinline__ void load_bias(const IgemmParams &p, int t, int n0, float b[8])
    {
        const int n = n0 + (t % VPR) * 8;
#pragma unroll
        for (int k = 0; k < 8; ++k) b[k] = 0.0f;
        if (p.epi.has_bias && n < p.N) load8(p.epi.bias_ptr, p.epi.bias_dtype, n, b);
    }

    // rows mq .. mq+31 from sC; output row-major with 8 | N (checked by the caller)
    static __device__ __forceinline__ void store_pass(const IgemmParams &p, const float *sC, int ldc, int t,
                                                      int mq, int n0, const float bias[8], const OperandRegs<NV> &r)
    {
        const Epilogue &e = p.epi;
        const int cv = t % VPR, r0 = t / VPR;
        const int n = n0 + cv * 8;
        const bool f32 = e.t_op >= 0 && e.t_dtype == DT_F32;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int row = r0 + SWEEP * i;
            const int m = mq + row;
            if (m < p.M && n < p.N) {
                float val[8];
                f32x4 lo = *(const f32x4 *)(sC + row * ldc + cv * 8);
                f32x4 hi = *(const f32x4 *)(sC + row * ldc + cv * 8 + 4);
#pragma unroll
                for (int k = 0; k < 4; ++k) { val[k] = lo[k]; val[4 + k] = hi[k]; }
                const int64_t off = (int64_t)m * p.ys_p + n;
                if (e.simple) {
#pragma unroll
                    for (int k = 0; k < 8; ++k) val[k] += bias[k];
                    if (e.t_op >= 0) {
                        float tt[8];
                        if (f32) {
#pragma unroll
                            for (int k = 0; k < 4; ++k) { tt[k] = __uint_as_float(r.lo[i][k]); tt[4 + k] = __uint_as_float(r.hi[i][k]); }
                        } else {
#pragma unroll
                            for (int k = 0; k < 4; ++k) {
                                tt[2 * k] = __uint_as_float(r.lo[i][k] << 16);
                                tt[2 * k + 1] = __uint_as_float(r.lo[i][k] & 0xffff0000u);
                            }
                        }
#pragma unroll
                        for (int k = 0; k < 8; ++k) val[k] = binop(e.t_op, val[k], tt[k]);
                    }
                    uint64_t codes = e.rest_ops;
                    for (int s = 0; s < e.rest_n; ++s, codes >>= 8) {
                        const int op = (int)(codes & 0xff);
                        if (op == E_RELU) {
#pragma unroll
                            for (int k = 0; k < 8; ++k) val[k] = val[k] > 0.0f ? val[k] : 0.0f;
                        } else {
#pragma unroll
                            for (int k = 0; k < 8; ++k) val[k] = unary_step(op, val[k]);
                        }
                    }
                } else {
                    chain8(e, val, off, n, 1, p.N);
                }
                store8(p.y, p.y_dtype, off, val);
            }
        }
    }

    // any output strides / ragged N: one element at a time, consecutive threads on consecutive rows
    static __device__ __forceinline__ void store_pass_scalar(const IgemmParams &p, const float *sC, int ldc, int t, int mq, int n0)
    {
        const Epilogue &e = p.epi;
        for (int idx = t; idx < 32 * BN; idx += 256) {
            int col = idx / 32, row = idx - col * 32;
            int m = mq + row, n = n0 + col;
            if (m < p.M && n < p.N) {
                int img = m / p.OHW;
                int pix = m - img * p.OHW;
                int64_t off = (int64_t)img * p.ys_n + (int64_t)pix * p.ys_p + (int64_t)n * p.ys_c;
                float val = sC[row * ldc + col];
                for (int s = 0; s < e.n_ops; ++s) val = epi_step(e, s, val, off, n);
                store_from_f32(p.y, p.y_dtype, off, val);
            }
        }
    }

    // LSTM gate math: packed column g*(BN/4)+u of the tile holds gate g of hidden unit bn*(BN/4)+u
    static __device__ __forceinline__ void gates_pass(const IgemmParams &p, const float *sC, int ldc, int t, int mq, int bn)
    {
        const Epilogue &e = p.epi;
        constexpr int U = BN / 4;
        for (int idx = t; idx < 32 * U; idx += 256) {
            int row = idx / U, u = idx - row * U;
            int m = mq + row, unit = bn * U + u;
            if (m < p.M && unit < p.hidden) {
                float z[4];
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    z[g] = sC[row * ldc + g * U + u];
                    for (int s = 0; s < e.n_ops; ++s)      // only E_BIAS steps reach a gate epilogue
                        z[g] += load_as_f32(epi_ptr(e, epi_arg(e, s)), epi_ptr_dtype(e, epi_arg(e, s)), g * p.hidden + unit);
                }
                float c_old = p.c_in[(int64_t)m * p.hidden + unit];
                float cn = sigmoidf_(z[1]) * c_old + sigmoidf_(z[0]) * tanhf_(z[2]);
                float hn = sigmoidf_(z[3]) * tanhf_(cn);
                p.c_out[(int64_t)m * p.hidden + unit] = cn;
                store_from_f32(p.h_out, p.h_dtype, (int64_t)m * p.hidden + unit, hn);
            }
        }
    }
};

}  // namespace rl

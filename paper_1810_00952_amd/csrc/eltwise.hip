// HBM-bound kernels for gfx950: the single-pass fused elementwise group, the
// stand-alone LSTM gate group, window reductions, layout change, weight
// packing and batch-norm folding.  All move 16-byte vectors per lane where the
// tensor's geometry allows and touch every input and output exactly once.
#include <algorithm>

#include "device_utils.h"

namespace rl {

// ---------------------------------------------------------------------------
// fused elementwise chain: y = chain(x, operands...), one 8-element vector per
// thread (one 16-byte access per bf16 tensor, two per f32 tensor), one pass, no
// grid-stride loop: many short-lived workgroups with streaming accesses get
// closest to the HBM rate on this part (four vectors per thread measured slower).
// When a per-channel operand is constant over runs of >= 8 elements (e.g. NCHW
// planes), a vector's channel comes from a multiply-high division by the run length.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void eltwise_kernel(const EltwiseParams p)
{
    const Epilogue &e = p.epi;
    const int64_t vi = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const bool nt = p.nt != 0;
    constexpr int UU = 4;
    if (p.v2 == UU) {
        // the common form on large 2-byte tensors: four vectors per thread, 256 vectors apart (every load instruction
        // still covers 64 consecutive vectors), all loads requested before anything is computed
        const int64_t va = (int64_t)blockIdx.x * (256 * UU) + threadIdx.x;
        float v[UU][8], tt[UU][8];
        float b[UU];
        bool live[UU];
#pragma unroll
        for (int u = 0; u < UU; ++u) {
            const int64_t vv = va + 256 * u;
            live[u] = vv < (p.n >> 3);
            const int64_t i0 = (live[u] ? vv : 0) << 3;
            if (nt) { load8_nt(p.x, p.x_dtype, i0, v[u]); load8_nt(e.t_ptr, e.t_dtype, i0, tt[u]); }
            else { load8(p.x, p.x_dtype, i0, v[u]); load8(e.t_ptr, e.t_dtype, i0, tt[u]); }
            b[u] = 0.0f;
            if (e.has_bias) {
                const uint32_t run = p.vec_per_run == 1 ? (uint32_t)vv : (__umulhi((uint32_t)vv, p.run_mul) >> p.run_sh);
                b[u] = load_as_f32(e.bias_ptr, e.bias_dtype, (int)(run % (uint32_t)p.ch_count));
            }
        }
#pragma unroll
        for (int u = 0; u < UU; ++u) {
#pragma unroll
            for (int k = 0; k < 8; ++k) v[u][k] = binop(e.t_op, v[u][k] + b[u], tt[u][k]);
            uint64_t codes = e.rest_ops;
            for (int st = 0; st < e.rest_n; ++st, codes >>= 8) {
                const int op = (int)(codes & 0xff);
                if (op == E_RELU) {
#pragma unroll
                    for (int k = 0; k < 8; ++k) v[u][k] = v[u][k] > 0.0f ? v[u][k] : 0.0f;
                } else {
#pragma unroll
                    for (int k = 0; k < 8; ++k) v[u][k] = unary_step(op, v[u][k]);
                }
            }
            if (live[u]) {
                const int64_t i0 = (va + 256 * u) << 3;
                if (nt) store8_nt(p.y, p.y_dtype, i0, v[u]);
                else store8(p.y, p.y_dtype, i0, v[u]);
            }
        }
        return;
    }
    if (vi < (p.n >> 3)) {
        const int64_t i0 = vi << 3;
        int ch_hint = -1;
        if (p.runs > 0) {
            const uint32_t run = p.vec_per_run == 1 ? (uint32_t)vi : (__umulhi((uint32_t)vi, p.run_mul) >> p.run_sh);
            ch_hint = (int)(run % (uint32_t)p.ch_count);
        }
        float v[8];
        if (e.simple && e.t_op >= 0 && (p.runs > 0) == (e.has_bias != 0)) {
            // the common form [per-run bias] one full-shape operand, operand-free steps: both tensors are
            // requested before anything is computed
            float tt[8];
            if (nt) { load8_nt(p.x, p.x_dtype, i0, v); load8_nt(e.t_ptr, e.t_dtype, i0, tt); }
            else { load8(p.x, p.x_dtype, i0, v); load8(e.t_ptr, e.t_dtype, i0, tt); }
            const float b = e.has_bias ? load_as_f32(e.bias_ptr, e.bias_dtype, ch_hint) : 0.0f;
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = binop(e.t_op, v[k] + b, tt[k]);
            uint64_t codes = e.rest_ops;
            for (int st = 0; st < e.rest_n; ++st, codes >>= 8) {
                const int op = (int)(codes & 0xff);
                if (op == E_RELU) {
#pragma unroll
                    for (int k = 0; k < 8; ++k) v[k] = v[k] > 0.0f ? v[k] : 0.0f;
                } else {
#pragma unroll
                    for (int k = 0; k < 8; ++k) v[k] = unary_step(op, v[k]);
                }
            }
        } else {
            if (nt) load8_nt(p.x, p.x_dtype, i0, v);
            else load8(p.x, p.x_dtype, i0, v);
            chain8(e, v, i0, i0, p.ch_inner, p.ch_count, ch_hint, nt);
        }
        if (nt) store8_nt(p.y, p.y_dtype, i0, v);
        else store8(p.y, p.y_dtype, i0, v);
    }
    // ragged tail (< 8 elements), one thread each, first workgroup
    if (blockIdx.x == 0) {
        const int64_t ti = ((p.n >> 3) << 3) + threadIdx.x;
        if (threadIdx.x < 8 && ti < p.n) {
            float v = load_as_f32(p.x, p.x_dtype, ti);
            int ch = (int)((ti / p.ch_inner) % p.ch_count);
            for (int s = 0; s < e.n_ops; ++s) v = epi_step(e, s, v, ti, ch);
            store_from_f32(p.y, p.y_dtype, ti, v);
        }
    }
}

hipError_t launch_eltwise(const EltwiseParams &p0, hipStream_t s)
{
    EltwiseParams p = p0;
    const int64_t nvec = p.n >> 3;
    // per-channel runs: 8 | ch_inner, so a vector never straddles a channel and the tensor has no ragged tail
    p.runs = 0; p.vec_per_run = 0; p.run_mul = 0; p.run_sh = 0;
    if (p.ch_count > 1 && p.ch_inner >= 8 && (p.ch_inner & 7) == 0 && p.n % p.ch_inner == 0 && nvec < ((int64_t)1 << 31) &&
        (p.ch_inner >> 3) < ((int64_t)1 << 31)) {
        p.vec_per_run = p.ch_inner >> 3;
        p.runs = 1;
        make_fast_div((uint32_t)p.vec_per_run, p.run_mul, p.run_sh);
    }
    // four vectors per thread: large 2-byte tensors in the common form without a ragged tail
    p.v2 = 0;
    {
        Epilogue e = p.epi;
        finalize_epilogue(e);
        const bool common = e.simple && e.t_op >= 0 && (p.runs > 0) == (e.has_bias != 0);
        // measured on 256x64x112x112: bf16 4.3-5.0 TB/s with one vector per thread, 5.4-5.7 with four; f32 is fastest
        // (5.6 TB/s) with its one 32-byte run per thread
        if (common && p.x_dtype == DT_BF16 && p.y_dtype == DT_BF16 && e.t_dtype == DT_BF16 && (p.n & 7) == 0 && p.n >= ((int64_t)32 << 20) &&
            nvec < ((int64_t)1 << 31))
            p.v2 = 4;
    }
    const int64_t blocks = std::max<int64_t>(1, p.v2 ? (nvec + 256 * p.v2 - 1) / (256 * p.v2) : (nvec + 255) / 256);
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    p.nt = p.n >= ((int64_t)32 << 20);           // tens of MB per tensor: beyond what the caches would keep for a consumer
    hipLaunchKernelGGL(eltwise_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// stand-alone LSTM gate group: z[B, 4H] in (i | f | g | o) blocks
// ---------------------------------------------------------------------------
template <typename V> __device__ __forceinline__ V ld_maybe_nt(const V *p, bool nt) { return nt ? __builtin_nontemporal_load(p) : *p; }
template <typename V> __device__ __forceinline__ void st_maybe_nt(V *p, V v, bool nt) { if (nt) __builtin_nontemporal_store(v, p); else *p = v; }

// one thread per four hidden units (16-byte accesses), one pass
__global__ __launch_bounds__(256) void lstm_gates_kernel(const GatesParams p)
{
    const int64_t total = (int64_t)p.B * p.H;
    const bool nt = p.nt != 0;
    if ((p.H & 3) == 0) {
        const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
        if (q < (total >> 2)) {
            int64_t idx = q << 2;
            int b = (int)(idx / p.H), u = (int)(idx - (int64_t)b * p.H);
            const float *zr = p.z + (int64_t)b * 4 * p.H + u;
            f32x4 zi = ld_maybe_nt((const f32x4 *)zr, nt), zf = ld_maybe_nt((const f32x4 *)(zr + p.H), nt);
            f32x4 zg = ld_maybe_nt((const f32x4 *)(zr + 2 * p.H), nt), zo = ld_maybe_nt((const f32x4 *)(zr + 3 * p.H), nt);
            f32x4 c = ld_maybe_nt((const f32x4 *)(p.c_in + idx), nt), cn;
            float hn[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                cn[k] = sigmoidf_(zf[k]) * c[k] + sigmoidf_(zi[k]) * tanhf_(zg[k]);
                hn[k] = sigmoidf_(zo[k]) * tanhf_(cn[k]);
            }
            st_maybe_nt((f32x4 *)(p.c_out + idx), cn, nt);
            if (p.h_dtype == DT_BF16) {
                u32x2 r;
                r[0] = f32_to_bf16_bits(hn[0]) | (f32_to_bf16_bits(hn[1]) << 16);
                r[1] = f32_to_bf16_bits(hn[2]) | (f32_to_bf16_bits(hn[3]) << 16);
                st_maybe_nt((u32x2 *)((uint16_t *)p.h_out + idx), r, nt);
            } else {
                f32x4 hv = {hn[0], hn[1], hn[2], hn[3]};
                st_maybe_nt((f32x4 *)((float *)p.h_out + idx), hv, nt);
            }
        }
    } else {
        const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
        if (idx < total) {
            int b = (int)(idx / p.H), u = (int)(idx - (int64_t)b * p.H);
            const float *zr = p.z + (int64_t)b * 4 * p.H + u;
            float cn = sigmoidf_(zr[p.H]) * p.c_in[idx] + sigmoidf_(zr[0]) * tanhf_(zr[2 * p.H]);
            p.c_out[idx] = cn;
            store_from_f32(p.h_out, p.h_dtype, idx, sigmoidf_(zr[3 * p.H]) * tanhf_(cn));
        }
    }
}

hipError_t launch_lstm_gates(const GatesParams &p0, hipStream_t s)
{
    GatesParams p = p0;
    const int64_t total = (int64_t)p.B * p.H;
    const int64_t work = (p.H & 3) == 0 ? (total + 3) / 4 : total;
    const int64_t blocks = std::max<int64_t>(1, (work + 255) / 256);
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    p.nt = total >= ((int64_t)8 << 20);
    hipLaunchKernelGGL(lstm_gates_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// window reductions on channel-last tensors; VEC channels per thread
// ---------------------------------------------------------------------------
template <typename T, int VEC> struct VecIO;
template <> struct VecIO<uint16_t, 8> {
    static __device__ void load(const uint16_t *p, float v[8]) { load8(p, DT_BF16, 0, v); }
    static __device__ void store(uint16_t *p, const float v[8]) { store8(p, DT_BF16, 0, v); }
};
template <> struct VecIO<float, 4> {
    static __device__ void load(const float *p, float v[4]) { f32x4 a = *(const f32x4 *)p; for (int k = 0; k < 4; ++k) v[k] = a[k]; }
    static __device__ void store(float *p, const float v[4]) { f32x4 a = {v[0], v[1], v[2], v[3]}; *(f32x4 *)p = a; }
};
template <> struct VecIO<uint16_t, 1> {
    static __device__ void load(const uint16_t *p, float v[1]) { v[0] = bf16_bits_to_f32(*p); }
    static __device__ void store(uint16_t *p, const float v[1]) { *p = (uint16_t)f32_to_bf16_bits(v[0]); }
};
template <> struct VecIO<float, 1> {
    static __device__ void load(const float *p, float v[1]) { v[0] = *p; }
    static __device__ void store(float *p, const float v[1]) { *p = v[0]; }
};

template <typename T, int VEC>
__global__ __launch_bounds__(256) void maxpool_nhwc_kernel(const PoolParams p)
{
    const int cv = p.C / VEC;
    const int64_t total = (int64_t)p.N * p.OH * p.OW * cv;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const T *x = (const T *)p.x;
    T *y = (T *)p.y;
    // consecutive workgroup ids go to different XCDs: give each XCD a contiguous run of the output, so that windows
    // that share input rows share an L2
    int64_t bid = blockIdx.x;
    {
        const int64_t per = gridDim.x / 8, main = per * 8;
        if (bid < main) bid = (bid % 8) * per + bid / 8;
    }
    for (int64_t idx = bid * blockDim.x + threadIdx.x; idx < total; idx += stride) {
        int c = (int)(idx % cv) * VEC;
        int64_t q = idx / cv;
        int ow = (int)(q % p.OW); q /= p.OW;
        int oh = (int)(q % p.OH);
        int n = (int)(q / p.OH);
        float best[VEC];
#pragma unroll
        for (int k = 0; k < VEC; ++k) best[k] = -INFINITY;
        for (int a = 0; a < p.KH; ++a) {
            int ih = oh * p.sh - p.ph + a;
            if ((unsigned)ih >= (unsigned)p.H) continue;
            for (int b = 0; b < p.KW; ++b) {
                int iw = ow * p.sw - p.pw + b;
                if ((unsigned)iw >= (unsigned)p.W) continue;
                float v[VEC];
                VecIO<T, VEC>::load(x + (((int64_t)n * p.H + ih) * p.W + iw) * p.C + c, v);
#pragma unroll
                for (int k = 0; k < VEC; ++k) best[k] = v[k] > best[k] ? v[k] : best[k];
            }
        }
        VecIO<T, VEC>::store(y + (((int64_t)n * p.OH + oh) * p.OW + ow) * p.C + c, best);
    }
}

// One workgroup per (image, slab of SLAB channel vectors): the 256 threads split the pixels 256 / SLAB ways,
// each sums its share in fp32, and the partial sums meet in LDS (fixed order, so the result does not depend
// on timing).  SLAB = 16 (sixteen pixel groups) gives four times the workgroups and a quarter of the serial
// loads per thread of SLAB = 64: the kernel is one memory latency after another, not bandwidth.
template <typename T, int VEC, int SLAB>
__global__ __launch_bounds__(256) void gavgpool_nhwc_kernel(const PoolParams p)
{
    constexpr int PG = 256 / SLAB;
    __shared__ float part[PG][SLAB][VEC];
    const int cv = p.C / VEC;
    const int slabs = (cv + SLAB - 1) / SLAB;
    const int n = blockIdx.x / slabs, slab = blockIdx.x - n * slabs;
    const int u = threadIdx.x % SLAB, g = threadIdx.x / SLAB;
    const int v = slab * SLAB + u;
    const T *x = (const T *)p.x;
    T *y = (T *)p.y;
    const int HW = p.H * p.W;
    float acc[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) acc[k] = 0.0f;
    if (v < cv)
        for (int q = g; q < HW; q += PG) {
            float t[VEC];
            VecIO<T, VEC>::load(x + ((int64_t)n * HW + q) * p.C + v * VEC, t);
#pragma unroll
            for (int k = 0; k < VEC; ++k) acc[k] += t[k];
        }
#pragma unroll
    for (int k = 0; k < VEC; ++k) part[g][u][k] = acc[k];
    __syncthreads();
    if (g == 0 && v < cv) {
        const float inv = 1.0f / (float)HW;
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            float sum = part[0][u][k];
#pragma unroll
            for (int j = 1; j < PG; ++j) sum += part[j][u][k];
            acc[k] = sum * inv;
        }
        VecIO<T, VEC>::store(y + (int64_t)n * p.C + v * VEC, acc);
    }
}

template <template <typename, int> class K>
struct PoolDispatch;

static inline unsigned grid_for(int64_t total)
{
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    if (blocks < 1) blocks = 1;
    return (unsigned)blocks;
}

hipError_t launch_maxpool_nhwc(const PoolParams &p, hipStream_t s)
{
    if (p.dtype == DT_BF16) {
        if (p.C % 8 == 0) hipLaunchKernelGGL((maxpool_nhwc_kernel<uint16_t, 8>), dim3(grid_for((int64_t)p.N * p.OH * p.OW * (p.C / 8))), dim3(256), 0, s, p);
        else hipLaunchKernelGGL((maxpool_nhwc_kernel<uint16_t, 1>), dim3(grid_for((int64_t)p.N * p.OH * p.OW * p.C)), dim3(256), 0, s, p);
    } else {
        if (p.C % 4 == 0) hipLaunchKernelGGL((maxpool_nhwc_kernel<float, 4>), dim3(grid_for((int64_t)p.N * p.OH * p.OW * (p.C / 4))), dim3(256), 0, s, p);
        else hipLaunchKernelGGL((maxpool_nhwc_kernel<float, 1>), dim3(grid_for((int64_t)p.N * p.OH * p.OW * p.C)), dim3(256), 0, s, p);
    }
    return hipGetLastError();
}

template <typename T, int VEC>
static hipError_t launch_gavgpool_t(const PoolParams &p, hipStream_t s)
{
    const int cv = p.C / VEC;
    // few workgroups of 64-vector slabs leave most of the chip idle: narrower slabs, more pixel groups
    const bool narrow = (int64_t)p.N * ((cv + 63) / 64) < 256 && p.H * p.W >= 16;
    const int slab = narrow ? 16 : 64;
    const int64_t nb = (int64_t)p.N * ((cv + slab - 1) / slab);
    if (nb <= 0 || nb > 0x7fffffff) return hipErrorInvalidValue;
    if (narrow) hipLaunchKernelGGL((gavgpool_nhwc_kernel<T, VEC, 16>), dim3((unsigned)nb), dim3(256), 0, s, p);
    else hipLaunchKernelGGL((gavgpool_nhwc_kernel<T, VEC, 64>), dim3((unsigned)nb), dim3(256), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_gavgpool_nhwc(const PoolParams &p, hipStream_t s)
{
    const bool wide = p.dtype == DT_BF16 ? p.C % 8 == 0 : p.C % 4 == 0;
    if (p.dtype == DT_BF16) return wide ? launch_gavgpool_t<uint16_t, 8>(p, s) : launch_gavgpool_t<uint16_t, 1>(p, s);
    return wide ? launch_gavgpool_t<float, 4>(p, s) : launch_gavgpool_t<float, 1>(p, s);
}

// ---------------------------------------------------------------------------
// layout change through a 32 x 32 LDS tile: src[n][r][q] -> dst[n][q][r]
// (R rows of Q contiguous elements become Q rows of R contiguous elements)
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T *__restrict__ src, T *__restrict__ dst, int R, int Q)
{
    __shared__ T tile[32][33];
    const int n = blockIdx.z;
    const int q0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;     // 32 x 8
    const T *s = src + (int64_t)n * R * Q;
    T *d = dst + (int64_t)n * R * Q;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        int r = r0 + ty + 8 * k, q = q0 + tx;
        if (r < R && q < Q) tile[ty + 8 * k][tx] = s[(int64_t)r * Q + q];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        int q = q0 + ty + 8 * k, r = r0 + tx;
        if (r < R && q < Q) d[(int64_t)q * R + r] = tile[tx][ty + 8 * k];
    }
}

// The same for R and Q multiples of the 16-byte vector (8 bf16 / 4 f32) and 16-byte aligned tensors, without
// LDS: a lane reads a VEC x VEC block as VEC row vectors, transposes it in registers and writes VEC column
// vectors.  A wave covers 8 x 8 such blocks; eight lanes read 128 contiguous bytes of a row, and eight lanes
// write 128 contiguous bytes of a result row.
template <typename T>
__global__ __launch_bounds__(256) void transpose_vec_kernel(const T *__restrict__ src, T *__restrict__ dst, int R, int Q, int tiles_r, int tiles_q,
                                                            int64_t total_tiles)
{
    constexpr int VEC = 16 / (int)sizeof(T);
    constexpr int TS = 8 * VEC;                       // tile side
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lr = lane >> 3, lq = lane & 7;
    for (int64_t tile = (int64_t)blockIdx.x * 4 + wave; tile < total_tiles; tile += (int64_t)gridDim.x * 4) {
        const int tq = (int)(tile % tiles_q);
        const int64_t rest = tile / tiles_q;
        const int tr = (int)(rest % tiles_r);
        const int64_t n = rest / tiles_r;
        const int r0 = tr * TS + lr * VEC, q0 = tq * TS + lq * VEC;
        if (r0 >= R || q0 >= Q) continue;             // R and Q are multiples of VEC: a block is inside or outside
        const T *sp = src + (n * R + r0) * Q + q0;
        u32x4 in[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) in[i] = *(const u32x4 *)(sp + (int64_t)i * Q);
        T *dp = dst + (n * Q + q0) * R + r0;
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            u32x4 o;
            if (sizeof(T) == 4) {
#pragma unroll
                for (int k = 0; k < 4; ++k) o[k] = in[k < VEC ? k : 0][j & 3];
            } else {
                // element j of row i is half (j & 1) of dword j >> 1; result dword k holds rows 2k and 2k + 1
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const uint32_t a = in[(2 * k) % VEC][(j >> 1) & 3], b = in[(2 * k + 1) % VEC][(j >> 1) & 3];
                    o[k] = (j & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
                }
            }
            *(u32x4 *)(dp + (int64_t)j * R) = o;
        }
    }
}

static hipError_t launch_transpose(const void *src, void *dst, int dtype, int N, int R, int Q, hipStream_t s)
{
    const int vec = dtype == DT_BF16 ? 8 : 4;
    if (R % vec == 0 && Q % vec == 0 && (((uintptr_t)src | (uintptr_t)dst) & 15) == 0 && N > 0) {
        const int ts = 8 * vec;
        const int tiles_r = (R + ts - 1) / ts, tiles_q = (Q + ts - 1) / ts;
        const int64_t total = (int64_t)N * tiles_r * tiles_q;
        const unsigned grid = (unsigned)std::min<int64_t>((total + 3) / 4, 256 * 64);
        if (dtype == DT_BF16) hipLaunchKernelGGL(transpose_vec_kernel<uint16_t>, dim3(grid), dim3(256), 0, s, (const uint16_t *)src, (uint16_t *)dst, R, Q, tiles_r, tiles_q, total);
        else hipLaunchKernelGGL(transpose_vec_kernel<float>, dim3(grid), dim3(256), 0, s, (const float *)src, (float *)dst, R, Q, tiles_r, tiles_q, total);
        return hipGetLastError();
    }
    dim3 grid((Q + 31) / 32, (R + 31) / 32, N);
    if (grid.y > 65535 || grid.z > 65535) return hipErrorInvalidValue;
    if (dtype == DT_BF16) hipLaunchKernelGGL(transpose_kernel<uint16_t>, grid, dim3(256), 0, s, (const uint16_t *)src, (uint16_t *)dst, R, Q);
    else hipLaunchKernelGGL(transpose_kernel<float>, grid, dim3(256), 0, s, (const float *)src, (float *)dst, R, Q);
    return hipGetLastError();
}

// general permutation: one element per thread, result-major (the writes coalesce, the reads gather)
template <typename T>
__global__ __launch_bounds__(256) void permute_kernel(const PermuteParams p)
{
    const T *x = (const T *)p.x;
    T *y = (T *)p.y;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < p.n; idx += (int64_t)gridDim.x * blockDim.x) {
        int64_t rem = idx, off = 0;
#pragma unroll
        for (int k = 5; k >= 0; --k)
            if (k < p.rank) {
                const int64_t q = rem / p.ydims[k];
                off += (rem - q * p.ydims[k]) * p.xstride[k];
                rem = q;
            }
        y[idx] = x[off];
    }
}

hipError_t launch_permute(const PermuteParams &p, hipStream_t s)
{
    if (p.rank < 0 || p.rank > 6 || p.n < 0) return hipErrorInvalidValue;
    if (p.n == 0) return hipSuccess;
    if (p.dtype == DT_BF16) hipLaunchKernelGGL(permute_kernel<uint16_t>, dim3(grid_for(p.n)), dim3(256), 0, s, p);
    else hipLaunchKernelGGL(permute_kernel<float>, dim3(grid_for(p.n)), dim3(256), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_nchw_to_nhwc(const void *src, void *dst, int32_t dtype, int32_t N, int32_t C, int32_t P, hipStream_t s)
{
    return launch_transpose(src, dst, dtype, N, C, P, s);
}

hipError_t launch_nhwc_to_nchw(const void *src, void *dst, int32_t dtype, int32_t N, int32_t C, int32_t P, hipStream_t s)
{
    return launch_transpose(src, dst, dtype, N, P, C, s);
}

// ---------------------------------------------------------------------------
// weight packing: src[O][C][T] -> dst[O'][T][C] with rows padded to Kp and
// optionally permuted (gate interleave)
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void pack_weight_kernel(const T *__restrict__ src, T *__restrict__ dst, int O, int C, int Tt,
                                                          int Kp, int perm_block)
{
    const int64_t total = (int64_t)O * Kp;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * blockDim.x) {
        int k = (int)(idx % Kp);
        int j = (int)(idx / Kp);
        int o = j;
        if (perm_block > 0) {
            int U = perm_block / 4;
            int blk = j / perm_block, r = j - blk * perm_block;
            int gate = r / U, u = r - gate * U;
            o = gate * (O / 4) + blk * U + u;
        }
        T v = 0;
        if (k < C * Tt) {
            int tap = k / C, c = k - tap * C;
            v = src[((int64_t)o * C + c) * Tt + tap];
        }
        dst[idx] = v;
    }
}

// second copy of a 64 x (9 x 64) bf16 weight in the fragment order of the kernel that keeps it in registers
__global__ __launch_bounds__(256) void pack_weight_frag64_kernel(const uint16_t *__restrict__ src, uint16_t *__restrict__ dst)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;             // 64 * 576 elements, grid 144
    const int e = idx & 7, lane = (idx >> 3) & 63, ks = (idx >> 9) & 3, ht = idx >> 11;
    const int h = ht / 9, tap = ht - 9 * h;
    const int o = 32 * h + (lane & 31), c = 16 * ks + 8 * (lane >> 5) + e;
    dst[idx] = src[(o * 64 + c) * 9 + tap];
}

hipError_t launch_pack_weight(const void *src, void *dst, int32_t dtype, int32_t O, int32_t C, int32_t T, int32_t Kp,
                              int32_t perm_block, hipStream_t s)
{
    if (perm_block == -1) {
        if (dtype != DT_BF16 || O != 64 || C != 64 || T != 9 || Kp != 576) return hipErrorInvalidValue;
        hipLaunchKernelGGL(pack_weight_kernel<uint16_t>, dim3(grid_for((int64_t)O * Kp)), dim3(256), 0, s, (const uint16_t *)src, (uint16_t *)dst, O, C, T, Kp, 0);
        hipLaunchKernelGGL(pack_weight_frag64_kernel, dim3(64 * 576 / 256), dim3(256), 0, s, (const uint16_t *)src, (uint16_t *)dst + 64 * 576);
        return hipGetLastError();
    }
    unsigned grid = grid_for((int64_t)O * Kp);
    if (dtype == DT_BF16) hipLaunchKernelGGL(pack_weight_kernel<uint16_t>, dim3(grid), dim3(256), 0, s, (const uint16_t *)src, (uint16_t *)dst, O, C, T, Kp, perm_block);
    else hipLaunchKernelGGL(pack_weight_kernel<float>, dim3(grid), dim3(256), 0, s, (const float *)src, (float *)dst, O, C, T, Kp, perm_block);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// stem convolutions: zero-padded 4-channel channel-last frame and matching weights (bf16)
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void stem_pad_kernel(const uint16_t *__restrict__ src, uint16_t *__restrict__ dst, int N, int C, int H,
                                                       int W, int Hp, int Wp, int ph, int pw)
{
    const int64_t total = (int64_t)N * Hp * Wp;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * blockDim.x) {
        const int wp = (int)(idx % Wp);
        const int64_t q = idx / Wp;
        const int hp = (int)(q % Hp);
        const int n = (int)(q / Hp);
        const int h = hp - ph, w = wp - pw;
        uint32_t v[4] = {0u, 0u, 0u, 0u};
        if ((unsigned)h < (unsigned)H && (unsigned)w < (unsigned)W) {
            const uint16_t *sp = src + (((int64_t)n * C) * H + h) * W + w;
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (c < C) v[c] = sp[(int64_t)c * H * W];
        }
        u32x2 o = {v[0] | (v[1] << 16), v[2] | (v[3] << 16)};
        *(u32x2 *)(dst + idx * 4) = o;
    }
}

hipError_t launch_stem_pad(const void *src, void *dst, int32_t N, int32_t C, int32_t H, int32_t W, int32_t Hp, int32_t Wp,
                           int32_t ph, int32_t pw, hipStream_t s)
{
    if (C < 1 || C > 4) return hipErrorInvalidValue;
    hipLaunchKernelGGL(stem_pad_kernel, dim3(grid_for((int64_t)N * Hp * Wp)), dim3(256), 0, s, (const uint16_t *)src, (uint16_t *)dst, N, C,
                       H, W, Hp, Wp, ph, pw);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void pack_weight_stem_kernel(const uint16_t *__restrict__ src, uint16_t *__restrict__ dst, int O, int C,
                                                               int KH, int KW, int Kp)
{
    const int64_t total = (int64_t)O * Kp;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * blockDim.x) {
        const int k = (int)(idx % Kp), o = (int)(idx / Kp);
        const int c = k & 3, px = (k >> 2) & 7, kh = k >> 5;      // kh = 2t + seg
        uint16_t v = 0;
        if (c < C && px < KW && kh < KH) v = src[(((int64_t)o * C + c) * KH + kh) * KW + px];
        dst[idx] = v;
    }
}

hipError_t launch_pack_weight_stem(const void *src, void *dst, int32_t O, int32_t C, int32_t KH, int32_t KW, int32_t Kp, hipStream_t s)
{
    hipLaunchKernelGGL(pack_weight_stem_kernel, dim3(grid_for((int64_t)O * Kp)), dim3(256), 0, s, (const uint16_t *)src, (uint16_t *)dst,
                       O, C, KH, KW, Kp);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// batch-norm folding, float64 arithmetic
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void fold_bn_kernel(const float *__restrict__ w, const float *__restrict__ gamma,
                                                      const float *__restrict__ beta, const float *__restrict__ mean,
                                                      const float *__restrict__ var, double eps, void *w_out, int out_dtype,
                                                      float *b_out, int64_t O, int64_t per_o)
{
    const int64_t total = O * per_o;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * blockDim.x) {
        int64_t o = idx / per_o;
        double scale = (double)gamma[o] / sqrt((double)var[o] + eps);
        float r = (float)((double)w[idx] * scale);
        store_from_f32(w_out, out_dtype, idx, r);
        if (idx == o * per_o) b_out[o] = (float)((double)beta[o] - (double)mean[o] * scale);
    }
}

hipError_t launch_fold_bn(const float *w, const float *gamma, const float *beta, const float *mean, const float *var,
                          double eps, void *w_out, int32_t out_dtype, float *b_out, int64_t O, int64_t per_o, hipStream_t s)
{
    hipLaunchKernelGGL(fold_bn_kernel, dim3(grid_for(O * per_o)), dim3(256), 0, s, w, gamma, beta, mean, var, eps, w_out,
                       out_dtype, b_out, O, per_o);
    return hipGetLastError();
}

}  // namespace rl

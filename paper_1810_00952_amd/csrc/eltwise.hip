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
// closest to the HBM rate on this part.  This kernel interprets any chain; the
// forms a fused group mostly takes have kernels of their own further down.
// When a per-channel operand is constant over runs of >= 8 elements (e.g. NCHW
// planes), a vector's channel comes from a multiply-high division by the run length.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void eltwise_kernel(const EltwiseParams p)
{
    const Epilogue &e = p.epi;
    const int64_t vi = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const bool nt = p.nt != 0;
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

// ---------------------------------------------------------------------------
// The forms fused groups mostly take -- y = steps( x [+ bias[channel]] [+ t] ) with x, t, y of one base type, an f32
// bias that is constant over runs of whole vectors and operand-free steps behind (none, one ReLU, or any) -- compiled per form: no program to interpret, a dozen
// registers per lane, so that a SIMD holds enough waves to cover the HBM latency.  One 16-byte vector of each
// tensor per thread (f32: two), streaming accesses for tensors the caches would not keep anyway.
// ---------------------------------------------------------------------------
// REST: the operand-free steps behind them: 0 none, 1 one ReLU, 2 up to eight steps of any kind, their codes in rest_ops
template <typename T, bool BIAS, bool TADD, int REST, bool NT>
__global__ __launch_bounds__(256) void eltwise_form_kernel(const T *__restrict__ x, const T *__restrict__ t, T *__restrict__ y,
                                                           const float *__restrict__ bias, int64_t nunit, uint32_t unit_per_run,
                                                           uint32_t run_mul, uint32_t run_sh, uint32_t ch_count, int rest_n, uint64_t rest_ops, int t_op)
{
    // a unit: the 16 bytes a lane moves per tensor (8 bf16 / 4 f32); consecutive lanes, consecutive units
    const int64_t vi = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (vi >= nunit) return;
    const u32x4 *xp = (const u32x4 *)x + vi;
    const u32x4 *tp = (const u32x4 *)t + vi;
    const u32x4 a = NT ? __builtin_nontemporal_load(xp) : *xp;
    u32x4 b = {0u, 0u, 0u, 0u};
    if (TADD) b = NT ? __builtin_nontemporal_load(tp) : *tp;
    float bv = 0.0f;
    if (BIAS) {
        const uint32_t run = unit_per_run == 1 ? (uint32_t)vi : (__umulhi((uint32_t)vi, run_mul) >> run_sh);
        bv = bias[run % ch_count];
    }
    constexpr int NE = 16 / (int)sizeof(T);
    float v[NE];
    if (sizeof(T) == 2) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v[2 * k] = __uint_as_float(a[k] << 16) + bv;
            v[2 * k + 1] = __uint_as_float(a[k] & 0xffff0000u) + bv;
            if (TADD) {
                // the full-shape operand: an addition in the forms with at most a ReLU behind, any of the six steps otherwise
                if (REST != 2) { v[2 * k] += __uint_as_float(b[k] << 16); v[2 * k + 1] += __uint_as_float(b[k] & 0xffff0000u); }
                else { v[2 * k] = binop(t_op, v[2 * k], __uint_as_float(b[k] << 16)); v[2 * k + 1] = binop(t_op, v[2 * k + 1], __uint_as_float(b[k] & 0xffff0000u)); }
            }
        }
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v[k] = __uint_as_float(a[k]) + bv;
            if (TADD) v[k] = REST != 2 ? v[k] + __uint_as_float(b[k]) : binop(t_op, v[k], __uint_as_float(b[k]));
        }
    }
    if (REST == 1) {
#pragma unroll
        for (int k = 0; k < NE; ++k) v[k] = v[k] > 0.0f ? v[k] : 0.0f;
    } else if (REST == 2) {
        uint64_t codes = rest_ops;
        for (int st = 0; st < rest_n; ++st, codes >>= 8) {
            const int op = (int)(codes & 0xff);
#pragma unroll
            for (int k = 0; k < NE; ++k) v[k] = unary_step(op, v[k]);
        }
    }
    u32x4 o;
    if (sizeof(T) == 2) {
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = pack_bf16x2(v[2 * k], v[2 * k + 1]);
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = __float_as_uint(v[k]);
    }
    u32x4 *yp = (u32x4 *)y + vi;
    if (NT) __builtin_nontemporal_store(o, yp);
    else *yp = o;
}

struct FormLaunch { int64_t nunit; uint32_t unit_per_run, run_mul, run_sh, ch_count; unsigned blocks; bool nt; };

template <typename T, bool BIAS, bool TADD, int REST>
static void launch_form_nt(const FormLaunch &f, hipStream_t s, const EltwiseParams &p, const Epilogue &e)
{
    const T *x = (const T *)p.x, *t = (const T *)e.t_ptr;
    T *y = (T *)p.y;
    const float *bias = (const float *)e.bias_ptr;
    if (f.nt) hipLaunchKernelGGL((eltwise_form_kernel<T, BIAS, TADD, REST, true>), dim3(f.blocks), dim3(256), 0, s, x, t, y, bias, f.nunit, f.unit_per_run, f.run_mul, f.run_sh, f.ch_count, (int)e.rest_n, (uint64_t)e.rest_ops, (int)e.t_op);
    else hipLaunchKernelGGL((eltwise_form_kernel<T, BIAS, TADD, REST, false>), dim3(f.blocks), dim3(256), 0, s, x, t, y, bias, f.nunit, f.unit_per_run, f.run_mul, f.run_sh, f.ch_count, (int)e.rest_n, (uint64_t)e.rest_ops, (int)e.t_op);
}
template <typename T, int REST>
static void launch_form_rest(bool bias, bool tadd, const FormLaunch &fl, hipStream_t s, const EltwiseParams &p, const Epilogue &e)
{
    const int f = (bias ? 2 : 0) | (tadd ? 1 : 0);
    switch (f) {
    case 0: launch_form_nt<T, false, false, REST>(fl, s, p, e); break;
    case 1: launch_form_nt<T, false, true, REST>(fl, s, p, e); break;
    case 2: launch_form_nt<T, true, false, REST>(fl, s, p, e); break;
    default: launch_form_nt<T, true, true, REST>(fl, s, p, e); break;
    }
}
template <typename T>
static void launch_form(bool bias, bool tadd, int rest, const FormLaunch &fl, hipStream_t s, const EltwiseParams &p, const Epilogue &e)
{
    if (rest == 0) launch_form_rest<T, 0>(bias, tadd, fl, s, p, e);
    else if (rest == 1) launch_form_rest<T, 1>(bias, tadd, fl, s, p, e);
    else launch_form_rest<T, 2>(bias, tadd, fl, s, p, e);
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
    const int64_t blocks = std::max<int64_t>(1, (nvec + 255) / 256);
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    p.nt = p.n >= ((int64_t)32 << 20);           // tens of MB per tensor: beyond what the caches would keep for a consumer
    {
        // y = [relu](x [+ bias] [+ t]) on whole 16-byte units of one base type: the kernels compiled per form
        Epilogue e = p.epi;
        finalize_epilogue(e);
        const int per = p.x_dtype == DT_BF16 ? 8 : 4;                 // elements per 16 bytes
        FormLaunch f{};
        f.nunit = p.n / per; f.unit_per_run = 1; f.ch_count = 1; f.nt = p.nt != 0;
        bool bias_ok = !e.has_bias;
        if (e.has_bias && e.bias_dtype == DT_F32 && e.bias_ptr && p.ch_count >= 1 && p.ch_inner >= per && p.ch_inner % per == 0 && p.n % p.ch_inner == 0 &&
            p.ch_inner / per < ((int64_t)1 << 31)) {
            bias_ok = true;
            f.unit_per_run = (uint32_t)(p.ch_inner / per); f.ch_count = (uint32_t)p.ch_count;
            make_fast_div(f.unit_per_run, f.run_mul, f.run_sh);
        }
        const bool t_ok = e.t_op < 0 || (e.t_dtype == p.x_dtype && e.t_ptr);
        // an operand that is not added takes the form with generic steps (which applies the operand's own step too)
        const int rest = (e.t_op >= 0 && e.t_op != E_ADD) ? 2 : e.rest_n == 0 ? 0 : e.relu_last ? 1 : 2;
        const int64_t fblocks = (f.nunit + 255) / 256;
        if (e.simple && bias_ok && t_ok && p.x_dtype == p.y_dtype && p.n % per == 0 && f.nunit >= 1 && f.nunit < ((int64_t)1 << 31) &&
            (((uintptr_t)p.x | (uintptr_t)p.y | (uintptr_t)e.t_ptr) & 15) == 0) {
            f.blocks = (unsigned)fblocks;
            if (p.x_dtype == DT_BF16) launch_form<uint16_t>(e.has_bias, e.t_op >= 0, rest, f, s, p, e);
            else launch_form<float>(e.has_bias, e.t_op >= 0, rest, f, s, p, e);
            return hipGetLastError();
        }
    }
    // the interpreting kernel moves two vectors per f32 tensor and thread and is faster with plain accesses whatever the
    // size (f32, 1 GB: 182 us plain, 199 us streaming; bf16: no difference)
    p.nt = 0;
    hipLaunchKernelGGL(eltwise_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// stand-alone LSTM gate group: z[B, 4H] in (i | f | g | o) blocks
// ---------------------------------------------------------------------------
// streaming or plain access, chosen at compile time.  (With the choice as a run-time argument the two branches hold the
// same access twice, the optimiser merges them into one before inlining, and the merged access keeps no streaming hint.)
template <bool NT, typename V> __device__ __forceinline__ V ld_maybe_nt(const V *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT, typename V> __device__ __forceinline__ void st_maybe_nt(V *p, V v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// one thread per four hidden units (16-byte accesses), one pass.  NT: streaming loads for tensors beyond the last-level cache
// (measured at 16384 rows of 1024 hidden units: 78.5 us plain, 68.1 us with streaming loads, 69.4-69.9 us with streaming stores as well, so
// the stores stay plain)
template <bool NT>
__global__ __launch_bounds__(256) void lstm_gates_kernel(const GatesParams p)
{
    const int64_t total = (int64_t)p.B * p.H;
    constexpr bool NTS = false;
    if ((p.H & 3) == 0) {
        const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
        if (q < (total >> 2)) {
            int64_t idx = q << 2;
            int b = (int)(idx / p.H), u = (int)(idx - (int64_t)b * p.H);
            const float *zr = p.z + (int64_t)b * 4 * p.H + u;
            f32x4 zi = ld_maybe_nt<NT>((const f32x4 *)zr), zf = ld_maybe_nt<NT>((const f32x4 *)(zr + p.H));
            f32x4 zg = ld_maybe_nt<NT>((const f32x4 *)(zr + 2 * p.H)), zo = ld_maybe_nt<NT>((const f32x4 *)(zr + 3 * p.H));
            f32x4 c = ld_maybe_nt<NT>((const f32x4 *)(p.c_in + idx)), cn;
            float hn[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                cn[k] = sigmoidf_(zf[k]) * c[k] + sigmoidf_(zi[k]) * tanhf_(zg[k]);
                hn[k] = sigmoidf_(zo[k]) * tanhf_(cn[k]);
            }
            st_maybe_nt<NTS>((f32x4 *)(p.c_out + idx), cn);
            if (p.h_dtype == DT_BF16) {
                u32x2 r;
                r[0] = f32_to_bf16_bits(hn[0]) | (f32_to_bf16_bits(hn[1]) << 16);
                r[1] = f32_to_bf16_bits(hn[2]) | (f32_to_bf16_bits(hn[3]) << 16);
                st_maybe_nt<NTS>((u32x2 *)((uint16_t *)p.h_out + idx), r);
            } else {
                f32x4 hv = {hn[0], hn[1], hn[2], hn[3]};
                st_maybe_nt<NTS>((f32x4 *)((float *)p.h_out + idx), hv);
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
    if (p.nt) hipLaunchKernelGGL(lstm_gates_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, p);
    else hipLaunchKernelGGL(lstm_gates_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, p);
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

// The 3x3 window (the pools of the convolutional graphs here) on tensors of fewer than 2^31 vectors: one thread
// per (pixel, channel vector), its coordinates by multiply-high divisions, the nine loads requested together from
// clamped coordinates and the taps outside the image discarded afterwards.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void maxpool3x3_nhwc_kernel(const PoolParams p)
{
    const uint32_t cv = (uint32_t)(p.C / VEC);
    const uint32_t total = (uint32_t)p.N * p.OH * p.OW * cv;
    // consecutive workgroup ids go to different XCDs: give each XCD a contiguous run of the output
    uint32_t bid = blockIdx.x;
    {
        const uint32_t per = gridDim.x / 8, main = per * 8;
        if (bid < main) bid = (bid % 8) * per + bid / 8;
    }
    const uint32_t idx = bid * 256 + threadIdx.x;
    if (idx >= total) return;
    const uint32_t q1 = cv == 1 ? idx : (__umulhi(idx, p.cv_mul) >> p.cv_sh);
    const uint32_t c = (idx - q1 * cv) * VEC;
    const uint32_t q2 = p.OW == 1 ? q1 : (__umulhi(q1, p.ow_mul) >> p.ow_sh);
    const int ow = (int)(q1 - q2 * p.OW);
    const uint32_t n = p.OH == 1 ? q2 : (__umulhi(q2, p.oh_mul) >> p.oh_sh);
    const int oh = (int)(q2 - n * p.OH);
    const T *x = (const T *)p.x + (int64_t)n * p.H * p.W * p.C + c;
    float v[9][VEC];
    bool ok[9];
#pragma unroll
    for (int a = 0; a < 3; ++a)
#pragma unroll
        for (int b = 0; b < 3; ++b) {
            const int ih = oh * p.sh - p.ph + a, iw = ow * p.sw - p.pw + b;
            ok[3 * a + b] = (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
            const int ihc = ih < 0 ? 0 : (ih >= p.H ? p.H - 1 : ih), iwc = iw < 0 ? 0 : (iw >= p.W ? p.W - 1 : iw);
            VecIO<T, VEC>::load(x + ((int64_t)ihc * p.W + iwc) * p.C, v[3 * a + b]);
        }
    float best[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) best[k] = -INFINITY;
#pragma unroll
    for (int tp = 0; tp < 9; ++tp)
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            const float t = ok[tp] ? v[tp][k] : -INFINITY;
            best[k] = t > best[k] ? t : best[k];
        }
    VecIO<T, VEC>::store((T *)p.y + (((int64_t)n * p.OH + oh) * p.OW + ow) * p.C + c, best);
}

static inline unsigned grid_for(int64_t total)
{
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    if (blocks < 1) blocks = 1;
    return (unsigned)blocks;
}

hipError_t launch_maxpool_nhwc(const PoolParams &p0, hipStream_t s)
{
    PoolParams p = p0;
    const int vec = p.dtype == DT_BF16 ? 8 : 4;
    if (p.KH == 3 && p.KW == 3 && p.C % vec == 0 && (int64_t)p.N * p.OH * p.OW * (p.C / vec) < ((int64_t)1 << 31) &&
        (int64_t)p.N * p.H * p.W * p.C < ((int64_t)1 << 40)) {
        make_fast_div((uint32_t)(p.C / vec), p.cv_mul, p.cv_sh);
        make_fast_div((uint32_t)p.OW, p.ow_mul, p.ow_sh);
        make_fast_div((uint32_t)p.OH, p.oh_mul, p.oh_sh);
        const unsigned grid = (unsigned)(((int64_t)p.N * p.OH * p.OW * (p.C / vec) + 255) / 256);
        if (p.dtype == DT_BF16) hipLaunchKernelGGL((maxpool3x3_nhwc_kernel<uint16_t, 8>), dim3(grid), dim3(256), 0, s, p);
        else hipLaunchKernelGGL((maxpool3x3_nhwc_kernel<float, 4>), dim3(grid), dim3(256), 0, s, p);
        return hipGetLastError();
    }
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
template <typename T, bool NT>
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
        for (int i = 0; i < VEC; ++i) in[i] = NT ? __builtin_nontemporal_load((const u32x4 *)(sp + (int64_t)i * Q)) : *(const u32x4 *)(sp + (int64_t)i * Q);
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
            if (NT) __builtin_nontemporal_store(o, (u32x4 *)(dp + (int64_t)j * R));
            else *(u32x4 *)(dp + (int64_t)j * R) = o;
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
        // tensors larger than the last-level cache: streaming accesses (bf16 256x64x112x112: 140 us against 154)
        const bool nt = (int64_t)N * R * Q * (dtype == DT_BF16 ? 2 : 4) >= ((int64_t)1 << 28);
        if (dtype == DT_BF16 && nt) hipLaunchKernelGGL((transpose_vec_kernel<uint16_t, true>), dim3(grid), dim3(256), 0, s, (const uint16_t *)src, (uint16_t *)dst, R, Q, tiles_r, tiles_q, total);
        else if (dtype == DT_BF16) hipLaunchKernelGGL((transpose_vec_kernel<uint16_t, false>), dim3(grid), dim3(256), 0, s, (const uint16_t *)src, (uint16_t *)dst, R, Q, tiles_r, tiles_q, total);
        else if (nt) hipLaunchKernelGGL((transpose_vec_kernel<float, true>), dim3(grid), dim3(256), 0, s, (const float *)src, (float *)dst, R, Q, tiles_r, tiles_q, total);
        else hipLaunchKernelGGL((transpose_vec_kernel<float, false>), dim3(grid), dim3(256), 0, s, (const float *)src, (float *)dst, R, Q, tiles_r, tiles_q, total);
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

template <typename T>
__global__ __launch_bounds__(256) void pack_gather_kernel(const T *__restrict__ src, T *__restrict__ dst, const GatherPack g)
{
    const int64_t total = (int64_t)g.R * g.Kp;
    const int Kreal = g.T * g.Cq;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * blockDim.x) {
        const int k = (int)(idx % g.Kp);
        const int64_t r = idx / g.Kp;
        T v = 0;
        if (k < Kreal) {
            const int tap = k / g.Cq, c = k - tap * g.Cq;
            const int ti = tap / g.TW, tj = tap - ti * g.TW;
            v = src[g.base + r * g.s_row + (int64_t)c * g.s_c + (int64_t)ti * g.s_ti + (int64_t)tj * g.s_tj];
        }
        dst[idx] = v;
    }
}

hipError_t launch_pack_gather(const void *src, void *dst, const GatherPack &g, hipStream_t s)
{
    if (g.R < 1 || g.Kp < 1 || g.T < 1 || g.Cq < 1 || g.TW < 1 || g.T % g.TW != 0 || (int64_t)g.T * g.Cq > g.Kp) return hipErrorInvalidValue;
    const unsigned grid = grid_for((int64_t)g.R * g.Kp);
    if (g.dtype == DT_BF16) hipLaunchKernelGGL(pack_gather_kernel<uint16_t>, dim3(grid), dim3(256), 0, s, (const uint16_t *)src, (uint16_t *)dst, g);
    else hipLaunchKernelGGL(pack_gather_kernel<float>, dim3(grid), dim3(256), 0, s, (const float *)src, (float *)dst, g);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// A channel-last tensor spread out with zeros: dst[n][s i][s j][:] = src[n][i][j][:], everything else 0 (dst is Hd x Wd
// pixels, at least (OH-1) s + 1 by (OW-1) s + 1).  What the gradient of a strided convolution with respect to its input
// convolves at stride 1.  One 16-byte vector per thread.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void dilate_nhwc_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, int64_t total, int OH, int OW,
                                                          int Hd, int Wd, int CV, int s)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int cv = (int)(idx % CV);
    const int64_t pix = idx / CV;
    const int wd = (int)(pix % Wd);
    const int64_t r = pix / Wd;
    const int hd = (int)(r % Hd);
    const int64_t n = r / Hd;
    u32x4 v = {0u, 0u, 0u, 0u};
    const int i = hd / s, j = wd / s;
    if (i * s == hd && j * s == wd && i < OH && j < OW) v = src[((n * OH + i) * OW + j) * CV + cv];
    dst[idx] = v;
}

hipError_t launch_dilate_nhwc(const void *src, void *dst, int32_t N, int32_t OH, int32_t OW, int32_t Hd, int32_t Wd, int32_t pixel_bytes, int32_t stride,
                              hipStream_t s)
{
    if (N < 1 || OH < 1 || OW < 1 || stride < 1 || pixel_bytes < 16 || pixel_bytes % 16 != 0 || Hd < (OH - 1) * stride + 1 || Wd < (OW - 1) * stride + 1 ||
        ((uintptr_t)src & 15) || ((uintptr_t)dst & 15))
        return hipErrorInvalidValue;
    const int64_t total = (int64_t)N * Hd * Wd * (pixel_bytes / 16);
    if (total >= ((int64_t)1 << 38)) return hipErrorInvalidValue;              // the grid stays below 2^30 workgroups
    hipLaunchKernelGGL(dilate_nhwc_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, (const u32x4 *)src, (u32x4 *)dst, total, OH, OW, Hd, Wd,
                       pixel_bytes / 16, stride);
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

// The same for even W and Wp and 4-byte aligned tensors: one thread per pair of frame pixels (one 16-byte store, so
// a wave writes a contiguous KB), each plane read as aligned dwords (two when the pair starts on an odd image
// column) instead of single elements.
template <int C>
__global__ __launch_bounds__(256) void stem_pad_pair_kernel(const uint16_t *__restrict__ src, uint16_t *__restrict__ dst, int N, int H, int W,
                                                            int Hp, int Wp2, int ph, int pw, uint32_t wp2_mul, uint32_t wp2_sh,
                                                            uint32_t hp_mul, uint32_t hp_sh)
{
    const uint32_t total = (uint32_t)N * Hp * Wp2;
    const uint32_t idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const uint32_t q = Wp2 == 1 ? idx : (__umulhi(idx, wp2_mul) >> wp2_sh);
    const int j = (int)(idx - q * Wp2);
    const uint32_t n = Hp == 1 ? q : (__umulhi(q, hp_mul) >> hp_sh);
    const int hp = (int)(q - n * Hp);
    const int h = hp - ph, w = 2 * j - pw;          // image position of the pair's first pixel
    uint32_t px0[4] = {0u, 0u, 0u, 0u}, px1[4] = {0u, 0u, 0u, 0u};
    if ((unsigned)h < (unsigned)H && w + 1 >= 0 && w < W) {
        const bool ok0 = w >= 0, ok1 = w + 1 < W;
        // aligned dwords: elements (e, e+1) with e = w rounded down to even, and the next pair when w is odd
        const int e = w & ~1;
        const int ea = e < 0 ? 0 : e, eb = e + 2 > W - 2 ? W - 2 : e + 2;
        const uint16_t *row = src + (((int64_t)n * C) * H + h) * W;
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const uint16_t *pr = row + (int64_t)c * H * W;
            const uint32_t a = *(const uint32_t *)(pr + ea);
            if (w & 1) {
                const uint32_t b = *(const uint32_t *)(pr + eb);
                px0[c] = ok0 ? (a >> 16) : 0u;                     // element e + 1 = w
                px1[c] = ok1 ? (b & 0xffffu) : 0u;                 // element e + 2 = w + 1
            } else {
                px0[c] = ok0 ? (a & 0xffffu) : 0u;
                px1[c] = ok1 ? (a >> 16) : 0u;
            }
        }
    }
    u32x4 o = {px0[0] | (px0[1] << 16), px0[2] | (px0[3] << 16), px1[0] | (px1[1] << 16), px1[2] | (px1[3] << 16)};
    *(u32x4 *)(dst + (size_t)idx * 8) = o;
}

hipError_t launch_stem_pad(const void *src, void *dst, int32_t N, int32_t C, int32_t H, int32_t W, int32_t Hp, int32_t Wp,
                           int32_t ph, int32_t pw, hipStream_t s)
{
    if (C < 1 || C > 4) return hipErrorInvalidValue;
    if (W % 2 == 0 && W >= 2 && Wp % 2 == 0 && (((uintptr_t)src & 3) == 0) && (((uintptr_t)dst & 15) == 0) && (int64_t)N * Hp * (Wp / 2) < ((int64_t)1 << 31)) {
        uint32_t m1, s1, m2, s2;
        make_fast_div((uint32_t)(Wp / 2), m1, s1);
        make_fast_div((uint32_t)Hp, m2, s2);
        const unsigned grid = (unsigned)(((int64_t)N * Hp * (Wp / 2) + 255) / 256);
        const uint16_t *sp = (const uint16_t *)src;
        uint16_t *dp = (uint16_t *)dst;
        switch (C) {
        case 1: hipLaunchKernelGGL(stem_pad_pair_kernel<1>, dim3(grid), dim3(256), 0, s, sp, dp, N, H, W, Hp, Wp / 2, ph, pw, m1, s1, m2, s2); break;
        case 2: hipLaunchKernelGGL(stem_pad_pair_kernel<2>, dim3(grid), dim3(256), 0, s, sp, dp, N, H, W, Hp, Wp / 2, ph, pw, m1, s1, m2, s2); break;
        case 3: hipLaunchKernelGGL(stem_pad_pair_kernel<3>, dim3(grid), dim3(256), 0, s, sp, dp, N, H, W, Hp, Wp / 2, ph, pw, m1, s1, m2, s2); break;
        default: hipLaunchKernelGGL(stem_pad_pair_kernel<4>, dim3(grid), dim3(256), 0, s, sp, dp, N, H, W, Hp, Wp / 2, ph, pw, m1, s1, m2, s2); break;
        }
        return hipGetLastError();
    }
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

// weights of the stem kernel that reads the channel-first input: contraction index 16 (c ceil(KH/2) + kh/2) + 8 (kh & 1) + j,
// window column j = kw + (pw & 1); zeros where the filter does not reach and past the last plane
__global__ __launch_bounds__(256) void pack_weight_stem_direct_kernel(const uint16_t *__restrict__ src, uint16_t *__restrict__ dst, int O, int C,
                                                                      int KH, int KW, int e)
{
    const int total = O * STEM_DIRECT_KP;
    for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += gridDim.x * blockDim.x) {
        const int k = idx % STEM_DIRECT_KP, o = idx / STEM_DIRECT_KP;
        const int khh = (KH + 1) >> 1;
        const int ks = k >> 4, kw = (k & 7) - e;
        const int c = ks / khh, kh = 2 * (ks - c * khh) + ((k >> 3) & 1);
        uint16_t v = 0;
        if (c < C && kh < KH && kw >= 0 && kw < KW) v = src[(((int64_t)o * C + c) * KH + kh) * KW + kw];
        dst[idx] = v;
    }
}

hipError_t launch_pack_weight_stem_direct(const void *src, void *dst, int32_t O, int32_t C, int32_t KH, int32_t KW, int32_t pw, hipStream_t s)
{
    if (O < 1 || O > (1 << 20) || C < 1 || KH < 1 || KW < 1 || C * ((KH + 1) / 2) * 16 > STEM_DIRECT_KP || KW + (pw & 1) > 8) return hipErrorInvalidValue;
    hipLaunchKernelGGL(pack_weight_stem_direct_kernel, dim3(grid_for((int64_t)O * STEM_DIRECT_KP)), dim3(256), 0, s, (const uint16_t *)src,
                       (uint16_t *)dst, O, C, KH, KW, pw & 1);
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

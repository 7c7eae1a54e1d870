// Implicit-GEMM contraction for gfx950, LDS-DMA variant: operand tiles go
// from global memory straight into LDS (buffer_load ... lds, 16 bytes per
// lane), three K tiles deep, with no staging registers and no LDS stores in
// the K loop.
//
//   C[m, n] = sum_k A[m, k] * Wp[n, k],  m = (image, oh, ow), n = out channel,
//   k = (kh, kw, c)
//
// Preconditions (checked by the planner): channel-last activations with
// C a multiple of the K tile (64 bf16 / 32 f32), so a K tile lies inside one
// filter tap and the tap state is wave-uniform; K a multiple of the tile and at
// least two tiles; KH*KW <= 32; operands below 2 GiB.
//
// Tile layout in LDS: rows of 128 bytes (8 chunks of 16 bytes), unpadded,
// because one DMA instruction writes 64 lanes x 16 bytes contiguously = 8 rows.
// Bank conflicts are avoided by choosing which global chunk each lane fetches:
// position p of row r holds chunk p ^ ((r >> 1) & 7), so the 16 rows read by a
// quarter-wave fragment load cover all 64 banks once.
//
// Padding taps and rows past M get a buffer offset outside the descriptor's
// range: the hardware then writes zeros into LDS without touching memory.
//
// Synchronisation: each stage is its own LDS array so that the compiler's
// wait-count insertion can tell DMA writes to one stage from fragment reads of
// another; the waits on the DMA itself are explicit (s_waitcnt vmcnt) and the
// workgroup barrier is the bare instruction, one per K tile:
//     wait(my DMAs of tile t) ; barrier ; issue DMA of tile t+2 ; MFMAs on tile t
// After the barrier every wave's part of tile t has landed and every wave has
// left tile t-1, whose stage the new DMA overwrites.
#include <algorithm>

#include "igemm_epilogue.h"

namespace rl {

namespace {

typedef __amdgpu_buffer_rsrc_t rsrc_t;
#define RL_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

__device__ __forceinline__ rsrc_t make_rsrc(const void *ptr, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc((void *)ptr, 0, bytes, 0x00020000);   // raw buffer, untyped dwords
}

template <typename T> struct Elem;
template <> struct Elem<float> { static constexpr int KV = 4; };
template <> struct Elem<uint16_t> { static constexpr int KV = 8; };

__device__ __forceinline__ void mma_chunk(f32x16 &acc, const u32x4 &a, const u32x4 &b, float)
{
#pragma unroll
    for (int j = 0; j < 4; ++j)
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[j]), __uint_as_float(b[j]), acc, 0, 0, 0);
}

__device__ __forceinline__ void mma_chunk(f32x16 &acc, const u32x4 &a, const u32x4 &b, uint16_t)
{
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding:
// vmcnt = bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)
template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

__device__ __forceinline__ void wg_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

constexpr int NUM_XCD = 8;
constexpr uint32_t OOB = 0x80000000u;

}  // namespace

template <typename T, int BM, int BN, bool GATES>
__global__ __launch_bounds__(256) void igemm_dma_kernel(const IgemmParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub; the body uses gfx950-only builtins
    constexpr int KV = Elem<T>::KV;
    constexpr int ES = (int)sizeof(T);
    constexpr int BKE = 8 * KV;               // K elements per tile (128 bytes per row)
    constexpr int WTM = BM / 2, WTN = BN / 2; // wave tile
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int AG = BM / 32, BG = BN / 32; // 8-row DMA groups per wave
    constexpr int LPT = AG + BG;              // DMA instructions per wave per tile
    constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
    constexpr int LDC = BN + 8;               // fp32 staging row (32 rows at a time)
    static_assert(32 * LDC * 4 <= STAGE, "epilogue staging must fit in one stage");

    __shared__ __attribute__((aligned(1024))) unsigned char st0[STAGE];
    __shared__ __attribute__((aligned(1024))) unsigned char st1[STAGE];
    __shared__ __attribute__((aligned(1024))) unsigned char st2[STAGE];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);   // wave-uniform by construction; keep it in an SGPR
    const int wm = wave >> 1, wn = wave & 1;

    // consecutive workgroup ids go to different XCDs; give each XCD a contiguous run of tiles
    const int nblk = p.nblk_m * p.nblk_n;
    int bid = blockIdx.x;
    {
        const int per = nblk / NUM_XCD, main = per * NUM_XCD;
        if (bid < main) bid = (bid % NUM_XCD) * per + bid / NUM_XCD;
    }
    const int bm = bid / p.nblk_n, bn = bid - bm * p.nblk_n;
    const int m0 = bm * BM, n0 = bn * BN;

    // The activation descriptor starts `bias` bytes before x so that the per-lane offset of a
    // row's tap (0,0) -- which lies above/left of the image for border pixels -- is never negative.
    const uint32_t bias = (uint32_t)(((int64_t)p.ph * p.xs_h + (int64_t)p.pw * p.xs_w) * ES);
    const rsrc_t rx = make_rsrc((const char *)p.x - bias, p.x_bytes + bias);
    const rsrc_t rx2 = make_rsrc(p.x2 ? p.x2 : p.x, p.x2 ? p.x2_bytes : p.x_bytes);
    const rsrc_t rw = make_rsrc(p.w, p.w_bytes);

    // ---- per-lane DMA state.  Lane l of a group writes LDS row (l >> 3), position (l & 7).
    const int r8 = lane >> 3, pos = lane & 7;
    uint32_t a_voff[AG], a_mask[AG], a2_voff[AG], b_voff[BG];
    int a_kc[AG];                       // first K element (within a tile) of the 16-byte chunk this lane fetches
#pragma unroll
    for (int i = 0; i < AG; ++i) {
        const int row = wave * 8 * AG + 8 * i + r8;
        const int chunk = pos ^ ((row >> 1) & 7);
        const int m = m0 + row;
        uint32_t mask = 0;
        int64_t off = 0;
        if (m < p.M) {
            int img = m / p.OHW;
            int pix = m - img * p.OHW;
            int oh = pix / p.OW;
            int ow = pix - oh * p.OW;
            int ih0 = oh * p.sh - p.ph, iw0 = ow * p.sw - p.pw;
            for (int kh = 0; kh < p.KH; ++kh)
                for (int kw = 0; kw < p.KW; ++kw)
                    if ((unsigned)(ih0 + kh) < (unsigned)p.H && (unsigned)(iw0 + kw) < (unsigned)p.W) mask |= 1u << (kh * p.KW + kw);
            off = ((int64_t)img * p.xs_n + (int64_t)ih0 * p.xs_h + (int64_t)iw0 * p.xs_w) * ES;
        }
        a_mask[i] = mask;
        a_kc[i] = chunk * KV;
        a_voff[i] = (uint32_t)(off + bias) + chunk * 16;
        a2_voff[i] = (uint32_t)((int64_t)m * p.x2s_n * ES) + chunk * 16;     // second operand of a concatenation: row m
    }
#pragma unroll
    for (int j = 0; j < BG; ++j) {
        const int row = wave * 8 * BG + 8 * j + r8;
        const int chunk = pos ^ ((row >> 1) & 7);
        int n = n0 + row;
        if (n > p.N - 1) n = p.N - 1;          // rows past N are computed on valid memory and never stored
        b_voff[j] = (uint32_t)((int64_t)n * p.Kp * ES) + chunk * 16;
    }

    // ---- wave-uniform K state of the tile to be issued next.  Issuing is unconditional so that
    // every K-loop body has the same number of DMA instructions in flight (the explicit vmcnt
    // waits count on it); past the last tile all lanes are sent out of range, which costs no
    // memory traffic and only zero-fills a stage nobody reads.
    // K tiles [kt0, nk) of the contraction's ceil(p.K / BKE) (>= 2): all of them, or this workgroup's slice.  Only a
    // one-tap contraction (dense, 1x1) may end in a partial tile: the weights are packed with zeros up to the tile,
    // the activation chunks past K are requested out of range.
    const int nk_all = (p.K + BKE - 1) / BKE;
    const int split = p.splits > 1 ? (int)blockIdx.y : 0;
    const int kt0 = p.splits > 1 ? split * p.split_tiles : 0;
    const int nk = p.splits > 1 ? min(nk_all, kt0 + p.split_tiles) : nk_all;
    int f_kt = kt0, f_c0 = 0, f_tap = 0, f_kh = 0, f_kw = 0;
    if (kt0 > 0) {
        const int tpt = p.KH * p.KW == 1 ? nk_all : p.C / BKE;      // K tiles per filter tap
        f_tap = kt0 / tpt;
        f_c0 = (kt0 - f_tap * tpt) * BKE;
        f_kh = f_tap / p.KW;
        f_kw = f_tap - f_kh * p.KW;
    }
#define RL_ISSUE(ST)                                                                                                  \
    {                                                                                                                 \
        const bool live = f_kt < nk;                                                                                  \
        const int k0 = f_kt * BKE;                                                                                    \
        const uint32_t soff_b = live ? (uint32_t)k0 * ES : 0u;                                                        \
        if (k0 < p.K1 || !live) {                                                                                     \
            const uint32_t tapbit = live ? (1u << f_tap) : 0u;                                                        \
            const uint32_t soff_a = live ? (uint32_t)(((int64_t)f_kh * p.xs_h + (int64_t)f_kw * p.xs_w + f_c0) * ES) : 0u; \
            const int krem = p.K - k0;      /* K elements from this tile's start on: >= BKE except in a partial last tile */ \
            _Pragma("unroll") for (int i = 0; i < AG; ++i)                                                            \
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, RL_LDS_PTR(ST + (wave * AG + i) * 1024), 16,             \
                                                         ((a_mask[i] & tapbit) && a_kc[i] < krem) ? a_voff[i] : OOB, soff_a, 0, 0); \
        } else {                                                                                                      \
            const uint32_t soff_a = (uint32_t)(k0 - p.K1) * ES;                                                       \
            _Pragma("unroll") for (int i = 0; i < AG; ++i)                                                            \
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rx2, RL_LDS_PTR(ST + (wave * AG + i) * 1024), 16,            \
                                                         a_mask[i] ? a2_voff[i] : OOB, soff_a, 0, 0);                 \
        }                                                                                                             \
        _Pragma("unroll") for (int j = 0; j < BG; ++j)                                                                \
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, RL_LDS_PTR(ST + A_BYTES + (wave * BG + j) * 1024), 16,       \
                                                     live ? b_voff[j] : OOB, soff_b, 0, 0);                           \
        ++f_kt;                                                                                                       \
        f_c0 += BKE;                                                                                                  \
        if (f_c0 >= p.C) {                                                                                            \
            f_c0 = 0;                                                                                                 \
            ++f_tap;                                                                                                  \
            if (++f_kw == p.KW) { f_kw = 0; ++f_kh; }                                                                 \
        }                                                                                                             \
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // ---- fragment addresses: row frow of a 32-row MFMA tile, chunk 2*ks + fhalf, swizzled
    const int frow = lane & 31, fhalf = lane >> 5;
    int f_off[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) f_off[ks] = frow * 128 + (((2 * ks + fhalf) ^ ((frow >> 1) & 7)) << 4);

#define RL_COMPUTE(ST)                                                                                                \
    {                                                                                                                 \
        _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) {                                                            \
            u32x4 fa[TM], fb[TN];                                                                                     \
            _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                            \
                fa[i] = *(const u32x4 *)(ST + (wm * WTM + i * 32) * 128 + f_off[ks]);                                 \
            _Pragma("unroll") for (int j = 0; j < TN; ++j)                                                            \
                fb[j] = *(const u32x4 *)(ST + A_BYTES + (wn * WTN + j * 32) * 128 + f_off[ks]);                       \
            _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                            \
                _Pragma("unroll") for (int j = 0; j < TN; ++j) mma_chunk(acc[i][j], fa[i], fb[j], T());               \
        }                                                                                                             \
    }

    // ---- K loop, three stages, unrolled by three so that every stage use names its array.
    // Tile kt lives in stage kt % 3.  Body: wait until my DMAs of tile kt have landed (the LPT
    // issued after them, for tile kt+1, may still fly), barrier, issue tile kt+2 into the stage
    // tile kt-1 just left, MFMAs on tile kt.
#define RL_BODY(CUR, NXT)     \
    {                         \
        wait_vmcnt<LPT>();    \
        wg_barrier();         \
        RL_ISSUE(NXT)         \
        RL_COMPUTE(CUR)       \
    }
    RL_ISSUE(st0)
    RL_ISSUE(st1)
    int kt = kt0;
#pragma unroll 1
    for (; kt + 3 <= nk; kt += 3) {
        RL_BODY(st0, st2)
        RL_BODY(st1, st0)
        RL_BODY(st2, st1)
    }
    if (kt < nk) {
        RL_BODY(st0, st2)
        if (kt + 1 < nk) RL_BODY(st1, st0)
    }
    wait_vmcnt<0>();           // the trailing out-of-range issues
#undef RL_BODY
#undef RL_COMPUTE
#undef RL_ISSUE

    // ---- epilogue: 32 rows at a time through LDS (stage 0's array), then 8 channels per thread;
    // the residual rows of the next pass are fetched while this pass is staged and stored
    using TE = TileEpilogue<BN>;
    float *sC = (float *)st0;
    if (!GATES && p.splits > 1) {
        // a slice of K: the bare fp32 sums, row-major [M][N], into this slice's part of the scratch tensor
        float *dst = p.partial + (int64_t)split * p.M * p.N;
#pragma unroll
        for (int q = 0; q < BM / 32; ++q) {
            wg_barrier();
            if (wm == q / TM) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        int row = 8 * (r >> 2) + 4 * fhalf + (r & 3);
                        int col = wn * WTN + j * 32 + frow;
                        sC[row * LDC + col] = acc[q % TM][j][r];
                    }
            }
            __syncthreads();
            for (int idx = t; idx < 32 * BN; idx += 256) {
                const int row = idx / BN, col = idx - row * BN;
                const int m = m0 + q * 32 + row, n = n0 + col;
                if (m < p.M && n < p.N) dst[(int64_t)m * p.N + n] = sC[row * LDC + col];
            }
        }
        return;
    }
    const bool rowmajor = (p.ys_n == (int64_t)p.OHW * p.ys_p) && p.ys_c == 1;
    const bool vec_ok = !GATES && rowmajor && (p.N & 7) == 0 && (p.ys_p & 7) == 0;
    const bool pre = vec_ok && p.epi.simple;
    float bias8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    OperandRegs<TE::NV> cur = {}, nxt = {};
    if (pre) {
        TE::load_bias(p, t, n0, bias8);
        TE::prefetch(p, t, m0, n0, cur);
    }
#pragma unroll
    for (int q = 0; q < BM / 32; ++q) {
        if (pre && q + 1 < BM / 32) TE::prefetch(p, t, m0 + (q + 1) * 32, n0, nxt);
        wg_barrier();                           // previous pass read out / last K tile consumed
        if (wm == q / TM) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int row = 8 * (r >> 2) + 4 * fhalf + (r & 3);
                    int col = wn * WTN + j * 32 + frow;
                    sC[row * LDC + col] = acc[q % TM][j][r];
                }
        }
        __syncthreads();
        const int mq = m0 + q * 32;
        if (GATES) TE::gates_pass(p, sC, LDC, t, mq, bn);
        else if (vec_ok) TE::store_pass(p, sC, LDC, t, mq, n0, bias8, cur);
        else TE::store_pass_scalar(p, sC, LDC, t, mq, n0);
        cur = nxt;
    }
#endif
}

// The second kernel of a split contraction: y[m, n] = epilogue(partial[0][m][n] + partial[1][m][n] + ...), one element
// per thread, slices added in order (so the result does not depend on timing), any output strides.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const IgemmParams p)
{
    const Epilogue &e = p.epi;
    const uint32_t total = (uint32_t)p.M * (uint32_t)p.N;            // below 2^31 (checked by the launcher): 32-bit index arithmetic
    for (uint32_t idx = blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += gridDim.x * blockDim.x) {
        const int m = (int)(idx / (uint32_t)p.N), n = (int)(idx - (uint32_t)m * (uint32_t)p.N);
        // eight slices' values are requested before the first is added (the additions stay in slice order)
        float val = 0.0f;
        for (int z0 = 0; z0 < p.splits; z0 += 8) {
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = z0 + j < p.splits ? p.partial[(int64_t)(z0 + j) * total + idx] : 0.0f;    // splits * total < 2^26 floats
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (z0 + j < p.splits) val = z0 + j == 0 ? v[j] : val + v[j];
        }
        const int img = m / p.OHW, pix = m - img * p.OHW;
        const int64_t off = (int64_t)img * p.ys_n + (int64_t)pix * p.ys_p + (int64_t)n * p.ys_c;
        for (int s = 0; s < e.n_ops; ++s) val = epi_step(e, s, val, off, n);
        store_from_f32(p.y, p.y_dtype, off, val);
    }
}

hipError_t launch_splitk_reduce(const IgemmParams &p, hipStream_t s)
{
    const int64_t total = (int64_t)p.M * p.N;
    if (total < 1 || total * p.splits >= (int64_t)1 << 31 || !p.partial) return hipErrorInvalidValue;
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)std::min<int64_t>((total + 255) / 256, 256 * 16)), dim3(256), 0, s, p);
    return hipGetLastError();
}

// The adding launch of a split dense contraction together with the small dense layer that consumes its result: one
// workgroup per row.  Threads add the slices of their columns in slice order and apply the first group's epilogue
// (and the rounding to the dtype the tensor between the groups has), the row meets in LDS, then every wave takes
// output columns in turn: lanes multiply a strided share of the row, the 64 shares are added in a fixed tree.
__global__ __launch_bounds__(256) void reduce_dense_kernel(const ReduceDenseParams p)
{
    __shared__ float hs[REDUCE_DENSE_MAX_N1];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int m = blockIdx.x;
    const int64_t slice = (int64_t)p.M * p.N1;
    for (int n = t; n < p.N1; n += 256) {
        const float *src = p.partial + (int64_t)m * p.N1 + n;
        float val = 0.0f;
        for (int z0 = 0; z0 < p.splits; z0 += 8) {
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = z0 + j < p.splits ? src[(int64_t)(z0 + j) * slice] : 0.0f;
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (z0 + j < p.splits) val = z0 + j == 0 ? v[j] : val + v[j];
        }
        const int64_t off = (int64_t)m * p.hs_n + (int64_t)n * p.hs_c;
        for (int s = 0; s < p.epi1.n_ops; ++s) val = epi_step(p.epi1, s, val, off, n);
        hs[n] = p.h_dtype == DT_BF16 ? round_bf16(val) : val;
    }
    __syncthreads();
    for (int j = wave; j < p.N2; j += 4) {
        float acc = 0.0f;
        for (int n = lane; n < p.N1; n += 64) acc += hs[n] * load_as_f32(p.w2, p.w_dtype, (int64_t)j * p.Kp2 + n);
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) acc += __shfl_xor(acc, d, 64);
        if (lane == 0) {
            const int64_t off = (int64_t)m * p.ys_n + (int64_t)j * p.ys_c;
            for (int s = 0; s < p.epi2.n_ops; ++s) acc = epi_step(p.epi2, s, acc, off, j);
            store_from_f32(p.y, p.y_dtype, off, acc);
        }
    }
}

hipError_t launch_reduce_dense(const ReduceDenseParams &p, hipStream_t s)
{
    if (!p.partial || !p.w2 || !p.y || p.splits < 2 || p.splits > 64 || p.M < 1 || p.M > 65535 || p.N1 < 1 || p.N1 > REDUCE_DENSE_MAX_N1 ||
        p.N2 < 1 || p.N2 > REDUCE_DENSE_MAX_N2 || p.Kp2 < p.N1 || (int64_t)p.M * p.N1 * p.splits >= (int64_t)1 << 31)
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(reduce_dense_kernel, dim3((unsigned)p.M), dim3(256), 0, s, p);
    return hipGetLastError();
}

// explicit instantiations (the host-side launch stubs of a kernel template with function-local
// __shared__ arrays are not emitted implicitly)
#define RL_INST(T, BM, BN, G) template __global__ void igemm_dma_kernel<T, BM, BN, G>(const IgemmParams);
RL_INST(uint16_t, 128, 128, false) RL_INST(uint16_t, 128, 64, false) RL_INST(uint16_t, 64, 64, false) RL_INST(uint16_t, 64, 64, true)
RL_INST(float, 128, 128, false) RL_INST(float, 128, 64, false) RL_INST(float, 64, 64, false) RL_INST(float, 64, 64, true)
#undef RL_INST

template <typename T, int BM, int BN, bool GATES>
static hipError_t launch_dma(const IgemmParams &p0, hipStream_t s)
{
    IgemmParams p = p0;
    {
        // a partial last K tile: one tap, no concatenation, weight rows padded to whole tiles
        constexpr int BKE = 128 / (int)sizeof(T);
        if (p.K % BKE != 0 && (p.KH * p.KW != 1 || p.K1 != p.K || p.x2 || p.Kp % BKE != 0 || p.Kp < p.K || GATES)) return hipErrorInvalidValue;
    }
    p.nblk_m = (p.M + BM - 1) / BM;
    p.nblk_n = (p.N + BN - 1) / BN;
    int64_t nblk = (int64_t)p.nblk_m * p.nblk_n;
    if (nblk <= 0 || nblk > 0x7fffffff) return hipErrorInvalidValue;
    if (p.splits > 1) {
        constexpr int BKE = 128 / (int)sizeof(T);
        const int nk = (p.K + BKE - 1) / BKE;
        // every slice holds at least one K tile and the slices cover K exactly once
        if (GATES || !p.partial || p.splits > 64 || (int64_t)p.M * p.N * p.splits >= (int64_t)1 << 31 || p.split_tiles < 1 || (int64_t)(p.splits - 1) * p.split_tiles >= nk ||
            (int64_t)p.splits * p.split_tiles < nk || (p.C % BKE != 0 && p.KH * p.KW != 1) || p.K1 != p.K)
            return hipErrorInvalidValue;
        hipLaunchKernelGGL((igemm_dma_kernel<T, BM, BN, GATES>), dim3((unsigned)nblk, (unsigned)p.splits), dim3(256), 0, s, p);
        hipError_t er = hipGetLastError();
        if (er != hipSuccess || p.skip_reduce) return er;
        return launch_splitk_reduce(p, s);
    }
    hipLaunchKernelGGL((igemm_dma_kernel<T, BM, BN, GATES>), dim3((unsigned)nblk), dim3(256), 0, s, p);
    return hipGetLastError();
}

template <typename T>
static hipError_t launch_dma_typed(const IgemmParams &p, const IgemmLaunch &l, hipStream_t s)
{
    if (l.gates) {
        if (l.tile != TILE_64x64) return hipErrorInvalidValue;
        return launch_dma<T, 64, 64, true>(p, s);
    }
    switch (l.tile) {
    case TILE_128x128: return launch_dma<T, 128, 128, false>(p, s);
    case TILE_128x64: return launch_dma<T, 128, 64, false>(p, s);
    default: return launch_dma<T, 64, 64, false>(p, s);
    }
}

hipError_t launch_igemm_dma(const IgemmParams &p, const IgemmLaunch &l, hipStream_t s)
{
    if (p.in_dtype == DT_BF16) return launch_dma_typed<uint16_t>(p, l, s);
    return launch_dma_typed<float>(p, l, s);
}

}  // namespace rl

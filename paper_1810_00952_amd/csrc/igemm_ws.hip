// Implicit-GEMM contraction for gfx950, bf16 in / fp32 accumulate, for narrow
// outputs (N <= 64 channels) whose whole packed weight matrix fits in LDS:
// weights stationary, persistent workgroups.
//
//   C[m, n] = sum_k A[m, k] * Wp[n, k],  m = (image, oh, ow), n = out channel,
//   k = (kh, kw, c)
//
// With N = 64 a tile's K loop is short (a few hundred cycles of MFMA work per
// 128 output pixels), so a kernel that starts a workgroup per tile spends most
// of its time in prologues, epilogues and launch tails, and re-fetches the
// same weights for every tile.  Here a workgroup (256 threads, 4 waves, one
// per CU) loads the weights once, as nk tiles of 64 rows x 128 bytes, and then
// walks a list of 128-pixel tiles.  Only activation tiles stream: they travel
// global -> LDS by direct loads (16 bytes per lane) through a ring of four
// stages that runs across tile boundaries, so the first K tiles of the next
// pixel tile are already in flight while the current one is finished.
//
// Each wave owns 32 pixels x 64 channels (two 32x32x16 MFMA tiles, weights as
// the row operand so that a lane holds one pixel).  K tiles are worked off in
// two phases of four MFMAs; fragments of the next phase are read while the
// current one runs, across K tiles too; a tile's four direct loads are issued
// one at a time between the MFMAs.  A wave streams exactly the activation rows
// it consumes, so the K loop needs no workgroup barrier.  LDS rows are 128 bytes,
// unpadded, 16-byte chunks XOR-swizzled by the row at load time.
//
// Epilogue per pixel tile: bias added in registers, accumulators parked as fp32
// in a wave-private 4 KB patch (16 pixels at a time), read back row-wise so
// that a lane finishes 8 consecutive channels of one pixel: residual (fetched
// the same way when the tile's K loop starts), ReLU, one rounding to bf16,
// 16-byte stores covering whole 128-byte output rows.
//
// Tiles are dealt so that each XCD (one L2) works on one contiguous run of the
// pixel axis: neighbouring tiles share filter-halo rows.
//
// Preconditions (checked by the planner): as for the pixel-on-lane kernel,
// plus N <= 64 and K <= 576.
#include "device_utils.h"

namespace rl {

namespace {

typedef __amdgpu_buffer_rsrc_t rsrc_t;
#define RL_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

__device__ __forceinline__ rsrc_t make_rsrc(const void *ptr, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc((void *)ptr, 0, bytes, 0x00020000);   // raw buffer, untyped dwords
}

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is six bits");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

__device__ __forceinline__ void wg_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

__device__ __forceinline__ uint32_t fast_div(uint32_t n, uint32_t d, uint32_t mul, uint32_t sh)
{
    return d == 1 ? n : (__umulhi(n, mul) >> sh);
}

constexpr int NUM_XCD = 8;
constexpr uint32_t OOB = 0x80000000u;
constexpr int WS_MAX_NK = 9;          // K tiles of stationary weights (9 x 8 KB)

}  // namespace

__global__ __launch_bounds__(256) void igemm_ws_kernel(const IgemmParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub; the body uses gfx950-only builtins
    constexpr int BM = 128, BKE = 64;
    constexpr int AG = BM / 32;                     // 8-row direct-load groups per wave per activation tile
    constexpr int LPT = AG;
    constexpr int A_BYTES = BM * 128, W_TILE = 64 * 128;
    constexpr int TN = 2;                           // wave tile: 32 pixels x 64 channels
    constexpr int NMMA = 8, KSP = 2, NPH = 2;

    __shared__ __attribute__((aligned(1024))) unsigned char sw[WS_MAX_NK * W_TILE];
    __shared__ __attribute__((aligned(1024))) unsigned char sa0[A_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char sa1[A_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char sa2[A_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char sa3[A_BYTES];
    __shared__ __attribute__((aligned(1024))) unsigned char spark[4 * 4096];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int nk = p.K / BKE;

    // ---- this workgroup's tiles: XCD x = blockIdx % 8 owns the run [x*per, (x+1)*per) of the pixel-tile
    // axis; its workgroups take the tiles of that run in turn
    const int ntile = (p.M + BM - 1) / BM;
    const int per = (ntile + NUM_XCD - 1) / NUM_XCD;
    const int xcd = blockIdx.x % NUM_XCD, slot = blockIdx.x / NUM_XCD, nslot = gridDim.x / NUM_XCD;
    const int run_end = min(ntile, (xcd + 1) * per);
    const int first = xcd * per + slot;
    const int my_tiles = first < run_end ? (run_end - first + nslot - 1) / nslot : 0;
    const int total = my_tiles * nk;                // K tiles this workgroup consumes
    if (total == 0) return;                         // whole workgroup leaves together

    const uint32_t halo = (uint32_t)(((int64_t)p.ph * p.xs_h + (int64_t)p.pw * p.xs_w) * 2);
    const rsrc_t rx = make_rsrc((const char *)p.x - halo, p.x_bytes + halo);
    const rsrc_t rw = make_rsrc(p.w, p.w_bytes);
    const Epilogue &e = p.epi;
    const bool has_res = e.t_op >= 0;
    const rsrc_t rres = make_rsrc(has_res ? e.t_ptr : p.w, has_res ? p.y_bytes : 0u);
    const rsrc_t ry = make_rsrc(p.y, p.y_bytes);

    // ---- stationary weights: K tile kt at sw + kt*8 KB, rows swizzled like the activation tiles
    const int r8 = lane >> 3, pos = lane & 7;
    for (int kt = 0; kt < nk; ++kt)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int row = wave * 16 + 8 * j + r8;
            const int chunk = pos ^ ((row >> 1) & 7);
            const int n = min(row, p.N - 1);                  // rows past N repeat a valid row and are never stored
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, RL_LDS_PTR(sw + kt * W_TILE + (wave * 2 + j) * 1024), 16,
                                                     (uint32_t)((int64_t)n * p.Kp * 2) + chunk * 16, (uint32_t)kt * 128u, 0, 0);
        }

    // ---- issue side: lane state of the pixel tile whose K tiles are being requested
    uint32_t a_voff[AG], a_mask[AG];
    int i_mt = first, i_kt = 0, i_g = 0;            // pixel tile, K tile, running K-tile count
    int f_c0 = 0, f_tap = 0, f_kh = 0, f_kw = 0;
#define RL_LANE_STATE(MT)                                                                                             \
    {                                                                                                                 \
        _Pragma("unroll") for (int i = 0; i < AG; ++i) {                                                              \
            const int row = wave * 8 * AG + 8 * i + r8;                                                               \
            const int chunk = pos ^ ((row >> 1) & 7);                                                                 \
            const int m = (MT) * BM + row;                                                                            \
            uint32_t mask = 0;                                                                                        \
            int64_t off = 0;                                                                                          \
            if (m < p.M) {                                                                                            \
                const int img = (int)fast_div((uint32_t)m, (uint32_t)p.OHW, p.div_ohw_mul, p.div_ohw_sh);             \
                const int pix = m - img * p.OHW;                                                                      \
                const int oh = (int)fast_div((uint32_t)pix, (uint32_t)p.OW, p.div_ow_mul, p.div_ow_sh);               \
                const int ow = pix - oh * p.OW;                                                                       \
                const int ih0 = oh * p.sh - p.ph, iw0 = ow * p.sw - p.pw;                                             \
                const int lo_h = max(0, -ih0), hi_h = max(lo_h, min(p.KH, p.H - ih0));                                \
                const int lo_w = max(0, -iw0), hi_w = max(lo_w, min(p.KW, p.W - iw0));                                \
                const uint32_t wmk = (uint32_t)(((1ull << hi_w) - 1) & ~((1ull << lo_w) - 1));                        \
                const uint32_t rows = (uint32_t)(((1ull << (hi_h * p.KW)) - 1) & ~((1ull << (lo_h * p.KW)) - 1));     \
                mask = (wmk * p.tap_rep) & rows;                                                                      \
                off = ((int64_t)img * p.xs_n + (int64_t)ih0 * p.xs_h + (int64_t)iw0 * p.xs_w) * 2;                    \
            }                                                                                                         \
            a_mask[i] = mask;                                                                                         \
            a_voff[i] = (uint32_t)(off + halo) + (uint32_t)(chunk >> 2) * p.seg_stride + (uint32_t)(chunk & 3) * 16u; \
        }                                                                                                             \
    }
    // latch the scalars of the next K tile to request; entering a new pixel tile recomputes the lane state
    bool t_live;
    uint32_t t_soff_a, t_tapbit;
#define RL_TILE_BEGIN                                                                                                 \
    {                                                                                                                 \
        t_live = i_g < total;                                                                                         \
        if (t_live && i_kt == 0 && i_g != 0) RL_LANE_STATE(i_mt)                                                      \
        t_tapbit = t_live ? (1u << f_tap) : 0u;                                                                       \
        t_soff_a = t_live ? (uint32_t)(((int64_t)f_kh * p.ts_h + (int64_t)f_kw * p.ts_w + f_c0) * 2) : 0u;            \
        ++i_g;                                                                                                        \
        f_c0 += BKE;                                                                                                  \
        if (f_c0 >= p.C) {                                                                                            \
            f_c0 = 0;                                                                                                 \
            ++f_tap;                                                                                                  \
            if (++f_kw == p.KW) { f_kw = 0; ++f_kh; }                                                                 \
        }                                                                                                             \
        if (++i_kt == nk) { i_kt = 0; i_mt += nslot; f_c0 = 0; f_tap = 0; f_kh = 0; f_kw = 0; }                       \
    }
#define RL_DMA(ST, D)                                                                                                 \
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, RL_LDS_PTR(ST + (wave * AG + (D)) * 1024), 16,                       \
                                             (a_mask[D] & t_tapbit) ? a_voff[D] : OOB, t_soff_a, 0, 0);
#define RL_ISSUE(ST)                                                                                                  \
    {                                                                                                                 \
        RL_TILE_BEGIN                                                                                                 \
        _Pragma("unroll") for (int d = 0; d < LPT; ++d) RL_DMA(ST, d)                                                 \
    }

    // ---- compute side
    f32x16 acc[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[j][q] = 0.0f;
    const int frow = lane & 31, fhalf = lane >> 5;
    int f_off[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) f_off[ks] = frow * 128 + (((2 * ks + fhalf) ^ ((frow >> 1) & 7)) << 4);
    int c_mt = first, c_kt = 0;                     // pixel tile and K tile being multiplied

    u32x4 fw[2][KSP][TN], fx[2][KSP];
    // fragments of phase PH of a K tile: activations from stage ST, weights of K tile WKT
#define RL_LOADP(ST, WKT, PH, SET)                                                                                    \
    {                                                                                                                 \
        const unsigned char *wb_ = sw + (WKT) * W_TILE;                                                               \
        _Pragma("unroll") for (int s_ = 0; s_ < KSP; ++s_) {                                                          \
            _Pragma("unroll") for (int j = 0; j < TN; ++j)                                                            \
                fw[SET][s_][j] = *(const u32x4 *)(wb_ + (j * 32) * 128 + f_off[(PH) * KSP + s_]);                     \
            fx[SET][s_] = *(const u32x4 *)(ST + (wave * 32) * 128 + f_off[(PH) * KSP + s_]);                          \
        }                                                                                                             \
        __builtin_amdgcn_sched_barrier(0);                                                                            \
    }
#define RL_MMAP(SET, PH, ISS)                                                                                         \
    {                                                                                                                 \
        _Pragma("unroll") for (int s_ = 0; s_ < KSP; ++s_)                                                            \
            _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                                          \
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fw[SET][s_][j]),          \
                                                                 __builtin_bit_cast(bf16x8, fx[SET][s_]), acc[j], 0, 0, 0); \
                const int q_ = ((PH) * KSP + s_) * TN + j;                                                            \
                _Pragma("unroll") for (int d = 0; d < LPT; ++d)                                                       \
                    if (d * NMMA / LPT == q_) RL_DMA(ISS, d)                                                          \
                __builtin_amdgcn_sched_barrier(0);                                                                    \
            }                                                                                                         \
    }

    // ---- epilogue state: bias in accumulator layout (fixed for the kernel), residual and output offsets per tile
    const int epix = lane & 31, ehalf = lane >> 5;
    constexpr int NPASS = 4;                        // 8 rows x 8 lanes per row-wise pass, 32 rows
    const int rr = lane >> 3, pp = lane & 7;
    f32x4 bias_r[TN][4];
    {
        const rsrc_t rb = make_rsrc(e.has_bias ? e.bias_ptr : p.w, e.has_bias ? (uint32_t)p.N * 4u : 0u);
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = 4 * ehalf + j * 32 + 8 * g;
                bias_r[j][g] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rb, n < p.N ? (uint32_t)n * 4u : OOB, 0, 0));
            }
    }
    u32x4 res_r[NPASS];
    uint32_t y_off[NPASS];
    int pA[NPASS];
#pragma unroll
    for (int q = 0; q < NPASS; ++q) {
        const int prow = (q & 1) * 8 + rr;          // row inside the 16-row parked patch
        pA[q] = 2 * pp + (prow & 1);
    }
    // request the residual rows of pixel tile MT (row-wise layout) and latch the output offsets
#define RL_RES_LOADS(MT)                                                                                              \
    {                                                                                                                 \
        _Pragma("unroll") for (int q = 0; q < NPASS; ++q) {                                                           \
            const int prow = (q & 1) * 8 + rr;                                                                        \
            const int cc = pp ^ ((prow & 15) >> 1);                                                                   \
            const int m = (MT) * BM + wave * 32 + (q >> 1) * 16 + prow, n = cc * 8;                                   \
            y_off[q] = (m < p.M && n < p.N) ? (uint32_t)(((int64_t)m * p.ys_p + n) * 2) : OOB;                        \
            res_r[q] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rres, y_off[q], 0, 0));        \
        }                                                                                                             \
    }
    const float lo = e.relu_last ? 0.0f : -INFINITY;
    unsigned char *park = spark + wave * 4096;
#define RL_EPILOGUE                                                                                                   \
    {                                                                                                                 \
        _Pragma("unroll") for (int h = 0; h < 2; ++h) {                                                               \
            if ((epix >> 4) == h) {                                                                                   \
                _Pragma("unroll") for (int j = 0; j < TN; ++j)                                                        \
                    _Pragma("unroll") for (int g = 0; g < 4; ++g) {                                                   \
                        const int prow = epix & 15;                                                                   \
                        const int c = j * 8 + 2 * g + ehalf;                                                          \
                        f32x4 v;                                                                                      \
                        _Pragma("unroll") for (int k = 0; k < 4; ++k) v[k] = acc[j][4 * g + k] + bias_r[j][g][k];     \
                        *(f32x4 *)(park + prow * 256 + ((c ^ prow) << 4)) = v;                                        \
                    }                                                                                                 \
            }                                                                                                         \
            wave_lds_exchange();                                                                                      \
            _Pragma("unroll") for (int q2 = 0; q2 < 2; ++q2) {                                                        \
                const int q = 2 * h + q2;                                                                             \
                const int prow = q2 * 8 + rr;                                                                         \
                const f32x4 a = *(const f32x4 *)(park + prow * 256 + pA[q] * 16);                                     \
                const f32x4 b = *(const f32x4 *)(park + prow * 256 + (pA[q] ^ 1) * 16);                               \
                const u32x4 r = res_r[q];                                                                             \
                float v[8];                                                                                           \
                _Pragma("unroll") for (int k = 0; k < 4; ++k) { v[k] = a[k]; v[4 + k] = b[k]; }                       \
                _Pragma("unroll") for (int k = 0; k < 4; ++k) {                                                       \
                    v[2 * k] += __uint_as_float(r[k] << 16);                                                          \
                    v[2 * k + 1] += __uint_as_float(r[k] & 0xffff0000u);                                              \
                }                                                                                                     \
                u32x4 o;                                                                                              \
                _Pragma("unroll") for (int k = 0; k < 4; ++k)                                                         \
                    o[k] = pack_bf16x2(fmaxf(v[2 * k], lo), fmaxf(v[2 * k + 1], lo));                                 \
                __builtin_amdgcn_raw_buffer_store_b128(o, ry, y_off[q], 0, 0);                                        \
            }                                                                                                         \
            wave_lds_exchange();                                                                                      \
        }                                                                                                             \
        _Pragma("unroll") for (int j = 0; j < TN; ++j)                                                                \
            _Pragma("unroll") for (int q = 0; q < 16; ++q) acc[j][q] = 0.0f;                                          \
    }

    // K tile g lives in stage g % 4.  After the counted wait the wave's own rows of tiles g and g+1 have
    // landed, g+2 is in flight and g+3 is requested into the stage tile g-1 just left.  A wave loads exactly
    // the 32 activation rows it multiplies and parks its results in its own patch, so after the weights are
    // in place the four waves share nothing they write: no barrier inside the loop, and the waves drift
    // apart, which spreads their requests and lets one wave's epilogue run beside the others' MFMAs.
    // The stage is picked by a switch so that every direct load and fragment read names its array.
#define RL_CORE(CUR, NXT, ISS)                                                                                        \
    {                                                                                                                 \
        RL_LOADP(CUR, c_kt, 1, 1)                                                                                     \
        RL_MMAP(0, 0, ISS)                                                                                            \
        RL_LOADP(NXT, nkt, 0, 0)                                                                                      \
        RL_MMAP(1, 1, ISS)                                                                                            \
    }

    RL_LANE_STATE(first)
    RL_ISSUE(sa0)
    RL_ISSUE(sa1)
    RL_ISSUE(sa2)
    wait_vmcnt<0>();                                // weights, bias and the first three tiles
    wg_barrier();
    RL_LOADP(sa0, 0, 0, 0)
#pragma unroll 1
    for (int g = 0; g < total; ++g) {
        wait_vmcnt<LPT>();
        asm volatile("" ::: "memory");
        RL_TILE_BEGIN
        if (c_kt == 0) RL_RES_LOADS(c_mt)
        const int nkt = c_kt + 1 == nk ? 0 : c_kt + 1;
        switch (g & 3) {
        case 0: RL_CORE(sa0, sa1, sa3) break;
        case 1: RL_CORE(sa1, sa2, sa0) break;
        case 2: RL_CORE(sa2, sa3, sa1) break;
        default: RL_CORE(sa3, sa0, sa2) break;
        }
        if (c_kt + 1 == nk) {
            RL_EPILOGUE
            c_kt = 0;
            c_mt += nslot;
        } else {
            ++c_kt;
        }
    }
    wait_vmcnt<0>();                                // trailing out-of-range requests and the last stores
#undef RL_CORE
#undef RL_EPILOGUE
#undef RL_RES_LOADS
#undef RL_MMAP
#undef RL_LOADP
#undef RL_ISSUE
#undef RL_DMA
#undef RL_TILE_BEGIN
#undef RL_LANE_STATE
#endif
}

hipError_t launch_igemm_ws(const IgemmParams &p, hipStream_t s)
{
    if (p.in_dtype != DT_BF16 || p.y_dtype != DT_BF16 || p.x2 || p.N > 64 || p.K % 64 != 0 || p.K / 64 > WS_MAX_NK || p.K < 64)
        return hipErrorInvalidValue;
    const int ntile = (p.M + 127) / 128;
    int grid = 256;                                 // one workgroup per CU, a multiple of the XCD count
    if (ntile < grid) grid = (ntile + NUM_XCD - 1) / NUM_XCD * NUM_XCD;
    hipLaunchKernelGGL(igemm_ws_kernel, dim3((unsigned)grid), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace rl

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
// global -> LDS by direct loads (16 bytes per lane) through a ring that takes
// whatever LDS the weights leave (5 or 7 stages of 16 KB) and runs across
// pixel-tile boundaries, so the first K tiles of the
// next pixel tile are in flight while the current one is finished.  When the
// group has a residual operand, its 128 x 64 tile travels through the same
// ring as one more tile behind the K tiles, and the epilogue reads it from LDS.
//
// Each wave owns 32 pixels x 64 channels (two 32x32x16 MFMA tiles, weights as
// the row operand so that a lane holds one pixel).  K tiles are worked off in
// two phases of four MFMAs; fragments of the next phase are read while the
// current one runs, across K tiles too; a tile's four direct loads are issued
// one at a time between the MFMAs.  A wave streams exactly the activation rows
// it consumes, so after the weights are
// in place the waves share nothing they write: the loop has no workgroup
// barrier and the waves drift apart, which spreads their memory requests.
//
// The direct loads are written as inline assembly and every wait on them is an
// explicit, counted s_waitcnt: with the compiler unaware of them the ring can
// be one array indexed at run time and the loop stays rolled (the compiler's
// own wait insertion would otherwise serialise each fragment read behind all
// loads in flight).  For the counts to hold, no other load may be in flight
// inside the loop: bias is fetched before it, the residual comes through the
// ring, and stores only make a counted wait stricter, never laxer (loads
// return in order among themselves).
//
// Epilogue per pixel tile, all in registers: a lane holds one pixel and, per
// group of four accumulator registers, four consecutive channels.  Bias, the
// residual (8 bytes from its tile in the ring), ReLU and the one rounding to
// bf16 are applied there; then the two half-waves, which hold the two halves of
// every 8-channel run of the same pixel, trade halves (v_permlane32_swap), so
// that each lane stores 16 bytes and a pixel's 32 bytes per instruction are
// contiguous.  No LDS round trip, so nothing but the residual read delays the
// next tile's MFMAs.
//
// Tiles are dealt so that each XCD (one L2) works on one contiguous run of the
// pixel axis: neighbouring tiles share filter-halo rows.
//
// Preconditions (checked by the planner): as for the pixel-on-lane kernel,
// plus N <= 64 and K <= 576.
#include "device_utils.h"

namespace rl {

namespace {

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

// raw buffer descriptor (untyped dwords, range-checked against `bytes`)
__device__ __forceinline__ u32x4 make_desc(const void *ptr, uint32_t bytes)
{
    const uint64_t a = (uint64_t)ptr;
    u32x4 d = {(uint32_t)a, (uint32_t)(a >> 32) & 0xffffu, bytes, 0x00020000u};
    return d;
}

// one direct load: 64 lanes x 16 bytes from desc[voff + soff] to LDS at lds_addr + lane*16
__device__ __forceinline__ void dma16(const u32x4 &desc, uint32_t lds_addr, uint32_t voff, uint32_t soff)
{
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :: "s"(lds_addr), "v"(voff), "s"(desc), "s"(soff) : "memory");
#endif
}

#define RL_WAIT_VM(N) asm volatile("s_waitcnt vmcnt(" #N ")" ::: "memory")

__device__ __forceinline__ uint32_t lds_addr_of(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}

constexpr int NUM_XCD = 8;
constexpr uint32_t OOB = 0x80000000u;
constexpr int WS_MAX_NK = 9;          // K tiles of stationary weights (9 x 8 KB)

}  // namespace

template <bool HAS_RES, int R>
__global__ __launch_bounds__(256) void igemm_ws_kernel(const IgemmParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub; the body uses gfx950-only builtins
    constexpr int BM = 128, BKE = 64;
    constexpr int LPT = 4;                          // direct loads per wave per tile: 4 groups of 8 rows
    constexpr int A_BYTES = BM * 128, W_TILE = 64 * 128;
    constexpr int TN = 2;                           // wave tile: 32 pixels x 64 channels
    constexpr int NMMA = 8, KSP = 2;

    // one block of LDS: the weights' nk tiles first, the ring behind them
    constexpr int LDS_BYTES = 152 * 1024;
    __shared__ __attribute__((aligned(1024))) unsigned char lds[LDS_BYTES];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int nk = p.K / BKE;
    const int T = nk + (HAS_RES ? 1 : 0);           // tiles streamed per pixel tile
    unsigned char *const sw = lds;
    unsigned char *const ring = lds + nk * W_TILE;
    static_assert(R == 5 || R == 7, "ring of 5 stages (up to 9 weight tiles) or 7 (up to 5)");

    // ---- this workgroup's pixel tiles: XCD x = blockIdx % 8 owns the run [x*per, (x+1)*per) of the
    // pixel-tile axis; its workgroups take the tiles of that run in turn
    const int ntile = (p.M + BM - 1) / BM;
    const int per = (ntile + NUM_XCD - 1) / NUM_XCD;
    const int xcd = blockIdx.x % NUM_XCD, slot = blockIdx.x / NUM_XCD, nslot = gridDim.x / NUM_XCD;
    const int run_end = min(ntile, (xcd + 1) * per);
    const int first = xcd * per + slot;
    const int my_tiles = first < run_end ? (run_end - first + nslot - 1) / nslot : 0;
    const int total = my_tiles * T;                 // tiles this workgroup streams
    if (total == 0) return;                         // whole workgroup leaves together

    const uint32_t halo = (uint32_t)(((int64_t)p.ph * p.xs_h + (int64_t)p.pw * p.xs_w) * 2);
    const u32x4 dx = make_desc((const char *)p.x - halo, p.x_bytes + halo);
    const u32x4 dw = make_desc(p.w, p.w_bytes);
    const Epilogue &e = p.epi;
    const u32x4 dres = make_desc(HAS_RES ? e.t_ptr : p.w, HAS_RES ? p.y_bytes : 0u);
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(p.y, 0, p.y_bytes, 0x00020000);

    const uint32_t sw_a = lds_addr_of(sw), ring_a = lds_addr_of(ring);

    // ---- stationary weights: K tile kt at sw + kt*8 KB, 16-byte chunks swizzled by the row like the
    // activation tiles (position q of row r holds chunk q ^ ((r >> 1) & 7))
    const int r8 = lane >> 3, pos = lane & 7;
    {
        uint32_t wv[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int row = wave * 16 + 8 * j + r8;
            const int chunk = pos ^ ((row >> 1) & 7);
            const int n = min(row, p.N - 1);                  // rows past N repeat a valid row and are never stored
            wv[j] = (uint32_t)((int64_t)n * p.Kp * 2) + chunk * 16;
        }
        for (int kt = 0; kt < nk; ++kt)
#pragma unroll
            for (int j = 0; j < 2; ++j) dma16(dw, sw_a + kt * W_TILE + (wave * 2 + j) * 1024, wv[j], (uint32_t)kt * 128u);
    }
    // bias in accumulator layout, fixed for the kernel (fetched here, before any counted wait)
    const int epix = lane & 31, ehalf = lane >> 5;
    f32x4 bias_r[TN][4];
    {
        const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc((void *)(e.has_bias ? e.bias_ptr : p.w), 0, e.has_bias ? (uint32_t)p.N * 4u : 0u, 0x00020000);
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = 4 * ehalf + j * 32 + 8 * g;
                bias_r[j][g] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rb, n < p.N ? (uint32_t)n * 4u : OOB, 0, 0));
            }
    }

    // ---- issue side.  Lane l < 32 decodes row l of the wave's 32 pixels once; the (row, chunk) layout
    // the direct loads need is then gathered with cross-lane reads.
    uint32_t a_voff[LPT], a_mask[LPT], r_voff[LPT];
    auto lane_state = [&](int mt) {
        const int m = mt * BM + wave * 32 + (lane & 31);
        uint32_t mask = 0, off = 0, roff = OOB;
        if (m < p.M) {
            const int img = (int)fast_div((uint32_t)m, (uint32_t)p.OHW, p.div_ohw_mul, p.div_ohw_sh);
            const int pix = m - img * p.OHW;
            const int oh = (int)fast_div((uint32_t)pix, (uint32_t)p.OW, p.div_ow_mul, p.div_ow_sh);
            const int ow = pix - oh * p.OW;
            const int ih0 = oh * p.sh - p.ph, iw0 = ow * p.sw - p.pw;
            const int lo_h = max(0, -ih0), hi_h = max(lo_h, min(p.KH, p.H - ih0));
            const int lo_w = max(0, -iw0), hi_w = max(lo_w, min(p.KW, p.W - iw0));
            const uint32_t wmk = (uint32_t)(((1ull << hi_w) - 1) & ~((1ull << lo_w) - 1));
            const uint32_t rows = (uint32_t)(((1ull << (hi_h * p.KW)) - 1) & ~((1ull << (lo_h * p.KW)) - 1));
            mask = (wmk * p.tap_rep) & rows;      // tap_rep has bit kh*KW set for every kh: no carries, wmk < 2^KW
            off = (uint32_t)(((int64_t)img * p.xs_n + (int64_t)ih0 * p.xs_h + (int64_t)iw0 * p.xs_w) * 2 + halo);
            roff = (uint32_t)((int64_t)m * p.ys_p * 2);
        }
#pragma unroll
        for (int d = 0; d < LPT; ++d) {
            const int row = 8 * d + r8;                       // row of the wave's 32 this lane fetches in group d
            const int chunk = pos ^ ((row >> 1) & 7);         // (wave*32 is a multiple of 16: same swizzle as the tile row)
            a_mask[d] = (uint32_t)__shfl((int)mask, row);
            a_voff[d] = (uint32_t)__shfl((int)off, row) + (uint32_t)(chunk >> 2) * p.seg_stride + (uint32_t)(chunk & 3) * 16u;
            if (HAS_RES) {
                const uint32_t rb = (uint32_t)__shfl((int)roff, row);
                r_voff[d] = (rb != OOB && chunk * 8 < p.N) ? rb + chunk * 16 : OOB;  // residual rows are swizzled like the rest
            }
        }
    };
    int i_mt = first, i_kt = 0, i_g = 0;            // pixel tile, tile within it, running tile count
    int f_c0 = 0, f_tap = 0, f_kh = 0, f_kw = 0;
    bool t_live, t_res;
    uint32_t t_soff, t_tapbit;
    // latch the scalars of the next tile to request; entering a new pixel tile recomputes the lane state
    auto tile_begin = [&]() {
        t_live = i_g < total;
        if (t_live && i_kt == 0 && i_g != 0) lane_state(i_mt);
        t_res = HAS_RES && i_kt == nk;
        t_tapbit = (t_live && !t_res) ? (1u << f_tap) : 0u;
        t_soff = (t_live && !t_res) ? (uint32_t)(((int64_t)f_kh * p.ts_h + (int64_t)f_kw * p.ts_w + f_c0) * 2) : 0u;
        ++i_g;
        // advance (c0, tap) and the tile counter with selects: taken branches are expensive at one wave per SIMD
        const bool tap_done = f_c0 + BKE >= p.C;
        const bool row_done = tap_done && f_kw + 1 == p.KW;
        const bool tile_done = i_kt + 1 == T;
        f_c0 = (tap_done || tile_done) ? 0 : f_c0 + BKE;
        f_tap = tile_done ? 0 : f_tap + (tap_done ? 1 : 0);
        f_kw = (row_done || tile_done) ? 0 : f_kw + (tap_done ? 1 : 0);
        f_kh = tile_done ? 0 : f_kh + (row_done ? 1 : 0);
        i_kt = tile_done ? 0 : i_kt + 1;
        i_mt += tile_done ? nslot : 0;
    };
    // direct load d of the latched tile into the stage at LDS address st
    auto dma = [&](uint32_t st, int d) {
        uint32_t v = (a_mask[d] & t_tapbit) ? a_voff[d] : OOB;
        if (HAS_RES) {
            if (t_res && t_live) v = r_voff[d];
            dma16(t_res ? dres : dx, st + (wave * LPT + d) * 1024, v, t_soff);
        } else {
            dma16(dx, st + (wave * LPT + d) * 1024, v, t_soff);
        }
    };

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
    int c_mt = first, c_kt = 0;                     // pixel tile and tile within it being consumed

    u32x4 fw[2][KSP][TN], fx[2][KSP];
    // fragments of phase PH of a K tile: activations from the stage at `st`, weights of K tile wkt
#define RL_LOADP(ST, WKT, PH, SET)                                                                                    \
    {                                                                                                                 \
        const unsigned char *wb_ = sw + (WKT) * W_TILE;                                                               \
        const unsigned char *ab_ = (ST) + (wave * 32) * 128;                                                          \
        _Pragma("unroll") for (int s_ = 0; s_ < KSP; ++s_) {                                                          \
            _Pragma("unroll") for (int j = 0; j < TN; ++j)                                                            \
                fw[SET][s_][j] = *(const u32x4 *)(wb_ + (j * 32) * 128 + f_off[(PH) * KSP + s_]);                     \
            fx[SET][s_] = *(const u32x4 *)(ab_ + f_off[(PH) * KSP + s_]);                                             \
        }                                                                                                             \
        __builtin_amdgcn_sched_barrier(0);                                                                            \
    }
    // the phase's four MFMAs; direct load d of the latched tile follows MFMA number 2d of the tile
#define RL_MMAP(SET, PH, ISS)                                                                                         \
    {                                                                                                                 \
        _Pragma("unroll") for (int s_ = 0; s_ < KSP; ++s_)                                                            \
            _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                                          \
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fw[SET][s_][j]),          \
                                                                 __builtin_bit_cast(bf16x8, fx[SET][s_]), acc[j], 0, 0, 0); \
                const int q_ = ((PH) * KSP + s_) * TN + j;                                                            \
                if (q_ % (NMMA / LPT) == 0) dma(ISS, q_ / (NMMA / LPT));                                              \
                __builtin_amdgcn_sched_barrier(0);                                                                    \
            }                                                                                                         \
    }

    // ---- epilogue of the wave's 32 x 64 tile of pixel tile c_mt
    const float lo = e.relu_last ? 0.0f : -INFINITY;
    auto epilogue = [&](const unsigned char *res_stage) {
        u32x2 pk[TN][4];                                                      // 4 channels of bf16 per register pair
        const unsigned char *rrow = res_stage + (wave * 32 + epix) * 128 + 8 * ehalf;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float v[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) v[k] = acc[j][4 * g + k] + bias_r[j][g][k];
                if (HAS_RES) {
                    const u32x2 r = *(const u32x2 *)(rrow + (((4 * j + g) ^ ((epix >> 1) & 7)) << 4));
                    v[0] += __uint_as_float(r[0] << 16); v[1] += __uint_as_float(r[0] & 0xffff0000u);
                    v[2] += __uint_as_float(r[1] << 16); v[3] += __uint_as_float(r[1] & 0xffff0000u);
                }
                pk[j][g][0] = pack_bf16x2(fmaxf(v[0], lo), fmaxf(v[1], lo));
                pk[j][g][1] = pack_bf16x2(fmaxf(v[2], lo), fmaxf(v[3], lo));
            }
        const int m = c_mt * BM + wave * 32 + epix;
        const uint32_t ybase = m < p.M ? (uint32_t)((int64_t)m * p.ys_p * 2) : OOB;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int G = 0; G < 2; ++G) {
                // lower half-wave keeps group 2G and receives its upper partner's, the upper half-wave keeps
                // group 2G+1 and receives its lower partner's: 8 consecutive channels per lane
                const u32x2 s0 = __builtin_amdgcn_permlane32_swap(pk[j][2 * G][0], pk[j][2 * G + 1][0], false, false);
                const u32x2 s1 = __builtin_amdgcn_permlane32_swap(pk[j][2 * G][1], pk[j][2 * G + 1][1], false, false);
                const u32x4 o = {s0[0], s1[0], s0[1], s1[1]};
                const int n = j * 32 + 16 * G + 8 * ehalf;
                __builtin_amdgcn_raw_buffer_store_b128(o, ry, (ybase != OOB && n < p.N) ? ybase + (uint32_t)n * 2u : OOB, 0, 0);
            }
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[j][q] = 0.0f;
    };

    // ---- stream.  Tile g lives in stage g % R.  After the counted wait the wave's own rows of tiles g
    // and g+1 have landed, g+2 .. g+R-2 are in flight and g+R-1 is requested into the stage tile g-1
    // just left.
    lane_state(first);
    for (int g0 = 0; g0 < R - 1; ++g0) {
        tile_begin();
#pragma unroll
        for (int d = 0; d < LPT; ++d) dma(ring_a + g0 * A_BYTES, d);
    }
    RL_WAIT_VM(0);                                  // weights, bias and the first tiles
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) asm volatile("" : "+v"(bias_r[j][g]));     // bias is in registers from here on
    wg_barrier();
    RL_LOADP(ring, 0, 0, 0)
    int s_cur = 0;                                  // stage of tile g
#pragma unroll 1
    for (int g = 0; g < total; ++g) {
        if (R == 5) RL_WAIT_VM(8);                  // at most (R - 3) tiles of 4 loads stay in flight
        else RL_WAIT_VM(16);
        const int s_nxt = s_cur + 1 == R ? 0 : s_cur + 1, s_iss = s_cur == 0 ? R - 1 : s_cur - 1;
        const unsigned char *cur = ring + s_cur * A_BYTES, *nxt = ring + s_nxt * A_BYTES;
        const uint32_t iss = ring_a + s_iss * A_BYTES;
        s_cur = s_nxt;
        tile_begin();
        if (!HAS_RES || c_kt < nk) {
            const int nkt = c_kt + 1 == nk ? 0 : c_kt + 1;
            RL_LOADP(cur, c_kt, 1, 1)
            RL_MMAP(0, 0, iss)
            if (!HAS_RES || c_kt + 1 < nk) RL_LOADP(nxt, nkt, 0, 0)           // the next tile is a K tile
            RL_MMAP(1, 1, iss)
            if (!HAS_RES && c_kt + 1 == nk) epilogue(cur);
        } else {
            // the residual tile: nothing to multiply, the epilogue reads it from its stage
#pragma unroll
            for (int d = 0; d < LPT; ++d) dma(iss, d);
            epilogue(cur);
            RL_LOADP(nxt, 0, 0, 0)
        }
        const bool c_done = c_kt + 1 == T;
        c_kt = c_done ? 0 : c_kt + 1;
        c_mt += c_done ? nslot : 0;
    }
    RL_WAIT_VM(0);                                  // trailing out-of-range requests
#undef RL_MMAP
#undef RL_LOADP
#endif
}

template __global__ void igemm_ws_kernel<false, 5>(const IgemmParams);
template __global__ void igemm_ws_kernel<true, 5>(const IgemmParams);
template __global__ void igemm_ws_kernel<false, 7>(const IgemmParams);
template __global__ void igemm_ws_kernel<true, 7>(const IgemmParams);

hipError_t launch_igemm_ws(const IgemmParams &p, hipStream_t s)
{
    if (p.in_dtype != DT_BF16 || p.y_dtype != DT_BF16 || p.x2 || p.N > 64 || p.N % 8 != 0 || p.K % 64 != 0 || p.K / 64 > WS_MAX_NK || p.K < 64)
        return hipErrorInvalidValue;
    const int ntile = (p.M + 127) / 128;
    int grid = 256;                                 // one workgroup per CU, a multiple of the XCD count
    if (ntile < grid) grid = (ntile + NUM_XCD - 1) / NUM_XCD * NUM_XCD;
    const bool deep = p.K / 64 <= 5;                // the weights leave room for a 7-stage ring
    const bool res = p.epi.t_op >= 0;
    if (res && deep) hipLaunchKernelGGL((igemm_ws_kernel<true, 7>), dim3((unsigned)grid), dim3(256), 0, s, p);
    else if (res) hipLaunchKernelGGL((igemm_ws_kernel<true, 5>), dim3((unsigned)grid), dim3(256), 0, s, p);
    else if (deep) hipLaunchKernelGGL((igemm_ws_kernel<false, 7>), dim3((unsigned)grid), dim3(256), 0, s, p);
    else hipLaunchKernelGGL((igemm_ws_kernel<false, 5>), dim3((unsigned)grid), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace rl

// 3x3, stride 1, pad 1 convolutions with C a multiple of 64 on image rows of at
// most 30 pixels (the later stages of a ResNet), bf16 in / fp32 accumulate /
// bf16 out, epilogue [f32 bias] [+ bf16 residual] [ReLU].
//
// The general implicit-GEMM kernel requests, for every K tile (one filter tap
// x 64 channels), a freshly gathered activation tile next to the weight tile,
// and on these shapes the time goes into those requests: a CU accepts about
// 80 bytes of direct loads per clock, while 128x64 and 128x128 tiles want 86
// and 58 per clock of MFMA work.  With stride 1 on an unchanged image size,
// tap (kh, kw) of flat pixel m (over all images) is flat input pixel
// m + (kh-1)*W + (kw-1), so the nine taps of a 64-channel slice can all be read
// from one copy of the input rows:
//   * K runs slice-major: for each 64-channel slice the block's "run", flat
//     input pixels m0 - W - 1 ... m0 + BM + W, 128 bytes each, is copied to LDS
//     once (double-buffered: the next slice's run arrives while this one is
//     multiplied) and serves nine K tiles; only the weight tiles (BN rows of
//     128 bytes, out of the ordinary packed matrix) are requested per K tile,
//     four stages deep.  That is 18 instead of 32 KB per 128x128 K tile, 10
//     instead of 24 per 128x64.
//   * A run pixel occupies 144 bytes in LDS (nine 16-byte units, the ninth
//     unused): the fragment reads of 16 consecutive pixels then fall into 16
//     different bank groups, and the address of tap (kh, kw) is the lane's own
//     address plus (kh*W + kw)*144.  Taps outside the image (including the
//     neighbour that wraps around an image row, or into the next image) are
//     redirected per lane to zeros (the never-fetched tail of the run buffer).
//   * Eight waves, two per SIMD.  A fragment read costs a wave as much issue
//     time as an MFMA; every read and every request follows an MFMA so that it
//     is issued while that MFMA executes.  Requests are counted by hand
//     (s_waitcnt vmcnt): every wave issues the same number per K tile (dead
//     ones go out of range and move nothing).
// MFMA roles and the epilogue are those of the pixel-on-lane kernel: weights
// as the row operand, accumulators plus bias parked as fp32 in LDS per wave,
// read back row-wise, residual, ReLU, one rounding, 16-byte stores.
//
// K order differs from the general kernel's (slice-major instead of tap-major),
// so results agree with it to fp32 summation order, not bit for bit.
//
// Preconditions (checked by the launcher and the planner): bf16 throughout,
// 3x3 / stride 1 / pad 1, C a multiple of 64, W <= 30, dense channel-last
// activations, output rows contiguous in n with N a multiple of 8, tensors
// below 2 GiB.
#include "device_utils.h"

namespace rl {

namespace {

typedef __amdgpu_buffer_rsrc_t rsrc_t;

__device__ __forceinline__ rsrc_t make_rsrc(const void *ptr, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc((void *)ptr, 0, bytes, 0x00020000);   // raw buffer, untyped dwords
}

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
#define RL_WAIT_LGKM0 asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory")

__device__ __forceinline__ void wg_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

__device__ __forceinline__ uint32_t lds_addr_of(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}

__device__ __forceinline__ uint32_t fast_div(uint32_t n, uint32_t d, uint32_t mul, uint32_t sh)
{
    return d == 1 ? n : (__umulhi(n, mul) >> sh);
}

template <int N> __device__ __forceinline__ void wait_vm()
{
    static_assert(N >= 0 && N < 64, "vmcnt is six bits");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
    asm volatile("" ::: "memory");
}

constexpr int NUM_XCD = 8;
constexpr uint32_t OOB = 0x80000000u;
constexpr int RUN_W_MAX = 30;                     // widest image row
constexpr int PITCH = 144;                        // bytes per run pixel in LDS

}  // namespace

// NB: weight-tile stages.  Weight tile u + NB - 1 is requested while tile u is multiplied, and at the end of a tile
// the requests of the last NB - 3 tiles may still be in flight: more stages, more time for a request to return.
template <int BM, int BN, int WGM, int WGN, int NB>
__global__ __launch_bounds__(WGM * WGN * 64) void conv3x3_run_kernel(const IgemmParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub; the body uses gfx950-only builtins
    constexpr int NW = WGM * WGN;
    constexpr int WTM = BM / WGM, WTN = BN / WGN, TM = WTM / 32, TN = WTN / 32;
    constexpr int RUN_PIX = BM + 2 * RUN_W_MAX + 2;               // longest run
    constexpr int RUN_LOADS = ((RUN_PIX * 9 + 63) / 64 + NW - 1) / NW;   // direct loads (64 units each) per wave per run
    constexpr int RUN_BYTES = RUN_LOADS * NW * 1024;
    constexpr int BG = BN / (8 * NW);                             // weight-tile loads (8 rows each) per wave per K tile
    constexpr int B_BYTES = BN * 128;
    constexpr int B_OFF = 2 * RUN_BYTES, LDS_BYTES = B_OFF + NB * B_BYTES;
    constexpr int PER_TILE = BG + 1;                              // requests per wave per K tile: the weights, one of the next run
    constexpr int FLY = NB - 3;                                   // tiles whose requests may be in flight at the end of a tile
    constexpr int NRD = TM + TN, NMM = TM * TN;                   // fragment reads and MFMAs per k-step
    static_assert(TM >= 1 && TN >= 1 && BG >= 1 && PER_TILE <= 4 && NB >= 4 && NB <= 6, "tile geometry");
    static_assert(RUN_LOADS <= 8 - FLY, "the next run is requested in the first K tiles of a slice and must have landed by the last");
    static_assert((RUN_LOADS * NW - 1) * 1024 >= RUN_PIX * PITCH, "the run buffer's last KB is the zero operand");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
    __shared__ __attribute__((aligned(1024))) unsigned char lds[LDS_BYTES];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave / WGN, wn = wave % WGN;
    const int W = p.W, HW = p.H * p.W, C = p.C;

    // consecutive workgroup ids go to different XCDs; give each XCD a contiguous run of tiles
    const int nblk = p.nblk_m * p.nblk_n;
    int bid = blockIdx.x;
    {
        const int per = nblk / NUM_XCD, main = per * NUM_XCD;
        if (bid < main) bid = (bid % NUM_XCD) * per + bid / NUM_XCD;
    }
    const int bm = bid / p.nblk_n, bn = bid - bm * p.nblk_n;
    const int m0 = bm * BM, n0 = bn * BN;

    const u32x4 dx = make_desc(p.x, p.x_bytes);
    const u32x4 dw = make_desc(p.w, p.w_bytes);
    const uint32_t lds_a = lds_addr_of(lds);
    const int frow = lane & 31, fhalf = lane >> 5;

    // ---- epilogue operands first (they are then the oldest requests in flight and never in the way of a count)
    const int epix = lane & 31, ehalf = lane >> 5;
    const Epilogue &e = p.epi;
    constexpr int LPR = WTN / 8;                   // lanes per output row of the wave tile (16 bytes of bf16 each)
    constexpr int RPP = 64 / LPR;                  // rows per row-wise pass
    constexpr int NPASS = WTM / RPP;
    constexpr int POSN = WTN / 4;                  // 16-byte fp32 positions per parked row
    constexpr int RP = 16 / POSN > 0 ? 16 / POSN : 1;   // parked rows per 256 bytes (all 64 banks)
    const int rr = lane / LPR, pp = lane % LPR;
    f32x4 bias_r[TN][4];
    u32x4 res_r[NPASS];
    uint32_t y_off[NPASS];                         // byte offset of the lane's 8 channels in pass q, or out of range
    int pA[NPASS];                                 // parked position read first in pass q
    const uint32_t y_bytes = p.y_bytes;
    {
        const bool has_res = e.t_op >= 0;
        // absent operands get an empty descriptor: every load then returns zeros without touching memory
        const rsrc_t rb = make_rsrc(e.has_bias ? e.bias_ptr : p.w, e.has_bias ? (uint32_t)p.N * 4u : 0u);
        const rsrc_t rres = make_rsrc(has_res ? e.t_ptr : p.w, has_res ? y_bytes : 0u);
        const int nb = n0 + wn * WTN + 4 * ehalf;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = nb + j * 32 + 8 * g;
                bias_r[j][g] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rb, n < p.N ? (uint32_t)n * 4u : OOB, 0, 0));
            }
#pragma unroll
        for (int q = 0; q < NPASS; ++q) {
            const int row = q * RPP + rr;
            const int key = (row / RP) & (POSN - 1);
            pA[q] = 2 * pp + (key & 1);
            const int cc = pp ^ (key >> 1);                  // 8-channel chunk this lane finishes in pass q
            const int m = m0 + wm * WTM + row, n = n0 + wn * WTN + cc * 8;
            y_off[q] = (m < p.M && n < p.N) ? (uint32_t)(((int64_t)m * p.ys_p + n) * 2) : OOB;
            res_r[q] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rres, y_off[q], 0, 0));
        }
    }

    // ---- request state.  Run: load k of the wave fills LDS units 64*(RUN_LOADS*wave + k) + lane of a run buffer;
    // unit u is 16-byte chunk u % 9 of run pixel u / 9 (chunk 8: padding; it fetches chunk 7 again rather than
    // nothing, lanes out of range in every request being slower than the 16 bytes they save).  Run pixel q is
    // flat input pixel m0 - W - 1 + q; outside the tensor or past the run: out of range, zeros.
    const int run_len = BM + 2 * W + 2;
    uint32_t r_voff[RUN_LOADS];
#pragma unroll
    for (int k = 0; k < RUN_LOADS; ++k) {
        const uint32_t u = (uint32_t)(64 * (RUN_LOADS * wave + k) + lane);
        const uint32_t px = u / 9u, c = u - 9u * px;
        const int q = m0 - W - 1 + (int)px;
        const bool ok = (int)px < run_len && q >= 0 && q < p.M;
        r_voff[k] = ok ? (uint32_t)((int64_t)q * C * 2) + (c < 8u ? c : 7u) * 16u : OOB;
    }
    // weights: lane l of load j fills row wave*8*BG + 8j + (l >> 3), position l & 7, with chunk position ^ key(row)
    uint32_t b_voff[BG];
    {
        const int r8 = lane >> 3, pos = lane & 7;
#pragma unroll
        for (int j = 0; j < BG; ++j) {
            const int row = wave * 8 * BG + 8 * j + r8;
            const int chunk = pos ^ ((row >> 1) & 7);
            int n = n0 + row;
            if (n > p.N - 1) n = p.N - 1;          // rows past N are computed on valid memory and never stored
            b_voff[j] = (uint32_t)((int64_t)n * p.Kp * 2) + chunk * 16;
        }
    }
    const int nsl = C / 64, NT = nsl * 9;
    // weight tile of K tile u = (slice s, tap tp): K offset tp*C + 64*s
    auto issue_b = [&](int d, int stage, int s, int tp, bool live) {
        dma16(dw, lds_a + B_OFF + stage * B_BYTES + (wave * BG + d) * 1024, live ? b_voff[d < BG ? d : 0] : OOB, live ? (uint32_t)((tp * C + 64 * s) * 2) : 0u);
    };
    // (a request that is only there to keep the count goes out of range, which writes zeros: it is aimed at the last
    // KB of the buffer, which lies past every run and holds nothing but such zeros)
    auto issue_r = [&](int k, int buf, int s, bool live) {
        dma16(dx, lds_a + buf * RUN_BYTES + (k < RUN_LOADS ? RUN_LOADS * wave + k : RUN_LOADS * NW - 1) * 1024,
              (live && k < RUN_LOADS) ? r_voff[k < RUN_LOADS ? k : 0] : OOB, live ? (uint32_t)(s * 128) : 0u);
    };

    // ---- prologue: run of slice 0, weight tiles 0 .. NB-2 (on their way while the lane state below is set up)
#pragma unroll
    for (int k = 0; k < RUN_LOADS; ++k) issue_r(k, 0, 0, true);
    // (each weight tile goes out with as many requests as a K tile of the loop issues, padded with ones that only
    // count, so that the loop's wait counts hold from its first tile on)
#pragma unroll
    for (int u = 0; u < NB - 1; ++u) {
#pragma unroll
        for (int d = 0; d < BG; ++d) issue_b(d, u, 0, u, u < NT);
#pragma unroll
        for (int d = BG; d < PER_TILE; ++d) issue_r(RUN_LOADS, 0, 0, false);
    }

    // ---- the lane's pixels: fragment base address in a run buffer, tap validity
    uint32_t fa[TM], tmask[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int j = wm * WTM + 32 * i + frow;
        fa[i] = (uint32_t)(j * PITCH + fhalf * 16);
        const int m = m0 + j;
        const int img = (int)fast_div((uint32_t)m, (uint32_t)HW, p.div_ohw_mul, p.div_ohw_sh);
        const int pix = m - img * HW;
        const int oh = (int)fast_div((uint32_t)pix, (uint32_t)W, p.div_ow_mul, p.div_ow_sh), ow = pix - oh * W;
        const uint32_t rows = (oh > 0 ? 0x007u : 0u) | 0x038u | (oh < p.H - 1 ? 0x1c0u : 0u);
        const uint32_t cols = (ow > 0 ? 0x049u : 0u) | 0x092u | (ow < W - 1 ? 0x124u : 0u);
        tmask[i] = m < p.M ? (rows & cols) : 0u;
    }
    // weight fragments: row frow of a 32-row MFMA tile of the wave's channels, chunk 2*ks + fhalf, swizzled
    uint32_t fb[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) fb[ks] = (uint32_t)(B_OFF + (wn * WTN + frow) * 128 + (((2 * ks + fhalf) ^ ((frow >> 1) & 7)) << 4));

    wait_vm<FLY * PER_TILE>();                      // all but weight tiles 2 .. NB-2
    wg_barrier();

    f32x16 acc[TM][TN];
    u32x4 fx[2][TM], fw[2][TN];
    uint32_t a0[TM], a0n[TM];                       // pixel fragment addresses of this K tile's tap and of the next one's
    // fragment read r of a k-step: r < TM: pixels, tile r; else weights, tile r - TM
    auto frag_read = [&](int r, int set, int ks, uint32_t bstage, const uint32_t *pix) {
        if (r < TM) fx[set][r < TM ? r : 0] = *(const u32x4 *)(lds + pix[r < TM ? r : 0] + ks * 32);
        else fw[set][r >= TM ? r - TM : 0] = *(const u32x4 *)(lds + fb[ks] + bstage + (r >= TM ? r - TM : 0) * 4096);
    };
    // addresses of tap tp in the run buffer at byte offset rb
    auto tap_addr = [&](int tp, uint32_t rb, uint32_t *out) {
        const uint32_t toff = (uint32_t)(((tp / 3) * W + tp % 3) * PITCH) + rb;
        const uint32_t zoff = rb + (uint32_t)(RUN_BYTES - 128);
#pragma unroll
        for (int i = 0; i < TM; ++i) out[i] = ((tmask[i] >> tp) & 1u) ? fa[i] + toff : zoff;
    };
    tap_addr(0, 0u, a0);
#pragma unroll
    for (int r = 0; r < NRD; ++r) frag_read(r, 0, 0, 0u, a0);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    __builtin_amdgcn_sched_barrier(0);

    int st_cur = 0;                                 // weight stage of the current K tile: u % NB
#pragma unroll 1
    for (int s = 0; s < nsl; ++s) {
        const uint32_t rb = (uint32_t)((s & 1) * RUN_BYTES), rbn = (uint32_t)(((s + 1) & 1) * RUN_BYTES);
        const bool more = s + 1 < nsl;
#pragma unroll
        for (int tp = 0; tp < 9; ++tp) {
            // K tile u = 9s + tp; on entry the barrier of this tile has been passed, the weight tiles u and u+1 and
            // this slice's run have landed, and the fragments of k-step 0 are in register set 0
            const int st_next = st_cur + 1 == NB ? 0 : st_cur + 1, st_iss = st_cur == 0 ? NB - 1 : st_cur - 1;
            const uint32_t bcur = (uint32_t)(st_cur * B_BYTES), bnext = (uint32_t)(st_next * B_BYTES);
            // this tile's requests: weight tile u + NB - 1 into the stage tile u - 1 has left, one piece of the next run
            const int tb = (tp + NB - 1) % 9, sb = s + (tp + NB - 1) / 9;
            const bool blive = sb < nsl;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const int set = ks & 1;
                int r = 0;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fw[set][j]), __builtin_bit_cast(bf16x8, fx[set][i]),
                                                                           acc[i][j], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                        // behind the MFMA: one fragment read of the next k-step (of the next tile after k-step 3) ...
                        if (r < NRD) { frag_read(r, set ^ 1, ks == 3 ? 0 : ks + 1, ks == 3 ? bnext : bcur, ks == 3 ? a0n : a0); ++r; }
                        // ... and, behind the first MFMA of k-step d, request d of the tile
                        if (i == 0 && j == 0) {
                            if (ks < BG) issue_b(ks, st_iss, sb, tb, blive);
                            else if (ks == BG) issue_r(tp, (s + 1) & 1, s + 1, more);
                            if (ks == 2) tap_addr(tp == 8 ? 0 : tp + 1, tp == 8 ? rbn : rb, a0n);   // the next tile's pixels
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
#pragma unroll
                for (; r < NRD; ++r) frag_read(r, set ^ 1, ks == 3 ? 0 : ks + 1, ks == 3 ? bnext : bcur, ks == 3 ? a0n : a0);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i) a0[i] = a0n[i];
            st_cur = st_next;
            wait_vm<FLY * PER_TILE>();              // everything but the last FLY tiles' requests: weight tile u + 2 has landed
            wg_barrier();
        }
    }
    wait_vm<0>();                                   // the trailing out-of-range requests
    wg_barrier();

    // ---- epilogue.  All waves are past their last fragment read; each wave works alone in its own piece of LDS.
    constexpr int WBYTES = WTM * WTN * 4, ROWB = WTN * 4;
    static_assert(NW * WBYTES <= LDS_BYTES, "LDS must hold the waves' parked tiles");
    unsigned char *park = lds + wave * WBYTES;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int row = i * 32 + epix;
                const int c = j * 8 + 2 * g + ehalf;                    // 4-channel chunk of the row
                const int pos = c ^ ((row / RP) & (POSN - 1));
                f32x4 v;
#pragma unroll
                for (int k = 0; k < 4; ++k) v[k] = acc[i][j][4 * g + k] + bias_r[j][g][k];
                *(f32x4 *)(park + row * ROWB + pos * 16) = v;
            }
    wave_lds_exchange();
    const rsrc_t ry = make_rsrc(p.y, y_bytes);
    const float lo = e.relu_last ? 0.0f : -INFINITY;
#pragma unroll
    for (int q = 0; q < NPASS; ++q) {
        const int row = q * RPP + rr;
        const f32x4 a = *(const f32x4 *)(park + row * ROWB + pA[q] * 16);
        const f32x4 b = *(const f32x4 *)(park + row * ROWB + (pA[q] ^ 1) * 16);
        const u32x4 rs = res_r[q];
        float v[8];
#pragma unroll
        for (int k = 0; k < 4; ++k) { v[k] = a[k]; v[4 + k] = b[k]; }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v[2 * k] += __uint_as_float(rs[k] << 16);
            v[2 * k + 1] += __uint_as_float(rs[k] & 0xffff0000u);
        }
        u32x4 o;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            o[k] = pack_bf16x2(fmaxf(v[2 * k], lo), fmaxf(v[2 * k + 1], lo));
        __builtin_amdgcn_raw_buffer_store_b128(o, ry, y_off[q], 0, 0);
    }
#endif
}

// The same contraction with K split over the waves: four waves, each multiplying the *whole* BM x BN tile for one of
// the four k-steps of every K tile (BM/32 + BN/32 fragment reads for BM/32 * BN/32 MFMAs: 0.75 per MFMA for 128x64,
// where a 32x32 wave tile needs two), and the four partial accumulator tiles summed through LDS at the end.
// Needs an even number of channel slices (the two fragment register sets alternate from K tile to K tile and a
// slice has nine).
template <int BM, int BN, int NB>
__global__ __launch_bounds__(256) void conv3x3_run_ks_kernel(const IgemmParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub; the body uses gfx950-only builtins
    constexpr int NW = 4;
    constexpr int TM = BM / 32, TN = BN / 32;
    constexpr int RUN_PIX = BM + 2 * RUN_W_MAX + 2;
    constexpr int RUN_LOADS = ((RUN_PIX * 9 + 63) / 64 + NW - 1) / NW;
    constexpr int RUN_BYTES = RUN_LOADS * NW * 1024;
    constexpr int BG = BN / (8 * NW);
    constexpr int B_BYTES = BN * 128;
    constexpr int B_OFF = 2 * RUN_BYTES;
    constexpr int PBYTES = BM * BN * 4;                           // one partial accumulator tile, fp32
    constexpr int LDS_BYTES = NW * PBYTES > B_OFF + NB * B_BYTES ? NW * PBYTES : B_OFF + NB * B_BYTES;
    constexpr int FLY = NB - 3;                                   // tiles whose requests may be in flight at the end of a tile
    constexpr int NR = (RUN_LOADS + 7 - FLY) / (8 - FLY);         // pieces of the next run requested per K tile
    constexpr int PER_TILE = BG + NR;
    constexpr int NRD = TM + TN, NMM = TM * TN;
    static_assert(BN == 64, "the finishing pass assumes rows of 64 channels");
    static_assert(BG >= 1 && 2 * PER_TILE <= NMM && NRD <= NMM - 1 && NB >= 4 && NB <= 6, "tile geometry");
    static_assert(NR * (8 - FLY) >= RUN_LOADS, "the next run is requested in the first K tiles of a slice and must have landed by the last");
    static_assert((RUN_LOADS * NW - 1) * 1024 >= RUN_PIX * PITCH, "the run buffer's last KB is the zero operand");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
    __shared__ __attribute__((aligned(1024))) unsigned char lds[LDS_BYTES];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);     // also the wave's k-step
    const int W = p.W, HW = p.H * p.W, C = p.C;

    const int nblk = p.nblk_m * p.nblk_n;
    int bid = blockIdx.x;
    {
        const int per = nblk / NUM_XCD, main = per * NUM_XCD;
        if (bid < main) bid = (bid % NUM_XCD) * per + bid / NUM_XCD;
    }
    // Channel-tile-major order when the weights of all channel tiles (N x K) would not stay in an XCD's L2 beside the
    // activations: each XCD then multiplies every pixel tile by one or two channel tiles' weights.
    int bm, bn;
    if (p.nmajor) { bn = bid / p.nblk_m; bm = bid - bn * p.nblk_m; }
    else { bm = bid / p.nblk_n; bn = bid - bm * p.nblk_n; }
    const int m0 = bm * BM, n0 = bn * BN;

    const u32x4 dx = make_desc(p.x, p.x_bytes);
    const u32x4 dw = make_desc(p.w, p.w_bytes);
    const uint32_t lds_a = lds_addr_of(lds);
    const int frow = lane & 31, fhalf = lane >> 5;

    // ---- operands of the finishing pass first: thread t finishes, in pass q, row 32q + t/8, channels 8*(t%8) .. +7
    const Epilogue &e = p.epi;
    constexpr int NPASS = BM / 32;
    const int rr = t >> 3, pp = t & 7;
    f32x4 bias_lo, bias_hi;
    u32x4 res_r[NPASS];
    uint32_t y_off[NPASS];
    const uint32_t y_bytes = p.y_bytes;
    {
        const bool has_res = e.t_op >= 0;
        const rsrc_t rb = make_rsrc(e.has_bias ? e.bias_ptr : p.w, e.has_bias ? (uint32_t)p.N * 4u : 0u);
        const rsrc_t rres = make_rsrc(has_res ? e.t_ptr : p.w, has_res ? y_bytes : 0u);
        const int n = n0 + 8 * pp;
        bias_lo = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rb, n < p.N ? (uint32_t)n * 4u : OOB, 0, 0));
        bias_hi = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rb, n < p.N ? (uint32_t)n * 4u + 16u : OOB, 0, 0));
#pragma unroll
        for (int q = 0; q < NPASS; ++q) {
            const int m = m0 + 32 * q + rr;
            y_off[q] = (m < p.M && n < p.N) ? (uint32_t)(((int64_t)m * p.ys_p + n) * 2) : OOB;
            res_r[q] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rres, y_off[q], 0, 0));
        }
    }

    // ---- request state (as in the kernel above)
    const int run_len = BM + 2 * W + 2;
    uint32_t r_voff[RUN_LOADS];
#pragma unroll
    for (int k = 0; k < RUN_LOADS; ++k) {
        const uint32_t u = (uint32_t)(64 * (RUN_LOADS * wave + k) + lane);
        const uint32_t px = u / 9u, c = u - 9u * px;
        const int q = m0 - W - 1 + (int)px;
        const bool ok = (int)px < run_len && q >= 0 && q < p.M;
        r_voff[k] = ok ? (uint32_t)((int64_t)q * C * 2) + (c < 8u ? c : 7u) * 16u : OOB;
    }
    uint32_t b_voff[BG];
    {
        const int r8 = lane >> 3, pos = lane & 7;
#pragma unroll
        for (int j = 0; j < BG; ++j) {
            const int row = wave * 8 * BG + 8 * j + r8;
            const int chunk = pos ^ ((row >> 1) & 7);
            int n = n0 + row;
            if (n > p.N - 1) n = p.N - 1;
            b_voff[j] = (uint32_t)((int64_t)n * p.Kp * 2) + chunk * 16;
        }
    }
    const int nsl = C / 64, NT = nsl * 9;
    auto issue_b = [&](int d, int stage, int s, int tp, bool live) {
        dma16(dw, lds_a + B_OFF + stage * B_BYTES + (wave * BG + d) * 1024, live ? b_voff[d < BG ? d : 0] : OOB, live ? (uint32_t)((tp * C + 64 * s) * 2) : 0u);
    };
    auto issue_r = [&](int k, int buf, int s, bool live) {
        dma16(dx, lds_a + buf * RUN_BYTES + (k < RUN_LOADS ? RUN_LOADS * wave + k : RUN_LOADS * NW - 1) * 1024,
              (live && k < RUN_LOADS) ? r_voff[k < RUN_LOADS ? k : 0] : OOB, live ? (uint32_t)(s * 128) : 0u);
    };
#pragma unroll
    for (int k = 0; k < RUN_LOADS; ++k) issue_r(k, 0, 0, true);
    // (each weight tile goes out with as many requests as a K tile of the loop issues, padded with ones that only
    // count, so that the loop's wait counts hold from its first tile on)
#pragma unroll
    for (int u = 0; u < NB - 1; ++u) {
#pragma unroll
        for (int d = 0; d < BG; ++d) issue_b(d, u, 0, u, u < NT);
#pragma unroll
        for (int d = BG; d < PER_TILE; ++d) issue_r(RUN_LOADS, 0, 0, false);
    }

    // ---- the lane's pixels (one per 32-row tile of the block): fragment address of the wave's k-step, tap validity
    uint32_t fa[TM], tmask[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int j = 32 * i + frow;
        fa[i] = (uint32_t)(j * PITCH + fhalf * 16 + wave * 32);
        const int m = m0 + j;
        const int img = (int)fast_div((uint32_t)m, (uint32_t)HW, p.div_ohw_mul, p.div_ohw_sh);
        const int pix = m - img * HW;
        const int oh = (int)fast_div((uint32_t)pix, (uint32_t)W, p.div_ow_mul, p.div_ow_sh), ow = pix - oh * W;
        const uint32_t rows = (oh > 0 ? 0x007u : 0u) | 0x038u | (oh < p.H - 1 ? 0x1c0u : 0u);
        const uint32_t cols = (ow > 0 ? 0x049u : 0u) | 0x092u | (ow < W - 1 ? 0x124u : 0u);
        tmask[i] = m < p.M ? (rows & cols) : 0u;
    }
    const uint32_t fbk = (uint32_t)(B_OFF + frow * 128 + (((2 * wave + fhalf) ^ ((frow >> 1) & 7)) << 4));

    wait_vm<FLY * PER_TILE>();                      // all but weight tiles 2 .. NB-2
    wg_barrier();

    f32x16 acc[TM][TN];
    u32x4 fx[2][TM], fw[2][TN];
    uint32_t an[TM], an2[TM];                       // pixel fragment addresses of the next K tile and of the one after it
    auto frag_read = [&](int r, int set, uint32_t bstage, const uint32_t *pix) {
        if (r < TM) fx[set][r < TM ? r : 0] = *(const u32x4 *)(lds + pix[r < TM ? r : 0]);
        else fw[set][r >= TM ? r - TM : 0] = *(const u32x4 *)(lds + fbk + bstage + (r >= TM ? r - TM : 0) * 4096);
    };
    auto tap_addr = [&](int tp, uint32_t rb, uint32_t *out) {
        const uint32_t toff = (uint32_t)(((tp / 3) * W + tp % 3) * PITCH) + rb;
        const uint32_t zoff = rb + (uint32_t)(RUN_BYTES - 128);
#pragma unroll
        for (int i = 0; i < TM; ++i) out[i] = ((tmask[i] >> tp) & 1u) ? fa[i] + toff : zoff;
    };
    tap_addr(0, 0u, an);
#pragma unroll
    for (int r = 0; r < NRD; ++r) frag_read(r, 0, 0u, an);
    tap_addr(1, 0u, an);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    __builtin_amdgcn_sched_barrier(0);

    int st_cur = 0;                                 // weight stage of the current K tile: u % NB
#pragma unroll 1
    for (int s2 = 0; s2 < nsl; s2 += 2) {
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            const int s = s2 + hh;
            const uint32_t rb = (uint32_t)(hh * RUN_BYTES), rbn = (uint32_t)((hh ^ 1) * RUN_BYTES);   // slice s lives in buffer s % 2
            const bool more = s + 1 < nsl;
#pragma unroll
            for (int tp = 0; tp < 9; ++tp) {
                // on entry: the barrier of K tile u = 9s + tp has been passed, weight tiles u and u+1 and this slice's
                // run have landed, the wave's fragments of tile u are in register set u % 2, an[] addresses tile u+1
                const int set = (hh * 9 + tp) & 1;
                const int st_next = st_cur + 1 == NB ? 0 : st_cur + 1, st_iss = st_cur == 0 ? NB - 1 : st_cur - 1;
                const uint32_t bnext = (uint32_t)(st_next * B_BYTES);
                const int tb = (tp + NB - 1) % 9, sb = s + (tp + NB - 1) / 9;
                const bool blive = sb < nsl;
                int q = 0;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fw[set][j]), __builtin_bit_cast(bf16x8, fx[set][i]),
                                                                           acc[i][j], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                        // behind the MFMA: one fragment read of the next tile, or the addresses of the tile after it,
                        // and after every second MFMA one request
                        if (q < NRD) frag_read(q, set ^ 1, bnext, an);
                        else if (q == NRD) tap_addr((tp + 2) % 9, tp >= 7 ? rbn : rb, an2);
                        if ((q & 1) && (q >> 1) < PER_TILE) {
                            const int d = q >> 1;
                            if (d < BG) issue_b(d, st_iss, sb, tb, blive);
                            else issue_r(NR * tp + (d - BG), (s + 1) & 1, s + 1, more);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                        ++q;
                    }
#pragma unroll
                for (int i = 0; i < TM; ++i) an[i] = an2[i];
                st_cur = st_next;
                wait_vm<FLY * PER_TILE>();          // everything but the last FLY tiles' requests: weight tile u + 2 has landed
                wg_barrier();
            }
        }
    }
    wait_vm<0>();
    wg_barrier();

    // ---- the four partial tiles go to LDS (16-byte chunks of a row XOR-swizzled by the row) ...
    {
        unsigned char *park = lds + wave * PBYTES;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int row = i * 32 + frow;
                    const int c = j * 8 + 2 * g + fhalf;                 // 4-channel chunk of the row, 0..15
                    f32x4 v;
#pragma unroll
                    for (int k = 0; k < 4; ++k) v[k] = acc[i][j][4 * g + k];
                    *(f32x4 *)(park + row * (BN * 4) + ((c ^ (row & 15)) << 4)) = v;
                }
    }
    RL_WAIT_LGKM0;
    wg_barrier();
    // ... and are summed row-wise: k-steps 0, 1, 2, 3 in that order, then bias, residual, ReLU, one rounding
    const rsrc_t ry = make_rsrc(p.y, y_bytes);
    const float lo = e.relu_last ? 0.0f : -INFINITY;
#pragma unroll
    for (int q = 0; q < NPASS; ++q) {
        const int row = 32 * q + rr;
        float v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const unsigned char *prow = lds + w * PBYTES + row * (BN * 4);
            const f32x4 a = *(const f32x4 *)(prow + (((2 * pp) ^ (row & 15)) << 4));
            const f32x4 b = *(const f32x4 *)(prow + (((2 * pp + 1) ^ (row & 15)) << 4));
#pragma unroll
            for (int k = 0; k < 4; ++k) { v[k] += a[k]; v[4 + k] += b[k]; }
        }
        const u32x4 rs = res_r[q];
#pragma unroll
        for (int k = 0; k < 4; ++k) { v[k] += bias_lo[k]; v[4 + k] += bias_hi[k]; }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v[2 * k] += __uint_as_float(rs[k] << 16);
            v[2 * k + 1] += __uint_as_float(rs[k] & 0xffff0000u);
        }
        u32x4 o;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            o[k] = pack_bf16x2(fmaxf(v[2 * k], lo), fmaxf(v[2 * k + 1], lo));
        __builtin_amdgcn_raw_buffer_store_b128(o, ry, y_off[q], 0, 0);
    }
#endif
}

template <int BM, int BN, int WGM, int WGN, int NB>
static hipError_t launch_run(const IgemmParams &p0, hipStream_t s)
{
    IgemmParams p = p0;
    p.nblk_m = (p.M + BM - 1) / BM;
    p.nblk_n = (p.N + BN - 1) / BN;
    int64_t nblk = (int64_t)p.nblk_m * p.nblk_n;
    if (nblk <= 0 || nblk > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL((conv3x3_run_kernel<BM, BN, WGM, WGN, NB>), dim3((unsigned)nblk), dim3(WGM * WGN * 64), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_conv3x3_run(const IgemmParams &p, const IgemmLaunch &l, hipStream_t s)
{
    // the kernel's addressing assumes exactly this geometry
    const int64_t HW = (int64_t)p.H * p.W;
    if (p.in_dtype != DT_BF16 || p.y_dtype != DT_BF16 || p.x2 || p.C < 64 || p.C % 64 != 0 || p.KH != 3 || p.KW != 3 || p.sh != 1 || p.sw != 1 ||
        p.ph != 1 || p.pw != 1 || p.OH != p.H || p.OW != p.W || p.W < 1 || p.W > RUN_W_MAX || p.K != 9 * p.C || p.Kp != p.K || p.N % 8 != 0 ||
        HW < 1 || p.M % HW != 0 || p.OHW != HW || p.xs_c != 1 || p.xs_w != p.C || p.xs_h != (int64_t)p.W * p.C || p.xs_n != HW * p.C ||
        p.ys_c != 1 || p.ys_n != HW * p.ys_p || (uint64_t)p.M * p.C * 2 >= 0x7fffffffull || p.x_bytes != (uint32_t)((uint64_t)p.M * p.C * 2) ||
        p.w_bytes < (uint32_t)((uint64_t)p.N * p.Kp * 2) || !p.epi.simple || (p.epi.has_bias && p.epi.bias_dtype != DT_F32) ||
        (p.epi.t_op >= 0 && (p.epi.t_op != E_ADD || p.epi.t_dtype != DT_BF16)) || (p.epi.rest_n != 0 && !p.epi.relu_last))
        return hipErrorInvalidValue;
    switch (l.tile) {
    case TILE_256x128: return launch_run<256, 128, 4, 2, 4>(p, s);      // 160 KB of LDS with four stages
    case TILE_128x128: return launch_run<128, 128, 2, 4, 5>(p, s);
    case TILE_128x64:
        if (l.run == 2) {
            if (p.C % 128 != 0) return hipErrorInvalidValue;      // each of the four waves takes whole k-steps of a 128-channel pair of slices
            IgemmParams q = p;
            q.nblk_m = (p.M + 127) / 128;
            q.nblk_n = (p.N + 63) / 64;
            hipLaunchKernelGGL((conv3x3_run_ks_kernel<128, 64, 6>), dim3((unsigned)(q.nblk_m * q.nblk_n)), dim3(256), 0, s, q);
            return hipGetLastError();
        }
        return launch_run<128, 64, 4, 2, 6>(p, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace rl

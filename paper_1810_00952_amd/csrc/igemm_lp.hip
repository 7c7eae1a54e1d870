// Implicit-GEMM contraction for gfx950, bf16 in / fp32 accumulate, with the
// output pixel on the lane axis of the MFMA result and a wave-private epilogue.
//
//   C[m, n] = sum_k A[m, k] * Wp[n, k],  m = (image, oh, ow), n = out channel,
//   k = (kh, kw, c)
//
// MFMA operand roles: the 32x32x16 instruction computes D[i][j] with lane l
// holding column j = l % 32 and rows i = 8*(r/4) + 4*(l/32) + r%4 in its 16
// result registers r.  Weights are fed as the row operand (i = channel) and
// activations as the column operand (j = pixel): a lane then owns one pixel
// and, per group of four registers, four consecutive channels.
//
// Operand tiles travel global -> LDS by direct loads (16 bytes per lane, one
// instruction fills 8 rows of 128 bytes), STAGES tiles deep.  Rows are 128
// bytes (one K tile of 64 bf16), unpadded; bank conflicts are avoided by
// choosing which global chunk a lane fetches: position q of row r holds chunk
// q ^ ((r >> 1) & 7).  Padding taps and rows past M get a buffer offset outside
// the descriptor's range, for which the hardware writes zeros into LDS without
// touching memory.
//
// K loop, one barrier per K tile.  With four stages, at the barrier of tile t
// the tiles t and t+1 have landed, t+2 is in flight and t+3 is issued into the
// stage tile t-1 just left; fragments of k-step s+1 are read from LDS into a
// second register set before the MFMAs of k-step s are issued, and the first
// fragments of tile t+1 are read before the barrier of t+1, so the matrix
// pipeline does not drain at the barrier.  The direct loads of a tile are not
// issued in one burst but one at a time between the MFMAs: a wave whose
// vector-memory queue is full stalls at the load, and the MFMAs behind it in
// program order would wait with it.  With three stages (smaller LDS
// footprint, two workgroups per CU) tile t+2 is issued at the barrier of t and
// fragment prefetch stays inside a tile.  Each stage is its own LDS array so
// that the compiler's wait-count insertion can tell direct loads into one
// stage from fragment reads of another; the waits on the direct loads
// themselves are explicit (s_waitcnt vmcnt), which is why every K-loop body
// issues the same number of them (issues past the last tile are sent out of
// range and cost no memory traffic).  The epilogue's operands (bias, residual)
// are requested right behind the first tiles, so their latency hides under
// the K loop; the first two waits count them in.
//
// Epilogue: after one barrier the stages are free and every wave owns a
// private piece of them.  It adds the bias to its accumulators and parks them
// there as fp32, 16 bytes (4 channels of one pixel) per lane and store, chunk
// positions XOR-swizzled by the row so that both the stores and the reads
// below are bank-conflict free.  It then reads them back row-wise -- a lane
// gets 8 consecutive channels of one pixel, the lanes of a row cover the row
// -- adds the residual (fetched with the same row-wise 16-byte accesses),
// applies ReLU, rounds once to bf16 and stores 16 bytes: whole output rows
// per instruction instead of 8-byte fragments scattered over 32 rows.
//
// Preconditions (checked by the planner): bf16 operands and output; channel-
// last activations with C a multiple of 64 so that a K tile lies inside one
// filter tap; K a multiple of 64; KH*KW <= 32; output rows contiguous in n with
// N a multiple of 8; epilogue of the form [f32 bias] [+ bf16 residual] [relu];
// every tensor below 2 GiB.
#include "device_utils.h"

namespace rl {

namespace {

typedef __amdgpu_buffer_rsrc_t rsrc_t;
#define RL_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

__device__ __forceinline__ rsrc_t make_rsrc(const void *ptr, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc((void *)ptr, 0, bytes, 0x00020000);   // raw buffer, untyped dwords
}

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding:
// vmcnt = bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)
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

// n / d for n < 2^31 with the host-computed multiplier (d >= 2) or d == 1
__device__ __forceinline__ uint32_t fast_div(uint32_t n, uint32_t d, uint32_t mul, uint32_t sh)
{
    return d == 1 ? n : (__umulhi(n, mul) >> sh);
}

constexpr int NUM_XCD = 8;
constexpr uint32_t OOB = 0x80000000u;

}  // namespace

// The workgroup's work: tile number bid_in of the contraction p.  YF32: the output is fp32 (no residual then).
// ANYACT: the operand-free steps behind bias and residual are any (up to eight, codes in the epilogue), not just one ReLU.
template <int BM, int BN, int WGM, int WGN, int STAGES, bool YF32 = false, bool ANYACT = false>
__device__ __forceinline__ void igemm_lp_body(const IgemmParams &p, const int bid_in)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub; the body uses gfx950-only builtins
    constexpr int NW = WGM * WGN;                   // waves: four (one per SIMD) or eight (two per SIMD)
    static_assert(NW == 4 || NW == 8, "four or eight waves");
    static_assert(STAGES == 3 || STAGES == 4, "three or four stages");
    constexpr int BKE = 64;                         // K elements per tile (128 bytes per row)
    constexpr int WTM = BM / WGM, WTN = BN / WGN;   // wave tile: pixels x channels
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int AG = BM / (8 * NW), BG = BN / (8 * NW);   // 8-row direct-load groups per wave
    static_assert(AG >= 1 && BG >= 1, "every wave requests rows of both operands");
    constexpr int LPT = AG + BG;                    // direct loads per wave per tile
    constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;

    __shared__ __attribute__((aligned(1024))) unsigned char st0[STAGE];
    __shared__ __attribute__((aligned(1024))) unsigned char st1[STAGE];
    __shared__ __attribute__((aligned(1024))) unsigned char st2[STAGE];
    __shared__ __attribute__((aligned(1024))) unsigned char st3[STAGES == 4 ? STAGE : 1024];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);   // wave-uniform by construction; keep it in an SGPR
    const int wm = wave / WGN, wn = wave % WGN;

    // consecutive workgroup ids go to different XCDs; give each XCD a contiguous run of tiles
    const int nblk = p.nblk_m * p.nblk_n;
    int bid = bid_in;
    {
        const int per = nblk / NUM_XCD, main = per * NUM_XCD;
        if (bid < main) bid = (bid % NUM_XCD) * per + bid / NUM_XCD;
    }
    // within a run, channel tiles in groups of eight and pixel tiles fastest inside a group: the 32 workgroups an XCD holds
    // at a time then share 4 x 8 operand tiles instead of 1 x 32 (wide matrices: 4096^3 952 -> 1015 TFLOP/s; with at most
    // eight channel tiles, as in the convolutional graphs, the order is the plain one)
    int bm, bn;
    {
        constexpr int GN = 8;
        const int grp = bid / (GN * p.nblk_m);
        const int within = bid - grp * GN * p.nblk_m;
        const int gw = min(GN, p.nblk_n - grp * GN);
        bm = within / gw; bn = grp * GN + (within - bm * gw);
    }
    const int m0 = bm * BM, n0 = bn * BN;

    // The activation descriptor starts `halo` bytes before x so that the per-lane offset of a
    // row's tap (0,0) -- which lies above/left of the image for border pixels -- is never negative.
    const uint32_t halo = (uint32_t)(((int64_t)p.ph * p.xs_h + (int64_t)p.pw * p.xs_w) * 2);
    const rsrc_t rx = make_rsrc((const char *)p.x - halo, p.x_bytes + halo);
    const rsrc_t rw = make_rsrc(p.w, p.w_bytes);

    // ---- per-lane direct-load state.  Lane l of a group writes LDS row (l >> 3), position (l & 7).
    const int r8 = lane >> 3, pos = lane & 7;
    uint32_t a_voff[AG], a_mask[AG], b_voff[BG];
#pragma unroll
    for (int i = 0; i < AG; ++i) {
        const int row = wave * 8 * AG + 8 * i + r8;
        const int chunk = pos ^ ((row >> 1) & 7);
        const int m = m0 + row;
        uint32_t mask = 0;
        int64_t off = 0;
        if (m < p.M) {
            const int img = (int)fast_div((uint32_t)m, (uint32_t)p.OHW, p.div_ohw_mul, p.div_ohw_sh);
            const int pix = m - img * p.OHW;
            const int oh = (int)fast_div((uint32_t)pix, (uint32_t)p.OW, p.div_ow_mul, p.div_ow_sh);
            const int ow = pix - oh * p.OW;
            const int ih0 = oh * p.sh - p.ph, iw0 = ow * p.sw - p.pw;
            // taps inside the image form a contiguous range of kh and of kw
            const int lo_h = max(0, -ih0), hi_h = max(lo_h, min(p.KH, p.H - ih0));
            const int lo_w = max(0, -iw0), hi_w = max(lo_w, min(p.KW, p.W - iw0));
            const uint32_t wmk = (uint32_t)(((1ull << hi_w) - 1) & ~((1ull << lo_w) - 1));
            const uint32_t rows = (uint32_t)(((1ull << (hi_h * p.KW)) - 1) & ~((1ull << (lo_h * p.KW)) - 1));
            mask = (wmk * p.tap_rep) & rows;      // tap_rep has bit kh*KW set for every kh: no carries, wmk < 2^KW
            off = ((int64_t)img * p.xs_n + (int64_t)ih0 * p.xs_h + (int64_t)iw0 * p.xs_w) * 2;
        }
        a_mask[i] = mask;
        // a K tile is two segments of 64 bytes, seg_stride bytes apart (64: one contiguous 128-byte run)
        a_voff[i] = (uint32_t)(off + halo) + (uint32_t)(chunk >> 2) * p.seg_stride + (uint32_t)(chunk & 3) * 16u;
    }
#pragma unroll
    for (int j = 0; j < BG; ++j) {
        const int row = wave * 8 * BG + 8 * j + r8;
        const int chunk = pos ^ ((row >> 1) & 7);
        int n = n0 + row;
        if (n > p.N - 1) n = p.N - 1;          // rows past N are computed on valid memory and never stored
        b_voff[j] = (uint32_t)((int64_t)n * p.Kp * 2) + chunk * 16;
    }

    // ---- wave-uniform K state of the tile to be issued next.  RL_TILE_BEGIN latches the scalars of
    // that tile and advances the state; RL_DMA(ST, d) then issues direct load d of the tile (A groups
    // first, then B groups) wherever the K loop wants it.
    const int nk = p.K / BKE;
    int f_kt = 0, f_c0 = 0, f_tap = 0, f_kh = 0, f_kw = 0;
    bool t_live;
    uint32_t t_soff_a, t_soff_b, t_tapbit;
#define RL_TILE_BEGIN                                                                                                 \
    {                                                                                                                 \
        t_live = f_kt < nk;                                                                                           \
        t_soff_b = t_live ? (uint32_t)(f_kt * BKE) * 2u : 0u;                                                         \
        t_tapbit = t_live ? (1u << f_tap) : 0u;                                                                       \
        t_soff_a = t_live ? (uint32_t)(((int64_t)f_kh * p.ts_h + (int64_t)f_kw * p.ts_w + f_c0) * 2) : 0u;            \
        ++f_kt;                                                                                                       \
        f_c0 += BKE;                                                                                                  \
        if (f_c0 >= p.C) {                                                                                            \
            f_c0 = 0;                                                                                                 \
            ++f_tap;                                                                                                  \
            if (++f_kw == p.KW) { f_kw = 0; ++f_kh; }                                                                 \
        }                                                                                                             \
    }
#define RL_DMA(ST, D)                                                                                                 \
    {                                                                                                                 \
        if ((D) < AG)                                                                                                 \
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rx, RL_LDS_PTR(ST + (wave * AG + (D)) * 1024), 16,               \
                                                     (a_mask[(D) < AG ? (D) : 0] & t_tapbit) ? a_voff[(D) < AG ? (D) : 0] : OOB, t_soff_a, 0, 0); \
        else                                                                                                          \
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, RL_LDS_PTR(ST + A_BYTES + (wave * BG + ((D) - AG)) * 1024), 16, \
                                                     t_live ? b_voff[(D) >= AG ? (D) - AG : 0] : OOB, t_soff_b, 0, 0); \
    }
#define RL_ISSUE(ST)                                                                                                  \
    {                                                                                                                 \
        RL_TILE_BEGIN                                                                                                 \
        _Pragma("unroll") for (int d = 0; d < LPT; ++d) RL_DMA(ST, d)                                                 \
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.0f;

    // ---- fragment addresses: row frow of a 32-row MFMA tile, chunk 2*ks + fhalf, swizzled
    const int frow = lane & 31, fhalf = lane >> 5;
    int f_off[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) f_off[ks] = frow * 128 + (((2 * ks + fhalf) ^ ((frow >> 1) & 7)) << 4);

    // A K tile is worked off in phases of four MFMAs (KSP k-steps each).  The fragments of a phase are
    // read into one of two register sets while the MFMAs of the phase before run from the other; the
    // tile's direct loads are spread between the MFMAs, one at a time, so that a full vector-memory
    // queue stalls the wave only while the matrix pipeline still has work.
    constexpr int NMMA = 4 * TM * TN;              // MFMAs per wave per K tile
    constexpr int KSP = 4 / (TM * TN);             // k-steps per phase
    constexpr int NPH = 4 / KSP;                   // phases per K tile
    static_assert(TM * TN == 1 || TM * TN == 2 || TM * TN == 4, "wave tile of one, two or four MFMA tiles");
    u32x4 fw[2][KSP][TN], fx[2][KSP][TM];
#define RL_LOADP(ST, PH, SET)                                                                                         \
    {                                                                                                                 \
        _Pragma("unroll") for (int s_ = 0; s_ < KSP; ++s_) {                                                          \
            _Pragma("unroll") for (int j = 0; j < TN; ++j)                                                            \
                fw[SET][s_][j] = *(const u32x4 *)(ST + A_BYTES + (wn * WTN + j * 32) * 128 + f_off[(PH) * KSP + s_]); \
            _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                            \
                fx[SET][s_][i] = *(const u32x4 *)(ST + (wm * WTM + i * 32) * 128 + f_off[(PH) * KSP + s_]);           \
        }                                                                                                             \
        __builtin_amdgcn_sched_barrier(0);   /* keep the reads ahead of the MFMAs that follow in program order */    \
    }
    // the phase's MFMAs; direct load d of the tile being issued into ISS follows MFMA number d*NMMA/LPT of the tile
#define RL_MMAP(SET, PH, ISS)                                                                                         \
    {                                                                                                                 \
        _Pragma("unroll") for (int s_ = 0; s_ < KSP; ++s_)                                                            \
            _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                            \
                _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                                      \
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fw[SET][s_][j]),   \
                                                                        __builtin_bit_cast(bf16x8, fx[SET][s_][i]), acc[i][j], 0, 0, 0); \
                    const int q_ = (((PH) * KSP + s_) * TM + i) * TN + j;                                             \
                    _Pragma("unroll") for (int d = 0; d < LPT; ++d)                                                   \
                        if (d * NMMA / LPT == q_) RL_DMA(ISS, d)                                                      \
                    __builtin_amdgcn_sched_barrier(0);                                                                \
                }                                                                                                     \
    }

    // ---- epilogue operands: requested behind the first tiles (see RL_EPI_LOADS below)
    const int epix = lane & 31, ehalf = lane >> 5;
    const Epilogue &e = p.epi;
    constexpr int LPR = WTN / 8;                   // lanes per output row of the wave tile (16 bytes of bf16 each)
    constexpr int RPP = 64 / LPR;                  // rows per row-wise pass
    constexpr int NPASS = WTM / RPP;
    constexpr int NEPI = TN * 4 + NPASS;           // vector-memory operations RL_EPI_LOADS issues
    constexpr int POSN = WTN / 4;                  // 16-byte fp32 positions per parked row
    constexpr int RP = 16 / POSN > 0 ? 16 / POSN : 1;   // parked rows per 256 bytes (all 64 banks)
    const int rr = lane / LPR, pp = lane % LPR;
    f32x4 bias_r[TN][4];
    u32x4 res_r[NPASS];
    uint32_t y_off[NPASS];                         // byte offset of the lane's 8 channels in pass q, or out of range
    int pA[NPASS];                                 // parked position read first in pass q
    const uint32_t y_bytes = p.y_bytes;
#define RL_EPI_LOADS                                                                                                  \
    {                                                                                                                 \
        const bool has_res = e.t_op >= 0;                                                                             \
        /* absent operands get an empty descriptor: every load then returns zeros without touching memory */         \
        const rsrc_t rb = make_rsrc(e.has_bias ? e.bias_ptr : p.w, e.has_bias ? (uint32_t)p.N * 4u : 0u);             \
        const rsrc_t rres = make_rsrc(has_res ? e.t_ptr : p.w, has_res ? y_bytes : 0u);                               \
        const int nb = n0 + wn * WTN + 4 * ehalf;                                                                     \
        _Pragma("unroll") for (int j = 0; j < TN; ++j)                                                                \
            _Pragma("unroll") for (int g = 0; g < 4; ++g) {                                                           \
                const int n = nb + j * 32 + 8 * g;                                                                    \
                bias_r[j][g] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rb, n < p.N ? (uint32_t)n * 4u : OOB, 0, 0)); \
            }                                                                                                         \
        _Pragma("unroll") for (int q = 0; q < NPASS; ++q) {                                                           \
            const int row = q * RPP + rr;                                                                             \
            const int key = (row / RP) & (POSN - 1);                                                                  \
            pA[q] = 2 * pp + (key & 1);                                                                               \
            const int cc = pp ^ (key >> 1);                  /* 8-channel chunk this lane finishes in pass q */      \
            const int m = m0 + wm * WTM + row, n = n0 + wn * WTN + cc * 8;                                            \
            y_off[q] = (m < p.M && n < p.N) ? (uint32_t)(((int64_t)m * p.ys_p + n) * (YF32 ? 4 : 2)) : OOB;           \
            res_r[q] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rres, y_off[q], 0, 0));        \
        }                                                                                                             \
    }

    int kt = 0;
    if (STAGES == 4) {
        // tile kt lives in stage kt % 4; S0 is the register set holding the tile's first phase
#define RL_BODY(CUR, NXT, ISS, INFLIGHT, S0)                                                                          \
    {                                                                                                                 \
        wait_vmcnt<INFLIGHT>();                                                                                       \
        wg_barrier();                                                                                                 \
        RL_TILE_BEGIN                                                                                                 \
        _Pragma("unroll") for (int ph = 0; ph < NPH; ++ph) {                                                          \
            if (ph + 1 < NPH) RL_LOADP(CUR, ph + 1 < NPH ? ph + 1 : 0, ((S0) + ph + 1) & 1)                           \
            else RL_LOADP(NXT, 0, ((S0) + ph + 1) & 1)                                                                \
            RL_MMAP(((S0) + ph) & 1, ph, ISS)                                                                         \
        }                                                                                                             \
    }
        constexpr int SODD = NPH & 1;              // one phase per tile: the register sets alternate from tile to tile
        RL_ISSUE(st0)
        RL_ISSUE(st1)
        RL_ISSUE(st2)
        RL_EPI_LOADS
        wait_vmcnt<2 * LPT + NEPI>();
        wg_barrier();
        RL_LOADP(st0, 0, 0)
        // first tile peeled: the epilogue operands are still in flight behind tile 2
        RL_BODY(st0, st1, st3, LPT + NEPI, 0)
        kt = 1;
#pragma unroll 1
        for (; kt + 4 <= nk; kt += 4) {
            RL_BODY(st1, st2, st0, LPT, SODD)
            RL_BODY(st2, st3, st1, LPT, 0)
            RL_BODY(st3, st0, st2, LPT, SODD)
            RL_BODY(st0, st1, st3, LPT, 0)
        }
        if (kt < nk) {
            RL_BODY(st1, st2, st0, LPT, SODD)
            if (kt + 1 < nk) {
                RL_BODY(st2, st3, st1, LPT, 0)
                if (kt + 2 < nk) RL_BODY(st3, st0, st2, LPT, SODD)
            }
        }
#undef RL_BODY
    } else {
        // tile kt lives in stage kt % 3
#define RL_BODY(CUR, ISS, INFLIGHT)                                                                                   \
    {                                                                                                                 \
        wait_vmcnt<INFLIGHT>();                                                                                       \
        wg_barrier();                                                                                                 \
        RL_TILE_BEGIN                                                                                                 \
        RL_LOADP(CUR, 0, 0)                                                                                           \
        _Pragma("unroll") for (int ph = 0; ph < NPH; ++ph) {                                                          \
            if (ph + 1 < NPH) RL_LOADP(CUR, ph + 1 < NPH ? ph + 1 : 0, (ph + 1) & 1)                                  \
            RL_MMAP(ph & 1, ph, ISS)                                                                                  \
        }                                                                                                             \
    }
        RL_ISSUE(st0)
        RL_ISSUE(st1)
        RL_EPI_LOADS
        RL_BODY(st0, st2, LPT + NEPI)
        kt = 1;
#pragma unroll 1
        for (; kt + 3 <= nk; kt += 3) {
            RL_BODY(st1, st0, LPT)
            RL_BODY(st2, st1, LPT)
            RL_BODY(st0, st2, LPT)
        }
        if (kt < nk) {
            RL_BODY(st1, st0, LPT)
            if (kt + 1 < nk) RL_BODY(st2, st1, LPT)
        }
#undef RL_BODY
    }
#undef RL_EPI_LOADS
    wait_vmcnt<0>();           // the trailing out-of-range issues
#undef RL_MMAP
#undef RL_LOADP
#undef RL_ISSUE
#undef RL_DMA
#undef RL_TILE_BEGIN

    // ---- epilogue.  All waves are past their last fragment read and every direct load has landed once
    // the barrier is crossed; from there on each wave works alone in its own piece of the stages.
    wg_barrier();
    constexpr int WBYTES = WTM * WTN * 4, ROWB = WTN * 4;
    static_assert((NW + STAGES - 1) / STAGES * WBYTES <= STAGE, "a stage must hold its waves' parked tiles");
    const int wsel = wave % STAGES;
    unsigned char *park = (wsel == 0 ? st0 : wsel == 1 ? st1 : wsel == 2 ? st2 : st3) + (wave / STAGES) * WBYTES;
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
    const float lo = (!ANYACT && e.relu_last) ? 0.0f : -INFINITY;
#pragma unroll
    for (int q = 0; q < NPASS; ++q) {
        const int row = q * RPP + rr;
        const f32x4 a = *(const f32x4 *)(park + row * ROWB + pA[q] * 16);
        const f32x4 b = *(const f32x4 *)(park + row * ROWB + (pA[q] ^ 1) * 16);
        const u32x4 r = res_r[q];
        float v[8];
#pragma unroll
        for (int k = 0; k < 4; ++k) { v[k] = a[k]; v[4 + k] = b[k]; }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v[2 * k] += __uint_as_float(r[k] << 16);
            v[2 * k + 1] += __uint_as_float(r[k] & 0xffff0000u);
        }
        if (ANYACT) {
            uint64_t codes = e.rest_ops;
            for (int st = 0; st < e.rest_n; ++st, codes >>= 8) {
                const int op = (int)(codes & 0xff);
#pragma unroll
                for (int k = 0; k < 8; ++k) v[k] = unary_step(op, v[k]);
            }
        }
        u32x4 o;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            o[k] = pack_bf16x2(fmaxf(v[2 * k], lo), fmaxf(v[2 * k + 1], lo));
        if (YF32) {
            const u32x4 o0 = {__float_as_uint(fmaxf(v[0], lo)), __float_as_uint(fmaxf(v[1], lo)), __float_as_uint(fmaxf(v[2], lo)), __float_as_uint(fmaxf(v[3], lo))};
            const u32x4 o1 = {__float_as_uint(fmaxf(v[4], lo)), __float_as_uint(fmaxf(v[5], lo)), __float_as_uint(fmaxf(v[6], lo)), __float_as_uint(fmaxf(v[7], lo))};
            __builtin_amdgcn_raw_buffer_store_b128(o0, ry, y_off[q], 0, 0);
            __builtin_amdgcn_raw_buffer_store_b128(o1, ry, y_off[q] != OOB ? y_off[q] + 16u : OOB, 0, 0);
        } else {
            __builtin_amdgcn_raw_buffer_store_b128(o, ry, y_off[q], 0, 0);
        }
    }
#endif
}

template <int BM, int BN, int WGM, int WGN, int STAGES>
__global__ __launch_bounds__(WGM * WGN * 64) void igemm_lp_kernel(const IgemmParams p)
{
    igemm_lp_body<BM, BN, WGM, WGN, STAGES>(p, (int)blockIdx.x);
}

// any operand-free steps behind bias and residual (tanh, sigmoid, a chain of them) instead of at most one ReLU
template <int BM, int BN, int WGM, int WGN, int STAGES>
__global__ __launch_bounds__(WGM * WGN * 64) void igemm_lp_anyact_kernel(const IgemmParams p)
{
    igemm_lp_body<BM, BN, WGM, WGN, STAGES, false, true>(p, (int)blockIdx.x);
}

// fp32 output (a projection whose result feeds further fp32 arithmetic: the recurrent executor's hoisted x . Wx^T)
template <int BM, int BN, int WGM, int WGN, int STAGES>
__global__ __launch_bounds__(WGM * WGN * 64) void igemm_lp_f32out_kernel(const IgemmParams p)
{
    igemm_lp_body<BM, BN, WGM, WGN, STAGES, true>(p, (int)blockIdx.x);
}

// Two independent contractions of the same tile shape in one launch: the first pa.nblk_m * pa.nblk_n workgroups work on
// pa, the rest on pb.  A stage's stride-2 convolution and its 1x1 projection each fill three quarters of the chip
// when launched alone; launched together, the short projection tiles run on the CUs the other leaves idle.
template <int BM, int BN, int WGM, int WGN, int STAGES>
__global__ __launch_bounds__(WGM * WGN * 64) void igemm_lp_pair_kernel(const IgemmParams pa, const IgemmParams pb)
{
    const int na = pa.nblk_m * pa.nblk_n;
    if ((int)blockIdx.x < na) igemm_lp_body<BM, BN, WGM, WGN, STAGES>(pa, (int)blockIdx.x);
    else igemm_lp_body<BM, BN, WGM, WGN, STAGES>(pb, (int)blockIdx.x - na);
}

#define RL_INST(BM, BN, WGM, WGN, ST) template __global__ void igemm_lp_kernel<BM, BN, WGM, WGN, ST>(const IgemmParams);
RL_INST(128, 128, 2, 4, 4) RL_INST(256, 128, 4, 2, 3) RL_INST(128, 64, 4, 1, 3) RL_INST(128, 64, 4, 1, 4) RL_INST(64, 64, 2, 2, 4)
#undef RL_INST

template <int BM, int BN, int WGM, int WGN, int STAGES>
static hipError_t launch_lp(const IgemmParams &p0, hipStream_t s, bool anyact)
{
    IgemmParams p = p0;
    p.nblk_m = (p.M + BM - 1) / BM;
    p.nblk_n = (p.N + BN - 1) / BN;
    int64_t nblk = (int64_t)p.nblk_m * p.nblk_n;
    if (nblk <= 0 || nblk > 0x7fffffff) return hipErrorInvalidValue;
    if (anyact) hipLaunchKernelGGL((igemm_lp_anyact_kernel<BM, BN, WGM, WGN, STAGES>), dim3((unsigned)nblk), dim3(WGM * WGN * 64), 0, s, p);
    else hipLaunchKernelGGL((igemm_lp_kernel<BM, BN, WGM, WGN, STAGES>), dim3((unsigned)nblk), dim3(WGM * WGN * 64), 0, s, p);
    return hipGetLastError();
}

template <int BM, int BN, int WGM, int WGN, int STAGES>
static hipError_t launch_lp_pair(const IgemmParams &a0, const IgemmParams &b0, hipStream_t s)
{
    IgemmParams a = a0, b = b0;
    a.nblk_m = (a.M + BM - 1) / BM; a.nblk_n = (a.N + BN - 1) / BN;
    b.nblk_m = (b.M + BM - 1) / BM; b.nblk_n = (b.N + BN - 1) / BN;
    const int64_t na = (int64_t)a.nblk_m * a.nblk_n, nb = (int64_t)b.nblk_m * b.nblk_n;
    if (na <= 0 || nb <= 0 || na + nb > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL((igemm_lp_pair_kernel<BM, BN, WGM, WGN, STAGES>), dim3((unsigned)(na + nb)), dim3(WGM * WGN * 64), 0, s, a, b);
    return hipGetLastError();
}

// the kernel variant launch_igemm_lp picks for a contraction (two contractions can share a launch when it is the same)
static int lp_variant(const IgemmParams &p, const IgemmLaunch &l)
{
    switch (l.tile) {
    case TILE_128x128: return 0;
    case TILE_256x128: return 1;
    case TILE_128x64: return (int64_t)((p.M + 127) / 128) * ((p.N + 63) / 64) <= 320 ? 2 : 3;
    default: return 4;
    }
}

bool igemm_lp_can_pair(const IgemmParams &a, const IgemmLaunch &la, const IgemmParams &b, const IgemmLaunch &lb)
{
    return la.lp && lb.lp && !la.ws && !lb.ws && !la.c64 && !lb.c64 && !la.run && !lb.run && !la.gates && !lb.gates && !a.x2 && !b.x2 &&
           !la.anyact && !lb.anyact &&
           a.in_dtype == DT_BF16 && b.in_dtype == DT_BF16 && a.y_dtype == DT_BF16 && b.y_dtype == DT_BF16 && lp_variant(a, la) == lp_variant(b, lb);
}

hipError_t launch_igemm_lp_pair(const IgemmParams &a, const IgemmLaunch &la, const IgemmParams &b, const IgemmLaunch &lb, hipStream_t s)
{
    if (!igemm_lp_can_pair(a, la, b, lb)) return hipErrorInvalidValue;
    switch (lp_variant(a, la)) {
    case 0: return launch_lp_pair<128, 128, 2, 4, 4>(a, b, s);
    case 1: return launch_lp_pair<256, 128, 4, 2, 3>(a, b, s);
    case 2:
        // together the two fill more than one workgroup per CU: three stages (72 KB), so that two share a CU and the
        // projection's short tiles run inside the stalls of the other's
        if ((int64_t)((a.M + 127) / 128) * ((a.N + 63) / 64) + (int64_t)((b.M + 127) / 128) * ((b.N + 63) / 64) > 320)
            return launch_lp_pair<128, 64, 4, 1, 3>(a, b, s);
        return launch_lp_pair<128, 64, 4, 1, 4>(a, b, s);
    case 3: return launch_lp_pair<128, 64, 4, 1, 3>(a, b, s);
    default: return launch_lp_pair<64, 64, 2, 2, 4>(a, b, s);
    }
}

template <int BM, int BN, int WGM, int WGN, int STAGES>
static hipError_t launch_lp_f32out(const IgemmParams &p0, hipStream_t s)
{
    IgemmParams p = p0;
    p.nblk_m = (p.M + BM - 1) / BM;
    p.nblk_n = (p.N + BN - 1) / BN;
    int64_t nblk = (int64_t)p.nblk_m * p.nblk_n;
    if (nblk <= 0 || nblk > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL((igemm_lp_f32out_kernel<BM, BN, WGM, WGN, STAGES>), dim3((unsigned)nblk), dim3(WGM * WGN * 64), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_igemm_lp(const IgemmParams &p, const IgemmLaunch &l, hipStream_t s)
{
    if (p.in_dtype == DT_BF16 && p.y_dtype == DT_F32 && !l.gates && !p.x2 && p.epi.t_op < 0) {
        // fp32 output: the two large tiles only
        if (l.tile == TILE_256x128) return launch_lp_f32out<256, 128, 4, 2, 3>(p, s);
        if (l.tile == TILE_128x128) return launch_lp_f32out<128, 128, 2, 4, 4>(p, s);
        return hipErrorInvalidValue;
    }
    if (p.in_dtype != DT_BF16 || p.y_dtype != DT_BF16 || l.gates || p.x2) return hipErrorInvalidValue;
    // the planner's flag and the chain must agree: one ReLU at most without it, other operand-free steps with it
    const bool anyact = l.anyact != 0;
    if (anyact != (p.epi.rest_n > 0 && !p.epi.relu_last)) return hipErrorInvalidValue;
    switch (l.tile) {
    case TILE_128x128:
        // eight waves of 64 pixels x 32 channels, two per SIMD: one wave's fragment reads and request stalls are
        // covered by the other's MFMAs (measured 4% faster than four waves of 64 x 64 on the ResNet shapes)
        return launch_lp<128, 128, 2, 4, 4>(p, s, anyact);
    case TILE_256x128:
        // eight waves of 64 x 64, two per SIMD, three stages of 48 KB
        return launch_lp<256, 128, 4, 2, 3>(p, s, anyact);
    case TILE_128x64:
        // few workgroups (at most one per CU anyway): four stages, so fragments are prefetched across the barrier;
        // many: three stages, so two workgroups share a CU and cover each other's barriers and epilogues
        if ((int64_t)((p.M + 127) / 128) * ((p.N + 63) / 64) <= 320) return launch_lp<128, 64, 4, 1, 4>(p, s, anyact);
        return launch_lp<128, 64, 4, 1, 3>(p, s, anyact);
    default: return launch_lp<64, 64, 2, 2, 4>(p, s, anyact);
    }
}

}  // namespace rl

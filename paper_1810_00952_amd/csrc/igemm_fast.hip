// Implicit-GEMM contraction for gfx950, fast path: channel-contiguous A rows
// (16-byte vector loads), packed K-contiguous weights.
//
//   C[m, n] = sum_k A[m, k] * Wp[n, k],  m = (image, oh, ow), n = out channel,
//   k = (kh, kw, c)
//
// Workgroup = 4 wavefronts (2 x 2) on a BM x BN tile, wave tile (BM/2)x(BN/2)
// of 32x32 MFMA accumulators.  K advances in tiles of 128 bytes per row.
// Global -> register fetches run two K tiles ahead of the MFMAs (two register
// sets), registers are parked in a two-stage LDS ring, one barrier per K tile.
// LDS rows carry 16 bytes of padding so the 16-byte fragment reads of
// consecutive rows hit distinct banks.  After the K loop the fp32 accumulators
// are staged through LDS once, so that the epilogue chain runs on 8 consecutive
// output channels per thread with 16-byte operand loads and 16-byte stores.
// Workgroup ids are remapped so that the tiles sharing activation rows run on
// one XCD (one L2).
#include "igemm_epilogue.h"

namespace rl {

namespace {

constexpr int ROW_STRIDE = 144;   // 128 data bytes + 16 pad
constexpr int CHUNKS = 8;         // 16-byte chunks per row per K tile
constexpr int NUM_XCD = 8;

typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void *ptr, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc((void *)ptr, 0, bytes, 0x00020000);   // raw buffer, 32-bit untyped data
}

template <typename T> struct Elem;
template <> struct Elem<float> { static constexpr int KV = 4; };
template <> struct Elem<uint16_t> { static constexpr int KV = 8; };

__device__ __forceinline__ void mma_chunk(f32x16 &acc, const u32x4 &a, const u32x4 &b, float)
{
    // four K=2 steps; lane half h supplies k = 4h + j for step j on both operands
#pragma unroll
    for (int j = 0; j < 4; ++j)
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[j]), __uint_as_float(b[j]), acc, 0, 0, 0);
}

__device__ __forceinline__ void mma_chunk(f32x16 &acc, const u32x4 &a, const u32x4 &b, uint16_t)
{
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}

}  // namespace

template <typename T, int BM, int BN, bool GATES>
__global__ __launch_bounds__(256) void igemm_fast_kernel(const IgemmParams p)
{
    constexpr int KV = Elem<T>::KV;
    constexpr int BKE = CHUNKS * KV;          // K elements per tile
    constexpr int WTM = BM / 2, WTN = BN / 2; // wave tile
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int APASS = BM / 32, BPASS = BN / 32;
    constexpr int A_BYTES = BM * ROW_STRIDE, B_BYTES = BN * ROW_STRIDE;
    constexpr int STAGE = A_BYTES + B_BYTES;
    constexpr int LDC = BN + 8;               // fp32 staging row; +8 keeps the two half-waves on different banks

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
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

    // Buffer resources: a lane whose tap falls outside the image (or past K) is
    // given an offset beyond the range, which the hardware answers with zeros
    // without touching memory -- no branches and no zero-fill in the loop.
    constexpr uint32_t OOB = 0x80000000u;
    constexpr int ES = (int)sizeof(T);
    const rsrc_t rx = make_rsrc(p.x, p.x_bytes);
    const rsrc_t rx2 = make_rsrc(p.x2 ? p.x2 : p.x, p.x2 ? p.x2_bytes : p.x_bytes);
    const rsrc_t rw = make_rsrc(p.w, p.w_bytes);

    // ---- per-thread loader state: one 16-byte chunk column, APASS + BPASS rows
    const int lchunk = t & 7, lrow = t >> 3;
    int a_off[APASS], a_ih0[APASS], a_iw0[APASS];      // byte offset of tap (0,0), top-left input coordinate
#pragma unroll
    for (int i = 0; i < APASS; ++i) {
        int m = m0 + lrow + 32 * i;
        if (m < p.M) {
            int img = m / p.OHW;
            int pix = m - img * p.OHW;
            int oh = pix / p.OW;
            int ow = pix - oh * p.OW;
            a_ih0[i] = oh * p.sh - p.ph;
            a_iw0[i] = ow * p.sw - p.pw;
            a_off[i] = (int)(((int64_t)img * p.xs_n + (int64_t)a_ih0[i] * p.xs_h + (int64_t)a_iw0[i] * p.xs_w) * ES);
        } else {
            a_ih0[i] = -(1 << 24);
            a_iw0[i] = 0;
            a_off[i] = 0;
        }
    }
    int b_off[BPASS];
#pragma unroll
    for (int i = 0; i < BPASS; ++i) {
        int n = n0 + lrow + 32 * i;
        if (n > p.N - 1) n = p.N - 1;          // rows past N are computed on valid memory and never stored
        b_off[i] = (int)((int64_t)n * p.Kp * ES);
    }
    // K split over workgroups (splits > 1): workgroup (tile, z = blockIdx.y) multiplies K tiles [z*per, (z+1)*per) and
    // leaves its bare fp32 sums in partial[z][M][N]; splitk_reduce_kernel adds the slices in order and finishes
    const int nk_all = (p.Kp + BKE - 1) / BKE;
    const int split = p.splits > 1 ? (int)blockIdx.y : 0;
    const int kt_begin = p.splits > 1 ? split * p.split_tiles : 0;
    const int kt_end = p.splits > 1 ? min(nk_all, kt_begin + p.split_tiles) : nk_all;
    int ktile0 = kt_begin * BKE;               // first k of the tile being fetched (uniform)
    int kc = ktile0 + lchunk * KV;             // k of this thread's chunk in that tile
    int c_cur, kh_cur, kw_cur;
    {
        int tap = kc / p.C;
        c_cur = kc - tap * p.C;
        kh_cur = tap / p.KW;
        kw_cur = tap - kh_cur * p.KW;
    }

    auto fetch = [&](u32x4 *ra, u32x4 *rb) {
        if (ktile0 < p.K1) {
            const bool kvalid = kc < p.K1;
            const int koff = (int)(((int64_t)kh_cur * p.xs_h + (int64_t)kw_cur * p.xs_w + c_cur) * ES);
#pragma unroll
            for (int i = 0; i < APASS; ++i) {
                int ih = a_ih0[i] + kh_cur, iw = a_iw0[i] + kw_cur;
                bool ok = kvalid && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
                ra[i] = __builtin_amdgcn_raw_buffer_load_b128(rx, ok ? (uint32_t)(a_off[i] + koff) : OOB, 0, 0);
            }
        } else {
            // second operand of a row concatenation (dense): row m of x2, column k - K1
            const bool kvalid = kc < p.K;
            const int koff = (kc - p.K1) * ES;
#pragma unroll
            for (int i = 0; i < APASS; ++i) {
                bool ok = kvalid && a_ih0[i] >= 0;
                ra[i] = __builtin_amdgcn_raw_buffer_load_b128(rx2, ok ? (uint32_t)((m0 + lrow + 32 * i) * (int)p.x2s_n * ES + koff) : OOB, 0, 0);
            }
        }
        const bool bvalid = kc < p.Kp;
#pragma unroll
        for (int i = 0; i < BPASS; ++i)
            rb[i] = __builtin_amdgcn_raw_buffer_load_b128(rw, bvalid ? (uint32_t)(b_off[i] + kc * ES) : OOB, 0, 0);
        // advance to the next K tile
        ktile0 += BKE;
        kc += BKE;
        c_cur += BKE;
        while (c_cur >= p.C) {
            c_cur -= p.C;
            if (++kw_cur == p.KW) { kw_cur = 0; ++kh_cur; }
        }
    };
    auto park = [&](int buf, const u32x4 *ra, const u32x4 *rb) {
        unsigned char *base = smem + buf * STAGE + lrow * ROW_STRIDE + lchunk * 16;
#pragma unroll
        for (int i = 0; i < APASS; ++i) *(u32x4 *)(base + i * 32 * ROW_STRIDE) = ra[i];
#pragma unroll
        for (int i = 0; i < BPASS; ++i) *(u32x4 *)(base + A_BYTES + i * 32 * ROW_STRIDE) = rb[i];
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    const int frow = lane & 31, fhalf = lane >> 5;
    auto compute = [&](int buf) {
        const unsigned char *a_base = smem + buf * STAGE + (wm * WTM + frow) * ROW_STRIDE + fhalf * 16;
        const unsigned char *b_base = smem + buf * STAGE + A_BYTES + (wn * WTN + frow) * ROW_STRIDE + fhalf * 16;
#pragma unroll
        for (int ks = 0; ks < CHUNKS / 2; ++ks) {
            u32x4 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[i] = *(const u32x4 *)(a_base + i * 32 * ROW_STRIDE + ks * 32);
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[j] = *(const u32x4 *)(b_base + j * 32 * ROW_STRIDE + ks * 32);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) mma_chunk(acc[i][j], fa[i], fb[j], T());
        }
    };

    // ---- K loop: register set 0 / 1 hold the tiles one and two ahead of the
    // MFMAs.  Fetches past the last tile return zeros, so the loop body has one
    // shape; an odd tile count is finished after the loop.
    const int nk = kt_end - kt_begin;
    u32x4 ra0[APASS], rb0[BPASS], ra1[APASS], rb1[BPASS];
    fetch(ra0, rb0);                 // tile 0
    fetch(ra1, rb1);                 // tile 1
    park(0, ra0, rb0);
    __syncthreads();
    int kt = 0;
#pragma unroll 1
    for (; kt + 2 <= nk; kt += 2) {
        fetch(ra0, rb0);             // tile kt + 2
        compute(0);                  // tile kt
        park(1, ra1, rb1);           // tile kt + 1
        __syncthreads();
        fetch(ra1, rb1);             // tile kt + 3
        compute(1);                  // tile kt + 1
        park(0, ra0, rb0);           // tile kt + 2
        __syncthreads();
    }
    if (kt < nk) {
        compute(0);                  // last tile of an odd count
        __syncthreads();
    }
    // every wave is past its last fragment read (each compute is followed by a barrier)

    // ---- stage fp32 accumulators in LDS: sC[row][col], row stride LDC floats
    float *sC = (float *)smem;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int row = wm * WTM + i * 32 + 8 * (r >> 2) + 4 * fhalf + (r & 3);
                int col = wn * WTN + j * 32 + frow;
                sC[row * LDC + col] = acc[i][j][r];
            }
    __syncthreads();

    if (!GATES && p.splits > 1) {
        float *dst = p.partial + (int64_t)split * p.M * p.N;
        for (int idx = t; idx < BM * BN; idx += 256) {
            const int row = idx / BN, col = idx - row * BN;
            const int m = m0 + row, n = n0 + col;
            if (m < p.M && n < p.N) dst[(int64_t)m * p.N + n] = sC[row * LDC + col];
        }
        return;
    }

    // ---- 32-row passes over the staged tile; the residual rows of the next pass are in flight
    // while this pass is stored
    using TE = TileEpilogue<BN>;
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
        const int mq = m0 + q * 32;
        const float *sq = sC + q * 32 * LDC;
        if (GATES) TE::gates_pass(p, sq, LDC, t, mq, bn);
        else if (vec_ok) TE::store_pass(p, sq, LDC, t, mq, n0, bias8, cur);
        else TE::store_pass_scalar(p, sq, LDC, t, mq, n0);
        cur = nxt;
    }
}

hipError_t launch_splitk_reduce(const IgemmParams &p, hipStream_t s);     // igemm_dma.hip

template <typename T, int BM, int BN, bool GATES>
static hipError_t launch_fast(const IgemmParams &p0, hipStream_t s)
{
    IgemmParams p = p0;
    p.nblk_m = (p.M + BM - 1) / BM;
    p.nblk_n = (p.N + BN - 1) / BN;
    size_t lds = 2 * (size_t)(BM + BN) * ROW_STRIDE;
    size_t stage_c = (size_t)BM * (BN + 8) * sizeof(float);
    if (stage_c > lds) lds = stage_c;
    auto kern = igemm_fast_kernel<T, BM, BN, GATES>;
    static bool attr_set = false;          // one flag per instantiation
    if (!attr_set && lds > 48 * 1024) {
        hipError_t er = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (er != hipSuccess) return er;
        attr_set = true;
    }
    int64_t nblk = (int64_t)p.nblk_m * p.nblk_n;
    if (nblk <= 0 || nblk > 0x7fffffff) return hipErrorInvalidValue;
    if (p.splits > 1) {
        constexpr int BKE = CHUNKS * Elem<T>::KV;
        const int nk = (p.Kp + BKE - 1) / BKE;
        // every slice holds at least one K tile and the slices cover K exactly once
        if (GATES || !p.partial || p.splits > 64 || (int64_t)p.M * p.N * p.splits >= (int64_t)1 << 31 || p.split_tiles < 1 ||
            (int64_t)(p.splits - 1) * p.split_tiles >= nk || (int64_t)p.splits * p.split_tiles < nk || p.x2)
            return hipErrorInvalidValue;
        hipLaunchKernelGGL(kern, dim3((unsigned)nblk, (unsigned)p.splits), dim3(256), lds, s, p);
        hipError_t er = hipGetLastError();
        if (er != hipSuccess) return er;
        return launch_splitk_reduce(p, s);
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)nblk), dim3(256), lds, s, p);
    return hipGetLastError();
}

template <typename T>
static hipError_t launch_fast_typed(const IgemmParams &p, const IgemmLaunch &l, hipStream_t s)
{
    if (l.gates) {
        if (l.tile != TILE_64x64) return hipErrorInvalidValue;
        return launch_fast<T, 64, 64, true>(p, s);
    }
    switch (l.tile) {
    case TILE_128x128: return launch_fast<T, 128, 128, false>(p, s);
    case TILE_128x64: return launch_fast<T, 128, 64, false>(p, s);
    default: return launch_fast<T, 64, 64, false>(p, s);
    }
}

hipError_t launch_igemm_fast(const IgemmParams &p, const IgemmLaunch &l, hipStream_t s)
{
    if (p.in_dtype == DT_BF16) return launch_fast_typed<uint16_t>(p, l, s);
    return launch_fast_typed<float>(p, l, s);
}

}  // namespace rl

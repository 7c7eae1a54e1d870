// Implicit-GEMM contraction kernels for gfx950 (conv2d and dense anchors of a
// fusion group) with the group's injective epilogue applied in registers.
// This file holds the gather variant (any element strides, any channel count:
// A elements are fetched one by one) and the dispatcher; the vector-load
// variant lives in igemm_fast.hip.
//
//   C[m, n] = sum_k A[m, k] * Wp[n, k]
//   m = (image, oh, ow)   n = output channel   k = (kh, kw, c)
//
// One workgroup = 256 threads = 4 wavefronts (2 x 2) computes a BM x BN tile.
// K is walked in tiles of 128 bytes per row (64 bf16 / 32 f32): each thread
// fetches 16-byte vectors from global memory into registers while the MFMAs of
// the previous tile run, then parks them in LDS (two buffers, one barrier per
// K tile).  LDS rows are padded by 16 bytes so that the 16-byte fragment reads
// of 32 consecutive rows fall on distinct banks.  The accumulators stay in
// registers (32x32 MFMA tiles, fp32) until the epilogue chain has been applied.
#include "device_utils.h"

namespace rl {

constexpr int ROW_STRIDE = 144;   // 128 data bytes + 16 pad
constexpr int CHUNKS = 8;         // 16-byte chunks per row per K tile

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

template <typename T, int BM, int BN, bool AVEC, bool GATES>
__global__ __launch_bounds__(256) void igemm_kernel(const IgemmParams p)
{
    constexpr int KV = Elem<T>::KV;
    constexpr int BKE = CHUNKS * KV;          // K elements per tile
    constexpr int WTM = BM / 2, WTN = BN / 2; // wave tile
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int APASS = BM / 32, BPASS = BN / 32;
    constexpr int A_BYTES = BM * ROW_STRIDE, B_BYTES = BN * ROW_STRIDE;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int STAGE = A_BYTES + B_BYTES;   // stage s: A tile at s*STAGE, B tile behind it

    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int bid = blockIdx.x;
    const int bm = bid / p.nblk_n, bn = bid - bm * p.nblk_n;
    const int m0 = bm * BM, n0 = bn * BN;

    const T *__restrict__ x = (const T *)p.x;
    const T *__restrict__ x2 = (const T *)p.x2;
    const T *__restrict__ w = (const T *)p.w;

    // ---- per-thread loader state
    const int lchunk = t & 7, lrow = t >> 3;
    int a_img[APASS], a_ih0[APASS], a_iw0[APASS];
#pragma unroll
    for (int i = 0; i < APASS; ++i) {
        int m = m0 + lrow + 32 * i;
        if (m < p.M) {
            int img = m / p.OHW;
            int pix = m - img * p.OHW;
            int oh = pix / p.OW;
            int ow = pix - oh * p.OW;
            a_img[i] = img;
            a_ih0[i] = oh * p.sh - p.ph;
            a_iw0[i] = ow * p.sw - p.pw;
        } else {
            a_img[i] = 0;
            a_ih0[i] = -(1 << 24);
            a_iw0[i] = 0;
        }
    }
    // K split over gridDim.y workgroups per tile (p.splits > 1): this one multiplies K tiles [kt0, kt0 + nk) and leaves
    // its bare fp32 sums in partial[blockIdx.y][M][N]; splitk_reduce_kernel adds the slices in order and finishes
    const int nk_all = (p.Kp + BKE - 1) / BKE;
    const int split = p.splits > 1 ? (int)blockIdx.y : 0;
    const int kt0 = p.splits > 1 ? split * p.split_tiles : 0;
    const int nk = p.splits > 1 ? max(0, min(nk_all - kt0, p.split_tiles)) : nk_all;
    int kc = kt0 * BKE + lchunk * KV;     // k of this thread's chunk in the current tile
    int c_cur = 0, kh_cur = 0, kw_cur = 0;
    if (AVEC) {
        int tap = kc / p.C;
        c_cur = kc - tap * p.C;
        kh_cur = tap / p.KW;
        kw_cur = tap - kh_cur * p.KW;
    }

    u32x4 ra[APASS], rb[BPASS];

    auto fetch = [&]() {
        if (AVEC) {
            const bool kvalid = kc < p.K;
            if (kc < p.K1) {
                const int64_t koff = (int64_t)kh_cur * p.xs_h + (int64_t)kw_cur * p.xs_w + c_cur;
#pragma unroll
                for (int i = 0; i < APASS; ++i) {
                    int ih = a_ih0[i] + kh_cur, iw = a_iw0[i] + kw_cur;
                    bool ok = kvalid && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
                    u32x4 v = {0u, 0u, 0u, 0u};
                    if (ok) {
                        const T *src = x + (int64_t)a_img[i] * p.xs_n + (int64_t)a_ih0[i] * p.xs_h + (int64_t)a_iw0[i] * p.xs_w + koff;
                        v = *(const u32x4 *)src;
                    }
                    ra[i] = v;
                }
            } else {
#pragma unroll
                for (int i = 0; i < APASS; ++i) {
                    bool ok = kvalid && a_ih0[i] >= 0;
                    u32x4 v = {0u, 0u, 0u, 0u};
                    if (ok) v = *(const u32x4 *)(x2 + (int64_t)a_img[i] * p.x2s_n + (kc - p.K1));
                    ra[i] = v;
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < APASS; ++i) {
                T tmp[KV];
#pragma unroll
                for (int e = 0; e < KV; ++e) {
                    int k = kc + e;
                    T val = 0;
                    if (k < p.K && a_ih0[i] > -(1 << 23)) {
                        if (k < p.K1) {
                            int tap = k / p.C;
                            int c = k - tap * p.C;
                            int kh = tap / p.KW;
                            int kw = tap - kh * p.KW;
                            int ih = a_ih0[i] + kh * (p.tap_dil_m1 + 1), iw = a_iw0[i] + kw * (p.tap_dil_m1 + 1);
                            bool on = true;
                            if (p.in_dil_m1 > 0) {           // only every (in_dil_m1 + 1)-th position of the virtual input holds a pixel
                                const int d = p.in_dil_m1 + 1;
                                on = ih >= 0 && iw >= 0 && ih % d == 0 && iw % d == 0;
                                ih = on ? ih / d : -1;
                                iw = on ? iw / d : -1;
                            }
                            if (on && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W)
                                val = x[(int64_t)a_img[i] * p.xs_n + (int64_t)c * p.xs_c + (int64_t)ih * p.xs_h + (int64_t)iw * p.xs_w];
                        } else {
                            val = x2[(int64_t)a_img[i] * p.x2s_n + (k - p.K1)];
                        }
                    }
                    tmp[e] = val;
                }
                ra[i] = *(const u32x4 *)tmp;
            }
        }
#pragma unroll
        for (int i = 0; i < BPASS; ++i) {
            int n = n0 + lrow + 32 * i;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (n < p.N && kc < p.Kp) v = *(const u32x4 *)(w + (int64_t)n * p.Kp + kc);
            rb[i] = v;
        }
    };
    auto advance = [&]() {
        kc += BKE;
        if (AVEC) {
            c_cur += BKE;
            while (c_cur >= p.C) {
                c_cur -= p.C;
                if (++kw_cur == p.KW) { kw_cur = 0; ++kh_cur; }
            }
        }
    };
    auto park = [&](int buf) {
#pragma unroll
        for (int i = 0; i < APASS; ++i)
            *(u32x4 *)(smem + buf * STAGE + (lrow + 32 * i) * ROW_STRIDE + lchunk * 16) = ra[i];
#pragma unroll
        for (int i = 0; i < BPASS; ++i)
            *(u32x4 *)(smem + buf * STAGE + A_BYTES + (lrow + 32 * i) * ROW_STRIDE + lchunk * 16) = rb[i];
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    if (nk > 0) {
        fetch();
        advance();
        park(0);
    }
    __syncthreads();

    const int frow = lane & 31, fhalf = lane >> 5;
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        const bool more = kt + 1 < nk;
        if (more) { fetch(); advance(); }
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
        if (more) park(buf ^ 1);
        __syncthreads();
    }

    if (!GATES && p.splits > 1) {
        float *dst = p.partial + (int64_t)split * p.M * p.N;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = n0 + wn * WTN + j * 32 + (lane & 31);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int m = m0 + wm * WTM + i * 32 + 8 * (r >> 2) + 4 * fhalf + (r & 3);
                    if (m < p.M && n < p.N) dst[(int64_t)m * p.N + n] = acc[i][j][r];
                }
            }
        return;
    }
    // ---- epilogue: chain applied to the accumulators in registers
    const Epilogue &e = p.epi;
    const bool rowmajor = (p.ys_n == (int64_t)p.OHW * p.ys_p);
    const int colq = lane & 31;

    // element (i, j, r) of this lane: row m, column n
    auto row_of = [&](int i, int r) { return m0 + wm * WTM + i * 32 + 8 * (r >> 2) + 4 * fhalf + (r & 3); };
    auto col_of = [&](int j) { return n0 + wn * WTN + j * 32 + colq; };
    auto off_of = [&](int m, int n) -> int64_t {
        if (rowmajor) return (int64_t)m * p.ys_p + (int64_t)n * p.ys_c;
        int img = m / p.OHW;
        int pix = m - img * p.OHW;
        return (int64_t)img * p.ys_n + (int64_t)pix * p.ys_p + (int64_t)n * p.ys_c;
    };
    auto chan_of = [&](int n) {
        if (!GATES) return n;
        int j = n - n0;                       // packed column inside the block tile
        return (j / (BN / 4)) * p.hidden + bn * (BN / 4) + (j % (BN / 4));
    };

    for (int s = 0; s < e.n_ops; ++s) {
        const int op = epi_op(e, s);
        if (op == E_BIAS) {
            const int a = epi_arg(e, s);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                int n = col_of(j);
                float b = (n < p.N) ? load_as_f32(epi_ptr(e, a), epi_ptr_dtype(e, a), chan_of(n)) : 0.0f;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] += b;
            }
        } else if (op == E_RELU) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] = acc[i][j][r] > 0.0f ? acc[i][j][r] : 0.0f;
        } else {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    int n = col_of(j);
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        int m = row_of(i, r);
                        if (m < p.M && n < p.N) acc[i][j][r] = epi_step(e, s, acc[i][j][r], off_of(m, n), n);
                    }
                }
        }
    }

    if (!GATES) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                int n = col_of(j);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int m = row_of(i, r);
                    if (m < p.M && n < p.N) store_from_f32(p.y, p.y_dtype, off_of(m, n), acc[i][j][r]);
                }
            }
    } else {
        // pre-activations of the block tile go through LDS so that one thread
        // sees the four gates of a hidden unit: packed column g*(BN/4)+u
        float *sC = (float *)smem;           // [BM][BN + 1]; all K-loop reads are behind the last barrier
        constexpr int LD = BN + 1;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int rl_ = wm * WTM + i * 32 + 8 * (r >> 2) + 4 * fhalf + (r & 3);
                    int cl_ = wn * WTN + j * 32 + colq;
                    sC[rl_ * LD + cl_] = acc[i][j][r];
                }
        __syncthreads();
        constexpr int U = BN / 4;
        for (int idx = t; idx < BM * U; idx += 256) {
            int row = idx / U, u = idx - row * U;
            int m = m0 + row, unit = bn * U + u;
            if (m < p.M && unit < p.hidden) {
                float zi = sC[row * LD + u], zf = sC[row * LD + U + u];
                float zg = sC[row * LD + 2 * U + u], zo = sC[row * LD + 3 * U + u];
                float c_old = p.c_in[(int64_t)m * p.hidden + unit];
                float cn = sigmoidf_(zf) * c_old + sigmoidf_(zi) * tanhf_(zg);
                float hn = sigmoidf_(zo) * tanhf_(cn);
                p.c_out[(int64_t)m * p.hidden + unit] = cn;
                store_from_f32(p.h_out, p.h_dtype, (int64_t)m * p.hidden + unit, hn);
            }
        }
    }
}

hipError_t launch_splitk_reduce(const IgemmParams &p, hipStream_t s);     // igemm_dma.hip

template <typename T, int BM, int BN, bool AVEC, bool GATES>
static hipError_t launch_one(const IgemmParams &p0, hipStream_t s)
{
    IgemmParams p = p0;
    p.nblk_m = (p.M + BM - 1) / BM;
    p.nblk_n = (p.N + BN - 1) / BN;
    size_t lds = 2 * (size_t)(BM + BN) * ROW_STRIDE;
    if (GATES) {
        size_t need = (size_t)BM * (BN + 1) * sizeof(float);
        if (need > lds) lds = need;
    }
    auto kern = igemm_kernel<T, BM, BN, AVEC, GATES>;
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
        if (GATES || AVEC || !p.partial || p.splits > 64 || (int64_t)p.M * p.N * p.splits >= (int64_t)1 << 31 || p.split_tiles < 1 ||
            (int64_t)p.splits * p.split_tiles < nk || p.x2)
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
static hipError_t launch_typed(const IgemmParams &p, const IgemmLaunch &l, hipStream_t s)
{
    if (l.tile != TILE_64x64) return hipErrorInvalidValue;
    return l.gates ? launch_one<T, 64, 64, false, true>(p, s) : launch_one<T, 64, 64, false, false>(p, s);
}

hipError_t launch_igemm_fast(const IgemmParams &p, const IgemmLaunch &l, hipStream_t s);
hipError_t launch_igemm_dma(const IgemmParams &p, const IgemmLaunch &l, hipStream_t s);
hipError_t launch_igemm_lp(const IgemmParams &p, const IgemmLaunch &l, hipStream_t s);
hipError_t launch_igemm_ws(const IgemmParams &p, hipStream_t s);

hipError_t launch_igemm(const IgemmParams &p, const IgemmLaunch &l, hipStream_t s)
{
    if (l.lp && l.c64) return launch_conv3x3_c64(p, s);
    if (l.lp && l.run) return launch_conv3x3_run(p, l, s);
    if (l.lp && l.ws) return launch_igemm_ws(p, s);
    if (l.lp) return launch_igemm_lp(p, l, s);
    if (l.avec && l.dma) return launch_igemm_dma(p, l, s);
    if (l.avec) return launch_igemm_fast(p, l, s);
    if (p.in_dtype == DT_BF16) return launch_typed<uint16_t>(p, l, s);
    return launch_typed<float>(p, l, s);
}

}  // namespace rl

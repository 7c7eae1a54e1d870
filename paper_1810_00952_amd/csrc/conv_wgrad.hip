// Gradient of a convolution with respect to its weights, bf16 in / fp32 accumulate, for batches of 64 images (or a
// multiple of 64: a workgroup then walks its row segment once per 64 images):
//   dw[o][c][a][b] = sum over (n, i, j) of dy[n][o][i][j] * x[n][c][s*i + a - ph][s*j + b - pw]
//
// The contraction runs over pixels and images, which are the SLOW axes of both operands as a plan stores them, while an
// MFMA wants eight consecutive contraction indices per lane.  Both operands are therefore transposed once (a step of the
// plan each, by the ordinary batched-transposition kernel) so that the 64 images are the fastest axis: dyT[pixel][o][n],
// xT[pixel][c][n].  Then, for ONE output pixel (i, j) and one filter tap (a, b),
//   dw_ab[o][c] += sum_n dyT[(i, j)][o][n] * xT[(s i + a - ph, s j + b - pw)][c][n]
// is a 64-deep contraction of two tiles whose rows (o, resp. c) are 128 contiguous bytes: exactly the [row][K tile]
// form every other contraction kernel here reads from LDS, a tap is a different pixel's tile (no per-lane masking: a
// tap outside the image is a tile of zeros for the whole workgroup), and any stride is address arithmetic.
//
// A workgroup owns an (o tile of 32*WO) x (c tile of 64) block of dw for ALL filter taps and a segment of one output
// row: wave (wo, wc) holds KH*KW accumulator tiles of 32 x 32.  It walks the segment's output pixels; per pixel it
// needs dy's tile (16 KB at WO = 4) and the x tiles of the KH x KW window, of which all but `stride` columns were
// already fetched for the pixel before: x tiles live in a ring of 3 rows x 5 columns (column w in slot w mod 5; a
// window of at most 3 columns plus at most 2 new ones for the next pixel never collide).  Everything arrives by
// direct global->LDS loads requested one pixel ahead; rows are XOR-swizzled by 16-byte chunk at load time so that the
// fragment reads are conflict-free.  Per pixel and wave: 4 dy fragments, then KH*KW*4 MFMAs each fed by one x
// fragment read issued three MFMAs earlier; one workgroup barrier per pixel.
//
// The sums of the workgroups that share a block of dw (one per row segment) go to a scratch tensor
// [segment][tap][O][C] in fp32 and are added in segment order by wgrad_reduce_kernel, which also writes dw in its
// declared order [O][C][KH][KW] and dtype: results do not depend on timing.
#include "device_utils.h"

namespace rl {

namespace {

__device__ __forceinline__ u32x4 make_desc(const void *ptr, uint32_t bytes)
{
    const uint64_t a = (uint64_t)ptr;
    u32x4 d = {(uint32_t)a, (uint32_t)(a >> 32) & 0xffffu, bytes, 0x00020000u};   // raw buffer, untyped dwords
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

constexpr int WG_CT = 64;                         // input channels of a workgroup's block
constexpr int WG_NB = 64;                         // images: the contraction depth of one pixel, one 128-byte row
constexpr int XT_BYTES = WG_CT * 128;             // an x tile: 8 KB
constexpr int RING_ROWS = 3, RING_COLS = 5;

}  // namespace

template <int WO, int KH, int KW>
__global__ __launch_bounds__(WO * 2 * 64) void conv_wgrad_kernel(const WgradParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub; the body uses gfx950-only builtins
    constexpr int NW = WO * 2;                    // waves
    constexpr int OT = WO * 32;                   // output channels of the block
    constexpr int DY_BYTES = OT * 128;
    constexpr int XI = 8 / NW;                    // direct loads per wave per x tile (8 in all)
    constexpr int T = KH * KW;
    constexpr int X_OFF = 2 * DY_BYTES, ZERO_OFF = X_OFF + RING_ROWS * RING_COLS * XT_BYTES;
    static_assert(NW == 8 || NW == 4, "eight or four waves");
    static_assert(KH <= RING_ROWS && KW <= 3, "window of at most 3 x 3 tiles");
    static_assert(ZERO_OFF + 128 <= 160 * 1024, "LDS");
    __shared__ __attribute__((aligned(1024))) unsigned char lds[ZERO_OFF + 128];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wo = wave % WO, wc = wave / WO;       // the wave's 32 output channels and 32 input channels of the block
    const int frow = lane & 31, fhalf = lane >> 5;

    // ---- this workgroup: block (ot, ct) of dw, segment `seg` of output row i
    const int ntile = p.n_ot * p.n_ct;
    const int chunk = blockIdx.x / ntile, tile = blockIdx.x - chunk * ntile;
    const int ot = tile / p.n_ct, ct = tile - ot * p.n_ct;
    const int i = chunk / p.nseg, seg = chunk - i * p.nseg;
    const int j0 = seg * p.L, j1 = min(p.OW, j0 + p.L);
    const int s = p.s;

    const u32x4 ddy = make_desc(p.dyT, p.dy_bytes);
    const u32x4 ddx = make_desc(p.xT, p.x_bytes);
    const uint32_t lds_a = lds_addr_of(lds);

    // ---- per-lane parts of the request addresses: lane l of a load fills row 8e + (l >> 3), position l & 7 of a tile,
    // with the row's 16-byte chunk (l & 7) ^ key(row); the pixel is a scalar offset
    uint32_t dy_voff[2], x_voff[XI];
#pragma unroll
    for (int d = 0; d < 2; ++d) {
        const int r = (wave * 2 + d) * 8 + (lane >> 3);
        dy_voff[d] = (uint32_t)(((int64_t)(ot * OT + r) * p.ys_o) * 2) + (uint32_t)(((lane & 7) ^ ((r >> 1) & 7)) * 16);
    }
#pragma unroll
    for (int d = 0; d < XI; ++d) {
        const int r = (wave * XI + d) * 8 + (lane >> 3);
        x_voff[d] = (uint32_t)(((int64_t)(ct * WG_CT + r) * p.xs_c) * 2) + (uint32_t)(((lane & 7) ^ ((r >> 1) & 7)) * 16);
    }
    uint32_t noff = 0;                              // byte offset of the current 64 images inside a row
    auto issue_dy = [&](int j, int buf) {
        const uint32_t soff = (uint32_t)(((int64_t)(i * p.OW + j) * p.ys_pix) * 2) + noff;
#pragma unroll
        for (int d = 0; d < 2; ++d) dma16(ddy, lds_a + buf * DY_BYTES + (wave * 2 + d) * 1024, dy_voff[d], soff);
    };
    // column w of the window rows, into its ring slots (rows and columns outside the image: nothing is fetched, the
    // taps that would read them read zeros instead)
    auto issue_col = [&](int w) {
        if (w < 0 || w >= p.W) return;
        const int cs = (w + RING_COLS) % RING_COLS;
#pragma unroll
        for (int a = 0; a < KH; ++a) {
            const int h = i * s + a - p.ph;
            if (h < 0 || h >= p.H) continue;
            const uint32_t soff = (uint32_t)(((int64_t)(h * p.W + w) * p.xs_pix) * 2) + noff;
#pragma unroll
            for (int d = 0; d < XI; ++d) dma16(ddx, lds_a + X_OFF + (a * RING_COLS + cs) * XT_BYTES + (wave * XI + d) * 1024, x_voff[d], soff);
        }
    };

    if (t < 32) *(uint32_t *)(lds + ZERO_OFF + t * 4) = 0u;

    // fragment addresses inside a tile: row (wave's 32 rows) x chunk 2 ks + fhalf, swizzled
    uint32_t fa_dy[4], fa_x[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        const int ra = wo * 32 + frow, rb = wc * 32 + frow;
        fa_dy[ks] = (uint32_t)(ra * 128 + (((2 * ks + fhalf) ^ ((ra >> 1) & 7)) << 4));
        fa_x[ks] = (uint32_t)(rb * 128 + (((2 * ks + fhalf) ^ ((rb >> 1) & 7)) << 4));
    }

    f32x16 acc[T];
#pragma unroll
    for (int tp = 0; tp < T; ++tp)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[tp][v] = 0.0f;

#pragma unroll 1
    for (int nc = 0; nc < p.nck; ++nc) {
    // ---- the first pixel's tiles of this group of 64 images (every wave has left the last group's tiles: the barrier
    // that ended its last pixel)
    noff = (uint32_t)nc * 128u;
    issue_dy(j0, 0);
#pragma unroll
    for (int b = 0; b < KW; ++b) issue_col(j0 * s + b - p.pw);
    RL_WAIT_VM(0);
    wg_barrier();

#pragma unroll 1
    for (int j = j0; j < j1; ++j) {
        const int buf = (j - j0) & 1;
        // the next pixel's tiles: dy, and the window columns this pixel's window does not hold
        if (j + 1 < j1) {
            issue_dy(j + 1, buf ^ 1);
            const int last = j * s + KW - 1 - p.pw;
#pragma unroll
            for (int b = 0; b < KW; ++b) {
                const int w = (j + 1) * s + b - p.pw;
                if (w > last) issue_col(w);
            }
        }
        // this pixel's taps: ring slot of each, or the zeros (scalars)
        uint32_t tap_off[T], tap_msk[T];
#pragma unroll
        for (int a = 0; a < KH; ++a)
#pragma unroll
            for (int b = 0; b < KW; ++b) {
                const int h = i * s + a - p.ph, w = j * s + b - p.pw;
                const bool ok = h >= 0 && h < p.H && w >= 0 && w < p.W;
                tap_off[a * KW + b] = ok ? (uint32_t)(X_OFF + (a * RING_COLS + (w + RING_COLS) % RING_COLS) * XT_BYTES) : (uint32_t)ZERO_OFF;
                tap_msk[a * KW + b] = ok ? 0xffffffffu : 0u;
            }
        constexpr int AHEAD = 3;                    // x fragments are read this many MFMAs before their own (an LDS read takes longer than an MFMA)
        u32x4 fdy[4], fx[AHEAD + 1];
        const unsigned char *dyb = lds + buf * DY_BYTES;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) fdy[ks] = *(const u32x4 *)(dyb + fa_dy[ks]);
#pragma unroll
        for (int u = 0; u < AHEAD && u < T * 4; ++u) fx[u] = *(const u32x4 *)(lds + tap_off[u >> 2] + (fa_x[u & 3] & tap_msk[u >> 2]));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < T * 4; ++u) {
            const int tp = u >> 2, ks = u & 3;
            if (u + AHEAD < T * 4) {
                const int tn = (u + AHEAD) >> 2, kn = (u + AHEAD) & 3;
                fx[(u + AHEAD) % (AHEAD + 1)] = *(const u32x4 *)(lds + tap_off[tn] + (fa_x[kn] & tap_msk[tn]));
                __builtin_amdgcn_sched_barrier(0);
            }
            acc[tp] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fdy[ks]), __builtin_bit_cast(bf16x8, fx[u % (AHEAD + 1)]), acc[tp], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        RL_WAIT_VM(0);                              // the next pixel's tiles have landed
        wg_barrier();                               // ... for every wave; and every wave has left this pixel's tiles
    }
    }

    // ---- this workgroup's sums: part[chunk][tap][o][c], accumulator register 4g + k of lane l: o = 8g + 4 (l >> 5) + k, c = l & 31
    float *out = p.part + ((int64_t)chunk * T * p.O + (ot * OT + wo * 32)) * p.C + ct * WG_CT + wc * 32 + frow;
#pragma unroll
    for (int tp = 0; tp < T; ++tp)
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int k = 0; k < 4; ++k)
                out[((int64_t)tp * p.O + 8 * g + 4 * fhalf + k) * p.C] = acc[tp][4 * g + k];
#endif
}

// dw[o][c][tap] = sum over segments of part[segment][tap][o][c], in a fixed order: a workgroup finishes 64 groups of four
// consecutive c; its sixteen waves each add up a contiguous share of the segments in order (four loads in flight at a
// time), and the first wave adds the sixteen shares in order.
constexpr int RED_WAVES = 16;
__global__ __launch_bounds__(64 * RED_WAVES) void wgrad_reduce_kernel(const float *__restrict__ part, void *out, int out_dtype, int chunks, int T, int O, int C)
{
    __shared__ f32x4 share[RED_WAVES][64];
    const int total4 = T * O * C / 4;
    const int lane = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const int item = blockIdx.x * 64 + lane;
    const int per = (chunks + RED_WAVES - 1) / RED_WAVES;
    const int c0 = grp * per, c1 = min(chunks, c0 + per);
    f32x4 sum = {0.0f, 0.0f, 0.0f, 0.0f};
    if (item < total4) {
        const f32x4 *src = (const f32x4 *)part + item;
        int sidx = c0;
        for (; sidx + 4 <= c1; sidx += 4) {
            const f32x4 v0 = src[(int64_t)sidx * total4], v1 = src[(int64_t)(sidx + 1) * total4];
            const f32x4 v2 = src[(int64_t)(sidx + 2) * total4], v3 = src[(int64_t)(sidx + 3) * total4];
            sum += v0; sum += v1; sum += v2; sum += v3;
        }
        for (; sidx < c1; ++sidx) sum += src[(int64_t)sidx * total4];
    }
    share[grp][lane] = sum;
    __syncthreads();
    if (grp != 0 || item >= total4) return;
    f32x4 tot = share[0][lane];
#pragma unroll
    for (int gidx = 1; gidx < RED_WAVES; ++gidx) tot += share[gidx][lane];
    const int idx = item * 4;
    const int c = idx % C, oc = idx / C, o = oc % O, tp = oc / O;
#pragma unroll
    for (int k = 0; k < 4; ++k) store_from_f32(out, out_dtype, ((int64_t)o * C + c + k) * T + tp, tot[k]);
}

bool conv_wgrad_ok(int32_t NB, int32_t O, int32_t C, int32_t KH, int32_t KW, int32_t s)
{
    return NB >= WG_NB && NB % WG_NB == 0 && O >= 64 && O % 64 == 0 && C >= 64 && C % 64 == 0 && ((KH == 3 && KW == 3) || (KH == 1 && KW == 1)) && (s == 1 || s == 2);
}

hipError_t launch_conv_wgrad(const WgradParams &p, hipStream_t s)
{
    const int64_t NB = (int64_t)p.nck * WG_NB;
    if (p.nck < 1 || p.nck > 64 || !conv_wgrad_ok((int32_t)NB, p.O, p.C, p.KH, p.KW, p.s) || !p.dyT || !p.xT || !p.part || ((uintptr_t)p.dyT & 15) || ((uintptr_t)p.xT & 15) ||
        ((uintptr_t)p.part & 3) || p.H < 1 || p.W < 1 || p.OH < 1 || p.OW < 1 || p.ph < 0 || p.pw < 0 || p.ph >= p.KH || p.pw >= p.KW ||
        p.OH != (p.H + 2 * p.ph - p.KH) / p.s + 1 || p.OW != (p.W + 2 * p.pw - p.KW) / p.s + 1 ||
        p.n_ct != p.C / WG_CT || (p.n_ot != p.O / 128 && p.n_ot != p.O / 64) || p.L < 1 || p.nseg != (p.OW + p.L - 1) / p.L ||
        p.ys_o < NB || p.ys_o % 8 != 0 || p.ys_pix % 8 != 0 || p.xs_c < NB || p.xs_c % 8 != 0 || p.xs_pix % 8 != 0 ||
        (uint64_t)p.dy_bytes != (uint64_t)p.OH * p.OW * p.O * NB * 2 || (uint64_t)p.x_bytes != (uint64_t)p.H * p.W * p.C * NB * 2 ||
        p.dy_bytes >= 0x7fffffffu || p.x_bytes >= 0x7fffffffu)
        return hipErrorInvalidValue;
    // every tile a workgroup requests lies inside its tensor: row (pixel, channel) starts at pixel*pix_stride + channel*ch_stride
    // and is 64 elements long; the largest such start over the tensor must leave room for the row
    const int64_t dy_last = (int64_t)(p.OH * p.OW - 1) * p.ys_pix + (int64_t)(p.O - 1) * p.ys_o + NB;
    const int64_t x_last = (int64_t)(p.H * p.W - 1) * p.xs_pix + (int64_t)(p.C - 1) * p.xs_c + NB;
    if (dy_last * 2 > (int64_t)p.dy_bytes || x_last * 2 > (int64_t)p.x_bytes) return hipErrorInvalidValue;
    const int64_t grid = (int64_t)p.OH * p.nseg * p.n_ot * p.n_ct;
    if (grid < 1 || grid > 0x7fffffff) return hipErrorInvalidValue;
    const bool wide = p.n_ot == p.O / 128 && p.O % 128 == 0;
    const bool k3 = p.KH == 3;
    if (wide && k3) hipLaunchKernelGGL((conv_wgrad_kernel<4, 3, 3>), dim3((unsigned)grid), dim3(512), 0, s, p);
    else if (wide) hipLaunchKernelGGL((conv_wgrad_kernel<4, 1, 1>), dim3((unsigned)grid), dim3(512), 0, s, p);
    else if (k3) hipLaunchKernelGGL((conv_wgrad_kernel<2, 3, 3>), dim3((unsigned)grid), dim3(256), 0, s, p);
    else hipLaunchKernelGGL((conv_wgrad_kernel<2, 1, 1>), dim3((unsigned)grid), dim3(256), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_wgrad_reduce(const float *part, void *out, int32_t out_dtype, int32_t chunks, int32_t T, int32_t O, int32_t C, hipStream_t s)
{
    if (!part || !out || chunks < 1 || T < 1 || O < 1 || C < 1 || (int64_t)T * O * C > 0x7fffffff) return hipErrorInvalidValue;
    if (C % 4 != 0 || ((uintptr_t)part & 15)) return hipErrorInvalidValue;
    const int total4 = T * O * C / 4;
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)((total4 + 63) / 64)), dim3(64 * RED_WAVES), 0, s, part, out, out_dtype, chunks, T, O, C);
    return hipGetLastError();
}

}  // namespace rl

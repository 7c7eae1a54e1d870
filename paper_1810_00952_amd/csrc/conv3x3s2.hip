// A stage's first block in one kernel: the 3x3 / stride 2 / pad 1 convolution and the 1x1 / stride 2 projection that
// reads the same input, bf16 in / fp32 accumulate / bf16 out, each with its own epilogue [f32 bias] [+ bf16 residual]
// [ReLU] and its own output.
//
// The projection reads x[2 oh, 2 ow], which is exactly the centre tap of the 3x3 window, so it is one more K tile of
// the same contraction with a second set of accumulators: the pixels of that tap are in LDS anyway.
//
// Run as implicit GEMMs that gather a fresh activation tile per K tile, the two convolutions are bound by their
// requests and by the start-up and wind-down of very short K loops.  Here, as in the stride-1 kernel next door, the
// input rows under a tile are copied to LDS once per 64-channel slice and serve every tap:
//   * A tile is 64 consecutive output pixels (flat over images and rows) x 128 output channels.  With even H and W,
//     flat output row R = img*OH + oh needs flat input rows 2R-1, 2R, 2R+1, and output column ow needs input columns
//     2ow-1, 2ow, 2ow+1; only the first of each can fall outside the image (oh = 0, ow = 0): those taps read zeros.
//   * The rows 2R0-1 .. 2R1+1 under the tile's output rows R0 .. R1 go to LDS with even and odd columns apart:
//     pixel (row r, column 2j + par) sits in slot (2r + par)*OW + j, 144 bytes per slot (nine 16-byte units, the
//     ninth unused).  The pixels that consecutive output pixels need for one tap are then consecutive slots, and
//     the address of tap (kh, kw) is the lane's own address plus a wave-uniform constant.
//   * K runs slice-major: per 64-channel slice the nine taps, with the projection's K tile right behind the centre
//     tap (same pixels, the projection's weights, the second accumulators): ten K tiles per slice, whose weight
//     tiles (128 rows x 128 bytes) stream through a ring of stages by direct loads.
//   * Four waves: wave (kq, nh) multiplies all 64 pixels by channels 64 nh .. +63 for the k-steps 2kq and 2kq+1 of
//     every K tile (four fragment reads for four MFMAs); the two partial sums of a tile meet in LDS at the end and
//     are finished row-wise: k-step pair 0 then 1, bias, residual, ReLU, one rounding, 16-byte stores.
// Results agree with the two convolutions run separately to fp32 summation order.
//
// Preconditions (checked by conv3x3s2_pair_ok, which the planner and the launcher share): bf16 throughout, the two
// contractions read the same dense channel-last tensor with even H and W and C a multiple of 64, have the same
// number of output channels (a multiple of 8), dense channel-last outputs, tensors below 2 GiB, and the rows under a
// tile fit the run buffer.
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
constexpr int PITCH = 144;                        // bytes per pixel slot in LDS
constexpr int S2_BM = 64, S2_BN = 128;
constexpr int S2_RL_A = 14, S2_RL_B = 18;         // run loads per wave of the two instances (56 KB / 72 KB of run buffer)
constexpr int S2_NB_A = 5, S2_NB_B = 5;            // weight-tile stages (six change nothing measurable)

// input rows under the 64 output pixels of a tile, at most
inline int s2_rows_max(int OW) { return 2 * ((OW - 1 + S2_BM - 1) / OW) + 3; }

}  // namespace

// RL: direct loads (64 units of 16 bytes) per wave per run.  NB: weight-tile stages; weight tile u + NB - 1 is
// requested while tile u is multiplied, and at a tile's end the requests of the last NB - 3 tiles may be in flight.
template <int RL, int NB>
__global__ __launch_bounds__(256) void conv3x3s2_pair_kernel(const IgemmParams p, const IgemmParams pd)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub; the body uses gfx950-only builtins
    constexpr int NW = 4, BM = S2_BM, BN = S2_BN;
    constexpr int RUN_BYTES = RL * NW * 1024;
    constexpr int BG = BN / (8 * NW);                             // weight-tile loads (8 rows each) per wave per K tile: 4
    constexpr int B_BYTES = BN * 128;
    constexpr int B_OFF = RUN_BYTES, Z_OFF = B_OFF + NB * B_BYTES;   // Z: one KB of zeros (masked taps read it)
    constexpr int LDS_BYTES = Z_OFF + 1024;
    constexpr int FLY = NB - 3;
    constexpr int PBYTES = BM * BN * 4;                           // one partial accumulator tile, fp32: 32 KB
    static_assert(4 * PBYTES <= LDS_BYTES && LDS_BYTES <= 160 * 1024, "LDS");
    static_assert(NB >= 4 && FLY * BG < 64, "ring depth");
    __shared__ __attribute__((aligned(1024))) unsigned char lds[LDS_BYTES];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int kq = wave & 1, nh = wave >> 1;        // k-step pair and channel half of the tile
    const int OW = p.OW, W = p.W, C = p.C;

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
    const u32x4 dw2 = make_desc(pd.w, pd.w_bytes);
    const uint32_t lds_a = lds_addr_of(lds);
    const int frow = lane & 31, fhalf = lane >> 5;

    // ---- geometry of the tile: output rows R0 .. R1 (flat over images), input rows Fb .. Fb + nrows - 1
    const int mlast = min(m0 + BM - 1, p.M - 1);
    const int R0 = (int)fast_div((uint32_t)m0, (uint32_t)OW, p.div_ow_mul, p.div_ow_sh);
    const int R1 = (int)fast_div((uint32_t)mlast, (uint32_t)OW, p.div_ow_mul, p.div_ow_sh);
    const int nrows = 2 * (R1 - R0) + 3;
    const int Fb = 2 * R0 - 1;
    const int Ftot = (p.M / p.OHW) * p.H;           // input rows of the whole tensor

    // ---- run requests: load k of the wave fills LDS units 64*(RL*wave + k) + lane; unit u is 16-byte chunk u % 9 of
    // slot u / 9 (chunk 8: padding, it fetches chunk 7 again); slot s = (2r + par)*OW + j is input pixel
    // (row Fb + r, column 2j + par).  Rows outside the tensor and slots past the tile's rows: out of range, zeros.
    uint32_t r_voff[RL];
#pragma unroll
    for (int k = 0; k < RL; ++k) {
        const uint32_t u = (uint32_t)(64 * (RL * wave + k) + lane);
        const uint32_t s = u / 9u, c = u - 9u * s;
        const uint32_t q = fast_div(s, (uint32_t)OW, p.div_ow_mul, p.div_ow_sh);
        const int j = (int)(s - q * (uint32_t)OW), r = (int)(q >> 1), par = (int)(q & 1u);
        const int F = Fb + r;
        const bool ok = r < nrows && F >= 0 && F < Ftot;
        r_voff[k] = ok ? (uint32_t)(((int64_t)F * W + 2 * j + par) * C * 2) + (c < 8u ? c : 7u) * 16u : OOB;
    }
    // weights: lane l of load d fills row wave*32 + 8d + (l >> 3), position l & 7, with chunk position ^ key(row)
    uint32_t b_voff[BG], b2_voff[BG];
    {
        const int r8 = lane >> 3, pos = lane & 7;
#pragma unroll
        for (int d = 0; d < BG; ++d) {
            const int row = wave * 8 * BG + 8 * d + r8;
            const int chunk = pos ^ ((row >> 1) & 7);
            int n = n0 + row;
            if (n > p.N - 1) n = p.N - 1;          // rows past N are computed on valid memory and never stored
            b_voff[d] = (uint32_t)((int64_t)n * p.Kp * 2) + chunk * 16;
            b2_voff[d] = (uint32_t)((int64_t)n * pd.Kp * 2) + chunk * 16;
        }
    }
    const int nsl = C / 64, NT = nsl * 10;
    // K tile v of a slice: taps 0..4, the projection, taps 5..8
    auto issue_b = [&](int d, int stage, int s, int v, bool live) {
        const uint32_t la = lds_a + B_OFF + stage * B_BYTES + (wave * BG + d) * 1024;
        if (v == 5) dma16(dw2, la, live ? b2_voff[d] : OOB, live ? (uint32_t)(64 * s * 2) : 0u);
        else dma16(dw, la, live ? b_voff[d] : OOB, live ? (uint32_t)((((v < 5 ? v : v - 1)) * C + 64 * s) * 2) : 0u);
    };
    auto issue_run = [&](int s) {
#pragma unroll
        for (int k = 0; k < RL; ++k) dma16(dx, lds_a + (RL * wave + k) * 1024, r_voff[k], (uint32_t)(s * 128));
    };

    // ---- prologue: run of slice 0, weight tiles 0 .. NB-2
    issue_run(0);
#pragma unroll
    for (int u = 0; u < NB - 1; ++u)
#pragma unroll
        for (int d = 0; d < BG; ++d) issue_b(d, u, 0, u, u < NT);
    if (t < 64) *(u32x4 *)(lds + Z_OFF + t * 16) = u32x4{0u, 0u, 0u, 0u};

    // ---- the lane's pixels: fragment base address in the run buffer (its k-step pair folded in), tap validity
    uint32_t fa[2], tmask[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int m = m0 + 32 * i + frow;
        const int mm = m < p.M ? m : p.M - 1;
        const int R = (int)fast_div((uint32_t)mm, (uint32_t)OW, p.div_ow_mul, p.div_ow_sh), ow = mm - R * OW;
        const int img = (int)fast_div((uint32_t)mm, (uint32_t)p.OHW, p.div_ohw_mul, p.div_ohw_sh);
        const int oh = R - img * p.OH;
        fa[i] = (uint32_t)((4 * (R - R0) * OW + ow) * PITCH + fhalf * 16 + kq * 64);
        const uint32_t rows = (oh > 0 ? 0x007u : 0u) | 0x1f8u;
        const uint32_t cols = (ow > 0 ? 0x049u : 0u) | 0x1b6u;
        tmask[i] = m < p.M ? (rows & cols) : 0u;
    }
    // weight fragments: row frow of a 32-row MFMA tile of the wave's 64 channels, chunk 2*ks + fhalf, swizzled
    uint32_t fb[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
        fb[kk] = (uint32_t)(B_OFF + (nh * 64 + frow) * 128 + (((2 * (2 * kq + kk) + fhalf) ^ ((frow >> 1) & 7)) << 4));

    wait_vm<FLY * BG>();                            // the run and weight tiles 0, 1
    RL_WAIT_LGKM0;
    wg_barrier();

    f32x16 acc[2][2], acc2[2][2];
    u32x4 fx[2][2], fw[2][2];
    uint32_t a0[2], a0n[2];
    // fragment read r of k-step kk: r < 2: pixels, tile r; else weights, tile r - 2
    auto frag_read = [&](int r, int kk, uint32_t bstage, const uint32_t *pix) {
        if (r < 2) fx[kk][r < 2 ? r : 0] = *(const u32x4 *)(lds + pix[r < 2 ? r : 0] + kk * 32);
        else fw[kk][r >= 2 ? r - 2 : 0] = *(const u32x4 *)(lds + fb[kk] + bstage + (r >= 2 ? r - 2 : 0) * 4096);
    };
    // addresses of tap tp: (kh, kw) -> slot offset ((2 kh + par) OW + dj), par/dj = 1/-1, 0/0, 1/0 for kw = 0, 1, 2
    auto tap_addr = [&](int tp, uint32_t *out) {
        const int kh = tp / 3, kw = tp % 3;
        const int par = kw == 1 ? 0 : 1, dj = kw == 0 ? -1 : 0;
        const int toff = ((2 * kh + par) * OW + dj) * PITCH;
#pragma unroll
        for (int i = 0; i < 2; ++i) out[i] = ((tmask[i] >> tp) & 1u) ? (uint32_t)((int)fa[i] + toff) : (uint32_t)(Z_OFF + fhalf * 16 + kq * 64);
    };
    tap_addr(0, a0);
#pragma unroll
    for (int r = 0; r < 4; ++r) frag_read(r, 0, 0u, a0);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) { acc[i][j][v] = 0.0f; acc2[i][j][v] = 0.0f; }
    __builtin_amdgcn_sched_barrier(0);

    int st_cur = 0;                                 // weight stage of the current K tile: u % NB
#pragma unroll 1
    for (int s = 0; s < nsl; ++s) {
        const bool more = s + 1 < nsl;
#pragma unroll
        for (int v = 0; v < 10; ++v) {
            // K tile u = 10 s + v.  On entry: the barrier of this tile has been passed, weight tiles u and u+1 and the
            // slice's run have landed, and the fragments of the wave's first k-step are in register set 0.
            const int st_next = st_cur + 1 == NB ? 0 : st_cur + 1, st_iss = st_cur == 0 ? NB - 1 : st_cur - 1;
            const uint32_t bcur = (uint32_t)(st_cur * B_BYTES), bnext = (uint32_t)(st_next * B_BYTES);
            // this tile's requests: weight tile u + NB - 1 into the stage tile u - 1 has left
            const int vb = (v + NB - 1) % 10, sb = s + (v + NB - 1) / 10;
            const bool blive = sb < nsl;
            const int tp_next = v + 1 < 5 ? v + 1 : (v + 1 == 5 ? 4 : (v + 1 == 10 ? 0 : v));   // tap of the next K tile
            const bool last_of_slice = v == 9;
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                int r = 0;
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        if (v == 5)
                            acc2[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fw[kk][j]), __builtin_bit_cast(bf16x8, fx[kk][i]),
                                                                                acc2[i][j], 0, 0, 0);
                        else
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fw[kk][j]), __builtin_bit_cast(bf16x8, fx[kk][i]),
                                                                               acc[i][j], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                        // behind the MFMA: one fragment read of the next k-step (after the tile's second k-step: of the
                        // next tile, whose pixels are not there yet when that tile opens a new slice) ...
                        if (kk == 0) frag_read(r, 1, bcur, a0);
                        else if (r >= 2 || !last_of_slice) frag_read(r, 0, bnext, a0n);
                        ++r;
                        // ... and, in the first k-step, one request of the tile and the next tile's pixel addresses
                        if (kk == 0) {
                            issue_b(2 * i + j, st_iss, sb, vb, blive);
                            if (i == 1 && j == 1) tap_addr(tp_next, a0n);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
            }
#pragma unroll
            for (int i = 0; i < 2; ++i) a0[i] = a0n[i];
            st_cur = st_next;
            wait_vm<FLY * BG>();                    // everything but the last FLY tiles' requests: weight tile u + 2 has landed
            wg_barrier();
            if (last_of_slice && more) {
                // every wave has left the run buffer: the next slice's rows (nothing multiplies meanwhile)
                issue_run(s + 1);
                wait_vm<0>();
                wg_barrier();
                frag_read(0, 0, 0u, a0);
                frag_read(1, 0, 0u, a0);
            }
        }
    }
    wait_vm<0>();                                   // the trailing out-of-range requests
    wg_barrier();

    // ---- operands of the finishing passes: thread t finishes, in pass q, row 16q + t/16, channels 8*(t%16) .. +7
    const int rr = t >> 4, pp = t & 15;
    const int nfin = n0 + 8 * pp;
    f32x4 bias_lo[2], bias_hi[2];
    u32x4 res_r[2][4];
    uint32_t y_off[2][4];
#pragma unroll
    for (int o = 0; o < 2; ++o) {
        const IgemmParams &po = o == 0 ? p : pd;
        const Epilogue &e = po.epi;
        const bool has_res = e.t_op >= 0;
        const rsrc_t rb = make_rsrc(e.has_bias ? e.bias_ptr : po.w, e.has_bias ? (uint32_t)po.N * 4u : 0u);
        const rsrc_t rres = make_rsrc(has_res ? e.t_ptr : po.w, has_res ? po.y_bytes : 0u);
        bias_lo[o] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rb, nfin < po.N ? (uint32_t)nfin * 4u : OOB, 0, 0));
        bias_hi[o] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rb, nfin < po.N ? (uint32_t)nfin * 4u + 16u : OOB, 0, 0));
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int m = m0 + 16 * q + rr;
            y_off[o][q] = (m < po.M && nfin < po.N) ? (uint32_t)(((int64_t)m * po.ys_p + nfin) * 2) : OOB;
            res_r[o][q] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rres, y_off[o][q], 0, 0));
        }
    }

    // ---- the partial tiles go to LDS (16-byte chunks of a 512-byte row XOR-swizzled by the row): output o, k-step pair kq
    // at (2 o + kq) * 32 KB ...
#pragma unroll
    for (int o = 0; o < 2; ++o) {
        unsigned char *park = lds + (2 * o + kq) * PBYTES;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int row = i * 32 + frow;
                    const int c = nh * 16 + j * 8 + 2 * g + fhalf;      // 4-channel chunk of the row, 0..31
                    f32x4 v;
#pragma unroll
                    for (int k = 0; k < 4; ++k) v[k] = o == 0 ? acc[i][j][4 * g + k] : acc2[i][j][4 * g + k];
                    *(f32x4 *)(park + row * (BN * 4) + ((c ^ (row & 31)) << 4)) = v;
                }
    }
    RL_WAIT_LGKM0;
    wg_barrier();
    // ... and are summed row-wise in k-step order, then bias, residual, ReLU, one rounding
#pragma unroll
    for (int o = 0; o < 2; ++o) {
        const IgemmParams &po = o == 0 ? p : pd;
        const rsrc_t ry = make_rsrc(po.y, po.y_bytes);
        const float lo = po.epi.relu_last ? 0.0f : -INFINITY;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int row = 16 * q + rr;
            float v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = 0.0f;
#pragma unroll
            for (int w = 0; w < 2; ++w) {
                const unsigned char *prow = lds + (2 * o + w) * PBYTES + row * (BN * 4);
                const f32x4 a = *(const f32x4 *)(prow + (((2 * pp) ^ (row & 31)) << 4));
                const f32x4 b = *(const f32x4 *)(prow + (((2 * pp + 1) ^ (row & 31)) << 4));
#pragma unroll
                for (int k = 0; k < 4; ++k) { v[k] += a[k]; v[4 + k] += b[k]; }
            }
            const u32x4 rs = res_r[o][q];
#pragma unroll
            for (int k = 0; k < 4; ++k) { v[k] += bias_lo[o][k]; v[4 + k] += bias_hi[o][k]; }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                v[2 * k] += __uint_as_float(rs[k] << 16);
                v[2 * k + 1] += __uint_as_float(rs[k] & 0xffff0000u);
            }
            u32x4 ov;
#pragma unroll
            for (int k = 0; k < 4; ++k)
                ov[k] = pack_bf16x2(fmaxf(v[2 * k], lo), fmaxf(v[2 * k + 1], lo));
            __builtin_amdgcn_raw_buffer_store_b128(ov, ry, y_off[o][q], 0, 0);
        }
    }
#endif
}

static bool s2_epilogue_ok(const Epilogue &e0)
{
    Epilogue e = e0;                                // the planner asks before the classification fields are filled in
    finalize_epilogue(e);
    return e.simple && (!e.has_bias || e.bias_dtype == DT_F32) && (e.t_op < 0 || (e.t_op == E_ADD && e.t_dtype == DT_BF16)) &&
           (e.rest_n == 0 || e.relu_last);
}

// a: the 3x3 / stride 2 / pad 1 convolution, b: the 1x1 / stride 2 / pad 0 projection of the same input.
// Pointers are not looked at (the planner asks before any are bound); the launcher compares them itself.
bool conv3x3s2_pair_ok(const IgemmParams &a, const IgemmLaunch &la, const IgemmParams &b, const IgemmLaunch &lb)
{
    if (!la.lp || !lb.lp || la.ws || lb.ws || la.c64 || lb.c64 || la.run || lb.run || la.gates || lb.gates || la.splits > 1 || lb.splits > 1 ||
        la.anyact || lb.anyact) return false;
    if (a.in_dtype != DT_BF16 || b.in_dtype != DT_BF16 || a.y_dtype != DT_BF16 || b.y_dtype != DT_BF16) return false;
    if (a.KH != 3 || a.KW != 3 || a.sh != 2 || a.sw != 2 || a.ph != 1 || a.pw != 1) return false;
    if (b.KH != 1 || b.KW != 1 || b.sh != 2 || b.sw != 2 || b.ph != 0 || b.pw != 0) return false;
    if (a.C != b.C || a.H != b.H || a.W != b.W || a.M != b.M || a.N != b.N || a.OH != b.OH || a.OW != b.OW || a.OHW != b.OHW) return false;
    if (a.C < 64 || a.C % 64 != 0 || a.N % 8 != 0 || a.H % 2 != 0 || a.W % 2 != 0 || a.OH * 2 != a.H || a.OW * 2 != a.W || a.OHW != a.OH * a.OW) return false;
    if (a.M < 1 || a.M % a.OHW != 0 || a.K != 9 * a.C || a.Kp != a.K || b.K != b.C || b.Kp != b.K) return false;
    const int64_t HW = (int64_t)a.H * a.W;
    for (const IgemmParams *q : {&a, &b}) {
        if (q->xs_c != 1 || q->xs_w != q->C || q->xs_h != (int64_t)q->W * q->C || q->xs_n != HW * q->C) return false;
        if (q->ys_c != 1 || q->ys_p < q->N || q->ys_n != (int64_t)q->OHW * q->ys_p) return false;
        if (!s2_epilogue_ok(q->epi)) return false;
        if ((uint64_t)q->M * (uint64_t)q->ys_p * 2 >= 0x7fffffffull) return false;
    }
    const uint64_t xb = (uint64_t)(a.M / a.OHW) * (uint64_t)HW * a.C * 2;
    if (xb >= 0x7fffffffull || a.x_bytes != (uint32_t)xb || b.x_bytes != (uint32_t)xb) return false;
    if (a.w_bytes < (uint64_t)a.N * a.Kp * 2 || b.w_bytes < (uint64_t)b.N * b.Kp * 2) return false;
    // the rows under a tile must fit the larger run buffer
    const int64_t units = (int64_t)s2_rows_max(a.OW) * 2 * a.OW * 9;
    return units <= (int64_t)S2_RL_B * 4 * 64;
}

hipError_t launch_conv3x3s2_pair(const IgemmParams &a0, const IgemmLaunch &la, const IgemmParams &b0, const IgemmLaunch &lb, hipStream_t s)
{
    if (!conv3x3s2_pair_ok(a0, la, b0, lb) || a0.x != b0.x || !a0.x || !a0.w || !b0.w || !a0.y || !b0.y) return hipErrorInvalidValue;
    IgemmParams a = a0, b = b0;
    a.nblk_m = (a.M + S2_BM - 1) / S2_BM;
    a.nblk_n = (a.N + S2_BN - 1) / S2_BN;
    const int64_t nblk = (int64_t)a.nblk_m * a.nblk_n;
    if (nblk <= 0 || nblk > 0x7fffffff) return hipErrorInvalidValue;
    const int64_t units = (int64_t)s2_rows_max(a.OW) * 2 * a.OW * 9;
    if (units <= (int64_t)S2_RL_A * 4 * 64) hipLaunchKernelGGL((conv3x3s2_pair_kernel<S2_RL_A, S2_NB_A>), dim3((unsigned)nblk), dim3(256), 0, s, a, b);
    else hipLaunchKernelGGL((conv3x3s2_pair_kernel<S2_RL_B, S2_NB_B>), dim3((unsigned)nblk), dim3(256), 0, s, a, b);
    return hipGetLastError();
}

}  // namespace rl

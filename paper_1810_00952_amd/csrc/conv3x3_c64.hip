// 3x3, stride 1, pad 1 convolution from 64 to 64 channels, bf16 in / fp32
// accumulate / bf16 out, with the epilogue [f32 bias] [+ bf16 residual] [ReLU]:
// the shape of a ResNet's first stage, where a general implicit-GEMM kernel
// spends its time requesting operands (a K loop of nine tiles, 72 KB of weights
// re-fetched by every workgroup, every input pixel fetched nine times) rather
// than multiplying.
//
// With 64 input channels a pixel is 128 bytes, exactly one K tile of the GEMM
// row of one filter tap, and with stride 1 on an unchanged image size the tap
// (kh, kw) of flat output pixel t (within its image) is flat input pixel
// t + (kh-1)*W + (kw-1).  So nothing needs to be expanded:
//   * Workgroups are persistent, two per CU (each XCD owns a contiguous run of
//     regions): while one is in its epilogue, at its barrier or requesting data,
//     the other one's waves keep the MFMA pipes busy.  A region is 128
//     consecutive output pixels of one image; wave (mh, nh) owns its pixels
//     64*mh .. +63 and output channels 32*nh .. +31.
//   * The weights are read once per workgroup into registers as MFMA
//     fragments, 144 registers per lane, from a copy that the weight packing
//     lays out in exactly that order (behind the usual 64 x 576 matrix), so
//     that every load is one contiguous KB per wave.
//   * The region's input pixels t0 - W - 1 ... t0 + 128 + W (a flat run of
//     130 + 2W pixels) are copied to LDS once by direct loads, double-buffered:
//     the next region's run arrives while this one is multiplied.  A pixel
//     occupies 144 bytes there (nine 16-byte units, the ninth unused): with
//     that pitch the fragment reads of 16 consecutive pixels fall into 16
//     different bank groups, and the address of tap (kh, kw) of the lane's
//     pixel is its own address plus (kh*W + kw)*144, a wave-uniform constant.
//   * Taps outside the image (which on a flat run includes the neighbour that
//     wraps around an image row) are redirected per lane to 128 bytes of zeros.
//   * A wave's instruction stream is serial, and its MFMAs are the only part
//     that has to take the time it takes; so the requests for the next run and
//     for this region's residual pieces are issued from inside the K loop, in
//     the slots between two MFMAs, where their address arithmetic is hidden.
// That leaves, per wave and region, 72 MFMAs, as many fragment reads, and one
// workgroup barrier per region.
//
// MFMA: weights are the row operand, so a lane holds one pixel and, per group
// of four accumulator registers, four consecutive channels.  Epilogue in
// registers: bias, residual (8-byte pieces in accumulator layout, requested at
// the start of the region), ReLU, one rounding to bf16; the two half-waves
// then trade halves (v_permlane32_swap) so that each lane stores 16 contiguous
// bytes.
//
// Preconditions (checked by the launcher and the planner): bf16 throughout,
// C = N = 64, 3x3, stride 1, pad 1, W <= 63, activations and output dense
// channel-last, tensors below 2 GiB.
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

constexpr int NUM_XCD = 8;
constexpr uint32_t OOB = 0x80000000u;
constexpr int CH = 64, NTAP = 9;
constexpr int C64_BM = 128;                       // pixels of a region
constexpr int W_MAX = 63;                         // widest image row: a run is BM + 2W + 2 pixels
constexpr int C64_RUN_PIX = C64_BM + 2 * W_MAX + 2;   // longest run: 256 pixels
constexpr uint32_t C64_W_BYTES = 64 * 9 * 64 * 2;     // the packed 64 x 576 matrix; the fragment-order copy follows it
constexpr int PITCH = 144;                        // bytes per pixel in LDS: nine 16-byte units, the last unused

}  // namespace

template <bool HAS_RES>
__global__ __launch_bounds__(256, 2) void conv3x3_c64_kernel(const IgemmParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub; the body uses gfx950-only builtins
    constexpr int RUN_LOADS = C64_RUN_PIX * 9 / 256;              // direct loads (64 units each) per wave per run: 9
    constexpr int RUN_BYTES = RUN_LOADS * 4 * 1024;               // one run buffer: 36 KB
    static_assert(C64_RUN_PIX * 9 % 256 == 0 && RUN_LOADS + 8 <= NTAP * 4, "LDS layout, one request per k-step");
    constexpr int BIAS_OFF = 2 * RUN_BYTES, ZERO_OFF = BIAS_OFF + CH * 4;
    constexpr int NSET = 3;                                       // fragment sets: reads run two k-steps ahead of the MFMAs
    __shared__ __attribute__((aligned(1024))) unsigned char lds[ZERO_OFF + 128];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int mh = wave & 1, nh = wave >> 1;        // pixel half, channel half of the region
    const int W = p.W, HW = p.H * p.W;
    const int n_img = p.M / HW;

    // ---- this workgroup's regions: XCD x = blockIdx % 8 owns the run [x*per, (x+1)*per) of the region
    // list (image-major); its workgroups take them in turn
    const int tpi = (HW + C64_BM - 1) / C64_BM;     // regions per image
    const int nreg = n_img * tpi;
    const int per = (nreg + NUM_XCD - 1) / NUM_XCD;
    const int xcd = blockIdx.x % NUM_XCD, slot = blockIdx.x / NUM_XCD, nslot = gridDim.x / NUM_XCD;
    const int run_end = min(nreg, (xcd + 1) * per);
    const int first = xcd * per + slot;
    const int my = first < run_end ? (run_end - first + nslot - 1) / nslot : 0;
    if (my == 0) return;                            // whole workgroup leaves together

    const u32x4 dx = make_desc(p.x, p.x_bytes);
    const uint32_t lds_a = lds_addr_of(lds);
    const int frow = lane & 31, fhalf = lane >> 5;
    const Epilogue &e = p.epi;
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(p.y, 0, p.y_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rres = __builtin_amdgcn_make_buffer_rsrc((void *)(HAS_RES ? e.t_ptr : p.w), 0, HAS_RES ? p.y_bytes : 0u, 0x00020000);
    const float lo = e.relu_last ? 0.0f : -INFINITY;

    // ---- requests.  Load k of the wave fills LDS units 64*(9*wave + k) + lane of a buffer; unit u is 16-byte chunk
    // u % 9 of pixel u / 9 (chunk 8: padding, nothing fetched).  Run pixel q is input pixel t0 - W - 1 + q of the
    // region's image; outside the image: out of range, zeros.
    const int run_len = C64_BM + 2 * W + 2;
    int rlane = lane;                               // the lane number as the request arithmetic sees it (see the loop)
    // q0: input pixel of run pixel 0 (may be negative); gbase: its byte offset (may wrap below zero; only used in range)
    auto run_voff = [&](int k, int q0, uint32_t gbase, bool live) -> uint32_t {
        const uint32_t u = (uint32_t)(64 * (RUN_LOADS * wave + k) + rlane);
        const uint32_t px = u / 9u, c = u - 9u * px;
        const int q = q0 + (int)px;
        // the padding unit fetches chunk 7 again (nobody reads it) rather than nothing: lanes out of range in every
        // request are slower than the 16 bytes they save
        const bool ok = live && (int)px < run_len && q >= 0 && q < HW;
        return ok ? gbase + px * 128u + (c < 8u ? c : 7u) * 16u : OOB;
    };
    auto run_issue = [&](int k, int buf, uint32_t voff) { dma16(dx, lds_a + buf * RUN_BYTES + (RUN_LOADS * wave + k) * 1024, voff, 0u); };
    {                                               // the first run, on its way while the weights are fetched
        const int img = first / tpi, t0 = (first - img * tpi) * C64_BM;
#pragma unroll
        for (int k = 0; k < RUN_LOADS; ++k) run_issue(k, 0, run_voff(k, t0 - W - 1, (uint32_t)(((int64_t)img * HW + t0 - W - 1) * 128), true));
    }

    // ---- weights: the fragment-order copy behind the packed matrix.  Fragment (tap, ks) of lane l of a wave with
    // channel half nh: 16 bytes at (((nh*9 + tap)*4 + ks)*64 + l)*16
    // (the bias is requested before them: a value requested behind the weights could only be used once they all
    // have arrived)
    float bias_v = 0.0f;
    if (t < CH && e.has_bias) bias_v = ((const float *)e.bias_ptr)[t];
    u32x4 wreg[NTAP][4];
    {
        const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void *)((const unsigned char *)p.w + C64_W_BYTES), 0, C64_W_BYTES, 0x00020000);
#pragma unroll
        for (int tp = 0; tp < NTAP; ++tp)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                wreg[tp][ks] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rw, (uint32_t)((((nh * NTAP + tp) * 4 + ks) * 64 + lane) * 16), 0, 0));
    }
    // bias and the zeros, in LDS for the whole kernel
    if (t < CH) *(float *)(lds + BIAS_OFF + t * 4) = bias_v;
    else if (t < CH + 32) *(uint32_t *)(lds + ZERO_OFF + (t - CH) * 4) = 0u;


    // the lane's two pixels within a region, and their fragment base addresses within a run buffer
    int pj[2];
    uint32_t fa[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        pj[i] = mh * 64 + 32 * i + frow;
        fa[i] = (uint32_t)(pj[i] * PITCH + fhalf * 16);
    }
    // the first run (this wave's part) has arrived once at most the 36 weight requests behind it are in flight; the
    // weights themselves are waited for tap by tap, by the compiler's own counting at their first use in the loop, so
    // that the first region starts multiplying while most of them are still on their way
    RL_WAIT_VM(36);
    RL_WAIT_LGKM0;                                  // bias and zeros written before the loop's first barrier

    f32x16 acc[2];
#pragma unroll 1
    for (int ri = 0; ri < my; ++ri) {
        const int reg = first + ri * nslot;
        const int img = reg / tpi, t0 = (reg - img * tpi) * C64_BM;
        const unsigned char *pa = lds + (ri & 1) * RUN_BYTES;
        const uint32_t zero_rel = (uint32_t)(ZERO_OFF - (int)((ri & 1) * RUN_BYTES));
        wg_barrier();                               // the whole run is there (each wave has waited for its part); every
                                                    // wave has left the other buffer
        // the next region's run is requested from inside the K loop (after the last one: nothing is fetched).  The
        // requests' per-lane address arithmetic is redone every time rather than kept in registers across the loop:
        // the register file is full of weights
        asm volatile("" : "+v"(rlane));
        const bool more = ri + 1 < my;
        const int nimg = (reg + nslot) / tpi, nt0 = (reg + nslot - nimg * tpi) * C64_BM;
        const uint32_t nrun_base = (uint32_t)(((int64_t)nimg * HW + nt0 - W - 1) * 128);

        // ---- the lane's pixels: tap validity and output offset (of its own 4-channel piece of group 0)
        uint32_t tmask[2], y_off[2];
        u32x2 res_r[2][4];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int tt = t0 + pj[i];
            const bool in = tt < HW;
            const int oh = (int)fast_div((uint32_t)tt, (uint32_t)W, p.div_ow_mul, p.div_ow_sh), ow = tt - oh * W;
            const uint32_t rows = (oh > 0 ? 0x007u : 0u) | 0x038u | (oh < p.H - 1 ? 0x1c0u : 0u);
            const uint32_t cols = (ow > 0 ? 0x049u : 0u) | 0x092u | (ow < W - 1 ? 0x124u : 0u);
            tmask[i] = in ? (rows & cols) : 0u;
            y_off[i] = in ? (uint32_t)((((int64_t)img * HW + tt) * CH + nh * 32 + 4 * fhalf) * 2) : OOB;
        }

        // ---- K loop: nine taps x four k-steps; fragments are read NSET-1 k-steps ahead of their MFMAs.
        // Address of (tap, pixel i, k-step ks): fa[i] + (kh*W + kw)*PITCH + 32*ks; an invalid tap reads zeros.
        u32x4 fx[NSET][2];
        uint32_t a0[2][2];
        auto read = [&](int s, int i) {
            const int tp = s >> 2, ks = s & 3;
            if (ks == 0) {
                const uint32_t toff = (uint32_t)(((tp / 3) * W + tp % 3) * PITCH);
                a0[tp & 1][i] = ((tmask[i] >> tp) & 1u) ? fa[i] + toff : zero_rel;
            }
            fx[s % NSET][i] = *(const u32x4 *)(pa + a0[tp & 1][i] + ks * 32);
        };
#pragma unroll
        for (int s = 0; s < NSET - 1; ++s) { read(s, 0); read(s, 1); }
        __builtin_amdgcn_sched_barrier(0);
        const f32x16 zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int s = 0; s < NTAP * 4; ++s) {
            const int tp = s >> 2, ks = s & 3;
            // every fragment read (which holds the wave for as long as an MFMA holds the pipe) and every other
            // instruction follows an MFMA, so that it is issued while that MFMA executes
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wreg[tp][ks]), __builtin_bit_cast(bf16x8, fx[s % NSET][0]),
                                                             s == 0 ? zero : acc[0], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (s + NSET - 1 < NTAP * 4) read(s + NSET - 1, 0);
            // the address of request s, or residual piece s - RUN_LOADS
            uint32_t voff = 0;
            if (s < RUN_LOADS) voff = run_voff(s, nt0 - W - 1, nrun_base, more);
            if (HAS_RES && s >= RUN_LOADS && s < RUN_LOADS + 8) {
                const int i = (s - RUN_LOADS) >> 2, g = (s - RUN_LOADS) & 3;
                res_r[i][g] = __builtin_bit_cast(u32x2, __builtin_amdgcn_raw_buffer_load_b64(rres, y_off[i] != OOB ? y_off[i] + 16u * g : OOB, 0, 0));
            }
            __builtin_amdgcn_sched_barrier(0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wreg[tp][ks]), __builtin_bit_cast(bf16x8, fx[s % NSET][1]),
                                                             s == 0 ? zero : acc[1], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (s + NSET - 1 < NTAP * 4) read(s + NSET - 1, 1);
            if (s < RUN_LOADS) run_issue(s, (ri + 1) & 1, voff);
            __builtin_amdgcn_sched_barrier(0);
        }

        RL_WAIT_VM(0);                              // the next run has long arrived; waiting here rather than at the barrier
                                                    // keeps this region's stores out of the wait
        // ---- epilogue in registers.  Accumulator register 4g + k of lane l, tile i: channel 32*nh + 8g + 4*(l >> 5) + k
        // of pixel 32i + (l & 31).  After the swap a lane holds 8 consecutive channels.
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            u32x2 pk[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 b = *(const f32x4 *)(lds + BIAS_OFF + (32 * nh + 8 * g + 4 * fhalf) * 4);
                float v[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) v[k] = acc[i][4 * g + k] + b[k];
                if (HAS_RES) {
                    const u32x2 r = res_r[i][g];
                    v[0] += __uint_as_float(r[0] << 16); v[1] += __uint_as_float(r[0] & 0xffff0000u);
                    v[2] += __uint_as_float(r[1] << 16); v[3] += __uint_as_float(r[1] & 0xffff0000u);
                }
                pk[g] = u32x2{pack_bf16x2(fmaxf(v[0], lo), fmaxf(v[1], lo)), pack_bf16x2(fmaxf(v[2], lo), fmaxf(v[3], lo))};
            }
            // y_off points at the lane's own 4-channel piece of group 0; the 16-byte store starts at channel
            // 16G + 8*fhalf of the wave's 32, i.e. 8*fhalf bytes further than 2 * (16G + 4*fhalf)
            const uint32_t yb = y_off[i] != OOB ? y_off[i] + (uint32_t)(8 * fhalf) : OOB;
#pragma unroll
            for (int G = 0; G < 2; ++G) {
                // lower half-wave keeps group 2G and receives its upper partner's, the upper half-wave keeps
                // group 2G+1 and receives its lower partner's: 8 consecutive channels per lane
                const u32x2 s0 = __builtin_amdgcn_permlane32_swap(pk[2 * G][0], pk[2 * G + 1][0], false, false);
                const u32x2 s1 = __builtin_amdgcn_permlane32_swap(pk[2 * G][1], pk[2 * G + 1][1], false, false);
                const u32x4 o = {s0[0], s1[0], s0[1], s1[1]};
                __builtin_amdgcn_raw_buffer_store_b128(o, ry, yb != OOB ? yb + 32u * G : OOB, 0, 0);
            }
        }
    }
#endif
}

hipError_t launch_conv3x3_c64(const IgemmParams &p, hipStream_t s)
{
    // the kernel's addressing assumes exactly this geometry
    const int64_t HW = (int64_t)p.H * p.W;
    if (p.in_dtype != DT_BF16 || p.y_dtype != DT_BF16 || p.x2 || p.C != CH || p.N != CH || p.KH != 3 || p.KW != 3 || p.sh != 1 || p.sw != 1 ||
        p.ph != 1 || p.pw != 1 || p.OH != p.H || p.OW != p.W || p.W < 1 || p.W > W_MAX || p.K != NTAP * CH || p.Kp != p.K ||
        HW < 1 || p.M % HW != 0 || p.xs_c != 1 || p.xs_w != CH || p.xs_h != (int64_t)p.W * CH || p.xs_n != HW * CH ||
        p.ys_c != 1 || p.ys_p != CH || p.ys_n != HW * CH || (uint64_t)p.M * CH * 2 >= 0x7fffffffull ||
        p.x_bytes != (uint32_t)((uint64_t)p.M * CH * 2) || p.y_bytes != p.x_bytes || p.w_bytes < 2 * C64_W_BYTES ||
        !p.epi.simple || (p.epi.has_bias && p.epi.bias_dtype != DT_F32) || (p.epi.t_op >= 0 && (p.epi.t_op != E_ADD || p.epi.t_dtype != DT_BF16)) ||
        (p.epi.rest_n != 0 && !p.epi.relu_last))
        return hipErrorInvalidValue;
    const int64_t nreg = (int64_t)(p.M / HW) * ((HW + C64_BM - 1) / C64_BM);
    int grid = 512;                                 // two workgroups per CU, a multiple of the XCD count
    if (nreg < grid) grid = (int)((nreg + NUM_XCD - 1) / NUM_XCD * NUM_XCD);
    if (p.epi.t_op >= 0) hipLaunchKernelGGL(conv3x3_c64_kernel<true>, dim3((unsigned)grid), dim3(256), 0, s, p);
    else hipLaunchKernelGGL(conv3x3_c64_kernel<false>, dim3((unsigned)grid), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace rl

// Few-channel stem convolution (stride 2) with its bias / ReLU epilogue and the 3x3 / stride 2 / pad 1 max-pool behind
// it in one kernel, reading the channel-first input as it is: no padded channel-last frame is written first.
// bf16 in / fp32 accumulate / bf16 out.  (stem_pool.hip is the same fusion on the 4-channel frame; this file replaces
// frame + kernel where the geometry allows: at most three input planes of even width, filter at most 8 rows high and,
// with an odd left padding, at most 7 columns wide.)
//
// A contraction index is (plane c, filter row kh, column j of an 8-pixel window): the 16 bytes a lane feeds an MFMA
// are eight neighbouring pixels of ONE plane row, so they can be read from a copy of the raw planes and nothing has to
// interleave channels.  The window of output column ox starts at the even pixel 2 ox - pw - e (e = pw & 1), so that
// every window is dword-aligned in a row that is itself copied from a dword-aligned position; filter column kw is window
// column kw + e and the window columns the filter does not cover meet zero weights (packed that way).  A k-step of 16
// is one plane and the filter rows 2r (lanes 0-31) and 2r + 1 (lanes 32-63); a filter row past the last one meets zero
// weights as well.  With three planes and seven filter rows that is 12 k-steps instead of the frame form's 14.
//
// Work unit, persistent workgroups (two per CU), weights in registers, staging tile and pooling: as in stem_pool.hip.
// The patch of a region -- rows 2*(14 tr - 1) - ph .. + 37 and 40 pixels from column 2*(16 tc - 1) - pw - e of every
// plane -- goes to LDS by 4-byte direct loads (a lane's dword lands at its own slot, so any arrangement can be
// requested): even and odd patch rows in separate areas, a row = [plane 0: 20 dwords][plane 1][plane 2][zeros], rows
// 81 dwords apart.  Output pixel (dy, dx), group (c, kh) then reads dwords 81 (dy + kh/2) + 20 c + dx .. + 3 of area
// kh & 1; 81 = 64 + 17 makes that the tile row 17 dy + dx plus a constant modulo the 64 banks, so the lanes of a wave
// read consecutive banks whatever the row wrap, and the two filter rows of a k-step differ by the constant distance
// between the areas.  Slots that hold nothing are requested out of range, which writes zeros.
#include "device_utils.h"

namespace rl {

namespace {

__device__ __forceinline__ u32x4 make_desc(const void *ptr, uint32_t bytes)
{
    const uint64_t a = (uint64_t)ptr;
    u32x4 d = {(uint32_t)a, (uint32_t)(a >> 32) & 0xffffu, bytes, 0x00020000u};   // raw buffer, untyped dwords
    return d;
}

// one direct load: 64 lanes x 4 bytes from desc[voff] to LDS at lds_addr + lane*4
__device__ __forceinline__ void dma4(const u32x4 &desc, uint32_t lds_addr, uint32_t voff)
{
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds"
                 :: "s"(lds_addr), "v"(voff), "s"(desc) : "memory");
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

typedef short i16x2 __attribute__((ext_vector_type(2)));
typedef u32x4 u32x4_dw __attribute__((aligned(4)));      // a 16-byte LDS read at dword alignment (two ds_read2_b32)

__device__ __forceinline__ uint32_t bf16x2_order(uint32_t b) { return b ^ (((b >> 15) & 0x00010001u) * 0x7fffu); }
__device__ __forceinline__ uint32_t pk_max_i16(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(i16x2, a), __builtin_bit_cast(i16x2, b)));
}
constexpr uint32_t LOWEST = 0x80008000u;          // below every mapped value

// staging-tile row order, see stem_pool.hip
__device__ __forceinline__ int stg_row(int m) { return (m & ~5) | ((m & 1) << 2) | ((m >> 2) & 1); }

constexpr int NUM_XCD = 8;
constexpr uint32_t OOB = 0x80000000u;
constexpr int TPH = 7, TPW = 8;                   // pooled pixels per region
constexpr int RH = 2 * TPH + 1, RW = 2 * TPW + 1; // convolution outputs a region needs: 15 x 17
constexpr int RPX = RH * RW;                      // 255 of the tile's 256 rows
constexpr int BM = 256, NCH = 64;
constexpr int NS = STEM_DIRECT_KP / 16;           // k-steps: 12 = (plane, pair of filter rows)
constexpr int PROWS = 2 * (RH + 1) + 6;           // patch rows (38: tile row 255 is a sixteenth output row; filters up to 8 high)
constexpr int ROWDW = 20;                         // dwords of a plane row under a region: 2*16 + 8 pixels
constexpr int CMAX = 3;
constexpr int PITCH = 81;                         // dwords from one row of an area to the next
constexpr int AROWS = PROWS / 2;                  // 19 rows per area
constexpr int AREA_DW = AROWS * PITCH;            // 1539 dwords
constexpr int PLOADS = ((2 * AREA_DW + 63) / 64 + 3) / 4 * 4;      // direct loads per patch: 52, thirteen per wave
constexpr int PATCH = PLOADS * 256;               // 13 KB
constexpr int STG_BYTES = BM * NCH * 2;
static_assert(PITCH >= CMAX * ROWDW && PITCH % 64 == RW, "a row holds three planes; bank-consecutive tile rows");
static_assert(RPX <= BM, "a region fits the tile");

}  // namespace

template <bool RELU>
__global__ __launch_bounds__(256, 2) void stem_pool_direct_kernel(const StemDirectParams q)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub; the body uses gfx950-only builtins
    __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * PATCH + STG_BYTES + 16];
    unsigned char *const stg = lds + 2 * PATCH;

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave >> 1, wn = wave & 1;        // the wave's half of the region's 256 rows and of the 64 channels

    // ---- this workgroup's regions: XCD x = blockIdx % 8 owns the run [x*per, (x+1)*per) of the region
    // list (image-major, then region rows, then region columns); its workgroups take them in turn
    const int ntr = (q.PH + TPH - 1) / TPH, ntc = (q.PW + TPW - 1) / TPW;
    const int nreg = q.n_img * ntr * ntc;
    const int per = (nreg + NUM_XCD - 1) / NUM_XCD;
    const int xcd = blockIdx.x % NUM_XCD, slot = blockIdx.x / NUM_XCD, nslot = gridDim.x / NUM_XCD;
    const int run_end = min(nreg, (xcd + 1) * per);
    const int first = xcd * per + slot;
    const int my = first < run_end ? (run_end - first + nslot - 1) / nslot : 0;
    if (my == 0) return;                            // whole workgroup leaves together

    const u32x4 dx = make_desc(q.x, q.x_bytes);
    const uint32_t lds_a = lds_addr_of(lds);
    const int frow = lane & 31, fhalf = lane >> 5;

    // ---- weights: the wave's 32 channels x 192, straight into registers (lane: channel wn*32 + frow, the eight
    // contraction indices 16 ks + 8 fhalf .. + 7 of every k-step), once
    u32x4 wreg[NS];
    {
        const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void *)q.w, 0, q.w_bytes, 0x00020000);
#pragma unroll
        for (int ks = 0; ks < NS; ++ks)
            wreg[ks] = __builtin_amdgcn_raw_buffer_load_b128(rw, (uint32_t)(((wn * 32 + frow) * STEM_DIRECT_KP + 16 * ks + 8 * fhalf) * 2), 0, 0);
    }
    // bias in accumulator layout (lane holds channels wn*32 + 8g + 4*fhalf .. +3)
    const Epilogue &e = q.epi;
    f32x4 bias_r[4];
    {
        const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc((void *)(e.has_bias ? e.bias_ptr : q.w), 0, e.has_bias ? (uint32_t)NCH * 4u : 0u, 0x00020000);
#pragma unroll
        for (int g = 0; g < 4; ++g)
            bias_r[g] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rb, (uint32_t)(wn * 32 + 8 * g + 4 * fhalf) * 4u, 0, 0));
    }

    // ---- fragment addresses inside a patch.  Tile row m = wm*128 + 32i + frow is output pixel (dy, dx) of the region:
    // byte 4 (81 dy + dx) of an area; k-step ks = (plane c, row pair r) adds r rows and 20 c dwords (the same for
    // every lane: scalars), and the lanes of the second half read the odd area.  A k-step past the last real one
    // reads what the first one reads, against zero weights.
    int fx_base[4], fx_ks[NS];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = wm * 128 + 32 * i + frow;
        const int dy = m / RW, dxx = m - dy * RW;
        fx_base[i] = (dy * PITCH + dxx + fhalf * AREA_DW) * 4;
    }
    const int khh = (q.KH + 1) >> 1;
#pragma unroll
    for (int ks = 0; ks < NS; ++ks) {
        const int c = ks / khh, r = ks - c * khh;
        fx_ks[ks] = c < q.C ? (r * PITCH + c * ROWDW) * 4 : 0;
    }
    // ---- patch requests: load k of the wave fills dword slots (wave*13 + k)*64 + lane = (area, row, column) with
    // column = (plane, dword d): patch row 2*row + area, pixels 2d and 2d + 1 of the plane's row.  Slots that hold
    // nothing (columns past the planes, past the second area) and pixels outside the image: out of range, zeros.
    constexpr int LPW = PLOADS / 4;
    int pt_rc[LPW];                                 // patch row << 8 | first pixel; an empty slot: a row never inside the image
    uint32_t pt_off[LPW];
#pragma unroll
    for (int k = 0; k < LPW; ++k) {
        const int sidx = (wave * LPW + k) * 64 + lane;
        const int area = sidx / AREA_DW, rem = sidx - area * AREA_DW;
        const int arow = rem / PITCH, col = rem - arow * PITCH;
        const int pl = col / ROWDW, d = col - pl * ROWDW;
        const bool holds = area < 2 && pl < q.C;
        const int prow = holds ? 2 * arow + area : 1 << 20;
        pt_rc[k] = (prow << 8) | (2 * d);
        pt_off[k] = holds ? (uint32_t)((((int64_t)pl * q.H + prow) * q.W + 2 * d) * 2) : 0u;
    }
    const int ecol = q.pw & 1;
    auto issue_patch = [&](int reg, int buf) {
        const int img = reg / (ntr * ntc), rr = reg - img * (ntr * ntc);
        const int tr = rr / ntc, tc = rr - tr * ntc;
        const int r0 = 2 * (2 * TPH * tr - 1) - q.ph, c0 = 2 * (2 * TPW * tc - 1) - q.pw - ecol;      // image row / (even) column of patch (0, 0)
        const uint32_t base = (uint32_t)((((int64_t)img * q.C * q.H + r0) * q.W + c0) * 2);        // may wrap below zero; only used when in range
#pragma unroll
        for (int k = 0; k < LPW; ++k) {
            const int ir = r0 + (pt_rc[k] >> 8), ic = c0 + (pt_rc[k] & 255);
            const bool ok = ir >= 0 && ir < q.H && ic >= 0 && ic + 1 < q.W;
            dma4(dx, lds_a + buf * PATCH + (wave * LPW + k) * 256, ok ? base + pt_off[k] : OOB);
        }
    };

    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(q.yp, 0, q.yp_bytes, 0x00020000);
    const float lo = RELU ? 0.0f : -INFINITY;

    // ---- pooling items of this thread (the same in every region), see stem_pool.hip
    int pl_pr[2], pl_pc[2], pl_addr[2][9];
    uint32_t pl_st[2];
    bool pl_live[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const int item = min(t + 256 * s, TPH * TPW * 8 - 1);
        const int pp = item >> 3, cq = item & 7;
        pl_pr[s] = pp / TPW; pl_pc[s] = pp - pl_pr[s] * TPW;
        pl_live[s] = t + 256 * s < TPH * TPW * 8;
        pl_st[s] = (uint32_t)((pl_pr[s] * q.PW + pl_pc[s]) * NCH + cq * 8) * 2u;
#pragma unroll
        for (int a = 0; a < 3; ++a)
#pragma unroll
            for (int b = 0; b < 3; ++b) {
                const int m = (2 * pl_pr[s] + a) * RW + 2 * pl_pc[s] + b;
                pl_addr[s][a * 3 + b] = stg_row(m) * 128 + ((cq ^ (m & 7)) << 4);
            }
    }
    constexpr int low_addr = STG_BYTES;             // 16 bytes of the lowest value behind the staging tile
    if (t == 0) *(u32x4 *)(stg + low_addr) = u32x4{LOWEST, LOWEST, LOWEST, LOWEST};   // stands in for window elements outside the image
    issue_patch(first, 0);

    f32x16 acc[4];
#pragma unroll 1
    for (int ri = 0; ri < my; ++ri) {
        const int reg = first + ri * nslot;
        const unsigned char *pa = lds + (ri & 1) * PATCH;
        RL_WAIT_VM(0);                              // this wave's part of the patch (and the last region's stores)
        wg_barrier();                               // the whole patch is there; the last region's pooling is done
        if (ri + 1 < my) issue_patch(reg + nslot, (ri + 1) & 1);
        // ---- K loop: 12 k-steps, fragments of the next one read while the current one is multiplied
        const f32x16 zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
        u32x4 fx[2][4];
        auto frag_addr = [&](int ks, int i) { return fx_ks[ks] + fx_base[i]; };
#pragma unroll
        for (int i = 0; i < 4; ++i) fx[0][i] = *(const u32x4_dw *)(pa + frag_addr(0, i));
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < NS; ++ks) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wreg[ks]), __builtin_bit_cast(bf16x8, fx[ks & 1][i]),
                                                                 ks == 0 ? zero : acc[i], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (ks + 1 < NS) {
                    fx[(ks + 1) & 1][i] = *(const u32x4_dw *)(pa + frag_addr(ks + 1, i));
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }

        // ---- finished bf16 values into the staging tile (row m in slot stg_row(m), chunk c at position c ^ (m & 7)), as 16-bit
        // integers in numeric order: after a ReLU that is the bf16 pattern itself.
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = wm * 128 + i * 32 + frow;
            unsigned char *dst = stg + stg_row(m) * 128 + fhalf * 8;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float v[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) v[k] = fmaxf(acc[i][4 * g + k] + bias_r[g][k], lo);
                u32x2 o = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
                if (!RELU) o = u32x2{bf16x2_order(o[0]), bf16x2_order(o[1])};
                *(u32x2 *)(dst + (((wn * 4 + g) ^ (m & 7)) << 4)) = o;
            }
        }
        wg_barrier();
        // ---- pooling.  All nine reads are issued before the first max; nothing branches.
        {
            const int img = reg / (ntr * ntc), rr = reg - img * (ntr * ntc);
            const int tr = rr / ntc, tc = rr - tr * ntc;
            const int oh0 = 2 * TPH * tr - 1, ow0 = 2 * TPW * tc - 1;
            const uint32_t reg_off = (uint32_t)((((int64_t)img * q.PH + TPH * tr) * q.PW + TPW * tc) * NCH) * 2u;
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                bool rok[3], cok[3];
#pragma unroll
                for (int a = 0; a < 3; ++a) {
                    const int oh = oh0 + 2 * pl_pr[s] + a, ow = ow0 + 2 * pl_pc[s] + a;
                    rok[a] = oh >= 0 && oh < q.OH;
                    cok[a] = ow >= 0 && ow < q.OW;
                }
                u32x4 r[9];
#pragma unroll
                for (int a = 0; a < 3; ++a)
#pragma unroll
                    for (int b = 0; b < 3; ++b) r[a * 3 + b] = *(const u32x4 *)(stg + ((rok[a] & cok[b]) ? pl_addr[s][a * 3 + b] : low_addr));
                u32x4 best = r[0];
#pragma unroll
                for (int w = 1; w < 9; ++w)
#pragma unroll
                    for (int k = 0; k < 4; ++k) best[k] = pk_max_i16(best[k], r[w][k]);
                if (!RELU) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) best[k] = bf16x2_order(best[k]);
                }
                const bool st_ok = pl_live[s] && TPH * tr + pl_pr[s] < q.PH && TPW * tc + pl_pc[s] < q.PW;
                __builtin_amdgcn_raw_buffer_store_b128(best, ry, st_ok ? reg_off + pl_st[s] : OOB, 0, 0);
            }
        }
    }
#endif
}

bool stem_direct_ok(int32_t C, int32_t H, int32_t W, int32_t KH, int32_t KW, int32_t ph, int32_t pw)
{
    return C >= 1 && C <= CMAX && H >= 1 && W >= 2 && W % 2 == 0 && KH >= 1 && KH <= 8 && KW >= 1 && KW + (pw & 1) <= 8 && ph >= 0 && pw >= 0 &&
           ph < 64 && pw < 64 && C * ((KH + 1) / 2) <= NS;
}

hipError_t launch_stem_pool_direct(const StemDirectParams &q, hipStream_t s)
{
    // the kernel's addressing assumes exactly this geometry
    if (!stem_direct_ok(q.C, q.H, q.W, q.KH, q.KW, q.ph, q.pw) || !q.x || !q.w || !q.yp || q.n_img < 1 ||
        ((uintptr_t)q.x & 3) != 0 || ((uintptr_t)q.w & 15) != 0 ||
        (uint64_t)q.n_img * q.C * q.H * q.W * 2 != (uint64_t)q.x_bytes || (uint64_t)q.x_bytes >= 0x7fffffffull ||
        q.w_bytes != (uint32_t)(NCH * STEM_DIRECT_KP * 2) ||
        q.OH != (q.H + 2 * q.ph - q.KH) / 2 + 1 || q.OW != (q.W + 2 * q.pw - q.KW) / 2 + 1 || q.OH < 1 || q.OW < 1 ||
        q.PH != (q.OH - 1) / 2 + 1 || q.PW != (q.OW - 1) / 2 + 1 ||
        q.epi.t_op >= 0 || !q.epi.simple || (q.epi.has_bias && q.epi.bias_dtype != DT_F32) || (q.epi.rest_n != 0 && !q.epi.relu_last) ||
        (uint64_t)q.n_img * q.PH * q.PW * NCH * 2 >= 0x7fffffffull || q.yp_bytes != (uint32_t)((uint64_t)q.n_img * q.PH * q.PW * NCH * 2))
        return hipErrorInvalidValue;
    const int ntr = (q.PH + TPH - 1) / TPH, ntc = (q.PW + TPW - 1) / TPW;
    const int64_t nreg = (int64_t)q.n_img * ntr * ntc;
    if (nreg > 0x7fffffff) return hipErrorInvalidValue;
    int grid = 512;                                 // two workgroups per CU, a multiple of the XCD count
    if (nreg < grid) grid = (int)((nreg + NUM_XCD - 1) / NUM_XCD * NUM_XCD);
    if (q.epi.relu_last) hipLaunchKernelGGL((stem_pool_direct_kernel<true>), dim3((unsigned)grid), dim3(256), 0, s, q);
    else hipLaunchKernelGGL((stem_pool_direct_kernel<false>), dim3((unsigned)grid), dim3(256), 0, s, q);
    return hipGetLastError();
}

}  // namespace rl

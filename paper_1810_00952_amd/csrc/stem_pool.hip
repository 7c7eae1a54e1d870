// Few-channel stem convolution (K = 256 after regrouping, 64 output channels)
// with its bias / ReLU epilogue AND the 3x3 stride-2 pad-1 max-pool that
// follows it, in one kernel, bf16 in / fp32 accumulate / bf16 out.
//
// Run as two kernels, the pair is bound by the traffic of the tensor between
// them: at batch 64 the stem writes 103 MB that the pool then reads back one
// and a half times, against 27 MB of input and 26 MB of pooled output.  Max
// commutes with everything monotone that the stem's epilogue does (adding the
// channel's bias, ReLU, rounding to bf16), so pooling the finished bf16 values
// in LDS gives bit for bit what the pool kernel computes from memory.
//
// Work unit: a region of 7 x 8 pooled pixels of one image, which needs the
// 15 x 17 = 255 convolution outputs around it (neighbouring regions share one
// row and one column of outputs: 14 % recomputation).  Those are the 256 rows
// of an implicit-GEMM tile; a wave multiplies 128 of them (four 32-row MFMA
// tiles) by 32 of the 64 channels; rows that fall outside the image are
// requested out of range (zeros) and ignored by the pooling.
//
// Workgroups are persistent, two per CU (each XCD owns a contiguous run of
// regions): staging and pooling are VALU and LDS work that keeps the MFMA pipe
// idle, and the second workgroup multiplies meanwhile.  That needs the kernel
// within 256 registers, which is why a wave takes half the channels: its share
// of the packed weights (32 KB in all) is read once into registers, 64 per
// lane, and stays there.  Activations are NOT expanded into GEMM rows on their
// way in: a GEMM row of this stem is 4 filter-row pairs x 2 rows x 8 pixels x
// 4 channels of the padded frame, and neighbouring output pixels share all but
// two of those pixels, so fetching rows tile by tile moves every input byte
// about fifteen times (and in half cache lines).  Instead the region's raw
// patch of the frame -- 38 rows x 40 pixels x 8 bytes = 12 KB -- is copied to
// LDS once (direct loads, twenty per region, into a 20 KB layout whose row
// pitch keeps the fragment reads free of bank conflicts) and the MFMA
// fragments are read straight out of it: the 16 bytes a lane needs for a
// k-step are 4 pixels of one frame row, and lanes that hold neighbouring
// output pixels read neighbouring 16-byte slots.  Two patch buffers: the next
// region's patch arrives while this one is multiplied.
//
// Per region: wait for the patch, barrier, request the next patch, 64 MFMAs
// per wave (as many fragment reads, each issued behind an MFMA), accumulators + bias, ReLU, rounded to bf16 into
// a 256-row staging tile in LDS (16-byte chunks XOR-swizzled by the row),
// barrier, then every thread pools one or two (pooled pixel, 8 channels)
// items, nine 16-byte reads each, and stores 16 bytes.  The staged values are
// kept as 16-bit integers in the numeric order of the bf16 values, so the max
// is a packed integer max and nothing in the pooling branches.
//
// Preconditions (checked by the launcher and the planner): the stem geometry
// of the pixel-on-lane path (4-channel padded frame, regrouped taps), exactly
// four K tiles, convolution stride 2, N = 64, epilogue [f32 bias] [relu],
// pool 3x3 / 2 / pad 1.
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

typedef short i16x2 __attribute__((ext_vector_type(2)));

// Two bf16 bit patterns -> two 16-bit integers whose signed order is the numeric order of the values (negative
// values get their low 15 bits flipped), and back: the map is its own inverse.  The pooling then is a packed
// integer max, with none of the floating-point max's NaN handling.
__device__ __forceinline__ uint32_t bf16x2_order(uint32_t b) { return b ^ (((b >> 15) & 0x00010001u) * 0x7fffu); }
__device__ __forceinline__ uint32_t pk_max_i16(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(i16x2, a), __builtin_bit_cast(i16x2, b)));
}
constexpr uint32_t LOWEST = 0x80008000u;          // below every mapped value

// Row m of the staging tile sits in 128-byte slot m with bits 0 and 2 exchanged.  A pooling read has eight
// lanes per row and rows two apart; the LDS serves lanes 0-15 and 16-31 of a half-wave four by four, a quad
// of the first sixteen together with the neighbouring quad of the second sixteen, so rows m and m + 4 must
// lie in different halves of the 256-byte bank line (measured: 4.9 cycles per read against 7.8 with row m
// in slot m; the 8-byte writes of the accumulator layout cost the same either way).
__device__ __forceinline__ int stg_row(int m) { return (m & ~5) | ((m & 1) << 2) | ((m >> 2) & 1); }

constexpr int NUM_XCD = 8;
constexpr uint32_t OOB = 0x80000000u;
constexpr int TPH = 7, TPW = 8;                   // pooled pixels per region
constexpr int RH = 2 * TPH + 1, RW = 2 * TPW + 1; // convolution outputs a region needs: 15 x 17
constexpr int RPX = RH * RW;                      // 255 of the tile's 256 rows
constexpr int BM = 256, NKT = 4, NCH = 64;
constexpr int PROWS = 2 * (RH + 1) + 6;           // frame rows under a region (38; one spare output row: tile row 255)
constexpr int PCH = (2 * RW + 6) / 2;             // 16-byte chunks (2 pixels x 4 channels) of a frame row under a region: 20
// The patch in LDS: even frame rows in one area, odd ones in another (a k-step reads rows of one parity), a row
// every 33 chunks.  Output pixel (dy, dx) then reads chunk 33 dy + dx + const, and 33 = 2*16 + 1 makes that
// tile row m = 17 dy + dx plus a constant modulo 16: the 32 rows of an MFMA tile read consecutive 16-byte bank
// groups, whatever the row wrap (measured: 4.0 cycles per fragment read against 6-7.5 with frame rows 20 chunks
// apart).  Chunks 20..32 of a row are requested out of range and never read.
constexpr int PCHS = 2 * 16 + 1;                  // chunks from one row of an area to the next
constexpr int AROWS = PROWS / 2;                  // 19 rows per area
constexpr int AREA = AROWS * PCHS * 16;           // 10 032 bytes
constexpr int PLOADS = (2 * AROWS * PCHS + 63) / 64;   // direct loads per patch: 20, five per wave
constexpr int PATCH = PLOADS * 1024;              // 20 KB
static_assert(PROWS % 2 == 0 && PCHS >= PCH, "two areas of whole rows");
constexpr int STG_BYTES = BM * NCH * 2;           // finished bf16 outputs of a region
static_assert(PLOADS % 4 == 0, "patch loads split evenly over the four waves");
static_assert(RPX <= BM, "a region fits the tile");

}  // namespace

// ODD: odd filter height: the second frame row of the last K tile meets zero weights only; its two k-steps are skipped
template <bool RELU, bool ODD>
__global__ __launch_bounds__(256, 2) void stem_pool_kernel(const StemPoolParams q)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub; the body uses gfx950-only builtins
    const IgemmParams &p = q.g;
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

    const u32x4 dx = make_desc(p.x, p.x_bytes);
    const u32x4 dw = make_desc(p.w, p.w_bytes);
    const uint32_t lds_a = lds_addr_of(lds);
    const int r8 = lane >> 3, pos = lane & 7;
    const int frow = lane & 31, fhalf = lane >> 5;

    // ---- weights: four K tiles of 64 rows x 128 bytes through the staging tile into registers, once
    u32x4 wreg[NKT][4];                             // the wave's 32 channels
    {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int row = wave * 16 + 8 * j + r8;
            const int chunk = pos ^ ((row >> 1) & 7);
            const uint32_t wv = (uint32_t)((int64_t)row * p.Kp * 2) + chunk * 16;      // N = 64 rows exactly
#pragma unroll
            for (int kt = 0; kt < NKT; ++kt) dma16(dw, lds_a + 2 * PATCH + kt * 8192 + (wave * 2 + j) * 1024, wv, (uint32_t)kt * 128u);
        }
        RL_WAIT_VM(0);
        wg_barrier();
#pragma unroll
        for (int kt = 0; kt < NKT; ++kt)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                wreg[kt][ks] = *(const u32x4 *)(stg + kt * 8192 + (wn * 32 + frow) * 128 + (((2 * ks + fhalf) ^ ((frow >> 1) & 7)) << 4));
    }
    // bias in accumulator layout (lane holds channels wn*32 + 8g + 4*fhalf .. +3)
    const Epilogue &e = p.epi;
    f32x4 bias_r[4];
    {
        const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc((void *)(e.has_bias ? e.bias_ptr : p.w), 0, e.has_bias ? (uint32_t)NCH * 4u : 0u, 0x00020000);
#pragma unroll
        for (int g = 0; g < 4; ++g)
            bias_r[g] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rb, (uint32_t)(wn * 32 + 8 * g + 4 * fhalf) * 4u, 0, 0));
    }

    // ---- fragment addresses inside a patch.  Tile row m = wm*128 + 32i + frow is output pixel (dy, dx) of the
    // region; its K tile kt, k-step ks is 16-byte chunk c = 2ks + fhalf of a 128-byte GEMM row, i.e. frame row
    // 2dy + 2kt + (c >> 2), pixels 2dx + 2(c & 3) and the next: area (c >> 2), row dy + kt, chunk dx + (c & 3).
    int fx_base[4], fx_ks[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = wm * 128 + 32 * i + frow;
        const int dy = m / RW, dxx = m - dy * RW;
        fx_base[i] = (dy * PCHS + dxx) * 16;
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        const int c = 2 * ks + fhalf;
        fx_ks[ks] = (c >> 2) * AREA + (c & 3) * 16;
    }
    // ---- patch requests: load k of the wave covers patch bytes (wave*5 + k)*1024 + lane*16, i.e. chunk slot
    // s = (wave*5 + k)*64 + lane = (area s / 627, row (s % 627) / 33, chunk s % 33): frame row
    // 2*(14 tr - 1) + 2*row + area, pixels 2*(16 tc - 1) + 2*chunk and the next.  Slots that hold nothing
    // (chunk >= 20, past the second area) and chunks outside the frame: out of range, zeros.
    const int Hp = p.H, Wp = p.W;                  // the padded frame
    int pt_row[PLOADS / 4], pt_col[PLOADS / 4];
    uint32_t pt_off[PLOADS / 4];
#pragma unroll
    for (int k = 0; k < PLOADS / 4; ++k) {
        const int sidx = (wave * (PLOADS / 4) + k) * 64 + lane;
        const int area = sidx / (AROWS * PCHS), rem = sidx - area * (AROWS * PCHS);
        const int arow = rem / PCHS, ch = rem - arow * PCHS;
        const bool holds = area < 2 && ch < PCH;
        pt_row[k] = holds ? 2 * arow + area : 1 << 20;        // an empty slot: never inside the frame
        pt_col[k] = holds ? 2 * ch : 0;
        pt_off[k] = holds ? (uint32_t)((pt_row[k] * Wp + pt_col[k]) * 8) : 0u;
    }
    auto issue_patch = [&](int reg, int buf) {
        const int img = reg / (ntr * ntc), rr = reg - img * (ntr * ntc);
        const int tr = rr / ntc, tc = rr - tr * ntc;
        const int fr0 = 2 * (2 * TPH * tr - 1), fc0 = 2 * (2 * TPW * tc - 1);
        const uint32_t base = (uint32_t)((((int64_t)img * Hp + fr0) * Wp + fc0) * 8);     // may wrap below zero; only used when in range
#pragma unroll
        for (int k = 0; k < PLOADS / 4; ++k) {
            const int fr = fr0 + pt_row[k], fc = fc0 + pt_col[k];
            const bool ok = fr >= 0 && fr < Hp && fc >= 0 && fc + 1 < Wp;
            dma16(dx, lds_a + buf * PATCH + (wave * (PLOADS / 4) + k) * 1024, ok ? base + pt_off[k] : OOB, 0u);
        }
    };

    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(q.yp, 0, q.yp_bytes, 0x00020000);
    const float lo = RELU ? 0.0f : -INFINITY;

    // ---- pooling items of this thread (the same in every region): item = (pooled pixel (pr, pc) of the region,
    // 8-channel chunk cq); 56 x 8 items over 256 threads, surplus threads redo the last item and do not store.
    // For each of the nine window elements the staging address is fixed; only whether its row / column lies in
    // the image depends on the region.
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
    constexpr int low_addr = STG_BYTES;             // 16 bytes of the lowest value behind the staging tile (written below)

    wg_barrier();                                   // every wave has its weights: the staging tile is free
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
        // ---- K loop: 16 (14) k-steps, fragments of the next one read while the current one is multiplied
        constexpr int NKS = NKT * 4 - (ODD ? 2 : 0);
        const f32x16 zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};   // the first k-step starts the sums
        u32x4 fx[2][4];
#pragma unroll
        for (int i = 0; i < 4; ++i) fx[0][i] = *(const u32x4 *)(pa + fx_base[i] + fx_ks[0]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kk = 0; kk < NKS; ++kk) {
            const int kt = kk >> 2, ks = kk & 3;
            // every fragment read of the next k-step follows an MFMA of this one, so that it is issued while that runs
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wreg[kt][ks]), __builtin_bit_cast(bf16x8, fx[kk & 1][i]),
                                                                 kk == 0 ? zero : acc[i], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (kk + 1 < NKS) {
                    const int kt1 = (kk + 1) >> 2, ks1 = (kk + 1) & 3;
                    fx[(kk + 1) & 1][i] = *(const u32x4 *)(pa + fx_base[i] + fx_ks[ks1] + kt1 * (PCHS * 16));
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
                    rok[a] = oh >= 0 && oh < p.OH;
                    cok[a] = ow >= 0 && ow < p.OW;
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


hipError_t launch_stem_pool(const StemPoolParams &q, hipStream_t s)
{
    const IgemmParams &p = q.g;
    // the kernel's addressing assumes exactly this geometry
    if (p.in_dtype != DT_BF16 || p.x2 || p.N != NCH || p.K != NKT * 64 || p.Kp != p.K || p.C != 64 || p.KW != 1 || p.KH != NKT || p.ph != 0 || p.pw != 0 || p.sh != 2 || p.sw != 2 ||
        p.H != (p.OH - 1) * 2 + 2 * NKT || p.W != (p.OW - 1) * 2 + 8 || p.xs_w != 4 || p.xs_h != (int64_t)p.W * 4 || p.xs_n != (int64_t)p.H * p.W * 4 ||
        (uint64_t)q.n_img * p.H * p.W * 8 != (uint64_t)p.x_bytes ||
        p.OH < 1 || p.OW < 1 || q.n_img < 1 || (int64_t)q.n_img * p.OHW != p.M || q.PH != (p.OH - 1) / 2 + 1 || q.PW != (p.OW - 1) / 2 + 1 ||
        p.epi.t_op >= 0 || !p.epi.simple || (p.epi.has_bias && p.epi.bias_dtype != DT_F32) || (p.epi.rest_n != 0 && !p.epi.relu_last) ||
        (uint64_t)q.n_img * q.PH * q.PW * NCH * 2 >= 0x7fffffffull || q.yp_bytes != (uint32_t)((uint64_t)q.n_img * q.PH * q.PW * NCH * 2) || !q.yp)
        return hipErrorInvalidValue;
    const int ntr = (q.PH + TPH - 1) / TPH, ntc = (q.PW + TPW - 1) / TPW;
    const int64_t nreg = (int64_t)q.n_img * ntr * ntc;
    if (nreg > 0x7fffffff) return hipErrorInvalidValue;
    int grid = 512;                                 // two workgroups per CU, a multiple of the XCD count
    if (nreg < grid) grid = (int)((nreg + NUM_XCD - 1) / NUM_XCD * NUM_XCD);
    if (q.kh != 2 * NKT && q.kh != 2 * NKT - 1) return hipErrorInvalidValue;
    const bool odd = q.kh == 2 * NKT - 1;
    if (p.epi.relu_last) {
        if (odd) hipLaunchKernelGGL((stem_pool_kernel<true, true>), dim3((unsigned)grid), dim3(256), 0, s, q);
        else hipLaunchKernelGGL((stem_pool_kernel<true, false>), dim3((unsigned)grid), dim3(256), 0, s, q);
    } else {
        if (odd) hipLaunchKernelGGL((stem_pool_kernel<false, true>), dim3((unsigned)grid), dim3(256), 0, s, q);
        else hipLaunchKernelGGL((stem_pool_kernel<false, false>), dim3((unsigned)grid), dim3(256), 0, s, q);
    }
    return hipGetLastError();
}

}  // namespace rl

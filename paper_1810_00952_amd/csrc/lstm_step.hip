// One LSTM time step with the input projection already done:
//
//   z[b, :]  = zx[b, :] + h_prev[b, :] . Wh^T + bias
//   i,f,g,o  = sigmoid, sigmoid, tanh, sigmoid of the four gate slices of z
//   c'       = f * c + i * g ;  h' = o * tanh(c')
//
// The recurrence leaves only a skinny contraction per step (batch x 4H x H with
// a batch of 64 or so) that has to finish before the next step can start, so
// what matters is latency and how many CUs share the weight traffic, not MFMA
// throughput.  A workgroup (4 waves) owns 32 batch rows x 8 hidden units
// (32 gate columns); with a batch of 64 and H = 1024 that is 256 workgroups,
// each reading its 64 KB weight slice (which stays in its XCD's L2 from step
// to step) and its 64 KB of h_prev: the split that moves the fewest bytes per
// CU when every CU has one workgroup.
//
// The K loop is split between the four waves: wave w takes K tiles w, w+4,
// w+8, ... in rounds of four.  A round requests everything it needs at once --
// the four 32-row h_prev tiles by direct loads (global -> LDS, 4 KB each, into
// the wave's private 16 KB), then the weight fragments of the four tiles
// straight into registers (a lane loads the 16 bytes the MFMA wants from it)
// -- so that one memory latency is paid per round, not per tile; H = 1024 is
// one round.  Nothing is shared between waves until the end, so the loop has
// no workgroup barrier.  The direct loads are inline assembly; the one wait on
// them counts the sixteen fragment loads issued after them as the only ones
// that may still be in flight, and the compiler's own waits on those
// fragments are exact because nothing is issued behind them.  Each wave ends
// with an fp32 partial sum of the whole 32 x 32 tile, parks it in its own LDS
// space, and after one barrier the 256 threads finish one (row, unit) pair
// each: sum of the four partials + zx + bias, gate arithmetic, c' and h'.
// The operands of that last part (zx, c, bias) are requested first of all.
//
// Weights are the packed cell weights [4H][Kp] bf16, gate-interleaved per 64
// rows (rows 64*T + 16*gate + u hold gate `gate` of unit 16*T + u), of which
// the recurrent columns start at k_off; zx uses the same column order.
// MFMA operand roles and LDS swizzle as in the contraction kernels (weights
// are the row operand, a lane holds one batch row).
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
#define RL_WAIT_LGKM0() asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory")

__device__ __forceinline__ uint32_t lds_addr_of(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}

constexpr uint32_t OOB = 0x80000000u;
constexpr int BM = 32, BNC = 32, UNITS = 8;       // batch rows, gate columns, hidden units per workgroup
constexpr int STAGE = BM * 128, NSTAGE = 4;       // one h_prev tile; tiles per round
constexpr int PSTRIDE = 36;                       // floats per parked row (32 + 4: spreads the banks)
static_assert(BM * PSTRIDE * 4 <= NSTAGE * STAGE && PSTRIDE >= BNC && BNC == 4 * UNITS, "a wave parks its partial tile in its own LDS space");

}  // namespace

__global__ __launch_bounds__(256) void lstm_step_kernel(const LstmStepParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass only needs the launch stub; the body uses gfx950-only builtins
    __shared__ __attribute__((aligned(1024))) unsigned char lds[4 * NSTAGE * STAGE];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int nb = blockIdx.x, m0 = blockIdx.y * BM;          // 8-unit column block, first batch row
    const int tile64 = nb >> 1, half = nb & 1;                // 64-row weight tile and which 8 of its 16 units
    const int unit0 = tile64 * 16 + half * UNITS;             // first hidden unit of the workgroup

    // ---- the last part's operands, requested first: thread t finishes (row, unit) pair t.
    // Plain range-checked buffer loads (out of range reads as zero), so nothing here branches or waits.
    constexpr int NPAIR = BM * UNITS / 256;                    // (row, unit) pairs per thread
    float zx_r[NPAIR][4], bias_r[NPAIR][4], c_r[NPAIR];
    {
        const __amdgpu_buffer_rsrc_t rz = __builtin_amdgcn_make_buffer_rsrc((void *)p.zx, 0, (uint32_t)p.B * 4u * (uint32_t)p.H * 4u, 0x00020000);
        const __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc((void *)p.c_in, 0, (uint32_t)p.B * (uint32_t)p.H * 4u, 0x00020000);
        const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc((void *)(p.bias ? p.bias : p.w), 0, p.bias ? 4u * (uint32_t)p.H * 4u : 0u, 0x00020000);
#pragma unroll
        for (int s = 0; s < NPAIR; ++s) {
            const int idx = t + 256 * s, row = idx >> 3, j = idx & 7;
            const int m = m0 + row, unit = unit0 + j;
            const bool live = m < p.B && unit < p.H;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int col = tile64 * 64 + g * 16 + half * UNITS + j;      // packed column of (gate g, unit)
                zx_r[s][g] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rz, live ? (uint32_t)(m * 4 * p.H + col) * 4u : OOB, 0, 0));
                bias_r[s][g] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rb, live ? (uint32_t)(g * p.H + unit) * 4u : OOB, 0, 0));
            }
            c_r[s] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rc, live ? (uint32_t)(m * p.H + unit) * 4u : OOB, 0, 0));
        }
    }
    asm volatile("" ::: "memory");

    // ---- direct-load state: lane l of a group writes LDS row (l >> 3), position (l & 7)
    const u32x4 dh = make_desc(p.h_prev, p.h_bytes);
    const int r8 = lane >> 3, pos = lane & 7;
    uint32_t a_voff[BM / 8];
#pragma unroll
    for (int i = 0; i < BM / 8; ++i) {
        const int row = 8 * i + r8, chunk = pos ^ ((row >> 1) & 7);
        const int m = m0 + row;
        a_voff[i] = m < p.B ? (uint32_t)((int64_t)m * p.H * 2) + chunk * 16 : OOB;
    }
    unsigned char *const ring = lds + wave * NSTAGE * STAGE;
    const uint32_t ring_a = lds_addr_of(ring);
    const int nk = p.H / 64;                                   // K tiles in all; this wave's are wave, wave + 4, ...
    const int nkw = nk > wave ? (nk - wave + 3) / 4 : 0;

    // fragment addressing: lane = (row frow of a 32-row MFMA tile, half fhalf of a 32-byte k-step)
    const int frow = lane & 31, fhalf = lane >> 5;
    int f_off[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) f_off[ks] = frow * 128 + (((2 * ks + fhalf) ^ ((frow >> 1) & 7)) << 4);
    // the lane's weight row: tile row frow = gate * 8 + unit-in-block
    uint32_t w_voff;
    {
        int wr = tile64 * 64 + (frow >> 3) * 16 + half * UNITS + (frow & 7);
        if (wr > 4 * p.H - 1) wr = 4 * p.H - 1;
        w_voff = (uint32_t)((int64_t)wr * p.Kp * 2) + (uint32_t)p.k_off * 2u + (uint32_t)fhalf * 16u;
    }
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void *)p.w, 0, p.w_bytes, 0x00020000);

    constexpr int TM = BM / 32;
    f32x16 acc[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[i][q] = 0.0f;

#pragma unroll 1
    for (int it0 = 0; it0 < nkw; it0 += NSTAGE) {
        // requests of the round: tiles past the wave's last go out of range (zeros), so the counts are fixed
#pragma unroll
        for (int q = 0; q < NSTAGE; ++q) {
            const bool live = it0 + q < nkw;
            const uint32_t k0 = (uint32_t)(wave + 4 * (it0 + q)) * 128u;      // byte offset of the K tile in a row
#pragma unroll
            for (int i = 0; i < BM / 8; ++i) dma16(dh, ring_a + q * STAGE + i * 1024, live ? a_voff[i] : OOB, live ? k0 : 0u);
        }
        u32x4 fw[NSTAGE][4];
#pragma unroll
        for (int q = 0; q < NSTAGE; ++q) {
            const bool live = it0 + q < nkw;
            const uint32_t k0 = (uint32_t)(wave + 4 * (it0 + q)) * 128u;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                fw[q][ks] = __builtin_amdgcn_raw_buffer_load_b128(rw, live ? w_voff + (uint32_t)ks * 32u : OOB, live ? k0 : 0u, 0);
        }
        RL_WAIT_VM(16);                                        // all but the sixteen fragment loads: every h_prev tile has landed
#pragma unroll
        for (int q = 0; q < NSTAGE; ++q) {
            const unsigned char *sa = ring + q * STAGE;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    const u32x4 fx = *(const u32x4 *)(sa + i * 32 * 128 + f_off[ks]);
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fw[q][ks]), __builtin_bit_cast(bf16x8, fx), acc[i], 0, 0, 0);
                }
            }
        }
        RL_WAIT_LGKM0();                                       // the tiles are read out: the next round may overwrite them
    }
    RL_WAIT_VM(0);

    // ---- park the wave's partial tile [row][gate column] as fp32 in its own ring space.  Accumulator
    // register 4g + k of lane l is (gate column 8g + 4*(l >> 5) + k, batch row 32i + (l & 31)).
    float *park = (float *)ring;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            f32x4 v;
#pragma unroll
            for (int k = 0; k < 4; ++k) v[k] = acc[i][4 * g + k];
            *(f32x4 *)(park + (32 * i + frow) * PSTRIDE + 8 * g + 4 * fhalf) = v;
        }
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    // ---- gate arithmetic: gate g of unit j sits in gate column 8g + j of every wave's partial tile
#pragma unroll
    for (int s = 0; s < NPAIR; ++s) {
        const int idx = t + 256 * s, row = idx >> 3, j = idx & 7;
        const int m = m0 + row, unit = unit0 + j;
        if (m < p.B && unit < p.H) {
            float z[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float a = 0.0f;
#pragma unroll
                for (int w = 0; w < 4; ++w) a += ((const float *)(lds + w * NSTAGE * STAGE))[row * PSTRIDE + 8 * g + j];
                z[g] = (a + zx_r[s][g]) + bias_r[s][g];
            }
            const float cn = sigmoidf_(z[1]) * c_r[s] + sigmoidf_(z[0]) * tanhf_(z[2]);
            const float hn = sigmoidf_(z[3]) * tanhf_(cn);
            p.c_out[(int64_t)m * p.H + unit] = cn;
            store_from_f32(p.h_out, p.h_dtype, (int64_t)m * p.H + unit, hn);
        }
    }
#endif
}

hipError_t launch_lstm_step(const LstmStepParams &p, hipStream_t s)
{
    // the kernel's addressing assumes exactly this geometry
    if (!p.h_prev || !p.w || !p.zx || !p.c_in || !p.c_out || !p.h_out || p.B < 1 || p.H < 64 || p.H % 64 != 0 || p.Kp < p.k_off + p.H ||
        (p.bias && p.bias_dtype != DT_F32) || p.k_off < 0 || p.k_off % 8 != 0 || p.Kp % 8 != 0 || (uint64_t)p.B * p.H * 16 >= 0x7fffffffull || (uint64_t)4 * p.H * p.Kp * 2 >= 0x7fffffffull ||
        p.h_bytes != (uint32_t)((uint64_t)p.B * p.H * 2) || p.w_bytes != (uint32_t)((uint64_t)4 * p.H * p.Kp * 2))
        return hipErrorInvalidValue;
    const dim3 grid((unsigned)(p.H / UNITS), (unsigned)((p.B + BM - 1) / BM));
    hipLaunchKernelGGL(lstm_step_kernel, grid, dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace rl

// Launch descriptors shared by the planner/executor (host) and the gfx950
// kernels.  Plain structs passed by value as kernel arguments.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rl {

enum { DT_F32 = 0, DT_BF16 = 1 };

// ---- injective epilogue program ------------------------------------------
// A fused group's injective operators form a chain over one running value v
// (the contraction's accumulator, or the first operand of an anchor-less
// group).  Each step is one op code and, for ops with a second operand, the
// index of that operand in the pointer table.
enum EpiOp : uint8_t {
    E_BIAS = 0,   // v += vec[channel]
    E_ADD, E_SUB, E_RSUB, E_MUL, E_DIV, E_RDIV,   // v = v op t[idx]   (R*: t[idx] op v)
    E_NEG, E_SQ, E_RELU, E_SIGMOID, E_TANH,
    E_ADD_VV, E_SUB_VV, E_DIV_VV,                 // both operands are the running value
    E_ROUND_BF16,                                 // cast to bf16 (value stays in a float register)
    E_NOP
};
#define RL_EPI_MAX_OPS 12
#define RL_EPI_MAX_PTRS 6

// Every field is 32 or 64 bits wide: the struct travels in the kernel-argument segment, where
// dword fields are fetched by scalar loads once per wave, while byte fields would be fetched by
// vector loads from that (host-visible) segment at microseconds apiece.
struct Epilogue {
    int32_t n_ops;
    uint32_t opw[RL_EPI_MAX_OPS / 4];     // op codes, 8 bits each
    uint32_t argw[RL_EPI_MAX_OPS / 4];    // pointer-table slots, 8 bits each
    uint32_t dtw;                         // dtype of pointer slot i in bits 4i .. 4i+3
    const void *ptr[RL_EPI_MAX_PTRS];
    // Host-side classification of the common form  [bias] [one full-shape operand step] operand-free*
    // (filled by finalize_epilogue; lets the kernels read fixed fields instead of walking the tables)
    int32_t simple;        // 1: the chain has that form and at most 8 trailing steps
    int32_t has_bias;
    int32_t t_op;          // EpiOp of the full-shape operand step, or -1
    int32_t bias_dtype, t_dtype;
    int32_t rest_n;        // trailing operand-free steps
    int32_t relu_last;     // 1: the trailing steps are exactly one ReLU
    uint64_t rest_ops;     // their op codes, 8 bits each, first step in the low byte
    const void *bias_ptr;
    const void *t_ptr;
};
inline void epi_set_op(Epilogue &e, int s, int op, int arg)
{
    e.opw[s >> 2] = (e.opw[s >> 2] & ~(0xffu << (8 * (s & 3)))) | ((uint32_t)op << (8 * (s & 3)));
    e.argw[s >> 2] = (e.argw[s >> 2] & ~(0xffu << (8 * (s & 3)))) | ((uint32_t)arg << (8 * (s & 3)));
}
inline int epi_host_op(const Epilogue &e, int s) { return (e.opw[s >> 2] >> (8 * (s & 3))) & 0xff; }
inline int epi_host_arg(const Epilogue &e, int s) { return (e.argw[s >> 2] >> (8 * (s & 3))) & 0xff; }
inline void epi_set_dtype(Epilogue &e, int slot, int dt) { e.dtw = (e.dtw & ~(0xfu << (4 * slot))) | ((uint32_t)dt << (4 * slot)); }
inline int epi_host_dtype(const Epilogue &e, int slot) { return (e.dtw >> (4 * slot)) & 0xf; }
// Derives the classification fields and the resolved pointers from the tables (call after ptr[] is final).
void finalize_epilogue(Epilogue &e);

// ---- implicit-GEMM contraction (conv2d and dense) ------------------------
// C[m, n] = sum_k A[m, k] * Wp[n, k], m = (image, oh, ow), n = output channel,
// k = (kh, kw, c).  A is gathered from x with element strides; Wp is the
// packed weight [N][Kp] (K contiguous, Kp a multiple of the 16-byte vector).
struct IgemmParams {
    const void *x;
    const void *x2;          // second operand of a row concatenation (dense): k >= K1 reads x2[m, k-K1]
    const void *w;
    void *y;
    int32_t M, N, K, Kp, K1;
    int32_t C, H, W, KH, KW, OH, OW, OHW, sh, sw, ph, pw;
    int64_t xs_n, xs_c, xs_h, xs_w;     // element strides of x
    int64_t x2s_n;                      // row stride of x2
    int64_t ys_n, ys_p, ys_c;           // element strides of y: image, pixel (oh*OW+ow), channel
    int32_t y_dtype;                    // DT_*
    int32_t in_dtype;
    Epilogue epi;
    // LSTM gate epilogue (mode GATES): packed column j of block tile holds gate j/(BN/4), unit j%(BN/4)
    const float *c_in; float *c_out; void *h_out; int32_t h_dtype; int32_t hidden;
    int32_t nblk_m, nblk_n;
    uint32_t x_bytes, x2_bytes, w_bytes;   // extents for range-checked buffer loads (vector-load variant)
    uint32_t y_bytes;                      // extent of y (and of a full-shape epilogue operand)
    uint32_t seg_stride;                   // bytes between the two 64-byte halves of an A row's K tile (64: contiguous)
    int64_t ts_h, ts_w;                    // element strides of one filter-tap step (xs_h, xs_w unless the taps are regrouped)
    uint32_t div_ohw_mul, div_ohw_sh, div_ow_mul, div_ow_sh;   // m / OHW and pix / OW by multiply-high (make_fast_div)
    uint32_t tap_rep;                      // bit kh*KW set for every kh < KH (KH*KW <= 32)
    // K split over `splits` workgroups per tile (direct-load variant only; 0 or 1: no split): workgroup (tile, z)
    // multiplies K tiles [z*per, (z+1)*per) and writes its fp32 sums to partial[z][M][N]; a second kernel adds the
    // slices in order z = 0, 1, ... and applies the epilogue
    // element-gather variant only (both zero: an ordinary convolution): filter taps tap_dil_m1 + 1 input pixels apart;
    // the input taken as if in_dil_m1 zeros stood between its pixels in both directions (H, W: the real extent)
    int32_t tap_dil_m1, in_dil_m1;
    int32_t nmajor;                        // conv3x3_run_ks_kernel: 1: tiles in channel-tile-major order
    int32_t splits, split_tiles;           // split_tiles: K tiles per slice
    float *partial;
    int32_t skip_reduce;                   // direct-load variant, splits > 1: the slices are added by the caller's next launch
};
// q = n / d for n < 2^31:  d == 1 ? n : (mulhi(n, mul) >> sh)
void make_fast_div(uint32_t d, uint32_t &mul, uint32_t &sh);

enum IgemmTile { TILE_128x128 = 0, TILE_128x64 = 1, TILE_64x64 = 2, TILE_256x128 = 3 /* pixel-on-lane variant only */, TILE_COUNT };
struct IgemmLaunch {
    int32_t tile;       // IgemmTile
    int32_t avec;       // 1: A rows are 16-byte-vector loadable (channel-contiguous, aligned)
    int32_t gates;      // 1: LSTM gate epilogue (tile must be TILE_64x64)
    int32_t dma;        // 1: K tiles go global -> LDS directly (needs avec, C and K multiples of the K tile, >= 2 tiles)
    int32_t lp;         // 1: pixel-on-lane variant with the register epilogue (bf16, [bias] [+residual] [relu])
    int32_t ws;         // 1 (with lp): weights-stationary persistent variant (N <= 64, K <= 576)
    int32_t c64;        // 1 (with lp): 3x3 / stride 1 / pad 1, 64 -> 64 channels, image rows of at most 63 pixels (conv3x3_c64.hip)
    int32_t run;        // 1 (with lp): 3x3 / stride 1 / pad 1, C a multiple of 64, image rows of at most 30 pixels, tile not 64x64 (conv3x3_run.hip);
                        // 2: its 128x64 form with K split over the waves (C a multiple of 128)
    int32_t splits;     // > 1 (with dma, no lp, no gates): K split over that many workgroups per tile (IgemmParams::splits)
    int32_t s2pair;     // 1 (first step of a pair): the pair runs as one stride-2 contraction with two accumulator sets (conv3x3s2.hip)
    int32_t anyact;     // 1 (with lp, no ws / c64 / run / pair): operand-free steps other than one ReLU behind bias and residual
};
hipError_t launch_igemm(const IgemmParams &p, const IgemmLaunch &l, hipStream_t s);

// The adding launch of a split dense contraction, and the small dense layer behind it, in one kernel: row m of
//   h = epi1(partial[0][m][:] + partial[1][m][:] + ...)         (slices in order; rounded to h_dtype as the tensor between
//   y[m][j] = epi2(sum_n h[n] * w2[j][n])                         the two groups would be)
// by one workgroup, h staying in LDS.  N1 <= 2048, N2 <= 64; w2 row-major with rows Kp2 elements apart.
struct ReduceDenseParams {
    const float *partial;
    int32_t splits, M, N1;
    Epilogue epi1;
    int64_t hs_n, hs_c;          // strides of h as the operands of epi1 are laid out
    int32_t h_dtype;
    const void *w2;
    int32_t w_dtype, N2, Kp2;
    Epilogue epi2;
    void *y;
    int32_t y_dtype;
    int64_t ys_n, ys_c;
};
constexpr int REDUCE_DENSE_MAX_N1 = 2048, REDUCE_DENSE_MAX_N2 = 64;
hipError_t launch_reduce_dense(const ReduceDenseParams &p, hipStream_t s);
// two independent pixel-on-lane contractions that use the same kernel variant, in one launch (igemm_lp.hip)
bool igemm_lp_can_pair(const IgemmParams &a, const IgemmLaunch &la, const IgemmParams &b, const IgemmLaunch &lb);
hipError_t launch_igemm_lp_pair(const IgemmParams &a, const IgemmLaunch &la, const IgemmParams &b, const IgemmLaunch &lb, hipStream_t s);
// a stage's 3x3 / stride 2 convolution (a) and the 1x1 / stride 2 projection of the same input (b) as one contraction with two
// accumulator sets (conv3x3s2.hip); the planner asks conv3x3s2_pair_ok before any pointer is bound
bool conv3x3s2_pair_ok(const IgemmParams &a, const IgemmLaunch &la, const IgemmParams &b, const IgemmLaunch &lb);
hipError_t launch_conv3x3s2_pair(const IgemmParams &a, const IgemmLaunch &la, const IgemmParams &b, const IgemmLaunch &lb, hipStream_t s);
hipError_t launch_conv3x3_c64(const IgemmParams &p, hipStream_t s);
hipError_t launch_conv3x3_run(const IgemmParams &p, const IgemmLaunch &l, hipStream_t s);

// ---- stem convolution + bias/ReLU + 3x3/2 max-pool in one kernel (stem_pool.hip) ----
struct StemPoolParams {
    IgemmParams g;                      // the stem contraction (x: padded frame, w: packed weights, N = 64, K = 256); y unused
    void *yp; uint32_t yp_bytes;        // pooled output [n_img, PH, PW, 64] bf16
    int32_t n_img, PH, PW;
    int32_t kh;                         // the filter's own height (2*g.KH or one less: the last frame row then meets zero weights and is skipped)
};
hipError_t launch_stem_pool(const StemPoolParams &q, hipStream_t s);

// ---- the same fusion reading the channel-first input itself (stem_direct.hip) ----
constexpr int STEM_DIRECT_KP = 192;     // contraction length of its packed weights: 12 k-steps of 16 = (plane, pair of filter rows) x 2 rows x 8 columns
struct StemDirectParams {
    const void *x; uint32_t x_bytes;    // [n_img, C, H, W] bf16, 4-byte aligned
    const void *w; uint32_t w_bytes;    // [64][STEM_DIRECT_KP] bf16 (launch_pack_weight_stem_direct)
    Epilogue epi;                       // [f32 bias] [relu]
    void *yp; uint32_t yp_bytes;        // pooled output [n_img, PH, PW, 64] bf16
    int32_t n_img, C, H, W, KH, KW, ph, pw, OH, OW, PH, PW;
};
bool stem_direct_ok(int32_t C, int32_t H, int32_t W, int32_t KH, int32_t KW, int32_t ph, int32_t pw);
hipError_t launch_stem_pool_direct(const StemDirectParams &q, hipStream_t s);
// weights [64, C, KH, KW] -> [64][STEM_DIRECT_KP]: index 16 (c ceil(KH/2) + kh/2) + 8 (kh & 1) + kw + (pw & 1), zeros elsewhere
hipError_t launch_pack_weight_stem_direct(const void *src, void *dst, int32_t O, int32_t C, int32_t KH, int32_t KW, int32_t pw, hipStream_t s);

// ---- gradient of a convolution with respect to its weights, batches that are multiples of 64 (conv_wgrad.hip) ----
struct WgradParams {
    const void *dyT; uint32_t dy_bytes;     // dy with the images as the fastest axis: element (pixel, o, n) at pixel*ys_pix + o*ys_o + n
    const void *xT; uint32_t x_bytes;       // x likewise: (pixel, c, n) at pixel*xs_pix + c*xs_c + n
    float *part;                            // [OH * nseg][KH*KW][O][C] fp32: the sums of the row segments
    int32_t O, C, H, W, OH, OW, KH, KW, s, ph, pw;
    int64_t ys_pix, ys_o, xs_pix, xs_c;     // in elements, multiples of 8
    int32_t nseg, L;                        // segments per output row, output pixels per segment
    int32_t n_ot, n_ct;                     // blocks of output channels (of 128, or of 64) and of input channels (of 64)
    int32_t nck;                            // groups of 64 images (the batch is 64 * nck)
};
bool conv_wgrad_ok(int32_t NB, int32_t O, int32_t C, int32_t KH, int32_t KW, int32_t s);
hipError_t launch_conv_wgrad(const WgradParams &p, hipStream_t s);
hipError_t launch_wgrad_reduce(const float *part, void *out, int32_t out_dtype, int32_t chunks, int32_t T, int32_t O, int32_t C, hipStream_t s);

// ---- one LSTM step on a precomputed input projection (lstm_step.hip) ------
struct LstmStepParams {
    const void *h_prev;                 // [B, H] bf16
    const void *w;                      // packed cell weights [4H][Kp] bf16, gate-interleaved per 64 rows
    const float *zx;                    // [B, 4H] f32: x_t . Wx^T in the packed column order
    const void *bias; int32_t bias_dtype;   // [4H] f32 in declaration order (i, f, g, o blocks), or null
    const float *c_in; float *c_out;    // [B, H] f32 (may alias)
    void *h_out; int32_t h_dtype;       // [B, H]
    int32_t B, H, Kp, k_off;            // k_off: first recurrent column of a weight row
    uint32_t h_bytes, w_bytes;
};
hipError_t launch_lstm_step(const LstmStepParams &p, hipStream_t s);

// ---- purely elementwise fused group ---------------------------------------
struct EltwiseParams {
    const void *x; int32_t x_dtype;     // first operand: initial running value
    void *y; int32_t y_dtype;
    int64_t n;                          // elements
    int64_t ch_inner; int32_t ch_count; // channel of flat index i = (i / ch_inner) % ch_count (for E_BIAS)
    Epilogue epi;
    // filled by launch_eltwise.  runs > 0: a per-channel operand is constant over runs of vec_per_run
    // 8-element vectors; the run of vector v is v / vec_per_run by multiply-high (make_fast_div)
    int64_t vec_per_run; int32_t runs; uint32_t run_mul, run_sh; int32_t nt;   // nt: streaming accesses
};
hipError_t launch_eltwise(const EltwiseParams &p, hipStream_t s);

struct GatesParams {
    const float *z; const float *c_in; float *c_out; void *h_out; int32_t h_dtype; int32_t B, H;
    int32_t nt;                         // streaming accesses (filled by launch_lstm_gates)
};
hipError_t launch_lstm_gates(const GatesParams &p, hipStream_t s);

// ---- window reductions (channel-last tensors [N, H, W, C]) ------------------
struct PoolParams {
    const void *x; void *y; int32_t dtype;
    int32_t N, C, H, W, OH, OW, KH, KW, sh, sw, ph, pw;
    // filled by launch_maxpool_nhwc: multiply-high constants (make_fast_div) for the divisions by C / vector, OW, OH
    uint32_t cv_mul, cv_sh, ow_mul, ow_sh, oh_mul, oh_sh;
};
hipError_t launch_maxpool_nhwc(const PoolParams &p, hipStream_t s);
hipError_t launch_gavgpool_nhwc(const PoolParams &p, hipStream_t s);   // y: [N, C]

// ---- layout change and weight packing -------------------------------------
// dst[n, p, c] (pixel-major, channel-last) <-> src[n, c, p]
hipError_t launch_nchw_to_nhwc(const void *src, void *dst, int32_t dtype, int32_t N, int32_t C, int32_t P, hipStream_t s);
hipError_t launch_nhwc_to_nchw(const void *src, void *dst, int32_t dtype, int32_t N, int32_t C, int32_t P, hipStream_t s);
// any permutation of up to six axes (element gather): y[i0..] = x[sum_k i_k * xstride[k]], i over ydims
struct PermuteParams {
    const void *x; void *y; int32_t dtype; int32_t rank;
    int64_t n;                          // elements
    int32_t ydims[6];                   // result shape
    int64_t xstride[6];                 // operand stride (elements) of the axis that result axis k comes from
};
hipError_t launch_permute(const PermuteParams &p, hipStream_t s);
// conv weight [O, C, KH*KW] -> [O, KH*KW, C] padded with zeros to Kp per row.
// perm_block > 0: output row j holds source row gate*(O/4) + blk*(perm_block/4) + u
// for j = blk*perm_block + gate*(perm_block/4) + u (LSTM gate interleave).
// perm_block == -1 (bf16, O = C = 64, T = 9, Kp = 576 only): the plain matrix is followed by a second copy in MFMA
// fragment order, dst2[(((h*9 + tap)*4 + ks)*64 + lane)*8 + e] = W[32h + lane%32][tap*64 + 16ks + 8*(lane/32) + e].
hipError_t launch_pack_weight(const void *src, void *dst, int32_t dtype, int32_t O, int32_t C, int32_t T,
                              int32_t Kp, int32_t perm_block, hipStream_t s);
// Few-channel stem convolutions (C <= 4, KW <= 8): the input is copied once into a zero-padded
// channel-last frame with 4 channels per pixel, dst[n][hp][wp][4] with image pixel (h, w) at
// (h + ph, w + pw); a run of 8 pixels then is 64 contiguous bytes and a K tile holds filter rows
// 2t and 2t+1 (8 pixels x 4 channels each).  The weights are packed to match:
// dst[o][((t*2 + seg)*8 + px)*4 + c] = src[o][c][2t+seg][px], zero outside the filter.
hipError_t launch_dilate_nhwc(const void *src, void *dst, int32_t N, int32_t OH, int32_t OW, int32_t Hd, int32_t Wd, int32_t pixel_bytes, int32_t stride,
                              hipStream_t s);
hipError_t launch_stem_pad(const void *src, void *dst, int32_t N, int32_t C, int32_t H, int32_t W, int32_t Hp, int32_t Wp,
                           int32_t ph, int32_t pw, hipStream_t s);
// Operand of a contraction gathered into the K-contiguous rows the kernels read: for row r < R and k < Kp,
// dst[r][k] = k < T*Cq ? src[base + r*s_row + (k % Cq)*s_c + (k / Cq / TW)*s_ti + (k / Cq % TW)*s_tj] : 0
// (element strides, possibly negative).  Serves the transposed, flipped and re-ordered operands of the gradient operators,
// at prepack time for params and as a step of the plan for activations.
struct GatherPack {
    int32_t dtype, R, Kp, T, Cq, TW;
    int64_t base, s_row, s_c, s_ti, s_tj;
};
hipError_t launch_pack_gather(const void *src, void *dst, const GatherPack &g, hipStream_t s);
hipError_t launch_pack_weight_stem(const void *src, void *dst, int32_t O, int32_t C, int32_t KH, int32_t KW, int32_t Kp, hipStream_t s);
// measurement aid (calibrate.hip): a chain of register-operand bf16 MFMAs per wave; out holds grid * 512 floats
hipError_t launch_mfma_peak(float *out, int32_t grid, int32_t iters, hipStream_t s);
hipError_t launch_fold_bn(const float *w, const float *gamma, const float *beta, const float *mean, const float *var,
                          double eps, void *w_out, int32_t out_dtype, float *b_out, int64_t O, int64_t per_o,
                          hipStream_t s);

}  // namespace rl

/*
 * CPU oracle: operator semantics written out as their plain definitions.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker for the GPU library; it
 * shares no code with it and nothing on the product path may call it.
 *
 * Every tensor is a dense row-major array of double (NCHW for rank 4).
 * Sums are accumulated in double in the textbook index order, with no
 * blocking, fusion or reordering.  The paper names these operators (conv2d,
 * max_pool, flatten_layer, linear, tanh in the decorator example of section
 * "Frontend"; + - * /, unary - and sq in the grammar figure) but defines none
 * of them; the definitions below are the standard ones and each is pinned by
 * the CPU tests against brute force, closed forms and invariants.
 *
 * OpenMP parallelism is over the outermost independent output index only; it
 * never splits a reduction, so results do not depend on the thread count.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* y[m,n] = sum_k x[m,k] * W[n,k]        ("linear"; weight stored [out, in]) */
void oracle_dense(const double *x, const double *w, double *y, int64_t M, int64_t N, int64_t K)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double s = 0.0;
            for (int64_t k = 0; k < K; ++k)
                s += x[m * K + k] * w[n * K + k];
            y[m * N + n] = s;
        }
}

/* Cross-correlation with zero padding, dilation 1, groups 1:
 * y[n,o,i,j] = sum_{c,a,b} xpad[n,c,i*sh-ph+a, j*sw-pw+b] * w[o,c,a,b],
 * OH = floor((H + 2 ph - KH)/sh) + 1 (computed by the caller and passed in). */
void oracle_conv2d(const double *x, const double *w, double *y,
                   int64_t N, int64_t C, int64_t H, int64_t W,
                   int64_t O, int64_t KH, int64_t KW,
                   int64_t sh, int64_t sw, int64_t ph, int64_t pw,
                   int64_t OH, int64_t OW)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t o = 0; o < O; ++o)
            for (int64_t i = 0; i < OH; ++i)
                for (int64_t j = 0; j < OW; ++j) {
                    double s = 0.0;
                    for (int64_t c = 0; c < C; ++c)
                        for (int64_t a = 0; a < KH; ++a) {
                            int64_t ih = i * sh - ph + a;
                            if (ih < 0 || ih >= H) continue;
                            for (int64_t b = 0; b < KW; ++b) {
                                int64_t iw = j * sw - pw + b;
                                if (iw < 0 || iw >= W) continue;
                                s += x[((n * C + c) * H + ih) * W + iw] * w[((o * C + c) * KH + a) * KW + b];
                            }
                        }
                    y[((n * O + o) * OH + i) * OW + j] = s;
                }
}

/* Partial derivatives of the two contractions, each written out as the sum it is by definition of the forward
 * operator (y = dense / conv2d above, L any scalar function of y, dy = dL/dy):
 *   dL/dx[m,k] = sum_n dy[m,n] * W[n,k]            dL/dW[n,k] = sum_m dy[m,n] * x[m,k]
 * These are the operators a reverse-mode gradient of a program (the paper's section "Automatic Differentiation",
 * node Grad) calls for every dense / conv2d it differentiates through; the paper gives no formula for them. */
void oracle_dense_grad_x(const double *dy, const double *w, double *dx, int64_t M, int64_t N, int64_t K)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            double s = 0.0;
            for (int64_t n = 0; n < N; ++n)
                s += dy[m * N + n] * w[n * K + k];
            dx[m * K + k] = s;
        }
}

void oracle_dense_grad_w(const double *dy, const double *x, double *dw, int64_t M, int64_t N, int64_t K)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            double s = 0.0;
            for (int64_t m = 0; m < M; ++m)
                s += dy[m * N + n] * x[m * K + k];
            dw[n * K + k] = s;
        }
}

/* dL/dx[n,c,h,w] = sum over every (o, a, b, i, j) whose forward term read x[n,c,h,w], i.e. with
 * h = i*sh - ph + a and w = j*sw - pw + b, of dy[n,o,i,j] * wt[o,c,a,b].  Written as the scatter it is. */
void oracle_conv2d_grad_x(const double *dy, const double *wt, double *dx,
                          int64_t N, int64_t C, int64_t H, int64_t W,
                          int64_t O, int64_t KH, int64_t KW,
                          int64_t sh, int64_t sw, int64_t ph, int64_t pw,
                          int64_t OH, int64_t OW)
{
    memset(dx, 0, (size_t)(N * C * H * W) * sizeof(double));
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t c = 0; c < C; ++c)
            for (int64_t o = 0; o < O; ++o)
                for (int64_t i = 0; i < OH; ++i)
                    for (int64_t j = 0; j < OW; ++j) {
                        double g = dy[((n * O + o) * OH + i) * OW + j];
                        for (int64_t a = 0; a < KH; ++a) {
                            int64_t ih = i * sh - ph + a;
                            if (ih < 0 || ih >= H) continue;
                            for (int64_t b = 0; b < KW; ++b) {
                                int64_t iw = j * sw - pw + b;
                                if (iw < 0 || iw >= W) continue;
                                dx[((n * C + c) * H + ih) * W + iw] += g * wt[((o * C + c) * KH + a) * KW + b];
                            }
                        }
                    }
}

/* dL/dwt[o,c,a,b] = sum_{n,i,j} dy[n,o,i,j] * xpad[n,c,i*sh-ph+a, j*sw-pw+b] */
void oracle_conv2d_grad_w(const double *dy, const double *x, double *dw,
                          int64_t N, int64_t C, int64_t H, int64_t W,
                          int64_t O, int64_t KH, int64_t KW,
                          int64_t sh, int64_t sw, int64_t ph, int64_t pw,
                          int64_t OH, int64_t OW)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t o = 0; o < O; ++o)
        for (int64_t c = 0; c < C; ++c)
            for (int64_t a = 0; a < KH; ++a)
                for (int64_t b = 0; b < KW; ++b) {
                    double s = 0.0;
                    for (int64_t n = 0; n < N; ++n)
                        for (int64_t i = 0; i < OH; ++i) {
                            int64_t ih = i * sh - ph + a;
                            if (ih < 0 || ih >= H) continue;
                            for (int64_t j = 0; j < OW; ++j) {
                                int64_t iw = j * sw - pw + b;
                                if (iw < 0 || iw >= W) continue;
                                s += dy[((n * O + o) * OH + i) * OW + j] * x[((n * C + c) * H + ih) * W + iw];
                            }
                        }
                    dw[((o * C + c) * KH + a) * KW + b] = s;
                }
}

/* y[outer, c, inner] = x[outer, c, inner] + b[c] */
void oracle_bias_add(const double *x, const double *b, double *y, int64_t outer, int64_t C, int64_t inner)
{
#pragma omp parallel for schedule(static)
    for (int64_t u = 0; u < outer; ++u)
        for (int64_t c = 0; c < C; ++c)
            for (int64_t v = 0; v < inner; ++v) {
                int64_t idx = (u * C + c) * inner + v;
                y[idx] = x[idx] + b[c];
            }
}

/* op: 0 add, 1 sub, 2 mul, 3 div (grammar figure, BinOp) */
void oracle_binary(int op, const double *a, const double *b, double *y, int64_t n)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        switch (op) {
        case 0: y[i] = a[i] + b[i]; break;
        case 1: y[i] = a[i] - b[i]; break;
        case 2: y[i] = a[i] * b[i]; break;
        default: y[i] = a[i] / b[i]; break;
        }
    }
}

/* op: 0 neg, 1 sq (grammar figure, UnaryOp), 2 relu, 3 sigmoid, 4 tanh */
void oracle_unary(int op, const double *x, double *y, int64_t n)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double v = x[i];
        switch (op) {
        case 0: y[i] = -v; break;
        case 1: y[i] = v * v; break;
        case 2: y[i] = v > 0.0 ? v : 0.0; break;
        case 3: y[i] = 1.0 / (1.0 + exp(-v)); break;
        default: y[i] = tanh(v); break;
        }
    }
}

/* Inference batch-norm: gamma * (x - mean) / sqrt(var + eps) + beta per channel. */
void oracle_batchnorm(const double *x, const double *gamma, const double *beta, const double *mean,
                      const double *var, double eps, double *y, int64_t N, int64_t C, int64_t HW)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t c = 0; c < C; ++c)
            for (int64_t v = 0; v < HW; ++v) {
                int64_t idx = (n * C + c) * HW + v;
                y[idx] = gamma[c] * (x[idx] - mean[c]) / sqrt(var[c] + eps) + beta[c];
            }
}

/* Folding that batch-norm into the preceding convolution's parameters:
 * scale[o] = gamma[o]/sqrt(var[o]+eps); w'[o,...] = w[o,...]*scale[o];
 * b'[o] = beta[o] - mean[o]*scale[o].  per_o = C*KH*KW. */
void oracle_fold_batchnorm(const double *w, const double *gamma, const double *beta, const double *mean,
                           const double *var, double eps, double *w_out, double *b_out, int64_t O, int64_t per_o)
{
    for (int64_t o = 0; o < O; ++o) {
        double scale = gamma[o] / sqrt(var[o] + eps);
        for (int64_t i = 0; i < per_o; ++i)
            w_out[o * per_o + i] = w[o * per_o + i] * scale;
        b_out[o] = beta[o] - mean[o] * scale;
    }
}

/* Max over the in-bounds taps of each window (out-of-bounds taps are ignored). */
void oracle_maxpool2d(const double *x, double *y, int64_t N, int64_t C, int64_t H, int64_t W,
                      int64_t KH, int64_t KW, int64_t sh, int64_t sw, int64_t ph, int64_t pw,
                      int64_t OH, int64_t OW)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t c = 0; c < C; ++c)
            for (int64_t i = 0; i < OH; ++i)
                for (int64_t j = 0; j < OW; ++j) {
                    double best = -INFINITY;
                    for (int64_t a = 0; a < KH; ++a) {
                        int64_t ih = i * sh - ph + a;
                        if (ih < 0 || ih >= H) continue;
                        for (int64_t b = 0; b < KW; ++b) {
                            int64_t iw = j * sw - pw + b;
                            if (iw < 0 || iw >= W) continue;
                            double v = x[((n * C + c) * H + ih) * W + iw];
                            if (v > best) best = v;
                        }
                    }
                    y[((n * C + c) * OH + i) * OW + j] = best;
                }
}

/* y[n,c] = mean over h,w of x[n,c,h,w] */
void oracle_global_avgpool(const double *x, double *y, int64_t N, int64_t C, int64_t HW)
{
#pragma omp parallel for schedule(static)
    for (int64_t nc = 0; nc < N * C; ++nc) {
        double s = 0.0;
        for (int64_t v = 0; v < HW; ++v) s += x[nc * HW + v];
        y[nc] = s / (double)HW;
    }
}

/* LSTM gate math on pre-activations z[B,4H] laid out as (i, f, g, o) blocks
 * of H columns each: c' = sigmoid(f) c + sigmoid(i) tanh(g); h' = sigmoid(o) tanh(c'). */
void oracle_lstm_gates(const double *z, const double *c, double *c_out, double *h_out, int64_t B, int64_t H)
{
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t u = 0; u < H; ++u) {
            const double *zr = z + b * 4 * H;
            double gi = 1.0 / (1.0 + exp(-zr[u]));
            double gf = 1.0 / (1.0 + exp(-zr[H + u]));
            double gg = tanh(zr[2 * H + u]);
            double go = 1.0 / (1.0 + exp(-zr[3 * H + u]));
            double cn = gf * c[b * H + u] + gi * gg;
            c_out[b * H + u] = cn;
            h_out[b * H + u] = go * tanh(cn);
        }
}

/* Nearest float32 (the C conversion rounds to nearest-even in the default mode). */
void oracle_round_f32(const double *x, double *y, int64_t n)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) y[i] = (double)(float)x[i];
}

/* Nearest bfloat16 (1 sign, 8 exponent, 7 fraction bits), ties to even,
 * directly from the double: keep the top 16 bits of the float32 encoding of
 * the correctly rounded value.  Done on the double's own bits so there is a
 * single rounding.  Finite inputs well inside the float32 range only. */
void oracle_round_bf16(const double *x, double *y, int64_t n)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double v = x[i];
        if (v == 0.0 || !isfinite(v)) { y[i] = v; continue; }
        int e;
        double m = frexp(fabs(v), &e);          /* |v| = m * 2^e, m in [0.5,1) */
        /* 8 significant bits: scale m to [128,256) and round to nearest even */
        double scaled = ldexp(m, 8);
        double r = nearbyint(scaled);           /* default rounding mode: ties-to-even */
        double out = ldexp(r, e - 8);
        y[i] = v < 0 ? -out : out;
    }
}

/* Threads the parallel loops above will use (for reporting). */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif

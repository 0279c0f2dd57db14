/*
 * CPU oracle for the merged ("input-weight local") operators of NetFuse.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  Nothing in the product path may call it, and
 * it shares no code, header, table or helper with the HIP sources.
 *
 * Principle (Section 3; Appendix A, Eq. 3-6): a merged operator gives exactly the
 * results of the M separate operators.  So every routine below loops over the
 * model index m and evaluates model m's ordinary operator on model m's slice of
 * the merged tensors; the merged layouts are touched only through the index maps
 * of Appendix A (x[C_in*m + c_in] = x_m[c_in], y_m[c_out] = y[C_out*m + c_out])
 * and of Section 3.1 (matrix multiplication: concatenation along a batch dim).
 *
 * Arithmetic: float inputs, every sum and every intermediate in double, one
 * conversion to float at the output.  When out_bf16 != 0 that float is then
 * rounded once more, to the nearest bfloat16 (ties to even), and returned as a
 * float holding that value -- the rounding a bf16-storage operator performs when
 * it writes its result.
 *
 * Parity pins: every routine is pinned by tests/test_oracle_*.py (brute force
 * against single-model definitions, library special cases at M = 1, closed
 * forms, permutation and isolation invariants).  No routine here is unpinned.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

enum { ACT_NONE = 0, ACT_RELU = 1, ACT_GELU = 2 };
enum { LAYOUT_BATCH = 0, LAYOUT_CHANNEL = 1 };

/* nearest-even rounding of a float to the bfloat16 grid; NaN stays NaN */
static float to_bf16_grid(float v)
{
    uint32_t u;
    memcpy(&u, &v, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) {          /* NaN: keep it quiet */
        u = (u | 0x00400000u) & 0xffff0000u;
    } else {
        uint32_t lsb = (u >> 16) & 1u;
        u = (u + 0x7fffu + lsb) & 0xffff0000u;
    }
    memcpy(&v, &u, 4);
    return v;
}

static float finish(double v, int out_bf16)
{
    float f = (float)v;
    return out_bf16 ? to_bf16_grid(f) : f;
}

/* ReLU, or GELU in its exact erf form 0.5 x (1 + erf(x / sqrt 2)) */
static double activate(double v, int act)
{
    if (act == ACT_RELU) return v > 0.0 ? v : (v != v ? v : 0.0);
    if (act == ACT_GELU) return 0.5 * v * (1.0 + erf(v * 0.70710678118654752440));
    return v;
}

/*
 * Merged matrix multiplication = batch matrix multiplication (Section 3.1,
 * "Matrix multiplication"): model m's input is multiplied with model m's weight
 * only.  X[M][N][K], W[M][K][Nout], bias[M][Nout] or NULL, residual[M][N][Nout]
 * or NULL, Y[M][N][Nout].   Y_m = act(X_m W_m + b_m) + R_m.
 */
void oracle_linear(const float *X, const float *W, const float *bias, const float *residual,
                   float *Y, int M, int N, int K, int Nout, int act, int out_bf16)
{
    #pragma omp parallel for collapse(2) schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int n = 0; n < N; ++n) {
            const float *Xm = X + (size_t)m * N * K;
            const float *Wm = W + (size_t)m * K * Nout;
            for (int j = 0; j < Nout; ++j) {
                double acc = 0.0;
                for (int k = 0; k < K; ++k)
                    acc += (double)Xm[(size_t)n * K + k] * (double)Wm[(size_t)k * Nout + j];
                if (bias) acc += (double)bias[(size_t)m * Nout + j];
                acc = activate(acc, act);
                size_t o = ((size_t)m * N + n) * Nout + j;
                if (residual) acc += (double)residual[o];
                Y[o] = finish(acc, out_bf16);
            }
        }
    }
}

/*
 * Merged convolution = grouped convolution with M*g groups (Section 3.1,
 * "Convolution" and "Operations with input-weight local computations";
 * Appendix A Eq. 2).  x[B][M*Cin][H][W], w[M*Cout][Cin/g][KH][KW],
 * y[B][M*Cout][Ho][Wo].  Output channel c belongs to group G = c / (Cout/g) and
 * reads input channels G*(Cin/g) ... G*(Cin/g) + Cin/g - 1 (Eq. 2's offset).
 * Zero padding, then valid cross-correlation (no kernel flip) with stride and
 * dilation.  Epilogue, in this order: + bias[c]; * scale[c] + shift[c] (both or
 * neither); + residual; activation.
 */
void oracle_conv2d(const float *x, const float *w, const float *bias, const float *scale,
                   const float *shift, const float *residual, float *y,
                   int M, int B, int Cin, int Cout, int g, int H, int Wd, int KH, int KW,
                   int stride, int pad, int dil, int act, int out_bf16)
{
    const int cig = Cin / g, cog = Cout / g;
    const int Ho = (H + 2 * pad - dil * (KH - 1) - 1) / stride + 1;
    const int Wo = (Wd + 2 * pad - dil * (KW - 1) - 1) / stride + 1;
    const int Ctot_in = M * Cin, Ctot_out = M * Cout;
    #pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b) {
        for (int c = 0; c < Ctot_out; ++c) {
            const int G = c / cog;                 /* which of the M*g groups */
            const int cbase = G * cig;             /* first input channel of that group */
            for (int oy = 0; oy < Ho; ++oy) {
                for (int ox = 0; ox < Wo; ++ox) {
                    double acc = 0.0;
                    for (int ci = 0; ci < cig; ++ci) {
                        for (int ky = 0; ky < KH; ++ky) {
                            const int iy = oy * stride + ky * dil - pad;
                            if (iy < 0 || iy >= H) continue;
                            for (int kx = 0; kx < KW; ++kx) {
                                const int ix = ox * stride + kx * dil - pad;
                                if (ix < 0 || ix >= Wd) continue;
                                double xv = x[(((size_t)b * Ctot_in + cbase + ci) * H + iy) * Wd + ix];
                                double wv = w[(((size_t)c * cig + ci) * KH + ky) * KW + kx];
                                acc += wv * xv;
                            }
                        }
                    }
                    if (bias) acc += (double)bias[c];
                    if (scale) acc = acc * (double)scale[c] + (double)shift[c];
                    size_t o = (((size_t)b * Ctot_out + c) * Ho + oy) * Wo + ox;
                    if (residual) acc += (double)residual[o];
                    acc = activate(acc, act);
                    y[o] = finish(acc, out_bf16);
                }
            }
        }
    }
}

/*
 * Merged layer normalisation = group normalisation with M groups (Section 3.1,
 * "Layer normalization"): the statistics of a row are taken over one model's H
 * features only.  layout BATCH: x[M][rows][H] (the output layout of the batch
 * matmul); layout CHANNEL: x[rows][M*H] (channel concatenation, the group-norm
 * form).  gamma, beta[M*H] are the M affine vectors concatenated.  residual (same
 * layout as x) or NULL is added before the statistics.  Biased variance.
 */
void oracle_layernorm(const float *x, const float *residual, const float *gamma,
                      const float *beta, float *y, int M, int rows, int H, double eps,
                      int layout, int out_bf16)
{
    #pragma omp parallel for collapse(2) schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int r = 0; r < rows; ++r) {
            size_t base = (layout == LAYOUT_BATCH) ? ((size_t)m * rows + r) * H
                                                   : ((size_t)r * M + m) * H;
            double mean = 0.0;
            for (int i = 0; i < H; ++i) {
                double v = x[base + i];
                if (residual) v += (double)residual[base + i];
                mean += v;
            }
            mean /= H;
            double var = 0.0;
            for (int i = 0; i < H; ++i) {
                double v = x[base + i];
                if (residual) v += (double)residual[base + i];
                var += (v - mean) * (v - mean);
            }
            var /= H;
            double rstd = 1.0 / sqrt(var + eps);
            for (int i = 0; i < H; ++i) {
                double v = x[base + i];
                if (residual) v += (double)residual[base + i];
                double o = (double)gamma[(size_t)m * H + i] * (v - mean) * rstd
                         + (double)beta[(size_t)m * H + i];
                y[base + i] = finish(o, out_bf16);
            }
        }
    }
}

/*
 * Merged batch normalisation, inference mode (Section 3.1: the computation is
 * per channel, so the M models' channels are simply concatenated).
 * x[B][M*C][HW]; gamma, beta, mean, var[M*C].
 * y = act(gamma (x - mean) / sqrt(var + eps) + beta + residual).
 */
void oracle_batchnorm(const float *x, const float *gamma, const float *beta, const float *mean,
                      const float *var, const float *residual, float *y, int M, int B, int C,
                      int HW, double eps, int act, int out_bf16)
{
    const int Ctot = M * C;
    #pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b) {
        for (int c = 0; c < Ctot; ++c) {
            double rstd = 1.0 / sqrt((double)var[c] + eps);
            for (int p = 0; p < HW; ++p) {
                size_t o = ((size_t)b * Ctot + c) * HW + p;
                double v = (double)gamma[c] * ((double)x[o] - (double)mean[c]) * rstd + (double)beta[c];
                if (residual) v += (double)residual[o];
                y[o] = finish(activate(v, act), out_bf16);
            }
        }
    }
}

/*
 * The per-channel constants of an inference batch normalisation, for use as a
 * convolution epilogue:  scale = gamma / sqrt(var + eps), shift = beta - mean*scale.
 * All arrays [n]; n = M*C merged channels (per merged channel, Section 3.1).
 */
void oracle_bn_fold(const float *gamma, const float *beta, const float *mean, const float *var,
                    float *scale, float *shift, int n, double eps)
{
    for (int c = 0; c < n; ++c) {
        double s = (double)gamma[c] / sqrt((double)var[c] + eps);
        scale[c] = (float)s;
        shift[c] = (float)((double)beta[c] - (double)mean[c] * s);
    }
}

/*
 * Merged attention.  Attention's two products are already batch matrix
 * multiplications over (sequence, head); merging M models multiplies the number
 * of independent problems by M (Section 3.1, "Operations with input-weight local
 * computations"), and softmax has no weights (Section 3.1, "Non-trainable
 * operations").  For each (m, b, head):
 *     s_ij = scale * sum_t Q_it K_jt (+ mask_j);  p_ij = softmax_j(s_ij);  O_it = sum_j p_ij V_jt.
 * Element (m, b, s, head, t) of Q, K, V lives at  ptr[m*stride_m + (b*S+s)*stride_row + head*d + t];
 * mask is additive, [M][B][S] over keys, or NULL;  O[M][B*S][heads*d] contiguous.
 */
void oracle_attention(const float *Q, const float *K, const float *V, const float *mask, float *O,
                      int M, int B, int S, int heads, int d, long stride_m, long stride_row,
                      double scale, int out_bf16)
{
    #pragma omp parallel for collapse(3) schedule(static)
    for (int m = 0; m < M; ++m) {
        for (int b = 0; b < B; ++b) {
            for (int h = 0; h < heads; ++h) {
                double p[S];
                for (int i = 0; i < S; ++i) {
                    const float *q = Q + (size_t)m * stride_m + ((size_t)b * S + i) * stride_row + (size_t)h * d;
                    double smax = -INFINITY;
                    for (int j = 0; j < S; ++j) {
                        const float *k = K + (size_t)m * stride_m + ((size_t)b * S + j) * stride_row + (size_t)h * d;
                        double s = 0.0;
                        for (int t = 0; t < d; ++t) s += (double)q[t] * (double)k[t];
                        s *= scale;
                        if (mask) s += (double)mask[((size_t)m * B + b) * S + j];
                        p[j] = s;
                        if (s > smax) smax = s;
                    }
                    double denom = 0.0;
                    for (int j = 0; j < S; ++j) { p[j] = exp(p[j] - smax); denom += p[j]; }
                    for (int t = 0; t < d; ++t) {
                        double acc = 0.0;
                        for (int j = 0; j < S; ++j) {
                            const float *v = V + (size_t)m * stride_m + ((size_t)b * S + j) * stride_row + (size_t)h * d;
                            acc += p[j] * (double)v[t];
                        }
                        O[((size_t)m * B * S + (size_t)b * S + i) * ((size_t)heads * d) + (size_t)h * d + t]
                            = finish(acc / denom, out_bf16);
                    }
                }
            }
        }
    }
}

/*
 * Max pooling (non-trainable, merges by concatenation: Section 3.1).  Per channel
 * of x[B][Ctot][H][W]; window k x k, stride, padding with -infinity (padded
 * positions never win).  y[B][Ctot][Ho][Wo], Ho = (H + 2 pad - k)/stride + 1.
 */
void oracle_maxpool2d(const float *x, float *y, int B, int Ctot, int H, int Wd, int k, int stride,
                      int pad, int out_bf16)
{
    const int Ho = (H + 2 * pad - k) / stride + 1, Wo = (Wd + 2 * pad - k) / stride + 1;
    #pragma omp parallel for schedule(static)
    for (int bc = 0; bc < B * Ctot; ++bc) {
        for (int oy = 0; oy < Ho; ++oy)
            for (int ox = 0; ox < Wo; ++ox) {
                double best = -INFINITY;
                for (int ky = 0; ky < k; ++ky)
                    for (int kx = 0; kx < k; ++kx) {
                        int iy = oy * stride + ky - pad, ix = ox * stride + kx - pad;
                        if (iy < 0 || iy >= H || ix < 0 || ix >= Wd) continue;
                        double v = x[((size_t)bc * H + iy) * Wd + ix];
                        if (v > best) best = v;
                    }
                y[((size_t)bc * Ho + oy) * Wo + ox] = finish(best, out_bf16);
            }
    }
}

/* Global average pooling (non-trainable): y[B][Ctot] = mean over the HW positions of x[B][Ctot][HW]. */
void oracle_avgpool_global(const float *x, float *y, int B, int Ctot, int HW, int out_bf16)
{
    #pragma omp parallel for schedule(static)
    for (int bc = 0; bc < B * Ctot; ++bc) {
        double acc = 0.0;
        for (int p = 0; p < HW; ++p) acc += (double)x[(size_t)bc * HW + p];
        y[bc] = finish(acc / HW, out_bf16);
    }
}

/*
 * The reshape-and-transpose inserted where consecutive merged operators disagree
 * on the merge dimension (Section 3.2, Algorithm 1):
 * to_channel != 0:  batch-merged src[M][rows][H]  ->  channel-merged dst[rows][M*H]
 * to_channel == 0:  the inverse.
 */
void oracle_merge_transpose(const float *src, float *dst, int M, int rows, int H, int to_channel)
{
    for (int m = 0; m < M; ++m)
        for (int r = 0; r < rows; ++r)
            for (int i = 0; i < H; ++i) {
                size_t ib = ((size_t)m * rows + r) * H + i;      /* batch-merged address   */
                size_t ic = ((size_t)r * M + m) * H + i;         /* channel-merged address */
                if (to_channel) dst[ic] = src[ib]; else dst[ib] = src[ic];
            }
}

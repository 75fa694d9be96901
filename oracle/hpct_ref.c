/*
 * CPU checker for the fused tensor operators.  TEST INFRASTRUCTURE ONLY:
 * it exists so that the GPU library's results can be compared with something
 * obviously correct, and to be timed as a reported CPU baseline.  The GPU
 * library never calls it and shares no source, header or table with it.
 *
 * Every function is the plain mathematical definition of its operator written
 * as nested loops: fp32 inputs are widened to double, every product and sum
 * is taken in double (an fp32*fp32 product is exact in double), libm
 * exp/tanh/sqrt in double, results returned as double.  Chains keep their
 * intermediates in double.  The only parallelism is an OpenMP pragma on the
 * outermost independent loop, the style of the CPU code in the paper's
 * Listing "CPU C Code without TVM dependency" (Section 3.5) and of its
 * VGG-16 case study (Section 5.3).  No blocking, no SIMD, no BLAS.
 *
 * Operator classes follow the paper's Table 1: Elementwise (add, sub, mul, div, sqrt, sin, cos, relu, ...),
 * Reduction (sum, mean, softmax), ComputeIntensive (matmul, conv).
 *
 * Parity pins: every function here is pinned by tests that do not run it
 * against itself (closed forms, invariants, brute force, textbook special
 * cases); none is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

/* ---- ComputeIntensive: matmul (Table 1) with a column-broadcast bias -------
 * Z[m][n] = bias[n] + sum_k X[m][k] * W[k][n];  X is [M,K], W is [K,N], both
 * row-major.  Dn[m][n] = |bias[n]| + sum_k |X[m][k]| |W[k][n]| is the scale
 * the contraction tolerance is normalised by.  bias may be NULL (= 0);
 * Dn may be NULL. */
void ref_gemm_bias(const float *X, const float *W, const float *bias,
                   int64_t M, int64_t K, int64_t N, double *Z, double *Dn)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            double b = bias ? (double)bias[n] : 0.0;
            double acc = b, mag = fabs(b);
            for (int64_t k = 0; k < K; ++k) {
                double a = (double)X[m * K + k], w = (double)W[k * N + n];
                acc += a * w;
                mag += fabs(a) * fabs(w);
            }
            Z[m * N + n] = acc;
            if (Dn) Dn[m * N + n] = mag;
        }
    }
}

/* ---- Elementwise: relu (Table 1), in place ------------------------------ */
void ref_relu(double *Z, int64_t count)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) Z[i] = Z[i] > 0.0 ? Z[i] : 0.0;
}

/* ---- Elementwise: multiplication by a constant, in place (the "Scale" of the
 * fused Gemm-Scale operator named in Section 5.2).  The constant is the fp32
 * value the GPU path receives, widened to double. */
void ref_scale(double *Z, int64_t count, float s)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) Z[i] = Z[i] * (double)s;
}

/* ---- Reduction: softmax (Table 1) over the last dimension ---------------
 * Y[r][n] = exp(Z[r][n] - max_n Z[r][.]) / sum_n exp(Z[r][n] - max). */
void ref_softmax_rows(const double *Z, int64_t rows, int64_t N, double *Y)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const double *z = Z + r * N;
        double *y = Y + r * N;
        double mx = z[0];
        for (int64_t n = 1; n < N; ++n) if (z[n] > mx) mx = z[n];
        double sum = 0.0;
        for (int64_t n = 0; n < N; ++n) { y[n] = exp(z[n] - mx); sum += y[n]; }
        for (int64_t n = 0; n < N; ++n) y[n] /= sum;
    }
}

/* ---- Elementwise chain: per-channel affine, relu, residual add ----------
 * T[p][i] = relu(X[p][i] * scale[c] + shift[c]) + R[p][i], with plane
 * p = n*C + c of an NCHW tensor and i running over the H*W plane.  The
 * residual is added after the relu. */
void ref_affine_relu_residual(const float *X, const float *scale, const float *shift,
                              const float *R, int64_t Nb, int64_t C, int64_t HW, double *T)
{
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < Nb * C; ++p) {
        int64_t c = p % C;
        double s = (double)scale[c], t = (double)shift[c];
        for (int64_t i = 0; i < HW; ++i) {
            double v = (double)X[p * HW + i] * s + t;
            v = v > 0.0 ? v : 0.0;
            T[p * HW + i] = v + (double)R[p * HW + i];
        }
    }
}

/* ---- Reduction: mean (Table 1) over each H*W plane = global average pool */
void ref_avgpool_planes(const double *T, int64_t planes, int64_t HW, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < planes; ++p) {
        double sum = 0.0;
        for (int64_t i = 0; i < HW; ++i) sum += T[p * HW + i];
        out[p] = sum / (double)HW;
    }
}

/* ---- Reduction: layer normalisation over the last dimension -------------
 * mu = sum x / N; var = sum (x-mu)^2 / N (biased); y = (x-mu)/sqrt(var+eps)
 * * gamma + beta.  gamma / beta may be NULL (= 1 / 0). */
void ref_layernorm_rows(const float *X, const float *gamma, const float *beta,
                        int64_t rows, int64_t N, double eps, double *Y)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const float *x = X + r * N;
        double mu = 0.0;
        for (int64_t n = 0; n < N; ++n) mu += (double)x[n];
        mu /= (double)N;
        double var = 0.0;
        for (int64_t n = 0; n < N; ++n) { double d = (double)x[n] - mu; var += d * d; }
        var /= (double)N;
        double inv = 1.0 / sqrt(var + eps);
        for (int64_t n = 0; n < N; ++n) {
            double g = gamma ? (double)gamma[n] : 1.0, b = beta ? (double)beta[n] : 0.0;
            Y[r * N + n] = ((double)x[n] - mu) * inv * g + b;
        }
    }
}

/* ---- Reduction: root-mean-square normalisation over the last dimension (the
 * layer normalisation of Table 1's Reduction class without the mean):
 *   y = x / sqrt(mean(x^2) + eps) * gamma.  gamma may be NULL (= 1). */
void ref_rmsnorm_rows(const float *X, const float *gamma, int64_t rows, int64_t N, double eps, double *Y)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const float *x = X + r * N;
        double ms = 0.0;
        for (int64_t n = 0; n < N; ++n) ms += (double)x[n] * (double)x[n];
        ms /= (double)N;
        double inv = 1.0 / sqrt(ms + eps);
        for (int64_t n = 0; n < N; ++n) Y[r * N + n] = (double)x[n] * inv * (gamma ? (double)gamma[n] : 1.0);
    }
}

/* ---- Reduction: group normalisation of an NCHW tensor (the "norm" of the
 * activation-and-norm fusions that Section 5.1 describes as Level-2 tasks; G = C is
 * instance normalisation, G = 1 layer normalisation over C, H and W).  The C
 * channels are split into G groups of C/G neighbours; for image n and group g
 *   mu = mean of x over the group's (C/G) H W elements, var = mean of (x - mu)^2 (biased),
 *   y[n][c][i] = (x[n][c][i] - mu) / sqrt(var + eps) * gamma[c] + beta[c].
 * gamma / beta may be NULL (= 1 / 0). */
void ref_groupnorm_nchw(const float *X, const float *gamma, const float *beta,
                        int64_t Nb, int64_t C, int64_t HW, int64_t G, double eps, double *Y)
{
    const int64_t Cg = C / G, L = Cg * HW;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < Nb * G; ++r) {
        const int64_t g = r % G;
        const float *x = X + r * L;
        double mu = 0.0;
        for (int64_t i = 0; i < L; ++i) mu += (double)x[i];
        mu /= (double)L;
        double var = 0.0;
        for (int64_t i = 0; i < L; ++i) { double d = (double)x[i] - mu; var += d * d; }
        var /= (double)L;
        double inv = 1.0 / sqrt(var + eps);
        for (int64_t i = 0; i < L; ++i) {
            int64_t c = g * Cg + i / HW;
            double ga = gamma ? (double)gamma[c] : 1.0, be = beta ? (double)beta[c] : 0.0;
            Y[r * L + i] = ((double)x[i] - mu) * inv * ga + be;
        }
    }
}

/* ---- Elementwise: tanh-form GELU, in place -------------------------------
 * 0.5 y (1 + tanh(sqrt(2/pi) (y + 0.044715 y^3))) */
void ref_gelu_tanh(double *Y, int64_t count)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        double y = Y[i];
        Y[i] = 0.5 * y * (1.0 + tanh(0.7978845608028654 * (y + 0.044715 * y * y * y)));
    }
}

/* ---- ComputeIntensive: conv (Table 1), NCHW ----------------------------------
 * Definition.  Let xp be the input plane extended by zeros outside
 * 0 <= row < H, 0 <= col < W.  Then
 *   out[n][k][y][x] = bias[k]
 *       + sum over c, r, s of  xp[n][c][y*stride - P + r*dil][x*stride - P + s*dil] * wt[k][c][r][s]
 * for 0 <= y < Ho = (H + 2P - (R-1)*dil - 1)/stride + 1 and 0 <= x < Wo likewise:
 * a cross-correlation (the filter is not flipped) with zero padding P, the bias
 * as the sum's first term, weights stored [K][C][R][S], output stored
 * [N][K][Ho][Wo].  This is the operator of the paper's VGG-16 case study
 * (Section 5.3) at stride 1, P = 1, R = S = 3, dil = 1, where Ho = H.
 * Dn (may be NULL) = |bias| + sum |xp| |wt| over the same terms: the
 * normaliser of the contraction tolerance. */
static double padded_at(const float *plane, int64_t H, int64_t W, int64_t row, int64_t col)
{
    return (row < 0 || row >= H || col < 0 || col >= W) ? 0.0 : (double)plane[row * W + col];
}

void ref_conv2d_nchw_bias(const float *in, const float *wt, const float *bias,
                          int64_t Nb, int64_t C, int64_t H, int64_t W, int64_t K,
                          int64_t R, int64_t S, int64_t stride, int64_t P, int64_t dil,
                          double *out, double *Dn)
{
    const int64_t Ho = (H + 2 * P - (R - 1) * dil - 1) / stride + 1, Wo = (W + 2 * P - (S - 1) * dil - 1) / stride + 1;
#pragma omp parallel for schedule(static)
    for (int64_t plane = 0; plane < Nb * K; ++plane) {   /* one output plane (n, k) per iteration */
        const int64_t n = plane / K, k = plane % K;
        const double first = bias ? (double)bias[k] : 0.0;
        for (int64_t y = 0; y < Ho; ++y) {
            for (int64_t x = 0; x < Wo; ++x) {
                double total = first, magnitude = fabs(first);
                for (int64_t c = 0; c < C; ++c) {
                    const float *xin = in + (n * C + c) * H * W;
                    const float *filt = wt + (k * C + c) * R * S;
                    for (int64_t r = 0; r < R; ++r) {
                        for (int64_t t = 0; t < S; ++t) {
                            const double v = padded_at(xin, H, W, y * stride - P + r * dil, x * stride - P + t * dil);
                            const double g = (double)filt[r * S + t];
                            total += v * g;
                            magnitude += fabs(v) * fabs(g);
                        }
                    }
                }
                out[(plane * Ho + y) * Wo + x] = total;
                if (Dn) Dn[(plane * Ho + y) * Wo + x] = magnitude;
            }
        }
    }
}

/* ---- Grouped conv (depthwise when groups = C = K): the conv above with the
 * input channels split into `groups` equal runs and the output channels
 * likewise; output channel k (group g = k / (K/groups)) sums only over the
 * C/groups input channels of its group, and its filter is wt[k][0 .. C/groups)
 * [R][S] (weights are [K][C/groups][R][S] contiguous).  groups = 1 is the conv
 * above; groups = C = K is the depthwise convolution of the MobileNetV2 blocks
 * (a model the paper's Section 5.2 names).  Same tap index, zero padding,
 * stride and dilation rules.  Dn as above. */
void ref_conv2d_nchw_grouped(const float *in, const float *wt, const float *bias,
                             int64_t Nb, int64_t C, int64_t H, int64_t W, int64_t K,
                             int64_t R, int64_t S, int64_t stride, int64_t P, int64_t dil,
                             int64_t groups, double *out, double *Dn)
{
    const int64_t Ho = (H + 2 * P - (R - 1) * dil - 1) / stride + 1, Wo = (W + 2 * P - (S - 1) * dil - 1) / stride + 1;
    const int64_t Cg = C / groups, Kg = K / groups;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t n = 0; n < Nb; ++n) {
        for (int64_t k = 0; k < K; ++k) {
            const int64_t c_first = (k / Kg) * Cg;
            for (int64_t h = 0; h < Ho; ++h) {
                for (int64_t w = 0; w < Wo; ++w) {
                    double b = bias ? (double)bias[k] : 0.0;
                    double sum = b, mag = fabs(b);
                    for (int64_t c = 0; c < Cg; ++c) {
                        for (int64_t kh = 0; kh < R; ++kh) {
                            for (int64_t kw = 0; kw < S; ++kw) {
                                int64_t ih = h * stride - P + kh * dil;
                                int64_t iw = w * stride - P + kw * dil;
                                if (ih >= 0 && ih < H && iw >= 0 && iw < W) {
                                    double a = (double)in[((n * C + c_first + c) * H + ih) * W + iw];
                                    double g = (double)wt[((k * Cg + c) * R + kh) * S + kw];
                                    sum += a * g;
                                    mag += fabs(a) * fabs(g);
                                }
                            }
                        }
                    }
                    int64_t o = ((n * K + k) * Ho + h) * Wo + w;
                    out[o] = sum;
                    if (Dn) Dn[o] = mag;
                }
            }
        }
    }
}

/* ---- Transposed conv ("Conv-Trans", a Level-2 operator the paper's Section 5.2
 * names), NCHW, the adjoint of the conv above with respect to its input:
 * every input element is scattered through the filter,
 *     out[n][k][ih*stride - P + kh*dil][iw*stride - P + kw*dil] += in[n][c][ih][iw] * wt[c][k][kh][kw],
 * positions outside the output dropped; out starts at bias[k].  Weights are
 * [C][K][R][S] contiguous (input channels first).  Output size
 * (H - 1)*stride - 2P + (R - 1)*dil + 1 (no extra output padding).
 * Dn (may be NULL) = |bias| + the same sum over absolute values. */
void ref_conv_transpose2d_nchw(const float *in, const float *wt, const float *bias,
                               int64_t Nb, int64_t C, int64_t H, int64_t W, int64_t K,
                               int64_t R, int64_t S, int64_t stride, int64_t P, int64_t dil,
                               double *out, double *Dn)
{
    const int64_t Ho = (H - 1) * stride - 2 * P + (R - 1) * dil + 1, Wo = (W - 1) * stride - 2 * P + (S - 1) * dil + 1;
#pragma omp parallel for schedule(static) collapse(2)
    for (int64_t n = 0; n < Nb; ++n) {
        for (int64_t k = 0; k < K; ++k) {        /* one output plane per iteration: no two threads write the same element */
            double *o = out + (n * K + k) * Ho * Wo;
            double *d = Dn ? Dn + (n * K + k) * Ho * Wo : NULL;
            double b = bias ? (double)bias[k] : 0.0;
            for (int64_t i = 0; i < Ho * Wo; ++i) { o[i] = b; if (d) d[i] = fabs(b); }
            for (int64_t c = 0; c < C; ++c) {
                for (int64_t ih = 0; ih < H; ++ih) {
                    for (int64_t iw = 0; iw < W; ++iw) {
                        double a = (double)in[((n * C + c) * H + ih) * W + iw];
                        for (int64_t kh = 0; kh < R; ++kh) {
                            for (int64_t kw = 0; kw < S; ++kw) {
                                int64_t oh = ih * stride - P + kh * dil;
                                int64_t ow = iw * stride - P + kw * dil;
                                if (oh >= 0 && oh < Ho && ow >= 0 && ow < Wo) {
                                    double g = (double)wt[((c * K + k) * R + kh) * S + kw];
                                    o[oh * Wo + ow] += a * g;
                                    if (d) d[oh * Wo + ow] += fabs(a) * fabs(g);
                                }
                            }
                        }
                    }
                }
            }
        }
    }
}

/* ---- Elementwise: relu6 = min(max(z, 0), 6), the activation of those blocks, in place */
void ref_relu6(double *Z, int64_t count)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) Z[i] = Z[i] < 0.0 ? 0.0 : (Z[i] > 6.0 ? 6.0 : Z[i]);
}

/* ---- Batched matmul - softmax - matmul ------------------------------------
 * For each batch b and query i:  s_j = scale * sum_d Q[b][i][d] K[b][j][d];
 * p = softmax_j(s) (two passes over one materialised row, not an online
 * recurrence);  O[b][i][d] = sum_j p_j V[b][j][d].
 * Dn[b][i][d] = sum_j p_j |V[b][j][d]| (may be NULL).
 * Q is [B,Lq,D], K and V are [B,Lk,D], row-major; Lk >= 1. */
void ref_attention(const float *Q, const float *K, const float *V,
                   int64_t B, int64_t Lq, int64_t Lk, int64_t D, double scale,
                   double *O, double *Dn)
{
#pragma omp parallel for schedule(static)
    for (int64_t bi = 0; bi < B * Lq; ++bi) {
        int64_t b = bi / Lq;
        const float *q = Q + bi * D;
        const float *Kb = K + b * Lk * D, *Vb = V + b * Lk * D;
        double *s = (double *)malloc((size_t)Lk * sizeof(double));
        double mx = -INFINITY;
        for (int64_t j = 0; j < Lk; ++j) {
            double acc = 0.0;
            for (int64_t d = 0; d < D; ++d) acc += (double)q[d] * (double)Kb[j * D + d];
            s[j] = acc * scale;
            if (s[j] > mx) mx = s[j];
        }
        double sum = 0.0;
        for (int64_t j = 0; j < Lk; ++j) { s[j] = exp(s[j] - mx); sum += s[j]; }
        for (int64_t j = 0; j < Lk; ++j) s[j] /= sum;
        for (int64_t d = 0; d < D; ++d) {
            double acc = 0.0, mag = 0.0;
            for (int64_t j = 0; j < Lk; ++j) {
                double v = (double)Vb[j * D + d];
                acc += s[j] * v;
                mag += s[j] * fabs(v);
            }
            O[bi * D + d] = acc;
            if (Dn) Dn[bi * D + d] = mag;
        }
        free(s);
    }
}

/* Threads the OpenMP loops above will use (reported next to baseline timings). */
#ifdef _OPENMP
#include <omp.h>
int ref_max_threads(void) { return omp_get_max_threads(); }
void ref_set_threads(int n) { if (n > 0) omp_set_num_threads(n); }
#else
int ref_max_threads(void) { return 1; }
void ref_set_threads(int n) { (void)n; }
#endif

/* ---- LayoutTransform (Table 1: "reshape, transpose"): out = contiguous copy
 * of a strided view.  out[i0]...[i_{nd-1}] (row-major over `shape`) =
 * in[sum_d i_d * stride[d]] (strides in elements, >= 0).  Values are copied as
 * 32-bit patterns, so the result is bit-exact by definition. */
void ref_layout_copy(const uint32_t *in, int32_t nd, const int64_t *shape, const int64_t *stride, uint32_t *out)
{
    int64_t total = 1;
    for (int32_t d = 0; d < nd; ++d) total *= shape[d];
#pragma omp parallel for schedule(static)
    for (int64_t lin = 0; lin < total; ++lin) {
        int64_t rem = lin, off = 0;
        for (int32_t d = nd - 1; d >= 0; --d) {
            off += (rem % shape[d]) * stride[d];
            rem /= shape[d];
        }
        out[lin] = in[off];
    }
}

/* ---- Hash dropout of the fused [Matmul, Dropout, Mean, Softmax] case study (Section 5.3).
 * The paper gives the random number of an element as a function of its linear
 * position and a seed:  u(t) = ((t' mod 1000) as fp32) / 1000.0f  with
 *     t' = mix(t),  mix: t ^= t >> 17, then t ^= t << 31, then t ^= t >> 8   (unsigned 64-bit)
 * and t = i*N + j + seed (wrapping) for row i, column j of an [M,N] tensor.
 * What is done with u is not printed; the reading taken is training-mode
 * dropout: the element becomes 0 when u < p (an fp32 comparison) and is
 * multiplied by 1 / (1 - p) otherwise. */
float ref_dropout_rand(uint64_t t)
{
    t ^= t >> 17;
    t ^= t << 31;
    t ^= t >> 8;
    return (float)(t % 1000u) / 1000.0f;
}

void ref_dropout_hash(double *Z, int64_t M, int64_t N, float p, uint64_t seed)
{
    const double survivor = 1.0 / (1.0 - (double)p);
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < M * N; ++e) {   /* e = i*N + j */
        const float u = ref_dropout_rand((uint64_t)e + seed);
        Z[e] = u < p ? 0.0 : Z[e] * survivor;
    }
}

/* ---- Reduction: mean (Table 1) over the last dimension: out[r] = (1/N) sum_n Z[r][n]. */
void ref_mean_rows(const double *Z, int64_t rows, int64_t N, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        double s = 0.0;
        for (int64_t n = 0; n < N; ++n) s += Z[r * N + n];
        out[r] = s / (double)N;
    }
}

/* ---- Elementwise: per-channel scale and shift (a folded batch-norm, the
 * "Conv2d BN" block named in Section 5.2) on an NCHW tensor held in double, in
 * place:  T[n][c][i] = T[n][c][i] * scale[c] + shift[c].  Either may be NULL. */
void ref_scale_shift_planes(double *T, const float *scale, const float *shift,
                            int64_t Nb, int64_t C, int64_t HW)
{
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < Nb * C; ++p) {
        const int64_t c = p % C;
        const double s = scale ? (double)scale[c] : 1.0, t = shift ? (double)shift[c] : 0.0;
        for (int64_t i = 0; i < HW; ++i) T[p * HW + i] = T[p * HW + i] * s + t;
    }
}

/* ---- Reduction: 2x2 max pooling with stride 2 over the planes of an NCHW
 * tensor (the pooling that closes each VGG-16 block, Section 5.3):
 * out[p][y][x] = max over dy,dx in {0,1} of T[p][2y+dy][2x+dx], for
 * y < H/2, x < W/2 (integer division: an odd last row or column is dropped). */
void ref_maxpool2x2_planes(const double *T, int64_t planes, int64_t H, int64_t W, double *out)
{
    const int64_t Hp = H / 2, Wp = W / 2;
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < planes; ++p) {
        for (int64_t y = 0; y < Hp; ++y) {
            for (int64_t x = 0; x < Wp; ++x) {
                double m = T[(p * H + 2 * y) * W + 2 * x];
                for (int64_t dy = 0; dy < 2; ++dy)
                    for (int64_t dx = 0; dx < 2; ++dx) {
                        double v = T[(p * H + 2 * y + dy) * W + 2 * x + dx];
                        if (v > m) m = v;
                    }
                out[(p * Hp + y) * Wp + x] = m;
            }
        }
    }
}

/* ---- Reduction: max pooling with a k x k window, stride s and padding p
 * (p < k) over the planes of an NCHW tensor - the pooling layers of the
 * networks that Section 5.1 names as Level-3 tasks (a ResNet's 3x3 / stride 2
 * / pad 1; the 2x2 / stride 2 above is the case k = 2, s = 2, p = 0):
 *   out[pl][oy][ox] = max over dy, dx in 0..k-1 of T[pl][oy s - p + dy][ox s - p + dx]
 * taken over the positions inside the image only (padding never wins), for
 * oy < (H + 2p - k) / s + 1, ox < (W + 2p - k) / s + 1 (integer division). */
void ref_maxpool2d_planes(const double *T, int64_t planes, int64_t H, int64_t W, int64_t k, int64_t s, int64_t p,
                          double *out)
{
    const int64_t Ho = (H + 2 * p - k) / s + 1, Wo = (W + 2 * p - k) / s + 1;
#pragma omp parallel for schedule(static)
    for (int64_t pl = 0; pl < planes; ++pl) {
        for (int64_t oy = 0; oy < Ho; ++oy) {
            for (int64_t ox = 0; ox < Wo; ++ox) {
                double m = -INFINITY;
                for (int64_t dy = 0; dy < k; ++dy)
                    for (int64_t dx = 0; dx < k; ++dx) {
                        int64_t iy = oy * s - p + dy, ix = ox * s - p + dx;
                        if (iy < 0 || iy >= H || ix < 0 || ix >= W) continue;
                        double v = T[(pl * H + iy) * W + ix];
                        if (v > m) m = v;
                    }
                out[(pl * Ho + oy) * Wo + ox] = m;
            }
        }
    }
}

/* ---- Reduction: average pooling with a k x k window, stride s and padding p
 * (p < k) over the planes of an NCHW tensor (Table 1 "mean" over windows; the
 * pooling of the transition layers of the Level-3 networks of Section 5.1):
 *   out[pl][oy][ox] = (1 / k^2) sum over dy, dx in 0..k-1 of T[pl][oy s - p + dy][ox s - p + dx],
 * positions outside the image counting as zeros (the divisor is always k^2), for
 * oy < (H + 2p - k) / s + 1, ox < (W + 2p - k) / s + 1 (integer division). */
void ref_avgpool2d_planes(const double *T, int64_t planes, int64_t H, int64_t W, int64_t k, int64_t s, int64_t p,
                          double *out)
{
    const int64_t Ho = (H + 2 * p - k) / s + 1, Wo = (W + 2 * p - k) / s + 1;
#pragma omp parallel for schedule(static)
    for (int64_t pl = 0; pl < planes; ++pl) {
        for (int64_t oy = 0; oy < Ho; ++oy) {
            for (int64_t ox = 0; ox < Wo; ++ox) {
                double acc = 0.0;
                for (int64_t dy = 0; dy < k; ++dy)
                    for (int64_t dx = 0; dx < k; ++dx) {
                        int64_t iy = oy * s - p + dy, ix = ox * s - p + dx;
                        if (iy < 0 || iy >= H || ix < 0 || ix >= W) continue;
                        acc += T[(pl * H + iy) * W + ix];
                    }
                out[(pl * Ho + oy) * Wo + ox] = acc / (double)(k * k);
            }
        }
    }
}

/* ---- Reduction (Table 1: "sum, mean" and the arg-reductions) over one axis of
 * a strided view.  The view has `nd` dims with `shape` and `stride` (elements,
 * >= 0); the output is the view with dim `axis` removed, row-major.
 *   op 0: sum      out_val = sum_r x_r
 *   op 1: mean     out_val = (sum_r x_r) / R
 *   op 2: argmax   out_idx = the smallest r with x_r = max_r x_r
 *   op 3: argmin   out_idx = the smallest r with x_r = min_r x_r
 *   op 4: max      out_val = max_r x_r
 *   op 5: min      out_val = min_r x_r
 * For op 0/1 out_abs (may be NULL) receives sum_r |x_r| (divided by R for the
 * mean), the scale a summation's rounding error is measured against.
 * Values are widened to double; comparisons of fp32 values are exact. */
void ref_reduce_axis(const float *in, int32_t nd, const int64_t *shape, const int64_t *stride,
                     int32_t axis, int32_t op, double *out_val, double *out_abs, int64_t *out_idx)
{
    int64_t outer = 1;
    for (int32_t d = 0; d < nd; ++d) if (d != axis) outer *= shape[d];
    const int64_t R = shape[axis], sR = stride[axis];
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < outer; ++o) {
        int64_t rem = o, base = 0;
        for (int32_t d = nd - 1; d >= 0; --d) {
            if (d == axis) continue;
            base += (rem % shape[d]) * stride[d];
            rem /= shape[d];
        }
        if (op <= 1) {
            double s = 0.0, a = 0.0;
            for (int64_t r = 0; r < R; ++r) {
                double x = (double)in[base + r * sR];
                s += x;
                a += fabs(x);
            }
            if (op == 1) { s /= (double)R; a /= (double)R; }
            out_val[o] = s;
            if (out_abs) out_abs[o] = a;
        } else if (op >= 4) {
            double bv = (double)in[base];
            for (int64_t r = 1; r < R; ++r) {
                double x = (double)in[base + r * sR];
                if (op == 4 ? x > bv : x < bv) bv = x;
            }
            out_val[o] = bv;
        } else {
            int64_t best = 0;
            double bv = (double)in[base];
            for (int64_t r = 1; r < R; ++r) {
                double x = (double)in[base + r * sR];
                if (op == 2 ? x > bv : x < bv) { bv = x; best = r; }
            }
            out_idx[o] = best;
        }
    }
}

/* ---- Batched matmul - softmax - matmul with a causal mask: query i attends
 * keys j <= i only (scores of later keys are minus infinity, i.e. those keys
 * are left out of the softmax):
 *   s_j = scale * sum_d Q[b][i][d] K[b][j][d],  j = 0 .. min(i, Lk-1)
 *   p = softmax over those j;  O[b][i][d] = sum_j p_j V[b][j][d].
 * Same layout and Dn as ref_attention. */
void ref_attention_causal(const float *Q, const float *K, const float *V,
                          int64_t B, int64_t Lq, int64_t Lk, int64_t D, double scale,
                          double *O, double *Dn)
{
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t bi = 0; bi < B * Lq; ++bi) {
        int64_t b = bi / Lq, i = bi % Lq;
        int64_t n = i + 1 < Lk ? i + 1 : Lk;   /* keys 0 .. n-1 */
        const float *q = Q + bi * D;
        const float *Kb = K + b * Lk * D, *Vb = V + b * Lk * D;
        double *s = (double *)malloc((size_t)n * sizeof(double));
        double mx = -INFINITY;
        for (int64_t j = 0; j < n; ++j) {
            double acc = 0.0;
            for (int64_t d = 0; d < D; ++d) acc += (double)q[d] * (double)Kb[j * D + d];
            s[j] = acc * scale;
            if (s[j] > mx) mx = s[j];
        }
        double sum = 0.0;
        for (int64_t j = 0; j < n; ++j) { s[j] = exp(s[j] - mx); sum += s[j]; }
        for (int64_t j = 0; j < n; ++j) s[j] /= sum;
        for (int64_t d = 0; d < D; ++d) {
            double acc = 0.0, mag = 0.0;
            for (int64_t j = 0; j < n; ++j) {
                double v = (double)Vb[j * D + d];
                acc += s[j] * v;
                mag += s[j] * fabs(v);
            }
            O[bi * D + d] = acc;
            if (Dn) Dn[bi * D + d] = mag;
        }
        free(s);
    }
}

/* ---- Elementwise chain on strided views (Table 1, Elementwise: "add, sub, mul,
 * div, sqrt, sin, cos, relu and etc.").  v = a[..] alone (bin < 0, b unused) or
 * a[..] (+, *, -, /) b[..] for bin = 0, 1, 2, 3; then the n_un unary steps un[0],
 * un[1], ... are applied to v in that order:
 *   0 max(v, 0)      1 tanh-form GELU      2 v * scale      3 sqrt(v)     4 sin(v)
 *   5 cos(v)         6 exp(v)              7 tanh(v)        8 1 / (1 + exp(-v))
 *   9 min(max(v, 0), 6)      10 |v|        11 -v        12 v * v        13 ln(v)
 *   14 v / (1 + exp(-v)) (SiLU)         15 v * min(max(v + 3, 0), 6) / 6 (hard swish)
 * Everything in double from the widened fp32 operands; libm supplies the
 * transcendental functions. */
void ref_eltwise_map(const float *a, const float *b, int32_t nd, const int64_t *shape,
                     const int64_t *sa, const int64_t *sb, int32_t bin, int32_t n_un,
                     const int32_t *un, float scale, double *out)
{
    int64_t total = 1;
    for (int32_t d = 0; d < nd; ++d) total *= shape[d];
#pragma omp parallel for schedule(static)
    for (int64_t lin = 0; lin < total; ++lin) {
        int64_t rem = lin, oa = 0, ob = 0;
        for (int32_t d = nd - 1; d >= 0; --d) {
            int64_t i = rem % shape[d];
            oa += i * sa[d];
            if (bin >= 0) ob += i * sb[d];
            rem /= shape[d];
        }
        double v = (double)a[oa];
        if (bin >= 0) {
            double y = (double)b[ob];
            v = bin == 0 ? v + y : bin == 1 ? v * y : bin == 2 ? v - y : v / y;
        }
        for (int32_t k = 0; k < n_un; ++k) {
            switch (un[k]) {
                case 0: v = v > 0.0 ? v : 0.0; break;
                case 1: v = 0.5 * v * (1.0 + tanh(0.7978845608028654 * (v + 0.044715 * v * v * v))); break;
                case 2: v = v * (double)scale; break;
                case 3: v = sqrt(v); break;
                case 4: v = sin(v); break;
                case 5: v = cos(v); break;
                case 6: v = exp(v); break;
                case 7: v = tanh(v); break;
                case 8: v = 1.0 / (1.0 + exp(-v)); break;
                case 9: v = v < 0.0 ? 0.0 : (v > 6.0 ? 6.0 : v); break;
                case 10: v = fabs(v); break;
                case 11: v = -v; break;
                case 12: v = v * v; break;
                case 13: v = log(v); break;
                case 14: v = v / (1.0 + exp(-v)); break;
                default: { double t = v + 3.0; t = t < 0.0 ? 0.0 : (t > 6.0 ? 6.0 : t); v = v * t / 6.0; } break;   /* 15: hard swish */
            }
        }
        out[lin] = v;
    }
}

/* ---- Elementwise (Table 1: "add, mul, relu") on two strided views of the same
 * shape; broadcasting is a stride of 0.  out[i0]..[i_{nd-1}] (row-major) =
 * f(a[sum i_d * sa[d]], b[sum i_d * sb[d]]) with f = a + b (op 0) or a * b
 * (op 1), followed by max(., 0) when relu != 0.  The fp32 operands are widened
 * to double (the product of two fp32 values is exact in double). */
void ref_eltwise_binary(const float *a, const float *b, int32_t nd, const int64_t *shape,
                        const int64_t *sa, const int64_t *sb, int32_t op, int32_t relu, double *out)
{
    int64_t total = 1;
    for (int32_t d = 0; d < nd; ++d) total *= shape[d];
#pragma omp parallel for schedule(static)
    for (int64_t lin = 0; lin < total; ++lin) {
        int64_t rem = lin, oa = 0, ob = 0;
        for (int32_t d = nd - 1; d >= 0; --d) {
            int64_t i = rem % shape[d];
            oa += i * sa[d];
            ob += i * sb[d];
            rem /= shape[d];
        }
        double x = (double)a[oa], y = (double)b[ob];
        double v = op == 0 ? x + y : x * y;
        out[lin] = (relu && v < 0.0) ? 0.0 : v;
    }
}

/*
 * CPU oracle for the dense tensor operators of "Tensor Program Optimization
 * with Probabilistic Programs" (arXiv 2205.13603).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the reference the GPU kernels are
 * compared with; nothing in the product library includes, links or calls it.
 * It shares no code with the HIP path.
 *
 * The paper's search space S(e0) contains only programs that are
 * semantically equal to the initial program e0 (Section 2; Section 3.1:
 * every transformation step maps e_{i-1} to an equivalent e_i).  So whatever
 * trace is chosen, the result is the operator's plain definition, and the
 * oracle is that definition written as nested loops, one loop per index of
 * the definition, no blocking, no reordering:
 *
 *   GEMM / batched matmul (Appendix A.2: GMM, TBG)
 *       C[b][i][j] = sum_k A[b][i][k] * B[b][k][j]
 *   conv2d NHWC with bias and ReLU (Appendix A.2: C2D, CBR; with groups: GRP - each group of Cout/groups
 *   output channels sums over its own Cin/groups input channels only)
 *       Y[n][oh][ow][co] = act(bias[co] + sum_{kh,kw,ci}
 *             Xpad[n][oh*s+kh-p][ow*s+kw-p][ci] * W[kh][kw][ci][co])
 *   depthwise conv2d NHWC (Appendix A.2: DEP)
 *       Y[n][oh][ow][c] = sum_{kh,kw} Xpad[n][oh*s+kh-p][ow*s+kw-p][c] * W[kh][kw][c]
 *   conv3d NDHWC with bias and ReLU (Appendix A.2: C3D), the same stride, padding and dilation on the three axes
 *       Y[n][od][oh][ow][co] = act(bias[co] + sum_{kd,kh,kw,ci}
 *             Xpad[n][od*s+kd*d-p][oh*s+kh*d-p][ow*s+kw*d-p][ci] * W[kd][kh][kw][ci][co])
 *   conv1d NWC with bias and ReLU (Appendix A.2: C1D)
 *       Y[n][ol][co] = act(bias[co] + sum_{k,ci} Xpad[n][ol*s + k*d - p][ci] * W[k][ci][co])
 *   transposed conv2d NHWC (Appendix A.2: T2D), the adjoint of the conv2d above in X:
 *       Y[n][ih*s+kh-p][iw*s+kw-p][co] += X[n][ih][iw][ci] * W[kh][kw][ci][co]   (then bias, ReLU)
 *       output size (H-1)*s - 2p + KH
 *   softmax over the last axis (Appendix A.2: SFM, batch x m x n)
 *       Y[r][j] = exp(X[r][j] - max_j X[r][j]) / sum_j exp(X[r][j] - max_j X[r][j])
 *   norm (Appendix A.2: NRM, batch x m x n)
 *       Y[b] = sqrt(sum_{i,j} X[b][i][j]^2)
 *
 * Readings where the paper is silent: cross-correlation (no kernel flip),
 * zero padding, output size floor((H + 2p - KH)/s) + 1, weights HWIO.
 * The appendix gives only the shapes of SFM and NRM: softmax is taken over
 * the last axis n of every (batch, m) row, in the shifted form above (equal
 * to exp(x_j) / sum exp(x_j) in exact arithmetic); the norm is the 2-norm of
 * all m*n elements of one batch entry (the Frobenius norm of the matrix), one
 * number per batch entry.
 *
 * Floating point inputs (fp32, fp16, bf16 bit patterns) are widened exactly
 * to double and accumulated in double, in index order.  int8 inputs are
 * accumulated in int32.  Outputs are dense row-major.
 *
 * Operands are addressed through element strides so that transposed layouts
 * (the TBG workload's fused transpose) need no copy.
 *
 * The outermost output loop carries an OpenMP pragma; it changes nothing in
 * the arithmetic of any output element.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORA_F32 = 0, ORA_F16 = 1, ORA_BF16 = 2, ORA_I8 = 3, ORA_F8E4M3 = 5 };

/* IEEE binary16 bit pattern -> double, exact. */
static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0) {
        v = (double)frac * (1.0 / 16777216.0); /* frac * 2^-24 (subnormal) */
    } else if (expo == 31) {
        if (frac == 0) {
            v = 1.0 / 0.0;
        } else {
            v = 0.0 / 0.0;
        }
    } else {
        double scale = 1.0;
        int e = expo - 15;
        int t;
        for (t = 0; t < e; ++t) scale *= 2.0;
        for (t = 0; t > e; --t) scale *= 0.5;
        v = (1.0 + (double)frac / 1024.0) * scale;
    }
    return sign ? -v : v;
}

/* bfloat16 bit pattern -> double: it is the high half of a binary32. */
static double bf16_bits_to_double(uint16_t b)
{
    uint32_t w = (uint32_t)b << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

/* 8-bit float of the OCP "E4M3" kind (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no
 * infinities, the all-ones exponent-and-mantissa pattern is NaN, largest finite value 448) -> double, exact. */
static double f8e4m3_bits_to_double(uint8_t b)
{
    int sign = (b >> 7) & 1;
    int expo = (b >> 3) & 0xf;
    int frac = b & 0x7;
    double v;
    if (expo == 15 && frac == 7) {
        v = 0.0 / 0.0;
    } else if (expo == 0) {
        v = (double)frac * (1.0 / 512.0); /* frac/8 * 2^-6 (subnormal) */
    } else {
        double scale = 1.0;
        int e = expo - 7;
        int t;
        for (t = 0; t < e; ++t) scale *= 2.0;
        for (t = 0; t > e; --t) scale *= 0.5;
        v = (1.0 + (double)frac / 8.0) * scale;
    }
    return sign ? -v : v;
}

static double load_elem(int dtype, const void *base, int64_t idx)
{
    switch (dtype) {
    case ORA_F32: return (double)((const float *)base)[idx];
    case ORA_F16: return half_bits_to_double(((const uint16_t *)base)[idx]);
    case ORA_BF16: return bf16_bits_to_double(((const uint16_t *)base)[idx]);
    case ORA_I8: return (double)((const int8_t *)base)[idx];
    case ORA_F8E4M3: return f8e4m3_bits_to_double(((const uint8_t *)base)[idx]);
    default: return 0.0 / 0.0;
    }
}

int ms_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Threads of the following calls (the benchmark's single-thread baseline); 0 restores the default. No arithmetic. */
void ms_oracle_set_threads(int n)
{
#ifdef _OPENMP
    static int initial = 0;
    if (!initial) initial = omp_get_max_threads();
    omp_set_num_threads(n > 0 ? n : initial);
#else
    (void)n;
#endif
}

/*
 * Type of the running sum of the three operators the benchmark times as its CPU baseline (matrix product, conv2d,
 * depthwise conv2d).  The oracle is built with double, always: that is what every test compares with.  The benchmark
 * additionally builds this file with -DORA_ACC_T=float into a library of its own, only to report how fast the same
 * plain loops run when they accumulate in the operator's own precision; no test loads that library.
 */
#ifndef ORA_ACC_T
#define ORA_ACC_T double
#endif

/* Exposed so that tests can pin the widening itself. */
double ms_oracle_widen(int dtype, const void *base, int64_t idx)
{
    return load_elem(dtype, base, idx);
}

/*
 * Batched matmul, floating point.  C is dense [nb][M][N] in double.
 * A element (b,i,k) sits at A[b*sAb + i*sAi + k*sAk]; B element (b,k,j) at
 * B[b*sBb + k*sBk + j*sBj].  Returns 0, or -1 on a bad dtype.
 */
int ms_oracle_bmm(int dtype, int64_t nb, int64_t M, int64_t N, int64_t K,
                  const void *A, int64_t sAb, int64_t sAi, int64_t sAk,
                  const void *B, int64_t sBb, int64_t sBk, int64_t sBj,
                  double *C)
{
    if (dtype != ORA_F32 && dtype != ORA_F16 && dtype != ORA_BF16 && dtype != ORA_F8E4M3) return -1;
    int64_t bi;
#pragma omp parallel for schedule(static)
    for (bi = 0; bi < nb * M; ++bi) {
        int64_t b = bi / M, i = bi % M;
        for (int64_t j = 0; j < N; ++j) {
            ORA_ACC_T acc = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double a = load_elem(dtype, A, b * sAb + i * sAi + k * sAk);
                double w = load_elem(dtype, B, b * sBb + k * sBk + j * sBj);
                acc += a * w;
            }
            C[(b * M + i) * N + j] = acc;
        }
    }
    return 0;
}

/* Batched matmul, int8 x int8 -> int32, exact. */
int ms_oracle_bmm_i8(int64_t nb, int64_t M, int64_t N, int64_t K,
                     const int8_t *A, int64_t sAb, int64_t sAi, int64_t sAk,
                     const int8_t *B, int64_t sBb, int64_t sBk, int64_t sBj,
                     int32_t *C)
{
    int64_t bi;
#pragma omp parallel for schedule(static)
    for (bi = 0; bi < nb * M; ++bi) {
        int64_t b = bi / M, i = bi % M;
        for (int64_t j = 0; j < N; ++j) {
            int32_t acc = 0;
            for (int64_t k = 0; k < K; ++k) {
                int32_t a = A[b * sAb + i * sAi + k * sAk];
                int32_t w = B[b * sBb + k * sBk + j * sBj];
                acc += a * w;
            }
            C[(b * M + i) * N + j] = acc;
        }
    }
    return 0;
}

static int64_t conv_out_size(int64_t in, int64_t k, int64_t s, int64_t p)
{
    int64_t span = in + 2 * p - k;
    if (span < 0) return 0;
    return span / s + 1;
}

int64_t ms_oracle_conv_out_size(int64_t in, int64_t k, int64_t s, int64_t p)
{
    return conv_out_size(in, k, s, p);
}

/*
 * conv2d, NHWC activations, HWIO weights, optional fp32 bias (NULL = none),
 * optional ReLU; tap (kh, kw) reads input element (oh*stride + kh*dilation - pad,
 * ow*stride + kw*dilation - pad), zero outside the image.  Y is dense [N][OH][OW][Cout] in double.
 */
int ms_oracle_conv2d_nhwc(int dtype, int64_t N, int64_t H, int64_t W_, int64_t Cin, int64_t Cout,
                          int64_t KH, int64_t KW, int64_t stride, int64_t pad, int64_t dilation, int64_t groups,
                          const void *X, const void *Wt, const float *bias, int relu,
                          double *Y)
{
    if (dtype != ORA_F32 && dtype != ORA_F16 && dtype != ORA_BF16) return -1;
    if (dilation < 1) return -1;
    /* grouped convolution: output channel co belongs to group co / (Cout/groups) and sees only the Cin/groups
       input channels of that group; W is [KH][KW][Cin/groups][Cout] */
    if (groups < 1 || Cin % groups || Cout % groups) return -1;
    int64_t Cg = Cin / groups, Ng = Cout / groups;
    /* a filter with taps `dilation` apart spans dilation*(K-1)+1 input elements */
    int64_t OH = conv_out_size(H, dilation * (KH - 1) + 1, stride, pad);
    int64_t OW = conv_out_size(W_, dilation * (KW - 1) + 1, stride, pad);
    int64_t row;
#pragma omp parallel for schedule(static)
    for (row = 0; row < N * OH; ++row) {
        int64_t n = row / OH, oh = row % OH;
        for (int64_t ow = 0; ow < OW; ++ow) {
            for (int64_t co = 0; co < Cout; ++co) {
                ORA_ACC_T acc = 0.0;
                for (int64_t kh = 0; kh < KH; ++kh) {
                    int64_t ih = oh * stride + kh * dilation - pad;
                    for (int64_t kw = 0; kw < KW; ++kw) {
                        int64_t iw = ow * stride + kw * dilation - pad;
                        for (int64_t ci = 0; ci < Cg; ++ci) {
                            double x = 0.0;
                            if (ih >= 0 && ih < H && iw >= 0 && iw < W_)
                                x = load_elem(dtype, X, ((n * H + ih) * W_ + iw) * Cin + (co / Ng) * Cg + ci);
                            double w = load_elem(dtype, Wt, ((kh * KW + kw) * Cg + ci) * Cout + co);
                            acc += x * w;
                        }
                    }
                }
                if (bias) acc += (double)bias[co];
                if (relu && acc < 0.0) acc = 0.0;
                Y[((n * OH + oh) * OW + ow) * Cout + co] = acc;
            }
        }
    }
    return 0;
}

/*
 * conv3d, NDHWC: X [N][D][H][W][Cin], W [KD][KH][KW][Cin][Cout], Y dense [N][OD][OH][OW][Cout] in double;
 * one stride, zero padding and dilation for the three axes, output size as for conv2d on each axis.
 */
int ms_oracle_conv3d_ndhwc(int dtype, int64_t N, int64_t D, int64_t H, int64_t W_, int64_t Cin, int64_t Cout,
                           int64_t KD, int64_t KH, int64_t KW, int64_t stride, int64_t pad, int64_t dilation,
                           const void *X, const void *Wt, const float *bias, int relu, double *Y)
{
    if (dtype != ORA_F32 && dtype != ORA_F16 && dtype != ORA_BF16) return -1;
    if (dilation < 1) return -1;
    int64_t OD = conv_out_size(D, dilation * (KD - 1) + 1, stride, pad);
    int64_t OH = conv_out_size(H, dilation * (KH - 1) + 1, stride, pad);
    int64_t OW = conv_out_size(W_, dilation * (KW - 1) + 1, stride, pad);
    int64_t row;
#pragma omp parallel for schedule(static)
    for (row = 0; row < N * OD * OH; ++row) {
        int64_t n = row / (OD * OH), od = (row / OH) % OD, oh = row % OH;
        for (int64_t ow = 0; ow < OW; ++ow)
            for (int64_t co = 0; co < Cout; ++co) {
                double acc = 0.0;
                for (int64_t kd = 0; kd < KD; ++kd) {
                    int64_t id = od * stride + kd * dilation - pad;
                    if (id < 0 || id >= D) continue;
                    for (int64_t kh = 0; kh < KH; ++kh) {
                        int64_t ih = oh * stride + kh * dilation - pad;
                        if (ih < 0 || ih >= H) continue;
                        for (int64_t kw = 0; kw < KW; ++kw) {
                            int64_t iw = ow * stride + kw * dilation - pad;
                            if (iw < 0 || iw >= W_) continue;
                            for (int64_t ci = 0; ci < Cin; ++ci)
                                acc += load_elem(dtype, X, (((n * D + id) * H + ih) * W_ + iw) * Cin + ci) *
                                       load_elem(dtype, Wt, (((kd * KH + kh) * KW + kw) * Cin + ci) * Cout + co);
                        }
                    }
                }
                if (bias) acc += (double)bias[co];
                if (relu && acc < 0.0) acc = 0.0;
                Y[(row * OW + ow) * Cout + co] = acc;
            }
    }
    return 0;
}

/*
 * conv1d, NWC: X [N][L][Cin], W [K][Cin][Cout], Y dense [N][OL][Cout] in double,
 * OL = floor((L + 2*pad - dilation*(K-1) - 1) / stride) + 1; zero padding at both ends.
 */
int ms_oracle_conv1d_nwc(int dtype, int64_t N, int64_t L, int64_t Cin, int64_t Cout, int64_t K,
                         int64_t stride, int64_t pad, int64_t dilation,
                         const void *X, const void *Wt, const float *bias, int relu, double *Y)
{
    if (dtype != ORA_F32 && dtype != ORA_F16 && dtype != ORA_BF16) return -1;
    if (dilation < 1) return -1;
    int64_t OL = conv_out_size(L, dilation * (K - 1) + 1, stride, pad);
    int64_t row;
#pragma omp parallel for schedule(static)
    for (row = 0; row < N * OL; ++row) {
        int64_t n = row / OL, ol = row % OL;
        for (int64_t co = 0; co < Cout; ++co) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                int64_t il = ol * stride + k * dilation - pad;
                if (il < 0 || il >= L) continue;
                for (int64_t ci = 0; ci < Cin; ++ci)
                    acc += load_elem(dtype, X, (n * L + il) * Cin + ci) * load_elem(dtype, Wt, (k * Cin + ci) * Cout + co);
            }
            if (bias) acc += (double)bias[co];
            if (relu && acc < 0.0) acc = 0.0;
            Y[row * Cout + co] = acc;
        }
    }
    return 0;
}

/*
 * Transposed conv2d, NHWC, in its scatter form: every input element adds its
 * contribution X * W[kh][kw] to the output position (ih*s + kh - p, iw*s + kw - p)
 * if that position exists.  W is [KH][KW][Cin][Cout].  Y is dense
 * [N][OH][OW][Cout] in double with OH = (H-1)*s - 2p + KH; bias and ReLU are
 * applied after all contributions have been added.  One thread per image, so
 * that no two threads add to the same output.
 */
int ms_oracle_conv2d_transposed_nhwc(int dtype, int64_t N, int64_t H, int64_t W_, int64_t Cin, int64_t Cout,
                                     int64_t KH, int64_t KW, int64_t stride, int64_t pad,
                                     const void *X, const void *Wt, const float *bias, int relu,
                                     double *Y)
{
    if (dtype != ORA_F32 && dtype != ORA_F16 && dtype != ORA_BF16) return -1;
    int64_t OH = (H - 1) * stride - 2 * pad + KH, OW = (W_ - 1) * stride - 2 * pad + KW;
    if (OH < 1 || OW < 1) return -1;
    int64_t n;
#pragma omp parallel for schedule(static)
    for (n = 0; n < N; ++n) {
        double *Yn = Y + n * OH * OW * Cout;
        for (int64_t i = 0; i < OH * OW * Cout; ++i) Yn[i] = 0.0;
        for (int64_t ih = 0; ih < H; ++ih)
            for (int64_t iw = 0; iw < W_; ++iw)
                for (int64_t kh = 0; kh < KH; ++kh) {
                    int64_t oh = ih * stride + kh - pad;
                    if (oh < 0 || oh >= OH) continue;
                    for (int64_t kw = 0; kw < KW; ++kw) {
                        int64_t ow = iw * stride + kw - pad;
                        if (ow < 0 || ow >= OW) continue;
                        for (int64_t ci = 0; ci < Cin; ++ci) {
                            double x = load_elem(dtype, X, ((n * H + ih) * W_ + iw) * Cin + ci);
                            for (int64_t co = 0; co < Cout; ++co)
                                Yn[(oh * OW + ow) * Cout + co] += x * load_elem(dtype, Wt, ((kh * KW + kw) * Cin + ci) * Cout + co);
                        }
                    }
                }
        for (int64_t i = 0; i < OH * OW; ++i)
            for (int64_t co = 0; co < Cout; ++co) {
                double v = Yn[i * Cout + co];
                if (bias) v += (double)bias[co];
                if (relu && v < 0.0) v = 0.0;
                Yn[i * Cout + co] = v;
            }
    }
    return 0;
}

/* depthwise conv2d, NHWC activations, weights [KH][KW][C], multiplier 1. */
int ms_oracle_dwconv2d_nhwc(int dtype, int64_t N, int64_t H, int64_t W_, int64_t C,
                            int64_t KH, int64_t KW, int64_t stride, int64_t pad,
                            const void *X, const void *Wt, double *Y)
{
    if (dtype != ORA_F32 && dtype != ORA_F16 && dtype != ORA_BF16) return -1;
    int64_t OH = conv_out_size(H, KH, stride, pad);
    int64_t OW = conv_out_size(W_, KW, stride, pad);
    int64_t row;
#pragma omp parallel for schedule(static)
    for (row = 0; row < N * OH; ++row) {
        int64_t n = row / OH, oh = row % OH;
        for (int64_t ow = 0; ow < OW; ++ow) {
            for (int64_t c = 0; c < C; ++c) {
                ORA_ACC_T acc = 0.0;
                for (int64_t kh = 0; kh < KH; ++kh) {
                    int64_t ih = oh * stride + kh - pad;
                    for (int64_t kw = 0; kw < KW; ++kw) {
                        int64_t iw = ow * stride + kw - pad;
                        if (ih >= 0 && ih < H && iw >= 0 && iw < W_) {
                            double x = load_elem(dtype, X, ((n * H + ih) * W_ + iw) * C + c);
                            double w = load_elem(dtype, Wt, (kh * KW + kw) * C + c);
                            acc += x * w;
                        }
                    }
                }
                Y[((n * OH + oh) * OW + ow) * C + c] = acc;
            }
        }
    }
    return 0;
}

/*
 * Softmax over the last axis: X is dense [rows][n], Y [rows][n] in double.
 * The maximum is subtracted before exponentiation (exp() of double from libm).
 */
int ms_oracle_softmax(int dtype, int64_t rows, int64_t n, const void *X, double *Y)
{
    if (dtype != ORA_F32 && dtype != ORA_F16 && dtype != ORA_BF16) return -1;
    int64_t r;
#pragma omp parallel for schedule(static)
    for (r = 0; r < rows; ++r) {
        double mx = load_elem(dtype, X, r * n);
        for (int64_t j = 1; j < n; ++j) {
            double x = load_elem(dtype, X, r * n + j);
            if (x > mx) mx = x;
        }
        double sum = 0.0;
        for (int64_t j = 0; j < n; ++j) sum += exp(load_elem(dtype, X, r * n + j) - mx);
        for (int64_t j = 0; j < n; ++j) Y[r * n + j] = exp(load_elem(dtype, X, r * n + j) - mx) / sum;
    }
    return 0;
}

/* 2-norm of each batch entry: X dense [nb][len], Y [nb] in double. */
int ms_oracle_norm(int dtype, int64_t nb, int64_t len, const void *X, double *Y)
{
    if (dtype != ORA_F32 && dtype != ORA_F16 && dtype != ORA_BF16) return -1;
    int64_t b;
#pragma omp parallel for schedule(static)
    for (b = 0; b < nb; ++b) {
        double acc = 0.0;
        for (int64_t k = 0; k < len; ++k) {
            double x = load_elem(dtype, X, b * len + k);
            acc += x * x;
        }
        Y[b] = sqrt(acc);
    }
    return 0;
}

/*
 * The split transformation (Section 3.1, the figure that splits loop i into
 * extents 32, 8, 4; Table 2 "split"): a loop of extent E becomes n nested
 * loops with extents f[0..n-1], outermost first, product E, and the original
 * index is recovered as i = ((i0*f1 + i1)*f2 + i2)...  This routine walks
 * the nest in order and writes the recovered index of each iteration.
 * Returns the iteration count, or -1 if out is too short.
 */
int64_t ms_oracle_split_walk(int n, const int64_t *f, int64_t *out, int64_t out_len)
{
    int64_t idx[16];
    int64_t count = 0;
    int d;
    if (n < 1 || n > 16) return -1;
    for (d = 0; d < n; ++d) {
        if (f[d] < 1) return -1;
        idx[d] = 0;
    }
    for (;;) {
        int64_t i = 0;
        for (d = 0; d < n; ++d) i = i * f[d] + idx[d];
        if (count >= out_len) return -1;
        out[count++] = i;
        d = n - 1;
        while (d >= 0 && ++idx[d] == f[d]) {
            idx[d] = 0;
            --d;
        }
        if (d < 0) break;
    }
    return count;
}

/*
 * Support set of sample-perfect-tile (Table 2): all ordered n-tuples of
 * positive integers whose product is the extent.  Brute force: try every
 * divisor at each position.  Writes tuples consecutively into out (n values
 * each) while room remains and returns the total number of tuples.
 */
static int64_t enum_rec(int64_t rest, int pos, int n, int64_t *cur, int64_t *out, int64_t cap, int64_t count)
{
    if (pos == n - 1) {
        cur[pos] = rest;
        if (out && count < cap) {
            int d;
            for (d = 0; d < n; ++d) out[count * n + d] = cur[d];
        }
        return count + 1;
    }
    for (int64_t f = 1; f <= rest; ++f) {
        if (rest % f) continue;
        cur[pos] = f;
        count = enum_rec(rest / f, pos + 1, n, cur, out, cap, count);
    }
    return count;
}

int64_t ms_oracle_perfect_tiles(int64_t extent, int n, int64_t *out, int64_t cap_tuples)
{
    int64_t cur[16];
    if (n < 1 || n > 16 || extent < 1) return -1;
    return enum_rec(extent, 0, n, cur, out, cap_tuples, 0);
}

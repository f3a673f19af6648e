/*
 * mdnn_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct CPU statement of the forward-propagation
 * (FPROP) minibatch convolution defined in Section 2 of the maxDNN paper
 * (arXiv 1501.06633): Nb multi-channel maps against a bank of No multi-channel
 * Sk x Sk filters, per-channel products summed over channels, a stride, an
 * optional padding offset with the image sitting in an apron of zeros, and a
 * final scale by a scalar alpha.
 *
 * It exists only so that tests, the smoke check and the benchmark's CPU
 * baseline leg have something independent to compare the GPU library with.
 * It shares no source, header, table or helper with the HIP path, and the HIP
 * path never calls it.
 *
 * Data layout (Section 3, first paragraph: the innermost dimension is the
 * batch for maps and the filter count for filters; the outer dimensions are
 * width, height and channel):
 *     in   [Nc][Hi][Wi][Nb]     fp32
 *     filt [Nc][Sk][Sk][No]     fp32   (row k=(c*Sk+ky)*Sk+kx of a K x No matrix)
 *     out  [No][Ho][Wo][Nb]     fp32
 *
 * Arithmetic: every product and every sum is taken in double; the result is
 * scaled by alpha in double and rounded to fp32 exactly once.
 *
 * Readings taken where the paper gives no formula:
 *   - cross-correlation (no filter flip): patch column k multiplies filter row
 *     k (Section 3, the patch-times-filter-matrix statement);
 *   - output size  Wo = floor((Wi + 2*pad - Sk)/stride) + 1  (it reproduces the
 *     input/output/kernel triples of Table 1);
 *   - one symmetric pad on all four sides, zeros outside the image;
 *   - alpha is applied once to the finished sum; out is overwritten.
 *
 * The data gradient (BPROP with respect to the input), which the paper only
 * conjectures to work the same way (abstract, Section 3.5), is written out too:
 * it is the adjoint of the map in -> out above, scaled by alpha.  Its pins are
 * the adjoint identity against the forward function, a scatter-add brute force,
 * torch's transposed convolution in float64 and delta tests.  So is the filter
 * gradient (BPROP with respect to the weights): the adjoint of the map
 * filt -> out.  Its pins: the same identity on the filter side (basis filters
 * included, which fixes every element separately), an accumulation over output
 * pixels of patch x gradient outer products in numpy, torch autograd in float64,
 * deltas, and planted-mistake tests.
 *
 * The plain matrix product in the convolution's operand layout (the SGEMM
 * the paper's conclusion measures itself against, and what a 1 x 1 filter
 * reduces the convolution to) closes the file.  Its pins: a hand-worked
 * case, the library's float64 matmul, identity operands, the forward function
 * at Sk = 1, and planted mistakes.
 *
 * Pins (tests/test_oracle_*.py, CPU only): brute-force im2col x GEMM in numpy
 * float64, the 1x1/stride-1 = plain matrix product identity, delta filters,
 * linearity in alpha / additivity, the all-ones closed form, exact-integer
 * data, translation equivariance, torch.nn.functional.conv2d in float64, the
 * Table 1 output sizes and hand-computed values of the complexity formula.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Output extent of one spatial dimension; returns 0 on success, 1 when the
 * arguments admit no output (filter larger than the padded image, etc.). */
int mdnn_oracle_out_dims(int Wi, int Hi, int Sk, int stride, int pad,
                         int* Wo, int* Ho)
{
    if (Wi < 1 || Hi < 1 || Sk < 1 || stride < 1 || pad < 0) return 1;
    if (Sk > Wi + 2 * pad || Sk > Hi + 2 * pad) return 1;
    *Wo = (Wi + 2 * pad - Sk) / stride + 1;
    *Ho = (Hi + 2 * pad - Sk) / stride + 1;
    return 0;
}

/* Algorithmic complexity, Section 2:  2 Nb Wo Ho (Nc Sk^2 + 1) No  FLOPs. */
uint64_t mdnn_oracle_flops(int Nb, int Wo, int Ho, int Nc, int No, int Sk)
{
    uint64_t per_output = (uint64_t)Nc * (uint64_t)Sk * (uint64_t)Sk + 1u;
    return 2u * (uint64_t)Nb * (uint64_t)Wo * (uint64_t)Ho * per_output * (uint64_t)No;
}

int mdnn_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Whole-tensor convolution.  All pointers are HOST memory.
 *   abs_sum  nullable; when given, receives for every output the sum of the
 *            absolute values of the products that went into it (the scale
 *            the acceptance tolerance is stated against), same layout as out.
 *   nthreads <= 0 means "all the OpenMP runtime offers".
 * Returns 0, or 1 on invalid dimensions / null pointers / allocation failure.
 *
 * The seven loops are o, y, x, c, ky, kx, n with n innermost (n is the
 * contiguous index of both in and out); OpenMP splits the o loop and nothing
 * else is blocked, fused or reordered.
 */
int mdnn_oracle_conv_fprop(const float* in, const float* filt, float* out,
                           double* abs_sum,
                           int Nb, int Wi, int Hi, int Nc, int No,
                           int Sk, int stride, int pad, float alpha,
                           int nthreads)
{
    int Wo, Ho;
    if (!in || !filt || !out) return 1;
    if (Nb < 1 || Nc < 1 || No < 1) return 1;
    if (mdnn_oracle_out_dims(Wi, Hi, Sk, stride, pad, &Wo, &Ho)) return 1;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
#else
    nthreads = 1;
#endif
    int failed = 0;

#pragma omp parallel num_threads(nthreads)
    {
        double* S = (double*)malloc(sizeof(double) * (size_t)Nb);
        double* A = (double*)malloc(sizeof(double) * (size_t)Nb);
        if (!S || !A) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(dynamic, 1)
            for (int o = 0; o < No; ++o) {
                for (int y = 0; y < Ho; ++y) {
                    for (int x = 0; x < Wo; ++x) {
                        for (int n = 0; n < Nb; ++n) { S[n] = 0.0; A[n] = 0.0; }
                        for (int c = 0; c < Nc; ++c) {
                            for (int ky = 0; ky < Sk; ++ky) {
                                int iy = y * stride - pad + ky;
                                if (iy < 0 || iy >= Hi) continue;      /* zero apron */
                                for (int kx = 0; kx < Sk; ++kx) {
                                    int ix = x * stride - pad + kx;
                                    if (ix < 0 || ix >= Wi) continue;  /* zero apron */
                                    const float* row =
                                        in + (((size_t)c * Hi + iy) * Wi + ix) * (size_t)Nb;
                                    double w = (double)
                                        filt[(((size_t)c * Sk + ky) * Sk + kx) * (size_t)No + o];
                                    for (int n = 0; n < Nb; ++n) {
                                        double p = (double)row[n] * w;
                                        S[n] += p;
                                        A[n] += fabs(p);
                                    }
                                }
                            }
                        }
                        size_t base = (((size_t)o * Ho + y) * Wo + x) * (size_t)Nb;
                        for (int n = 0; n < Nb; ++n)
                            out[base + n] = (float)((double)alpha * S[n]);
                        if (abs_sum)
                            for (int n = 0; n < Nb; ++n) abs_sum[base + n] = A[n];
                    }
                }
            }
        }
        free(S);
        free(A);
    }
    return failed;
}

/*
 * The same definition evaluated at a list of output positions only, one by
 * one, so that a parity test at full layer size can check sampled outputs.
 *   idx      npts x 4 ints: (o, y, x, n) per point
 *   out_val  npts floats   (alpha * sum, rounded once)
 *   abs_val  npts doubles  (sum of |products|), nullable
 * Returns 0, or 1 on invalid arguments (including an index out of range).
 */
int mdnn_oracle_conv_fprop_points(const float* in, const float* filt,
                                  const int32_t* idx, int64_t npts,
                                  float* out_val, double* abs_val,
                                  int Nb, int Wi, int Hi, int Nc, int No,
                                  int Sk, int stride, int pad, float alpha)
{
    int Wo, Ho;
    if (!in || !filt || !idx || !out_val || npts < 0) return 1;
    if (Nb < 1 || Nc < 1 || No < 1) return 1;
    if (mdnn_oracle_out_dims(Wi, Hi, Sk, stride, pad, &Wo, &Ho)) return 1;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t i = 0; i < npts; ++i) {
        int o = idx[4 * i + 0], y = idx[4 * i + 1], x = idx[4 * i + 2], n = idx[4 * i + 3];
        if (o < 0 || o >= No || y < 0 || y >= Ho || x < 0 || x >= Wo || n < 0 || n >= Nb) {
            bad |= 1;
            continue;
        }
        double S = 0.0, A = 0.0;
        for (int c = 0; c < Nc; ++c)
            for (int ky = 0; ky < Sk; ++ky)
                for (int kx = 0; kx < Sk; ++kx) {
                    int iy = y * stride - pad + ky;
                    int ix = x * stride - pad + kx;
                    if (iy < 0 || iy >= Hi || ix < 0 || ix >= Wi) continue;
                    double p = (double)in[(((size_t)c * Hi + iy) * Wi + ix) * (size_t)Nb + n] *
                               (double)filt[(((size_t)c * Sk + ky) * Sk + kx) * (size_t)No + o];
                    S += p;
                    A += fabs(p);
                }
        out_val[i] = (float)((double)alpha * S);
        if (abs_val) abs_val[i] = A;
    }
    return bad;
}

/*
 * Data gradient of the convolution above (BPROP w.r.t. the input):
 *   din[c][iy][ix][n] = alpha * sum_{o,ky,kx} dout[o][y][x][n] * filt[c][ky][kx][o]
 * over those (ky,kx) for which  y = (iy + pad - ky)/stride  and  x = (ix + pad - kx)/stride
 * are integers inside the output map -- i.e. over every forward term in which
 * in[c][iy][ix][n] took part.  din has the layout and size of `in`; input
 * pixels no filter window reaches get 0.  abs_sum as in the forward function.
 * Loops: c, iy, ix, o, ky, kx, n (n innermost), OpenMP over c only.
 */
int mdnn_oracle_conv_bprop_data(const float* dout, const float* filt, float* din,
                                double* abs_sum,
                                int Nb, int Wi, int Hi, int Nc, int No,
                                int Sk, int stride, int pad, float alpha,
                                int nthreads)
{
    int Wo, Ho;
    if (!dout || !filt || !din) return 1;
    if (Nb < 1 || Nc < 1 || No < 1) return 1;
    if (mdnn_oracle_out_dims(Wi, Hi, Sk, stride, pad, &Wo, &Ho)) return 1;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
#else
    nthreads = 1;
#endif
    int failed = 0;

#pragma omp parallel num_threads(nthreads)
    {
        double* S = (double*)malloc(sizeof(double) * (size_t)Nb);
        double* A = (double*)malloc(sizeof(double) * (size_t)Nb);
        if (!S || !A) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(dynamic, 1)
            for (int c = 0; c < Nc; ++c) {
                for (int iy = 0; iy < Hi; ++iy) {
                    for (int ix = 0; ix < Wi; ++ix) {
                        for (int n = 0; n < Nb; ++n) { S[n] = 0.0; A[n] = 0.0; }
                        for (int o = 0; o < No; ++o) {
                            for (int ky = 0; ky < Sk; ++ky) {
                                int ty = iy + pad - ky;                 /* = y * stride */
                                if (ty < 0 || ty % stride != 0 || ty / stride >= Ho) continue;
                                for (int kx = 0; kx < Sk; ++kx) {
                                    int tx = ix + pad - kx;
                                    if (tx < 0 || tx % stride != 0 || tx / stride >= Wo) continue;
                                    const float* row = dout +
                                        (((size_t)o * Ho + ty / stride) * Wo + tx / stride) * (size_t)Nb;
                                    double w = (double)
                                        filt[(((size_t)c * Sk + ky) * Sk + kx) * (size_t)No + o];
                                    for (int n = 0; n < Nb; ++n) {
                                        double p = (double)row[n] * w;
                                        S[n] += p;
                                        A[n] += fabs(p);
                                    }
                                }
                            }
                        }
                        size_t base = (((size_t)c * Hi + iy) * Wi + ix) * (size_t)Nb;
                        for (int n = 0; n < Nb; ++n)
                            din[base + n] = (float)((double)alpha * S[n]);
                        if (abs_sum)
                            for (int n = 0; n < Nb; ++n) abs_sum[base + n] = A[n];
                    }
                }
            }
        }
        free(S);
        free(A);
    }
    return failed;
}

/*
 * Filter gradient of the convolution above (BPROP w.r.t. the weights):
 *   dfilt[c][ky][kx][o] = alpha * sum_{y,x,n} in[c][y*stride-pad+ky][x*stride-pad+kx][n] * dout[o][y][x][n]
 * with apron reads contributing 0 -- every forward term in which filt[c][ky][kx][o]
 * took part, weighted by the gradient of the output it went into.  dfilt has the
 * layout and size of `filt`.  abs_sum as in the forward function.
 * Loops: c, ky, kx, o, y, x, n (n innermost), OpenMP over c only.
 */
int mdnn_oracle_conv_bprop_filter(const float* in, const float* dout, float* dfilt,
                                  double* abs_sum,
                                  int Nb, int Wi, int Hi, int Nc, int No,
                                  int Sk, int stride, int pad, float alpha,
                                  int nthreads)
{
    int Wo, Ho;
    if (!in || !dout || !dfilt) return 1;
    if (Nb < 1 || Nc < 1 || No < 1) return 1;
    if (mdnn_oracle_out_dims(Wi, Hi, Sk, stride, pad, &Wo, &Ho)) return 1;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
#else
    nthreads = 1;
#endif

#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int c = 0; c < Nc; ++c) {
        for (int ky = 0; ky < Sk; ++ky) {
            for (int kx = 0; kx < Sk; ++kx) {
                for (int o = 0; o < No; ++o) {
                    double S = 0.0, A = 0.0;
                    for (int y = 0; y < Ho; ++y) {
                        int iy = y * stride - pad + ky;
                        if (iy < 0 || iy >= Hi) continue;       /* zero apron */
                        for (int x = 0; x < Wo; ++x) {
                            int ix = x * stride - pad + kx;
                            if (ix < 0 || ix >= Wi) continue;
                            const float* a = in + (((size_t)c * Hi + iy) * Wi + ix) * (size_t)Nb;
                            const float* g = dout + (((size_t)o * Ho + y) * Wo + x) * (size_t)Nb;
                            for (int n = 0; n < Nb; ++n) {
                                double p = (double)a[n] * (double)g[n];
                                S += p;
                                A += fabs(p);
                            }
                        }
                    }
                    size_t e = (((size_t)c * Sk + ky) * Sk + kx) * (size_t)No + o;
                    dfilt[e] = (float)((double)alpha * S);
                    if (abs_sum) abs_sum[e] = A;
                }
            }
        }
    }
    return 0;
}

/*
 * The same definition at selected filter elements only: idx holds npts rows
 * (c, ky, kx, o).  For layers whose whole gradient is too slow to evaluate here.
 * Returns 0, or 1 when an argument or an index is out of range.
 */
int mdnn_oracle_conv_bprop_filter_points(const float* in, const float* dout,
                                         const int* idx, long long npts,
                                         float* val, double* abs_val,
                                         int Nb, int Wi, int Hi, int Nc, int No,
                                         int Sk, int stride, int pad, float alpha)
{
    int Wo, Ho;
    if (!in || !dout || !idx || !val || npts < 0) return 1;
    if (Nb < 1 || Nc < 1 || No < 1) return 1;
    if (mdnn_oracle_out_dims(Wi, Hi, Sk, stride, pad, &Wo, &Ho)) return 1;
    int bad = 0;

#pragma omp parallel for schedule(dynamic, 4) reduction(|:bad)
    for (long long i = 0; i < npts; ++i) {
        int c = idx[4 * i + 0], ky = idx[4 * i + 1], kx = idx[4 * i + 2], o = idx[4 * i + 3];
        if (c < 0 || c >= Nc || ky < 0 || ky >= Sk || kx < 0 || kx >= Sk || o < 0 || o >= No) {
            bad |= 1;
            continue;
        }
        double S = 0.0, A = 0.0;
        for (int y = 0; y < Ho; ++y) {
            int iy = y * stride - pad + ky;
            if (iy < 0 || iy >= Hi) continue;
            for (int x = 0; x < Wo; ++x) {
                int ix = x * stride - pad + kx;
                if (ix < 0 || ix >= Wi) continue;
                const float* a = in + (((size_t)c * Hi + iy) * Wi + ix) * (size_t)Nb;
                const float* g = dout + (((size_t)o * Ho + y) * Wo + x) * (size_t)Nb;
                for (int n = 0; n < Nb; ++n) {
                    double p = (double)a[n] * (double)g[n];
                    S += p;
                    A += fabs(p);
                }
            }
        }
        val[i] = (float)((double)alpha * S);
        if (abs_val) abs_val[i] = A;
    }
    return bad;
}

/*
 * The data gradient at selected input elements only: idx holds npts rows
 * (c, iy, ix, n).  Same definition as mdnn_oracle_conv_bprop_data.
 * Returns 0, or 1 when an argument or an index is out of range.
 */
int mdnn_oracle_conv_bprop_data_points(const float* dout, const float* filt,
                                       const int* idx, long long npts,
                                       float* val, double* abs_val,
                                       int Nb, int Wi, int Hi, int Nc, int No,
                                       int Sk, int stride, int pad, float alpha)
{
    int Wo, Ho;
    if (!dout || !filt || !idx || !val || npts < 0) return 1;
    if (Nb < 1 || Nc < 1 || No < 1) return 1;
    if (mdnn_oracle_out_dims(Wi, Hi, Sk, stride, pad, &Wo, &Ho)) return 1;
    int bad = 0;

#pragma omp parallel for schedule(dynamic, 16) reduction(|:bad)
    for (long long i = 0; i < npts; ++i) {
        int c = idx[4 * i + 0], iy = idx[4 * i + 1], ix = idx[4 * i + 2], n = idx[4 * i + 3];
        if (c < 0 || c >= Nc || iy < 0 || iy >= Hi || ix < 0 || ix >= Wi || n < 0 || n >= Nb) {
            bad |= 1;
            continue;
        }
        double S = 0.0, A = 0.0;
        for (int o = 0; o < No; ++o)
            for (int ky = 0; ky < Sk; ++ky) {
                int ty = iy + pad - ky;                     /* = y * stride */
                if (ty < 0 || ty % stride != 0 || ty / stride >= Ho) continue;
                for (int kx = 0; kx < Sk; ++kx) {
                    int tx = ix + pad - kx;
                    if (tx < 0 || tx % stride != 0 || tx / stride >= Wo) continue;
                    double p = (double)dout[(((size_t)o * Ho + ty / stride) * Wo + tx / stride) * (size_t)Nb + n] *
                               (double)filt[(((size_t)c * Sk + ky) * Sk + kx) * (size_t)No + o];
                    S += p;
                    A += fabs(p);
                }
            }
        val[i] = (float)((double)alpha * S);
        if (abs_val) abs_val[i] = A;
    }
    return bad;
}

/*
 * Plain single-precision matrix product in the operand layout the convolution
 * uses: the paper's conclusion measures the kernel against SGEMM, and with a
 * 1 x 1 filter the per-coordinate product of Section 3 is nothing else.
 *
 *   a  [K][N]  fp32   (the filter matrix: row k, column o)
 *   b  [K][M]  fp32   (the input: row k, column m)
 *   c  [N][M]  fp32   c[o][m] = alpha * sum_k a[k][o] * b[k][m]
 *
 * Products and sums in double, one rounding at the end, abs_sum (nullable,
 * [N][M] doubles) the sum of |products| as in the convolution.  Three loops
 * o, m, k; OpenMP splits the o loop.  Returns 0, or 1 on invalid arguments.
 */
int mdnn_oracle_sgemm_tn(const float* a, const float* b, float* c, double* abs_sum,
                         int N, int M, int K, float alpha, int nthreads)
{
    if (!a || !b || !c) return 1;
    if (N < 1 || M < 1 || K < 1) return 1;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
#else
    nthreads = 1;
#endif
#pragma omp parallel for num_threads(nthreads) schedule(dynamic, 1)
    for (int o = 0; o < N; ++o) {
        for (int m = 0; m < M; ++m) {
            double s = 0.0, ab = 0.0;
            for (int k = 0; k < K; ++k) {
                double p = (double)a[(size_t)k * N + o] * (double)b[(size_t)k * M + m];
                s += p;
                ab += fabs(p);
            }
            c[(size_t)o * M + m] = (float)((double)alpha * s);
            if (abs_sum) abs_sum[(size_t)o * M + m] = ab;
        }
    }
    return 0;
}

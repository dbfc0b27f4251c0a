/*
 * CPU oracle for the per-block distillation step -- layer primitives, fp64, direct loops.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may call, link or load this file; it shares
 * no code with the HIP library.  It exists so that the GPU results can be compared with an obviously
 * correct, slow statement of what the method computes.
 *
 * What it follows.  The paper (section 3.1, Eq. 3) trains a replacement block g_k on the local loss
 * between the teacher block's activations f_k(x) and g_k applied to the same block input; section 3.2
 * fixes the replacement block as a stack of "depthwise separable + batch normalisation + ReLU" layers.
 * The paper gives no formulas for the layers themselves, so each function below is the textbook
 * definition written out as nested loops (cross-correlation, zero padding 1, NCHW, weights OIHW).
 * Every tensor is a contiguous double array.
 *
 * Readings taken where the paper is silent (the complete list lives with the block driver, block.py):
 * convolutions are cross-correlations without bias, 3x3 kernels pad one zero on all four sides also at
 * stride 2 (input index = stride*out + k - 1), output size floor((H-1)/stride)+1, the 1x1 projection
 * reads input index stride*out, BatchNorm uses the batch mean and the biased batch variance.
 *
 * Parallelism: OpenMP over (image, channel) only -- no blocking, no reordering of the definition.
 */
#include <math.h>
#include <stddef.h>
#include <string.h>

#define IDX4(n, c, h, w, C, H, W) ((((size_t)(n) * (C) + (c)) * (H) + (h)) * (W) + (w))

static int out_dim(int in, int s) { return (in - 1) / s + 1; }

/* z[n,o,i,j] = sum_{c,ky,kx} Wt[o,c,ky,kx] * a[n,c,s*i+ky-1,s*j+kx-1]   (out of range reads are 0) */
void ref_conv3x3_fwd(const double *a, const double *Wt, double *z, int N, int Ci, int Co, int H, int W, int s)
{
    const int Ho = out_dim(H, s), Wo = out_dim(W, s);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int o = 0; o < Co; ++o) {
            double *zp = z + IDX4(n, o, 0, 0, Co, Ho, Wo);
            memset(zp, 0, sizeof(double) * (size_t)Ho * Wo);
            for (int c = 0; c < Ci; ++c)
                for (int ky = 0; ky < 3; ++ky)
                    for (int kx = 0; kx < 3; ++kx) {
                        const double wv = Wt[((size_t)(o * Ci + c) * 3 + ky) * 3 + kx];
                        for (int i = 0; i < Ho; ++i) {
                            const int y = s * i + ky - 1;
                            if (y < 0 || y >= H) continue;
                            const double *ap = a + IDX4(n, c, y, 0, Ci, H, W);
                            for (int j = 0; j < Wo; ++j) {
                                const int x = s * j + kx - 1;
                                if (x < 0 || x >= W) continue;
                                zp[i * Wo + j] += wv * ap[x];
                            }
                        }
                    }
        }
}

/* dW[o,c,ky,kx] = sum_{n,i,j} dz[n,o,i,j] * a[n,c,s*i+ky-1,s*j+kx-1] */
void ref_conv3x3_wgrad(const double *dz, const double *a, double *dW, int N, int Ci, int Co, int H, int W, int s)
{
    const int Ho = out_dim(H, s), Wo = out_dim(W, s);
#pragma omp parallel for collapse(2) schedule(static)
    for (int o = 0; o < Co; ++o)
        for (int c = 0; c < Ci; ++c)
            for (int ky = 0; ky < 3; ++ky)
                for (int kx = 0; kx < 3; ++kx) {
                    double acc = 0.0;
                    for (int n = 0; n < N; ++n)
                        for (int i = 0; i < Ho; ++i) {
                            const int y = s * i + ky - 1;
                            if (y < 0 || y >= H) continue;
                            for (int j = 0; j < Wo; ++j) {
                                const int x = s * j + kx - 1;
                                if (x < 0 || x >= W) continue;
                                acc += dz[IDX4(n, o, i, j, Co, Ho, Wo)] * a[IDX4(n, c, y, x, Ci, H, W)];
                            }
                        }
                    dW[((size_t)(o * Ci + c) * 3 + ky) * 3 + kx] = acc;
                }
}

/* da[n,c,y,x] = sum over (o,ky,kx,i,j) with s*i+ky-1==y, s*j+kx-1==x of Wt[o,c,ky,kx] * dz[n,o,i,j].
 * Written as a scatter of every forward term, which is the transpose of the forward map by construction. */
void ref_conv3x3_dgrad(const double *dz, const double *Wt, double *da, int N, int Ci, int Co, int H, int W, int s)
{
    const int Ho = out_dim(H, s), Wo = out_dim(W, s);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < Ci; ++c) {
            double *dp = da + IDX4(n, c, 0, 0, Ci, H, W);
            memset(dp, 0, sizeof(double) * (size_t)H * W);
            for (int o = 0; o < Co; ++o)
                for (int ky = 0; ky < 3; ++ky)
                    for (int kx = 0; kx < 3; ++kx) {
                        const double wv = Wt[((size_t)(o * Ci + c) * 3 + ky) * 3 + kx];
                        for (int i = 0; i < Ho; ++i) {
                            const int y = s * i + ky - 1;
                            if (y < 0 || y >= H) continue;
                            for (int j = 0; j < Wo; ++j) {
                                const int x = s * j + kx - 1;
                                if (x < 0 || x >= W) continue;
                                dp[y * W + x] += wv * dz[IDX4(n, o, i, j, Co, Ho, Wo)];
                            }
                        }
                    }
        }
}

/* u[n,c,i,j] = sum_{ky,kx} D[c,ky,kx] * a[n,c,s*i+ky-1,s*j+kx-1] */
void ref_dw3x3_fwd(const double *a, const double *D, double *u, int N, int C, int H, int W, int s)
{
    const int Ho = out_dim(H, s), Wo = out_dim(W, s);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int i = 0; i < Ho; ++i)
                for (int j = 0; j < Wo; ++j) {
                    double acc = 0.0;
                    for (int ky = 0; ky < 3; ++ky) {
                        const int y = s * i + ky - 1;
                        if (y < 0 || y >= H) continue;
                        for (int kx = 0; kx < 3; ++kx) {
                            const int x = s * j + kx - 1;
                            if (x < 0 || x >= W) continue;
                            acc += D[(c * 3 + ky) * 3 + kx] * a[IDX4(n, c, y, x, C, H, W)];
                        }
                    }
                    u[IDX4(n, c, i, j, C, Ho, Wo)] = acc;
                }
}

/* dD[c,ky,kx] = sum_{n,i,j} du[n,c,i,j] * a[n,c,s*i+ky-1,s*j+kx-1] */
void ref_dw3x3_wgrad(const double *du, const double *a, double *dD, int N, int C, int H, int W, int s)
{
    const int Ho = out_dim(H, s), Wo = out_dim(W, s);
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c)
        for (int ky = 0; ky < 3; ++ky)
            for (int kx = 0; kx < 3; ++kx) {
                double acc = 0.0;
                for (int n = 0; n < N; ++n)
                    for (int i = 0; i < Ho; ++i) {
                        const int y = s * i + ky - 1;
                        if (y < 0 || y >= H) continue;
                        for (int j = 0; j < Wo; ++j) {
                            const int x = s * j + kx - 1;
                            if (x < 0 || x >= W) continue;
                            acc += du[IDX4(n, c, i, j, C, Ho, Wo)] * a[IDX4(n, c, y, x, C, H, W)];
                        }
                    }
                dD[(c * 3 + ky) * 3 + kx] = acc;
            }
}

/* da = transpose of ref_dw3x3_fwd applied to du (scatter of every forward term) */
void ref_dw3x3_dgrad(const double *du, const double *D, double *da, int N, int C, int H, int W, int s)
{
    const int Ho = out_dim(H, s), Wo = out_dim(W, s);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            double *dp = da + IDX4(n, c, 0, 0, C, H, W);
            memset(dp, 0, sizeof(double) * (size_t)H * W);
            for (int i = 0; i < Ho; ++i)
                for (int j = 0; j < Wo; ++j) {
                    const double g = du[IDX4(n, c, i, j, C, Ho, Wo)];
                    for (int ky = 0; ky < 3; ++ky) {
                        const int y = s * i + ky - 1;
                        if (y < 0 || y >= H) continue;
                        for (int kx = 0; kx < 3; ++kx) {
                            const int x = s * j + kx - 1;
                            if (x < 0 || x >= W) continue;
                            dp[y * W + x] += D[(c * 3 + ky) * 3 + kx] * g;
                        }
                    }
                }
        }
}

/* 1x1 convolution with stride (pad 0): z[n,o,i,j] = sum_c P[o,c] * a[n,c,s*i,s*j].  s=1 is the pointwise conv. */
void ref_conv1x1_fwd(const double *a, const double *P, double *z, int N, int Ci, int Co, int H, int W, int s)
{
    const int Ho = out_dim(H, s), Wo = out_dim(W, s);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int o = 0; o < Co; ++o) {
            double *zp = z + IDX4(n, o, 0, 0, Co, Ho, Wo);
            memset(zp, 0, sizeof(double) * (size_t)Ho * Wo);
            for (int c = 0; c < Ci; ++c) {
                const double wv = P[(size_t)o * Ci + c];
                for (int i = 0; i < Ho; ++i)
                    for (int j = 0; j < Wo; ++j)
                        zp[i * Wo + j] += wv * a[IDX4(n, c, s * i, s * j, Ci, H, W)];
            }
        }
}

/* dP[o,c] = sum_{n,i,j} dz[n,o,i,j] * a[n,c,s*i,s*j] */
void ref_conv1x1_wgrad(const double *dz, const double *a, double *dP, int N, int Ci, int Co, int H, int W, int s)
{
    const int Ho = out_dim(H, s), Wo = out_dim(W, s);
#pragma omp parallel for collapse(2) schedule(static)
    for (int o = 0; o < Co; ++o)
        for (int c = 0; c < Ci; ++c) {
            double acc = 0.0;
            for (int n = 0; n < N; ++n)
                for (int i = 0; i < Ho; ++i)
                    for (int j = 0; j < Wo; ++j)
                        acc += dz[IDX4(n, o, i, j, Co, Ho, Wo)] * a[IDX4(n, c, s * i, s * j, Ci, H, W)];
            dP[(size_t)o * Ci + c] = acc;
        }
}

/* da[n,c,s*i,s*j] = sum_o P[o,c] * dz[n,o,i,j]; positions not hit by the stride get 0 */
void ref_conv1x1_dgrad(const double *dz, const double *P, double *da, int N, int Ci, int Co, int H, int W, int s)
{
    const int Ho = out_dim(H, s), Wo = out_dim(W, s);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < Ci; ++c) {
            double *dp = da + IDX4(n, c, 0, 0, Ci, H, W);
            memset(dp, 0, sizeof(double) * (size_t)H * W);
            for (int o = 0; o < Co; ++o) {
                const double wv = P[(size_t)o * Ci + c];
                for (int i = 0; i < Ho; ++i)
                    for (int j = 0; j < Wo; ++j)
                        dp[(s * i) * W + s * j] += wv * dz[IDX4(n, o, i, j, Co, Ho, Wo)];
            }
        }
}

/* BatchNorm, training mode, over (N, H, W) per channel; HW = H*W.
 *   mean_c = sum z / m,  var_c = sum (z-mean)^2 / m (biased),  rstd_c = 1/sqrt(var+eps),
 *   xhat = (z-mean)*rstd,  b = gamma*xhat + beta.      m = N*HW                                     */
void ref_bn_fwd(const double *z, const double *gamma, const double *beta, double eps,
                double *xhat, double *b, double *mean, double *rstd, int N, int C, int HW)
{
    const double m = (double)N * HW;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        double s1 = 0.0;
        for (int n = 0; n < N; ++n)
            for (int p = 0; p < HW; ++p) s1 += z[((size_t)n * C + c) * HW + p];
        const double mu = s1 / m;
        double s2 = 0.0;
        for (int n = 0; n < N; ++n)
            for (int p = 0; p < HW; ++p) {
                const double d = z[((size_t)n * C + c) * HW + p] - mu;
                s2 += d * d;
            }
        const double r = 1.0 / sqrt(s2 / m + eps);
        mean[c] = mu;
        rstd[c] = r;
        for (int n = 0; n < N; ++n)
            for (int p = 0; p < HW; ++p) {
                const size_t k = ((size_t)n * C + c) * HW + p;
                const double xh = (z[k] - mu) * r;
                xhat[k] = xh;
                b[k] = gamma[c] * xh + beta[c];
            }
    }
}

/* Backward of ref_bn_fwd through the batch mean and variance:
 *   dbeta_c = sum g,  dgamma_c = sum g*xhat,
 *   dz = gamma*rstd/m * (m*g - dbeta - xhat*dgamma)                                                  */
void ref_bn_bwd(const double *g, const double *xhat, const double *gamma, const double *rstd,
                double *dz, double *dgamma, double *dbeta, int N, int C, int HW)
{
    const double m = (double)N * HW;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        double sb = 0.0, sg = 0.0;
        for (int n = 0; n < N; ++n)
            for (int p = 0; p < HW; ++p) {
                const size_t k = ((size_t)n * C + c) * HW + p;
                sb += g[k];
                sg += g[k] * xhat[k];
            }
        dbeta[c] = sb;
        dgamma[c] = sg;
        const double f = gamma[c] * rstd[c] / m;
        for (int n = 0; n < N; ++n)
            for (int p = 0; p < HW; ++p) {
                const size_t k = ((size_t)n * C + c) * HW + p;
                dz[k] = f * (m * g[k] - sb - xhat[k] * sg);
            }
    }
}

/* Number of OpenMP threads the loops above will use (for reporting the CPU baseline). */
#ifdef _OPENMP
#include <omp.h>
int ref_num_threads(void) { return omp_get_max_threads(); }
#else
int ref_num_threads(void) { return 1; }
#endif

/* Runs every loop of the CPU oracle's C file on small ragged shapes, every buffer a heap block of exactly the size the
 * call needs, so that AddressSanitizer and UndefinedBehaviorSanitizer see any index that leaves a tensor.  Built and
 * run by tests/test_sanitizers.py with -fsanitize=address,undefined; prints "ok" on success. */
#include <stdio.h>
#include <stdlib.h>

void ref_conv3x3_fwd(const double *a, const double *Wt, double *z, int N, int Ci, int Co, int H, int W, int s);
void ref_conv3x3_wgrad(const double *dz, const double *a, double *dW, int N, int Ci, int Co, int H, int W, int s);
void ref_conv3x3_dgrad(const double *dz, const double *Wt, double *da, int N, int Ci, int Co, int H, int W, int s);
void ref_dw3x3_fwd(const double *a, const double *D, double *u, int N, int C, int H, int W, int s);
void ref_dw3x3_wgrad(const double *du, const double *a, double *dD, int N, int C, int H, int W, int s);
void ref_dw3x3_dgrad(const double *du, const double *D, double *da, int N, int C, int H, int W, int s);
void ref_conv1x1_fwd(const double *a, const double *P, double *z, int N, int Ci, int Co, int H, int W, int s);
void ref_conv1x1_wgrad(const double *dz, const double *a, double *dP, int N, int Ci, int Co, int H, int W, int s);
void ref_conv1x1_dgrad(const double *dz, const double *P, double *da, int N, int Ci, int Co, int H, int W, int s);
void ref_bn_fwd(const double *z, const double *gamma, const double *beta, double eps, double *xhat, double *b, double *mean,
                double *rstd, int N, int C, int HW);
void ref_bn_bwd(const double *g, const double *xhat, const double *gamma, const double *rstd, double *dz, double *dgamma,
                double *dbeta, int N, int C, int HW);
int ref_num_threads(void);

static double *buf(size_t n, unsigned seed) {
  double *p = (double *)malloc((n ? n : 1) * sizeof(double));
  if (!p) exit(3);
  for (size_t i = 0; i < n; ++i) {
    seed = seed * 1664525u + 1013904223u;
    p[i] = (double)(seed >> 8) / 8388608.0 - 1.0;
  }
  return p;
}

static int out_dim(int in, int s) { return (in - 1) / s + 1; }

static void one(int N, int Ci, int Co, int H, int W, int s) {
  const int Ho = out_dim(H, s), Wo = out_dim(W, s);
  const size_t na = (size_t)N * Ci * H * W, nz = (size_t)N * Co * Ho * Wo, nu = (size_t)N * Ci * Ho * Wo;
  double *a = buf(na, 1), *Wt = buf((size_t)Co * Ci * 9, 2), *z = buf(nz, 3), *dW = buf((size_t)Co * Ci * 9, 4), *da = buf(na, 5);
  ref_conv3x3_fwd(a, Wt, z, N, Ci, Co, H, W, s);
  ref_conv3x3_wgrad(z, a, dW, N, Ci, Co, H, W, s);
  ref_conv3x3_dgrad(z, Wt, da, N, Ci, Co, H, W, s);
  double *D = buf((size_t)Ci * 9, 6), *u = buf(nu, 7), *dD = buf((size_t)Ci * 9, 8);
  ref_dw3x3_fwd(a, D, u, N, Ci, H, W, s);
  ref_dw3x3_wgrad(u, a, dD, N, Ci, H, W, s);
  ref_dw3x3_dgrad(u, D, da, N, Ci, H, W, s);
  double *P = buf((size_t)Co * Ci, 9), *dP = buf((size_t)Co * Ci, 10);
  ref_conv1x1_fwd(a, P, z, N, Ci, Co, H, W, s);          /* strided 1x1: reads a[s*i][s*j], writes Ho x Wo */
  ref_conv1x1_wgrad(z, a, dP, N, Ci, Co, H, W, s);
  ref_conv1x1_dgrad(z, P, da, N, Ci, Co, H, W, s);
  double *g = buf(Co, 11), *be = buf(Co, 12), *xh = buf(nz, 13), *b = buf(nz, 14), *mu = buf(Co, 15), *rs = buf(Co, 16);
  double *dz = buf(nz, 17), *dg = buf(Co, 18), *db = buf(Co, 19);
  ref_bn_fwd(z, g, be, 1e-5, xh, b, mu, rs, N, Co, Ho * Wo);
  ref_bn_bwd(b, xh, g, rs, dz, dg, db, N, Co, Ho * Wo);
  free(a); free(Wt); free(z); free(dW); free(da); free(D); free(u); free(dD); free(P); free(dP);
  free(g); free(be); free(xh); free(b); free(mu); free(rs); free(dz); free(dg); free(db);
}

int main(void) {
  const int shapes[][6] = {{1, 1, 1, 1, 1, 1}, {2, 3, 5, 7, 9, 1}, {3, 4, 2, 9, 11, 2}, {2, 2, 6, 1, 7, 2}, {1, 5, 3, 2, 2, 1},
                           {2, 3, 3, 8, 1, 2}, {4, 1, 2, 3, 3, 1}};
  for (unsigned i = 0; i < sizeof shapes / sizeof shapes[0]; ++i)
    one(shapes[i][0], shapes[i][1], shapes[i][2], shapes[i][3], shapes[i][4], shapes[i][5]);
  if (ref_num_threads() < 1) return 2;
  printf("ok\n");
  return 0;
}

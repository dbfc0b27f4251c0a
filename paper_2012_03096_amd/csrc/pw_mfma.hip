// 1x1 convolution (the student's pointwise conv, its data gradient, the projection shortcut) on the fp32
// matrix cores, written for what bounds it: HBM.  z[n,o,p] = sum_c A[o,c] * in[n,c,p].
//
// The weight matrix is small, the pixel dimension huge, and in NCHW 32 consecutive pixels of one channel
// are 128 contiguous bytes -- exactly the B operand of one half of a v_mfma_f32_32x32x2_f32 (lane l holds
// B[k = l/32][pixel l%32]).  So the activations never touch LDS: every wave loads its B operands straight
// from global memory into registers, coalesced, through a ring of PW_D steps in flight, and only the
// weights (all K rows of the workgroup's channel tile, at most 128 x 128 floats per stage) are staged in
// LDS once per 128 input channels.  After that staging no barrier is needed: the four waves of a
// workgroup own disjoint pixel columns and run independently.
#include "conv_mfma_kernel.h"

namespace pbkd {

constexpr int PW_D = 8;        // B-operand loads in flight per wave, in MFMA steps
constexpr int PW_KS = 128;     // input channels per LDS stage of the weights

template <int MB, int NB>
__global__ __launch_bounds__(256, 2) void pw_mfma_kernel(PwArgs p) {
  constexpr int BM = MB * 32;
  extern __shared__ float smem[];   // [PW_KS][BM]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l31 = lane & 31, lh = lane >> 5;
  const int m0 = blockIdx.y * BM;
  const int HWo = p.Ho * p.Wo;
  const long long P = (long long)p.N * HWo;
  const int nsteps = p.nchunks * (KC1 / 2);    // MFMA steps over the zero-padded K

  ptrdiff_t inoff[NB];
  size_t outoff[NB];
  bool pvalid[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    long long g = ((long long)blockIdx.x * 4 + wave) * (NB * 32) + nb * 32 + l31;
    pvalid[nb] = g < P;
    if (!pvalid[nb]) g = P - 1;               // read a real pixel, never store it
    const int n = (int)(g / HWo);
    const int r = (int)(g - (long long)n * HWo);
    const int i = r / p.Wo, j = r - i * p.Wo;
    inoff[nb] = (ptrdiff_t)n * p.Cin * p.HWin + (ptrdiff_t)(p.stride * i) * p.Win + p.stride * j;
    outoff[nb] = (size_t)n * p.Cout * HWo + r;
  }
  auto bload = [&](int t, int nb) -> float {
    int k = 2 * t + lh;
    if (k > p.Cin - 1) k = p.Cin - 1;          // padded K: the weight rows are zero there
    return p.in[inoff[nb] + (ptrdiff_t)k * p.HWin];
  };

  floatx16 acc[MB][NB];
#pragma unroll
  for (int a = 0; a < MB; ++a)
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  float ring[PW_D][NB];
#pragma unroll
  for (int d = 0; d < PW_D; ++d)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) ring[d][nb] = bload(d < nsteps ? d : nsteps - 1, nb);

  const float *wsrc = p.wpk + (size_t)blockIdx.y * p.nchunks * (KC1 * BM);
  const int aoff = l31 + lh * BM;
  for (int s0 = 0; s0 < nsteps; s0 += PW_KS / 2) {
    const int steps = (nsteps - s0 < PW_KS / 2) ? nsteps - s0 : PW_KS / 2;   // multiple of 16
    __syncthreads();
    {
      typedef float f4 __attribute__((ext_vector_type(4)));
      const f4 *src = reinterpret_cast<const f4 *>(wsrc + (size_t)s0 * 2 * BM);
      f4 *dst = reinterpret_cast<f4 *>(smem);
      const int n4 = steps * 2 * BM / 4;
      for (int e = tid; e < n4; e += 256) dst[e] = src[e];
    }
    __syncthreads();
    float av[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) av[mb] = smem[aoff + 32 * mb];
    for (int tt = 0; tt < steps; tt += PW_D) {
#pragma unroll
      for (int d = 0; d < PW_D; ++d) {
        const int t = s0 + tt + d;
        float bv[NB], nav[MB];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) bv[nb] = ring[d][nb];
        {
          int tn = t + PW_D;
          if (tn > nsteps - 1) tn = nsteps - 1;
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) ring[d][nb] = bload(tn, nb);
        }
        {
          int ln = tt + d + 1;                   // next step's weights (wraps harmlessly on the last step)
          if (ln > steps - 1) ln = steps - 1;
#pragma unroll
          for (int mb = 0; mb < MB; ++mb) nav[mb] = smem[ln * 2 * BM + aoff + 32 * mb];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
          for (int nb = 0; nb < NB; ++nb)
            acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[mb], bv[nb], acc[mb][nb], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) av[mb] = nav[mb];
      }
    }
  }

  // ---- store: accumulator register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int o = m0 + mb * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
      if (o < p.Cout) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
          if (pvalid[nb]) p.out[outoff[nb] + (size_t)o * HWo] = acc[mb][nb][r];
      }
    }

  // ---- per-channel (sum, sum of squares) over this workgroup's pixels, for BatchNorm
  if (p.stat_partial) {
    __syncthreads();
    float *red = smem;   // [4 waves][BM][2]
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const float v = pvalid[nb] ? acc[mb][nb][r] : 0.f;
          s1 += v;
          s2 += v * v;
        }
        s1 = half32_sum(s1);
        s2 = half32_sum(s2);
        if (l31 == 0) {
          const int row = mb * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
          red[(wave * BM + row) * 2 + 0] = s1;
          red[(wave * BM + row) * 2 + 1] = s2;
        }
      }
    __syncthreads();
    for (int e = tid; e < BM; e += 256) {
      const int o = m0 + e;
      if (o < p.Cout) {
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          s1 += red[(w * BM + e) * 2 + 0];
          s2 += red[(w * BM + e) * 2 + 1];
        }
        float *dst = p.stat_partial + ((size_t)blockIdx.x * p.Cout + o) * 2;
        dst[0] = s1;
        dst[1] = s2;
      }
    }
  }
}

PwGeom pw_geom(int N, int Cin, int Cout, int Ho, int Wo) {
  // (MB, NB) = (channel blocks of 32 per workgroup, pixel blocks of 32 per wave).  Prefer the largest
  // tile that still gives two workgroups per compute unit; else the one with the most workgroups.
  static const int kMB[4] = {4, 4, 2, 2}, kNB[4] = {2, 1, 2, 1};
  const long long P = (long long)N * Ho * Wo;
  auto blocks = [&](int v) { return (long long)cdiv(Cout, kMB[v] * 32) * ((P + 4 * kNB[v] * 32 - 1) / (4 * kNB[v] * 32)); };
  int v = 3;
  const int first = (Cout > 64) ? 0 : 2;
  for (int i = first; i < 4; ++i)
    if (blocks(i) >= 512) { v = i; break; }
  PwGeom g;
  g.variant = v;
  g.bm = kMB[v] * 32;
  g.mtiles = cdiv(Cout, g.bm);
  g.nchunks = cdiv(Cin, KC1);
  g.a_floats = KC1 * g.bm;
  g.n_ptiles = (int)((P + 4 * kNB[v] * 32 - 1) / (4 * kNB[v] * 32));
  g.lds_bytes = (size_t)PW_KS * g.bm * sizeof(float);
  return g;
}

hipError_t init_pw_attributes() {
  hipError_t e;
#define PBKD_SET(MB, NB)                                                                                    \
  e = hipFuncSetAttribute(reinterpret_cast<const void *>(&pw_mfma_kernel<MB, NB>),                          \
                          hipFuncAttributeMaxDynamicSharedMemorySize, MAX_LDS);                             \
  if (e != hipSuccess) return e;
  PBKD_SET(4, 2) PBKD_SET(4, 1) PBKD_SET(2, 2) PBKD_SET(2, 1)
#undef PBKD_SET
  return hipSuccess;
}

hipError_t launch_pw(const PwArgs &a, hipStream_t s) {
  if (a.N <= 0 || a.Cin <= 0 || a.Cout <= 0 || a.g.mtiles > 65535) return hipErrorInvalidValue;
  const dim3 grid(a.g.n_ptiles, a.g.mtiles), block(256);
  switch (a.g.variant) {
    case 0: hipLaunchKernelGGL((pw_mfma_kernel<4, 2>), grid, block, a.g.lds_bytes, s, a); break;
    case 1: hipLaunchKernelGGL((pw_mfma_kernel<4, 1>), grid, block, a.g.lds_bytes, s, a); break;
    case 2: hipLaunchKernelGGL((pw_mfma_kernel<2, 2>), grid, block, a.g.lds_bytes, s, a); break;
    case 3: hipLaunchKernelGGL((pw_mfma_kernel<2, 1>), grid, block, a.g.lds_bytes, s, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace pbkd

// Implicit-GEMM convolution on the fp32 matrix cores of gfx950 (v_mfma_f32_32x32x2_f32), staged
// through LDS.  Serves the teacher's 3x3 convolutions, the student's pointwise 1x1 (forward and data
// gradient), the 1x1 projection shortcut and a trainable full 3x3 first layer.
//
// GEMM view: M = Cout, N = output pixels, K = taps*Cin.  A = weights, B = activations, so that the 32
// MFMA columns held by 32 consecutive lanes are 32 consecutive pixels and stores to NCHW coalesce.
// A workgroup (4 waves) owns a tile of 64*WGM output channels x 64*(4/WGM) pixels; a pixel tile is
// nimg whole images x TH x TW (powers of two), so small feature maps pack several images per tile.
// Per step of KC input channels the block stages the weights [taps][KC][BM] and ONE halo tile of the
// input [KC][nimg][IH][IW]; the nine taps are read from that halo tile with a constant offset, no
// im2col is materialised.
#include "pbkd_internal.h"

namespace pbkd {

typedef float floatx16 __attribute__((ext_vector_type(16)));

template <int TAPS, int KC, int WGM>
__global__ __launch_bounds__(256) void conv_mfma_kernel(ConvArgs p) {
  constexpr int WGN = 4 / WGM;
  constexpr int BM = WGM * 64;
  constexpr int PAD = (TAPS == 9) ? 1 : 0;
  extern __shared__ float smem[];
  float *As = smem;                    // [TAPS*KC][BM]
  float *Bs = smem + TAPS * KC * BM;   // [KC][PL]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WGM, wn = wave / WGM;
  const int l31 = lane & 31, lh = lane >> 5;

  int pt = blockIdx.x;
  const int tx = pt % p.g.tiles_x;
  pt /= p.g.tiles_x;
  const int ty = pt % p.g.tiles_y;
  const int tn = pt / p.g.tiles_y;
  const int m0 = blockIdx.y * BM;
  const int lTW = p.g.lTW, lTH = p.g.lTH;
  const int TW = 1 << lTW, TH = 1 << lTH;
  const int x0 = tx * TW, y0 = ty * TH, n0 = tn * p.g.nimg;
  const int IH = p.g.IH, IW = p.g.IW, PL = p.g.PL;
  const int s = p.stride;
  const int HWo = p.Ho * p.Wo;

  int pixoff[2];
  bool pvalid[2];
  size_t outoff[2];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    const int pn = wn * 64 + nb * 32 + l31;
    const int img = pn >> (lTW + lTH);
    const int rem = pn & (TH * TW - 1);
    const int i = rem >> lTW, j = rem & (TW - 1);
    pixoff[nb] = (img * IH + s * i) * IW + s * j + lh * PL;
    const int n = n0 + img, y = y0 + i, x = x0 + j;
    pvalid[nb] = (n < p.N) && (y < p.Ho) && (x < p.Wo);
    outoff[nb] = (size_t)n * p.Cout * HWo + (size_t)y * p.Wo + x;
  }
  const int aoff = wm * 64 + l31 + lh * BM;

  floatx16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  const int HW = p.H * p.W;
  const int IHW = IH * IW;
  for (int c0 = 0; c0 < p.Cin; c0 += KC) {
    __syncthreads();
    // ---- weights -> LDS
    for (int e = tid; e < TAPS * KC * BM; e += 256) {
      const int m = e & (BM - 1);
      const int r = e / BM;
      const int kc = r % KC, tap = r / KC;
      const int c = c0 + kc, o = m0 + m;
      float v = 0.f;
      if (c < p.Cin && o < p.Cout)
        v = p.wgt_km ? p.wgt[((size_t)tap * p.Cin + c) * p.Cout + o] : p.wgt[((size_t)o * p.Cin + c) * TAPS + tap];
      As[e] = v;
    }
    // ---- input halo tile -> LDS (BatchNorm+ReLU of the producer applied here; padding stays 0)
    for (int q = tid; q < PL; q += 256) {
      const int img = q / IHW;
      const int r = q - img * IHW;
      const int iy = r / IW;
      const int ix = r - iy * IW;
      const int n = n0 + img, y = y0 * s - PAD + iy, x = x0 * s - PAD + ix;
      const bool ok = (n < p.N) && (y >= 0) && (y < p.H) && (x >= 0) && (x < p.W);
      const float *src = p.in + ((ptrdiff_t)n * p.Cin + c0) * HW + (ptrdiff_t)y * p.W + x;   // only read if ok
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) {
        const int c = c0 + kc;
        float v = 0.f;
        if (ok && c < p.Cin) {
          v = src[(size_t)kc * HW];
          if (p.in_scale) v = fmaxf(fmaf(v, p.in_scale[c], p.in_shift[c]), 0.f);
        }
        Bs[kc * PL + q] = v;
      }
    }
    __syncthreads();
    // ---- MFMA over taps x channel pairs
#pragma unroll
    for (int tap = 0; tap < TAPS; ++tap) {
      const int toff = (TAPS == 9) ? ((tap / 3) * IW + (tap % 3)) : 0;
#pragma unroll
      for (int kk = 0; kk < KC; kk += 2) {
        const float a0 = As[(tap * KC + kk) * BM + aoff];
        const float a1 = As[(tap * KC + kk) * BM + aoff + 32];
        const float b0 = Bs[kk * PL + pixoff[0] + toff];
        const float b1 = Bs[kk * PL + pixoff[1] + toff];
        acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
        acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
        acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
        acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
      }
    }
  }

  // ---- store: accumulator register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int o = m0 + wm * 64 + mb * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
      if (o < p.Cout) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
          if (pvalid[nb]) p.out[outoff[nb] + (size_t)o * HWo] = acc[mb][nb][r];
      }
    }

  // ---- per-channel (sum, sum of squares) of this pixel tile, for BatchNorm's batch statistics
  if (p.stat_partial) {
    __syncthreads();
    float *red = smem;   // [WGN][BM][2]
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float v0 = pvalid[0] ? acc[mb][0][r] : 0.f;
        const float v1 = pvalid[1] ? acc[mb][1][r] : 0.f;
        float s1 = v0 + v1;
        float s2 = v0 * v0 + v1 * v1;
#pragma unroll
        for (int d = 16; d >= 1; d >>= 1) {
          s1 += __shfl_xor(s1, d, 64);
          s2 += __shfl_xor(s2, d, 64);
        }
        if (l31 == 0) {
          const int row = wm * 64 + mb * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
          red[(wn * BM + row) * 2 + 0] = s1;
          red[(wn * BM + row) * 2 + 1] = s2;
        }
      }
    __syncthreads();
    for (int e = tid; e < BM; e += 256) {
      const int o = m0 + e;
      if (o < p.Cout) {
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int w = 0; w < WGN; ++w) {
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

constexpr int KC9 = 8;    // input channels per step, 3x3
constexpr int KC1 = 32;   // input channels per step, 1x1

ConvGeom conv_geom(int taps, int N, int Cout, int Ho, int Wo, int stride) {
  ConvGeom g;
  g.wgm = (Cout > 64) ? 2 : 1;
  const int BN = (4 / g.wgm) * 64;
  int TW = pow2ceil(Wo);
  if (TW > 32) TW = 32;
  int TH = pow2ceil(Ho);
  if (TH > BN / TW) TH = BN / TW;
  g.lTW = ilog2(TW);
  g.lTH = ilog2(TH);
  g.nimg = BN / (TW * TH);
  const int halo = (taps == 9) ? 2 : 0;
  g.IH = stride * (TH - 1) + 1 + halo;
  g.IW = stride * (TW - 1) + 1 + halo;
  g.PL = g.nimg * g.IH * g.IW;
  g.tiles_x = cdiv(Wo, TW);
  g.tiles_y = cdiv(Ho, TH);
  g.tiles_n = cdiv(N, g.nimg);
  g.n_ptiles = g.tiles_x * g.tiles_y * g.tiles_n;
  g.kc = (taps == 9) ? KC9 : KC1;
  const int BM = g.wgm * 64;
  size_t fl = (size_t)taps * g.kc * BM + (size_t)g.kc * g.PL;
  const size_t red = (size_t)(4 / g.wgm) * BM * 2;
  if (fl < red) fl = red;
  g.lds_bytes = fl * sizeof(float);
  return g;
}

static constexpr int MAX_LDS = 160 * 1024;

hipError_t init_conv_attributes() {
  hipError_t e;
#define PBKD_SET(k)                                                                                              \
  e = hipFuncSetAttribute(reinterpret_cast<const void *>(&k), hipFuncAttributeMaxDynamicSharedMemorySize, MAX_LDS); \
  if (e != hipSuccess) return e;
  PBKD_SET((conv_mfma_kernel<9, KC9, 1>))
  PBKD_SET((conv_mfma_kernel<9, KC9, 2>))
  PBKD_SET((conv_mfma_kernel<1, KC1, 1>))
  PBKD_SET((conv_mfma_kernel<1, KC1, 2>))
#undef PBKD_SET
  return hipSuccess;
}

hipError_t launch_conv(int taps, const ConvArgs &a, hipStream_t s) {
  if (a.g.lds_bytes > (size_t)MAX_LDS) return hipErrorInvalidValue;
  if (a.N <= 0 || a.Cout <= 0 || a.Cin <= 0) return hipErrorInvalidValue;
  const int BM = a.g.wgm * 64;
  dim3 grid(a.g.n_ptiles, cdiv(a.Cout, BM));
  dim3 block(256);
  if (taps == 9) {
    if (a.g.wgm == 1)
      hipLaunchKernelGGL((conv_mfma_kernel<9, KC9, 1>), grid, block, a.g.lds_bytes, s, a);
    else
      hipLaunchKernelGGL((conv_mfma_kernel<9, KC9, 2>), grid, block, a.g.lds_bytes, s, a);
  } else if (taps == 1) {
    if (a.g.wgm == 1)
      hipLaunchKernelGGL((conv_mfma_kernel<1, KC1, 1>), grid, block, a.g.lds_bytes, s, a);
    else
      hipLaunchKernelGGL((conv_mfma_kernel<1, KC1, 2>), grid, block, a.g.lds_bytes, s, a);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// Pointwise weight gradient dP[o,c] = sum_k dz[o,k] * u[c,k], k = (image, pixel): M = Cout, N = Cin,
// K = N*H*W.  A workgroup owns a 64x64 tile of dP and a contiguous range of K (split-K); its four waves
// each take a quarter of every staged 64-wide K chunk and are summed through LDS at the end.  Rows are
// padded to 65 floats so that the 32 lanes of an MFMA operand (32 different rows, same k) hit 32 banks.
constexpr int WG_KP = 64;
constexpr int WG_KPS = WG_KP + 1;

__global__ __launch_bounds__(256) void pw_wgrad_kernel(WgradArgs p) {
  __shared__ float As[64 * WG_KPS];
  __shared__ float Bs[64 * WG_KPS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l31 = lane & 31, lh = lane >> 5;
  const int m0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int split = blockIdx.z;
  const long long K = (long long)p.N * p.HW;
  const int kk_t = tid & 63;     // this thread's k within a chunk
  const int row_t = tid >> 6;    // first row it loads; then every 4th

  floatx16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  const int ch_begin = split * p.g.chunks_per_split;
  for (int ch = ch_begin; ch < ch_begin + p.g.chunks_per_split; ++ch) {
    const long long k = (long long)ch * WG_KP + kk_t;
    const bool kok = k < K;
    const int n = kok ? (int)(k / p.HW) : 0;
    const int px = kok ? (int)(k - (long long)n * p.HW) : 0;
    __syncthreads();
#pragma unroll 4
    for (int i = 0; i < 16; ++i) {
      const int row = row_t + 4 * i;
      const int o = m0 + row, c = c0 + row;
      float va = 0.f, vb = 0.f;
      if (kok && o < p.Co) va = p.dz[((size_t)n * p.Co + o) * p.HW + px];
      if (kok && c < p.Ci) vb = p.u[((size_t)n * p.Ci + c) * p.HW + px];
      As[row * WG_KPS + kk_t] = va;
      Bs[row * WG_KPS + kk_t] = vb;
    }
    __syncthreads();
    const int kb = wave * 16 + lh;
#pragma unroll
    for (int ks = 0; ks < 16; ks += 2) {
      const float a0 = As[l31 * WG_KPS + kb + ks];
      const float a1 = As[(32 + l31) * WG_KPS + kb + ks];
      const float b0 = Bs[l31 * WG_KPS + kb + ks];
      const float b1 = Bs[(32 + l31) * WG_KPS + kb + ks];
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
    }
  }

  // ---- sum the four waves' tiles through LDS (wave 0 collects), fixed order
  float *red = As;   // 64*64 floats needed, As+Bs are contiguous? no: use As (64*65 floats >= 4096)
  for (int w = 1; w < 4; ++w) {
    __syncthreads();
    if (wave == w) {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int r = 0; r < 16; ++r) red[((mb * 2 + nb) * 16 + r) * 64 + lane] = acc[mb][nb][r];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[mb][nb][r] += red[((mb * 2 + nb) * 16 + r) * 64 + lane];
    }
  }
  if (wave == 0) {
    float *dst = p.partial + (size_t)split * p.Co * p.Ci;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int o = m0 + mb * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
        if (o < p.Co) {
#pragma unroll
          for (int nb = 0; nb < 2; ++nb) {
            const int c = c0 + nb * 32 + l31;
            if (c < p.Ci) dst[(size_t)o * p.Ci + c] = acc[mb][nb][r];
          }
        }
      }
  }
}

WgradGeom wgrad_geom(int N, int Co, int Ci, int HW) {
  WgradGeom g;
  g.tiles_m = cdiv(Co, 64);
  g.tiles_n = cdiv(Ci, 64);
  const long long K = (long long)N * HW;
  const int nchunks = (int)((K + WG_KP - 1) / WG_KP);
  int want = cdiv(1024, g.tiles_m * g.tiles_n);
  if (want < 1) want = 1;
  if (want > nchunks) want = nchunks;
  g.chunks_per_split = cdiv(nchunks, want);
  g.splits = cdiv(nchunks, g.chunks_per_split);
  return g;
}

hipError_t launch_pw_wgrad(const WgradArgs &a, hipStream_t s) {
  if (a.g.splits <= 0 || a.g.splits > 65535) return hipErrorInvalidValue;
  dim3 grid(a.g.tiles_n, a.g.tiles_m, a.g.splits);
  hipLaunchKernelGGL(pw_wgrad_kernel, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace pbkd

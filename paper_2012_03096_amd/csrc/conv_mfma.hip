// Implicit-GEMM convolution on the fp32 matrix cores of gfx950 (v_mfma_f32_32x32x2_f32), staged
// through LDS.  Serves the teacher's 3x3 convolutions, the student's pointwise 1x1 (forward and data
// gradient), the 1x1 projection shortcut and a trainable full 3x3 first layer.
//
// GEMM view: M = Cout, N = output pixels, K = taps*Cin.  A = weights, B = activations, so that the 32
// MFMA columns held by 32 consecutive lanes are 32 consecutive pixels and stores to NCHW coalesce.
// A workgroup (4 waves) owns a tile of 128x128, 64x256, 64x128 or 64x64 (channels x pixels), picked so that
// at least two workgroups can share a compute unit whenever the problem is large enough; a pixel tile is
// nimg whole images x TH x TW (powers of two), so small feature maps pack several images per tile.
// Per step of KC input channels the block stages the weights [taps][KC][BM] and ONE halo tile of the
// input [KC][nimg][IH][IW]; the nine taps are read from that halo tile with a constant offset, no
// im2col is materialised.
#include <cstdlib>

#include "conv_mfma_kernel.h"

namespace pbkd {

// Tile choice.  Large tiles reuse staged operands best, so take the largest tile that still gives every
// one of the 256 compute units a workgroup, else the smallest (measured on the VGG/ResNet shapes: 128x128
// for 16x16 maps with 128 channels, 64x128 for 8x8 maps, 64x64 for 4x4 and 2x2 maps, 64x256 when there
// are only 64 output channels).  PBKD_CONV_TILE=0..3 overrides the choice (tuning aid).
ConvGeom conv_geom(int taps, int N, int Cin, int Cout, int Ho, int Wo, int stride) {
  static const int kBM[4] = {128, 64, 64, 64}, kBN[4] = {128, 256, 128, 64};
  const long long pixels = (long long)N * Ho * Wo;
  auto blocks = [&](int t) { return (long long)cdiv(Cout, kBM[t]) * ((pixels + kBN[t] - 1) / kBN[t]); };
  const int order_wide[4] = {0, 1, 2, 3}, order_narrow[3] = {1, 2, 3};
  const int *order = (Cout > 64) ? order_wide : order_narrow;
  const int n_order = (Cout > 64) ? 4 : 3;
  int tile = order[n_order - 1];
  for (int i = 0; i < n_order; ++i)
    if (blocks(order[i]) >= 256) { tile = order[i]; break; }
  if (const char *env = std::getenv("PBKD_CONV_TILE")) {
    const int t = std::atoi(env);
    if (t >= 0 && t < 4) tile = t;
  }
  ConvGeom g;
  g.tile = tile;
  g.bm = kBM[tile];
  const int BN = kBN[tile];
  g.kc = (taps == 9) ? KC9 : KC1;
  g.mtiles = cdiv(Cout, g.bm);
  g.nchunks = cdiv(Cin, g.kc);
  g.a_floats = taps * g.kc * g.bm;
  int TW = pow2ceil(Wo);
  if (TW > 32) TW = 32;
  int TH = pow2ceil(Ho);
  if (TH > BN / TW) TH = BN / TW;
  g.lTW = ilog2(TW);
  g.lTH = ilog2(TH);
  g.nimg = BN / (TW * TH);
  g.IH = stride * (TH - 1) + 3;
  g.IW = stride * (TW - 1) + 3;
  // LDS strides: 32 consecutive output pixels of a wave (rows of TW, images of TH*TW) must fall into 32
  // different banks for every tap, so the row stride is made congruent to TW and the image stride to
  // TH*TW modulo 32 (stride-1 convolutions; with stride 2 a two-way conflict remains)
  g.IWS = g.IW;
  if (TW < 32) while (g.IWS % 32 != TW % 32) ++g.IWS;
  g.IMS = g.IH * g.IWS;
  if (TH * TW < 32) while (g.IMS % 32 != (TH * TW) % 32) ++g.IMS;
  g.PLd = g.nimg * g.IH * g.IW;
  g.PL = g.nimg * g.IMS;
  if (2 * ((size_t)g.a_floats + (size_t)g.kc * g.PL) * sizeof(float) > 128 * 1024) {   // tiny maps: padding would not fit
    g.IWS = g.IW;
    g.IMS = g.IH * g.IW;
    g.PL = g.PLd;
  }
  g.tiles_x = cdiv(Wo, TW);
  g.tiles_y = cdiv(Ho, TH);
  g.tiles_n = cdiv(N, g.nimg);
  g.n_ptiles = g.tiles_x * g.tiles_y * g.tiles_n;
  size_t fl = 2 * ((size_t)g.a_floats + (size_t)g.kc * g.PL);
  const size_t red = (size_t)4 * g.bm * 2;
  if (fl < red) fl = red;
  g.lds_bytes = fl * sizeof(float);
  return g;
}

hipError_t init_conv_attributes() {
  hipError_t e;
  if ((e = conv_tile0_init()) != hipSuccess) return e;
  if ((e = conv_tile1_init()) != hipSuccess) return e;
  if ((e = conv_tile2_init()) != hipSuccess) return e;
  return conv_tile3_init();
}

hipError_t launch_conv(int taps, const ConvArgs &a, hipStream_t s) {
  if (a.g.lds_bytes > (size_t)MAX_LDS) return hipErrorInvalidValue;
  if (a.N <= 0 || a.Cout <= 0 || a.Cin <= 0) return hipErrorInvalidValue;
  switch (a.g.tile) {
    case 0: return conv_tile0_launch(taps, a, s);
    case 1: return conv_tile1_launch(taps, a, s);
    case 2: return conv_tile2_launch(taps, a, s);
    case 3: return conv_tile3_launch(taps, a, s);
    default: return hipErrorInvalidValue;
  }
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

// Second form, used whenever H*W is a multiple of 4: no LDS for the operands at all.  Both dz[o,:] and
// u[c,:] are contiguous along the reduction index (pixels), and a sum does not care in which order its
// terms are taken: every lane loads 4 consecutive pixels of its row as one 16-byte vector -- lanes 0..31
// the first four of a group of eight pixels, lanes 32..63 the second four -- and the four MFMA steps that
// follow pair element s of the A vector with element s of the B vector, i.e. K index (8g + s, 8g + 4 + s).
// The four waves of a workgroup take groups g = wave, wave + 4, ... of the workgroup's pixel range, so
// together they consume whole 128-byte lines of every row; WG2_D groups per wave are kept in flight.
constexpr int WG2_D = 4;

__global__ __launch_bounds__(256, 2) void pw_wgrad2_kernel(WgradArgs p) {
  __shared__ float red[64 * 64];
  typedef float f4 __attribute__((ext_vector_type(4)));
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l31 = lane & 31, lh = lane >> 5;
  const int m0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int split = blockIdx.z;
  const long long K = (long long)p.N * p.HW;
  const long long ngroups = (K + 7) / 8;
  const long long g_begin = (long long)split * p.g.chunks_per_split * (WG_KP / 8);
  long long g_end = g_begin + (long long)p.g.chunks_per_split * (WG_KP / 8);
  if (g_end > ngroups) g_end = ngroups;

  size_t rowa[2], rowb[2];
  bool oka[2], okb[2];
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    int o = m0 + b * 32 + l31, c = c0 + b * 32 + l31;
    oka[b] = o < p.Co;
    okb[b] = c < p.Ci;
    if (!oka[b]) o = p.Co - 1;
    if (!okb[b]) c = p.Ci - 1;
    rowa[b] = (size_t)o * p.HW;
    rowb[b] = (size_t)c * p.HW;
  }
  const f4 zero4 = {0.f, 0.f, 0.f, 0.f};
  auto load = [&](long long g, f4 (&a)[2], f4 (&b)[2]) {
    long long q = g * 8 + 4 * lh;
    const bool ok = (g < g_end) && (q < K);    // K is a multiple of 4, so q < K covers q..q+3
    if (!ok) q = 0;
    const int n = (int)(q / p.HW);
    const int px = (int)(q - (long long)n * p.HW);
    const float *pa = p.dz + (size_t)n * p.Co * p.HW + px;
    const float *pb = p.u + (size_t)n * p.Ci * p.HW + px;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const f4 va = *reinterpret_cast<const f4 *>(pa + rowa[i]);
      const f4 vb = *reinterpret_cast<const f4 *>(pb + rowb[i]);
      a[i] = (ok && oka[i]) ? va : zero4;
      b[i] = (ok && okb[i]) ? vb : zero4;
    }
  };

  floatx16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  f4 ra[WG2_D][2], rb[WG2_D][2];
#pragma unroll
  for (int d = 0; d < WG2_D; ++d) load(g_begin + wave + 4 * d, ra[d], rb[d]);
  const long long mine = (g_end - g_begin - wave + 3) / 4;   // groups of this wave (may be <= 0)
  for (long long i = 0; i < mine; i += WG2_D) {
#pragma unroll
    for (int d = 0; d < WG2_D; ++d) {
      f4 ca[2], cb[2];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        ca[j] = ra[d][j];
        cb[j] = rb[d][j];
      }
      load(g_begin + wave + 4 * (i + d + WG2_D), ra[d], rb[d]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(ca[0][e], cb[0][e], acc[0][0], 0, 0, 0);
        acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(ca[0][e], cb[1][e], acc[0][1], 0, 0, 0);
        acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(ca[1][e], cb[0][e], acc[1][0], 0, 0, 0);
        acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(ca[1][e], cb[1][e], acc[1][1], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // ---- sum the four waves' tiles through LDS (wave 0 collects), fixed order
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
  // about 1.5 workgroups per compute unit: every split costs one 64x64 partial tile of traffic
  int want = cdiv(384, g.tiles_m * g.tiles_n);
  if (want < 1) want = 1;
  if (want > nchunks) want = nchunks;
  g.chunks_per_split = cdiv(nchunks, want);
  g.splits = cdiv(nchunks, g.chunks_per_split);
  return g;
}

hipError_t launch_pw_wgrad(const WgradArgs &a, hipStream_t s) {
  if (a.g.splits <= 0 || a.g.splits > 65535) return hipErrorInvalidValue;
  dim3 grid(a.g.tiles_n, a.g.tiles_m, a.g.splits);
  if (a.HW % 4 == 0)
    hipLaunchKernelGGL(pw_wgrad2_kernel, grid, dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL(pw_wgrad_kernel, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace pbkd

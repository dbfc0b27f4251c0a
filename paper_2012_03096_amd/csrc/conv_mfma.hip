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

// Software pipeline.  The LDS holds two copies of (weights, input tile).  While the matrix cores work
// on chunk k from copy k&1, the global loads of chunk k+1 are issued a few per MFMA step during the first
// half of the chunk and land in registers; during the last quarter they are written, again a few per
// step, into the other copy (BatchNorm+ReLU of the producing layer applied at that point), and one
// barrier per chunk closes the hand-over.  The LDS operands of MFMA step t+1 are fetched before the four
// MFMAs of step t are issued.  Nothing but those four MFMAs sits between two scheduling fences, so a
// single wave per SIMD keeps its matrix pipe busy while it does all the staging itself.
template <int VW> struct VecOf;
template <> struct VecOf<4> { typedef float type __attribute__((ext_vector_type(4))); };
template <> struct VecOf<2> { typedef float type __attribute__((ext_vector_type(2))); };

template <int TAPS, int KC, int WGM, int BSLOTS>
__global__ __launch_bounds__(256, (TAPS == 9) ? 1 : 2) void conv_mfma_kernel(ConvArgs p) {
  constexpr int WGN = 4 / WGM;
  constexpr int BM = WGM * 64;
  constexpr int PAD = (TAPS == 9) ? 1 : 0;
  constexpr int A_FLOATS = TAPS * KC * BM;
  constexpr int A_PT = A_FLOATS / 256;          // weights staged per thread and chunk
  constexpr int VW = (A_PT % 4 == 0) ? 4 : 2;
  constexpr int NA = A_PT / VW;                 // vector loads of weights per thread and chunk
  constexpr int NB = BSLOTS * KC;               // scalar loads of inputs per thread and chunk
  constexpr int NL = NA + NB;
  constexpr int T = TAPS * KC / 2;              // MFMA steps (K = 2 each) per chunk
  constexpr int L_STEPS = T / 2;                // global loads are issued during steps [0, L_STEPS)
  constexpr int LPS = (NL + L_STEPS - 1) / L_STEPS;
  constexpr int S_STEPS = (T / 4 > 0) ? T / 4 : 1;
  constexpr int S_BEGIN = T - S_STEPS;          // LDS writes happen during steps [S_BEGIN, T)
  constexpr int SPS = (NL + S_STEPS - 1) / S_STEPS;
  static_assert(A_FLOATS % 256 == 0 && A_PT % VW == 0, "weight tile must divide evenly over the workgroup");
  typedef typename VecOf<VW>::type avec_t;
  extern __shared__ float smem[];
  const int PL = p.g.PL;
  float *As = smem;                    // [2][TAPS*KC][BM]
  float *Bs = smem + 2 * A_FLOATS;     // [2][KC][PL]

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
  const int IH = p.g.IH, IW = p.g.IW;
  const int s = p.stride;
  // a 3x3 tile is staged densely (halo included) and read with the stride; a 1x1 tile holds just the
  // pixels that are used, gathered with the stride from global memory
  const int sl_ = (TAPS == 9) ? s : 1;
  const int HWo = p.Ho * p.Wo;
  const int HW = p.H * p.W;
  const int IHW = IH * IW;
  const int nchunks = p.g.nchunks;
  const bool bn = (p.in_scale != nullptr);

  // ---- where this lane's two pixel columns sit in the staged tile and in the output
  int pixoff[2];
  bool pvalid[2];
  size_t outoff[2];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    const int pn = wn * 64 + nb * 32 + l31;
    const int img = pn >> (lTW + lTH);
    const int rem = pn & (TH * TW - 1);
    const int i = rem >> lTW, j = rem & (TW - 1);
    pixoff[nb] = (img * IH + sl_ * i) * IW + sl_ * j + lh * PL;
    const int n = n0 + img, y = y0 + i, x = x0 + j;
    pvalid[nb] = (n < p.N) && (y < p.Ho) && (x < p.Wo);
    outoff[nb] = (size_t)n * p.Cout * HWo + (size_t)y * p.Wo + x;
  }
  const int aoff = wm * 64 + l31 + lh * BM;

  // ---- which input-tile elements this thread stages (same positions in every chunk)
  ptrdiff_t goff[BSLOTS];
  bool gok[BSLOTS];
#pragma unroll
  for (int sl = 0; sl < BSLOTS; ++sl) {
    const int q = tid + 256 * sl;
    const int img = q / IHW;
    const int r = q - img * IHW;
    const int iy = r / IW;
    const int ix = r - iy * IW;
    const int n = n0 + img;
    const int y = (TAPS == 9) ? (y0 * s - PAD + iy) : (y0 + iy) * s;
    const int x = (TAPS == 9) ? (x0 * s - PAD + ix) : (x0 + ix) * s;
    gok[sl] = (q < PL) && (n < p.N) && (y >= 0) && (y < p.H) && (x >= 0) && (x < p.W);
    goff[sl] = (ptrdiff_t)n * p.Cin * HW + (ptrdiff_t)y * p.W + x;
  }
  const float *wsrc = p.wpk + (size_t)blockIdx.y * nchunks * A_FLOATS + (size_t)tid * VW;

  avec_t avec[NA];
  float breg[NB];
  float scn[KC], shn[KC];   // BatchNorm scale / shift of the channels being staged

  auto load_item = [&](int idx, int chunk) {
    if (idx < NA) {
      avec[idx] = *reinterpret_cast<const avec_t *>(wsrc + (size_t)chunk * A_FLOATS + (size_t)idx * 256 * VW);
    } else {
      const int jb = idx - NA, sl = jb / KC, kc = jb % KC;
      const int c = chunk * KC + kc;
      breg[jb] = (gok[sl] && c < p.Cin) ? p.in[goff[sl] + (ptrdiff_t)c * HW] : 0.f;
    }
  };
  auto load_affine = [&](int chunk) {
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      const int c = chunk * KC + kc;
      const bool on = bn && (c < p.Cin);
      scn[kc] = on ? p.in_scale[c] : 1.f;
      shn[kc] = on ? p.in_shift[c] : 0.f;
    }
  };
  auto store_item = [&](int idx, int buf) {
    if (idx < NA) {
      *reinterpret_cast<avec_t *>(As + buf * A_FLOATS + (tid + 256 * idx) * VW) = avec[idx];
    } else {
      const int jb = idx - NA, sl = jb / KC, kc = jb % KC;
      const int q = tid + 256 * sl;
      if (q < PL) {
        float v = breg[jb];
        if (bn && gok[sl]) v = fmaxf(fmaf(v, scn[kc], shn[kc]), 0.f);   // padding stays exactly zero
        Bs[(buf * KC + kc) * PL + q] = v;
      }
    }
  };

  floatx16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  load_affine(0);
#pragma unroll
  for (int idx = 0; idx < NL; ++idx) load_item(idx, 0);
#pragma unroll
  for (int idx = 0; idx < NL; ++idx) store_item(idx, 0);
  __syncthreads();
  for (int k = 0; k < nchunks; ++k) {
    const bool more = (k + 1 < nchunks);
    const float *Ab = As + (k & 1) * A_FLOATS + aoff;
    const float *Bb = Bs + (k & 1) * KC * PL;
    float a0 = Ab[0], a1 = Ab[32];
    float b0 = Bb[pixoff[0]], b1 = Bb[pixoff[1]];
    if (more) load_affine(k + 1);
#pragma unroll
    for (int t = 0; t < T; ++t) {
      float na0 = 0.f, na1 = 0.f, nb0 = 0.f, nb1 = 0.f;
      if (t + 1 < T) {
        const int tap = (t + 1) / (KC / 2), kk = 2 * ((t + 1) % (KC / 2));
        const int toff = (TAPS == 9) ? ((tap / 3) * IW + (tap % 3)) : 0;
        na0 = Ab[(tap * KC + kk) * BM];
        na1 = Ab[(tap * KC + kk) * BM + 32];
        nb0 = Bb[kk * PL + pixoff[0] + toff];
        nb1 = Bb[kk * PL + pixoff[1] + toff];
      }
      if (more) {
        if (t < L_STEPS) {
#pragma unroll
          for (int i = 0; i < LPS; ++i)
            if (t * LPS + i < NL) load_item(t * LPS + i, k + 1);
        }
        if (t >= S_BEGIN) {
#pragma unroll
          for (int i = 0; i < SPS; ++i)
            if ((t - S_BEGIN) * SPS + i < NL) store_item((t - S_BEGIN) * SPS + i, (k + 1) & 1);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      a0 = na0; a1 = na1; b0 = nb0; b1 = nb1;
    }
    __syncthreads();
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
    float *red = smem;   // [WGN][BM][2]; the last chunk's barrier has already passed
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

static int bslots_for(int PL) {
  const int need = cdiv(PL, 256);
  if (need <= 1) return 1;
  if (need <= 2) return 2;
  if (need <= 3) return 3;
  if (need <= 5) return 5;
  if (need <= 8) return 8;
  return 0;
}

ConvGeom conv_geom(int taps, int N, int Cin, int Cout, int Ho, int Wo, int stride) {
  ConvGeom g;
  g.wgm = (Cout > 64) ? 2 : 1;
  g.bm = 64 * g.wgm;
  g.kc = (taps == 9) ? KC9 : KC1;
  g.mtiles = cdiv(Cout, g.bm);
  g.nchunks = cdiv(Cin, g.kc);
  g.a_floats = taps * g.kc * g.bm;
  const int BN = (4 / g.wgm) * 64;
  int TW = pow2ceil(Wo);
  if (TW > 32) TW = 32;
  int TH = pow2ceil(Ho);
  if (TH > BN / TW) TH = BN / TW;
  g.lTW = ilog2(TW);
  g.lTH = ilog2(TH);
  g.nimg = BN / (TW * TH);
  g.IH = (taps == 9) ? stride * (TH - 1) + 3 : TH;
  g.IW = (taps == 9) ? stride * (TW - 1) + 3 : TW;
  g.PL = g.nimg * g.IH * g.IW;
  g.tiles_x = cdiv(Wo, TW);
  g.tiles_y = cdiv(Ho, TH);
  g.tiles_n = cdiv(N, g.nimg);
  g.n_ptiles = g.tiles_x * g.tiles_y * g.tiles_n;
  const int BM = g.wgm * 64;
  size_t fl = 2 * ((size_t)taps * g.kc * BM + (size_t)g.kc * g.PL);
  const size_t red = (size_t)(4 / g.wgm) * BM * 2;
  if (fl < red) fl = red;
  g.lds_bytes = fl * sizeof(float);
  return g;
}

static constexpr int MAX_LDS = 160 * 1024;

template <int TAPS, int KC, int WGM, int BSLOTS>
static hipError_t conv_set_attr() {
  return hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_mfma_kernel<TAPS, KC, WGM, BSLOTS>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, MAX_LDS);
}
template <int TAPS, int KC, int WGM>
static hipError_t conv_set_attr_slots() {
  hipError_t e;
  if ((e = conv_set_attr<TAPS, KC, WGM, 1>()) != hipSuccess) return e;
  if constexpr (TAPS == 1) {
    return hipSuccess;   // a 1x1 tile is compact: never more than 256 staged floats per channel
  } else {
    if ((e = conv_set_attr<TAPS, KC, WGM, 2>()) != hipSuccess) return e;
    if ((e = conv_set_attr<TAPS, KC, WGM, 3>()) != hipSuccess) return e;
    if ((e = conv_set_attr<TAPS, KC, WGM, 5>()) != hipSuccess) return e;
    return conv_set_attr<TAPS, KC, WGM, 8>();
  }
}

hipError_t init_conv_attributes() {
  hipError_t e;
  if ((e = conv_set_attr_slots<9, KC9, 1>()) != hipSuccess) return e;
  if ((e = conv_set_attr_slots<9, KC9, 2>()) != hipSuccess) return e;
  if ((e = conv_set_attr_slots<1, KC1, 1>()) != hipSuccess) return e;
  return conv_set_attr_slots<1, KC1, 2>();
}

template <int TAPS, int KC, int WGM>
static hipError_t conv_launch_slots(const ConvArgs &a, dim3 grid, hipStream_t s) {
  const dim3 block(256);
  if constexpr (TAPS == 1) {
    if (bslots_for(a.g.PL) != 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL((conv_mfma_kernel<TAPS, KC, WGM, 1>), grid, block, a.g.lds_bytes, s, a);
  } else {
    switch (bslots_for(a.g.PL)) {
      case 1: hipLaunchKernelGGL((conv_mfma_kernel<TAPS, KC, WGM, 1>), grid, block, a.g.lds_bytes, s, a); break;
      case 2: hipLaunchKernelGGL((conv_mfma_kernel<TAPS, KC, WGM, 2>), grid, block, a.g.lds_bytes, s, a); break;
      case 3: hipLaunchKernelGGL((conv_mfma_kernel<TAPS, KC, WGM, 3>), grid, block, a.g.lds_bytes, s, a); break;
      case 5: hipLaunchKernelGGL((conv_mfma_kernel<TAPS, KC, WGM, 5>), grid, block, a.g.lds_bytes, s, a); break;
      case 8: hipLaunchKernelGGL((conv_mfma_kernel<TAPS, KC, WGM, 8>), grid, block, a.g.lds_bytes, s, a); break;
      default: return hipErrorInvalidValue;
    }
  }
  return hipGetLastError();
}

hipError_t launch_conv(int taps, const ConvArgs &a, hipStream_t s) {
  if (a.g.lds_bytes > (size_t)MAX_LDS) return hipErrorInvalidValue;
  if (a.N <= 0 || a.Cout <= 0 || a.Cin <= 0) return hipErrorInvalidValue;
  const int BM = a.g.wgm * 64;
  const dim3 grid(a.g.n_ptiles, cdiv(a.Cout, BM));
  if (taps == 9) return a.g.wgm == 1 ? conv_launch_slots<9, KC9, 1>(a, grid, s) : conv_launch_slots<9, KC9, 2>(a, grid, s);
  if (taps == 1) return a.g.wgm == 1 ? conv_launch_slots<1, KC1, 1>(a, grid, s) : conv_launch_slots<1, KC1, 2>(a, grid, s);
  return hipErrorInvalidValue;
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

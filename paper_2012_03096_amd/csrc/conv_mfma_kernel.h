// Device code of the implicit-GEMM convolution on the fp32 matrix cores (see conv_mfma.hip for the
// overview).  Included by the translation units that instantiate one workgroup tile each.
#pragma once
#include "pbkd_internal.h"

namespace pbkd {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Staging schedule inside a chunk of T MFMA steps: the next chunk's global loads are issued during the
// first T/LOAD_DIV steps and written to LDS during the last T/STORE_DIV steps.
#ifndef PBKD_CONV_LOAD_DIV
#define PBKD_CONV_LOAD_DIV 2
#endif
#ifndef PBKD_CONV_STORE_DIV
#define PBKD_CONV_STORE_DIV 4
#endif

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

template <int TAPS, int KC, int WGM, int MB, int NB, int BSLOTS>
__global__ __launch_bounds__(256, (TAPS == 9 && MB * NB == 4) ? 1 : 2) void conv_mfma_kernel(ConvArgs p) {
  constexpr int WGN = 4 / WGM;
  constexpr int BM = WGM * MB * 32;     // output channels per workgroup
  constexpr int WN = NB * 32;           // pixels per wave
  constexpr int PAD = (TAPS == 9) ? 1 : 0;
  constexpr int A_FLOATS = TAPS * KC * BM;
  constexpr int A_PT = A_FLOATS / 256;          // weights staged per thread and chunk
  constexpr int VW = (A_PT % 4 == 0) ? 4 : 2;
  constexpr int NA = A_PT / VW;                 // vector loads of weights per thread and chunk
  constexpr int NBL = BSLOTS * KC;              // scalar loads of inputs per thread and chunk
  constexpr int NL = NA + NBL;
  constexpr int T = TAPS * KC / 2;              // MFMA steps (K = 2 each) per chunk
  constexpr int L_STEPS = (T / PBKD_CONV_LOAD_DIV > 0) ? T / PBKD_CONV_LOAD_DIV : 1;   // global loads are issued during steps [0, L_STEPS)
  constexpr int LPS = (NL + L_STEPS - 1) / L_STEPS;
  constexpr int S_STEPS = (T / PBKD_CONV_STORE_DIV > 0) ? T / PBKD_CONV_STORE_DIV : 1;
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
  int pixoff[NB];
  bool pvalid[NB];
  size_t outoff[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int pn = wn * WN + nb * 32 + l31;
    const int img = pn >> (lTW + lTH);
    const int rem = pn & (TH * TW - 1);
    const int i = rem >> lTW, j = rem & (TW - 1);
    pixoff[nb] = (img * IH + sl_ * i) * IW + sl_ * j + lh * PL;
    const int n = n0 + img, y = y0 + i, x = x0 + j;
    pvalid[nb] = (n < p.N) && (y < p.Ho) && (x < p.Wo);
    outoff[nb] = (size_t)n * p.Cout * HWo + (size_t)y * p.Wo + x;
  }
  const int aoff = wm * (MB * 32) + l31 + lh * BM;

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
  float breg[NBL];
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

  floatx16 acc[MB][NB];
#pragma unroll
  for (int a = 0; a < MB; ++a)
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

#ifdef PBKD_EXP_CLOCK
  const long long exp_c0 = clock64(), exp_w0 = wall_clock64();
#endif
  load_affine(0);
#pragma unroll
  for (int idx = 0; idx < NL; ++idx) load_item(idx, 0);
#pragma unroll
  for (int idx = 0; idx < NL; ++idx) store_item(idx, 0);
  __syncthreads();
#ifdef PBKD_EXP_CLOCK
  long long exp_tc = 0, exp_tb = 0;
#endif
  for (int k = 0; k < nchunks; ++k) {
#ifdef PBKD_EXP_CLOCK
    const long long exp_a = clock64();
#endif
    const bool more = (k + 1 < nchunks);
    const float *Ab = As + (k & 1) * A_FLOATS + aoff;
    const float *Bb = Bs + (k & 1) * KC * PL;
    float av[MB], bv[NB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) av[mb] = Ab[32 * mb];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) bv[nb] = Bb[pixoff[nb]];
    if (more) load_affine(k + 1);
#pragma unroll
    for (int t = 0; t < T; ++t) {
      float nav[MB], nbv[NB];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) nav[mb] = 0.f;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) nbv[nb] = 0.f;
      if (t + 1 < T) {
        const int tap = (t + 1) / (KC / 2), kk = 2 * ((t + 1) % (KC / 2));
        const int toff = (TAPS == 9) ? ((tap / 3) * IW + (tap % 3)) : 0;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) nav[mb] = Ab[(tap * KC + kk) * BM + 32 * mb];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) nbv[nb] = Bb[kk * PL + pixoff[nb] + toff];
      }
      if (more) {
        if (t < L_STEPS) {
#pragma unroll
          for (int i = 0; i < LPS; ++i)
#ifndef PBKD_EXP_NOLOAD
            if (t * LPS + i < NL) load_item(t * LPS + i, k + 1);
#endif
            ;
        }
        if (t >= S_BEGIN) {
#pragma unroll
          for (int i = 0; i < SPS; ++i)
#ifndef PBKD_EXP_NOSTORE
            if ((t - S_BEGIN) * SPS + i < NL) store_item((t - S_BEGIN) * SPS + i, (k + 1) & 1);
#endif
            ;
        }
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
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) bv[nb] = nbv[nb];
    }
#ifdef PBKD_EXP_CLOCK
    const long long exp_b = clock64();
#endif
#ifndef PBKD_EXP_NOBARRIER
    __syncthreads();
#endif
#ifdef PBKD_EXP_CLOCK
    exp_tc += exp_b - exp_a;
    exp_tb += clock64() - exp_b;
#endif
  }

#ifdef PBKD_EXP_CLOCK
  if (tid == 0 && blockIdx.x == 0 && blockIdx.y == 0) {
    const long long c1 = clock64(), w1 = wall_clock64();
    p.stat_partial[0] = (float)(c1 - exp_c0);
    p.stat_partial[1] = (float)(w1 - exp_w0);
    p.stat_partial[2] = (float)exp_tc;
    p.stat_partial[3] = (float)exp_tb;
  }
  if (blockIdx.x == 0 && blockIdx.y == 0) return;
#endif
  // ---- store: accumulator register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int o = m0 + wm * (MB * 32) + mb * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
      if (o < p.Cout) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
          if (pvalid[nb]) p.out[outoff[nb] + (size_t)o * HWo] = acc[mb][nb][r];
      }
    }

  // ---- per-channel (sum, sum of squares) of this pixel tile, for BatchNorm's batch statistics
  if (p.stat_partial) {
    float *red = smem;   // [WGN][BM][2]; the last chunk's barrier has already passed
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
#pragma unroll
        for (int d = 16; d >= 1; d >>= 1) {
          s1 += __shfl_xor(s1, d, 64);
          s2 += __shfl_xor(s2, d, 64);
        }
        if (l31 == 0) {
          const int row = wm * (MB * 32) + mb * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
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
constexpr int MAX_LDS = 160 * 1024;

inline int conv_bslots_for(int PL) {
  const int need = cdiv(PL, 256);
  if (need <= 1) return 1;
  if (need <= 2) return 2;
  if (need <= 3) return 3;
  if (need <= 5) return 5;
  if (need <= 8) return 8;
  return 0;
}

// One workgroup tile = one (WGM, MB, NB): instantiates the kernels, raises their LDS limit, launches.
template <int WGM, int MB, int NB>
struct ConvTile {
  template <int TAPS, int KC, int BSLOTS>
  static hipError_t attr() {
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_mfma_kernel<TAPS, KC, WGM, MB, NB, BSLOTS>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, MAX_LDS);
  }
  static hipError_t init() {
    hipError_t e;
    if ((e = attr<1, KC1, 1>()) != hipSuccess) return e;
    if ((e = attr<9, KC9, 1>()) != hipSuccess) return e;
    if ((e = attr<9, KC9, 2>()) != hipSuccess) return e;
    if ((e = attr<9, KC9, 3>()) != hipSuccess) return e;
    if ((e = attr<9, KC9, 5>()) != hipSuccess) return e;
    return attr<9, KC9, 8>();
  }
  static hipError_t launch(int taps, const ConvArgs &a, hipStream_t s) {
    const dim3 grid(a.g.n_ptiles, a.g.mtiles), block(256);
    const int bs = conv_bslots_for(a.g.PL);
    if (taps == 1) {
      if (bs != 1) return hipErrorInvalidValue;
      hipLaunchKernelGGL((conv_mfma_kernel<1, KC1, WGM, MB, NB, 1>), grid, block, a.g.lds_bytes, s, a);
    } else if (taps == 9) {
      switch (bs) {
        case 1: hipLaunchKernelGGL((conv_mfma_kernel<9, KC9, WGM, MB, NB, 1>), grid, block, a.g.lds_bytes, s, a); break;
        case 2: hipLaunchKernelGGL((conv_mfma_kernel<9, KC9, WGM, MB, NB, 2>), grid, block, a.g.lds_bytes, s, a); break;
        case 3: hipLaunchKernelGGL((conv_mfma_kernel<9, KC9, WGM, MB, NB, 3>), grid, block, a.g.lds_bytes, s, a); break;
        case 5: hipLaunchKernelGGL((conv_mfma_kernel<9, KC9, WGM, MB, NB, 5>), grid, block, a.g.lds_bytes, s, a); break;
        case 8: hipLaunchKernelGGL((conv_mfma_kernel<9, KC9, WGM, MB, NB, 8>), grid, block, a.g.lds_bytes, s, a); break;
        default: return hipErrorInvalidValue;
      }
    } else {
      return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
};

// tile ids (ConvGeom::tile): 0 = 128 ch x 128 px, 1 = 64 x 256, 2 = 64 x 128, 3 = 64 x 64
hipError_t conv_tile0_init();
hipError_t conv_tile1_init();
hipError_t conv_tile2_init();
hipError_t conv_tile3_init();
hipError_t conv_tile0_launch(int taps, const ConvArgs &a, hipStream_t s);
hipError_t conv_tile1_launch(int taps, const ConvArgs &a, hipStream_t s);
hipError_t conv_tile2_launch(int taps, const ConvArgs &a, hipStream_t s);
hipError_t conv_tile3_launch(int taps, const ConvArgs &a, hipStream_t s);

}  // namespace pbkd

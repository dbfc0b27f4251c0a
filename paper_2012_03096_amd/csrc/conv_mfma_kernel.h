// Device code of the implicit-GEMM convolution on the fp32 matrix cores (see conv_mfma.hip for the
// overview).  Included by the translation units that instantiate one workgroup tile each.
#pragma once
#include "pbkd_internal.h"

namespace pbkd {

typedef float floatx16 __attribute__((ext_vector_type(16)));


// Work split inside a workgroup of 8 waves: waves 0-3 do nothing but fetch MFMA operands from LDS and
// issue MFMAs (each owns a sub-tile of MB x NB blocks of 32 x 32); waves 4-7 are loaders: while the
// matrix cores work on chunk k from LDS copy k&1 they fetch chunk k+1 from global memory (weights as
// contiguous 16-byte vectors of the pre-packed image, the input halo tile element by element), apply the
// producing layer's BatchNorm+ReLU, and write copy (k+1)&1.  One barrier per chunk hands over.  Keeping
// vector-memory instructions out of the MFMA waves matters: issuing them between MFMAs cost those waves
// about a quarter of their matrix throughput, whatever the data's latency.  In the MFMA waves the LDS
// operands of step t+1 are fetched before the MFMAs of step t issue, fenced so the compiler keeps it so.
template <int VW> struct VecOf;
template <> struct VecOf<4> { typedef float type __attribute__((ext_vector_type(4))); };
template <> struct VecOf<2> { typedef float type __attribute__((ext_vector_type(2))); };

template <int TAPS, int KC, int WGM, int MB, int NB, int BSLOTS>
__global__ __launch_bounds__(512) void conv_mfma_kernel(ConvArgs p) {
  constexpr int WGN = 4 / WGM;
  constexpr int BM = WGM * MB * 32;     // output channels per workgroup
  constexpr int WN = NB * 32;           // pixels per wave
  constexpr int PAD = (TAPS == 9) ? 1 : 0;
  constexpr int A_FLOATS = TAPS * KC * BM;
  constexpr int A_PT = A_FLOATS / 256;          // weights staged per loader thread and chunk
  constexpr int VW = (A_PT % 4 == 0) ? 4 : 2;
  constexpr int NA = A_PT / VW;                 // vector loads of weights per loader thread and chunk
  constexpr int T = TAPS * KC / 2;              // MFMA steps (K = 2 each) per chunk
  static_assert(A_FLOATS % 256 == 0 && A_PT % VW == 0, "weight tile must divide evenly over the loader waves");
  typedef typename VecOf<VW>::type avec_t;
  extern __shared__ float smem[];
  const int PL = p.g.PL;
  float *As = smem;                    // [2][TAPS*KC][BM]
  float *Bs = smem + 2 * A_FLOATS;     // [2][KC][PL]

  const bool loader = threadIdx.x >= 256;
  const int tid = threadIdx.x & 255, lane = tid & 63, wave = tid >> 6;
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
  const int IH = p.g.IH, IW = p.g.IW, IWS = p.g.IWS, IMS = p.g.IMS;
  const int s = p.stride;
  const int HWo = p.Ho * p.Wo;
  const int HW = p.H * p.W;
  const int IHW = IH * IW;
  const int nchunks = p.g.nchunks;

  floatx16 acc[MB][NB];
#pragma unroll
  for (int a = 0; a < MB; ++a)
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  // where this lane's pixel columns sit in the staged tile and in the output (MFMA waves)
  int pixoff[NB];
  bool pvalid[NB];
  size_t outoff[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int pn = wn * WN + nb * 32 + l31;
    const int img = pn >> (lTW + lTH);
    const int rem = pn & (TH * TW - 1);
    const int i = rem >> lTW, j = rem & (TW - 1);
    pixoff[nb] = img * IMS + (s * i) * IWS + s * j + lh * PL;
    const int n = n0 + img, y = y0 + i, x = x0 + j;
    pvalid[nb] = (n < p.N) && (y < p.Ho) && (x < p.Wo) && !loader;
    outoff[nb] = (size_t)n * p.Cout * HWo + (size_t)y * p.Wo + x;
  }

  if (loader) {
    // ------------------------------------------------------------------ loader waves
    const bool bn = (p.in_scale != nullptr);
    ptrdiff_t goff[BSLOTS];
    int loff[BSLOTS];      // where the element goes in the staged tile; -1: this slot is beyond the tile
    bool gok[BSLOTS];
#pragma unroll
    for (int sl = 0; sl < BSLOTS; ++sl) {
      const int q = tid + 256 * sl;
      const int img = q / IHW;
      const int r = q - img * IHW;
      const int iy = r / IW;
      const int ix = r - iy * IW;
      const int n = n0 + img, y = y0 * s - PAD + iy, x = x0 * s - PAD + ix;
      const bool in_tile = q < p.g.PLd;
      gok[sl] = in_tile && (n < p.N) && (y >= 0) && (y < p.H) && (x >= 0) && (x < p.W);
      goff[sl] = (ptrdiff_t)n * p.Cin * HW + (ptrdiff_t)y * p.W + x;
      loff[sl] = in_tile ? img * IMS + iy * IWS + ix : -1;
    }
    const float *wsrc = p.wpk + (size_t)blockIdx.y * nchunks * A_FLOATS + (size_t)tid * VW;
    for (int k = 0; k <= nchunks; ++k) {
      if (k < nchunks) {
        avec_t avec[NA];
        float breg[BSLOTS][KC];
#pragma unroll
        for (int i = 0; i < NA; ++i)
          avec[i] = *reinterpret_cast<const avec_t *>(wsrc + (size_t)k * A_FLOATS + (size_t)i * 256 * VW);
#pragma unroll
        for (int sl = 0; sl < BSLOTS; ++sl)
#pragma unroll
          for (int kc = 0; kc < KC; ++kc) {
            const int c = k * KC + kc;
            breg[sl][kc] = (gok[sl] && c < p.Cin) ? p.in[goff[sl] + (ptrdiff_t)c * HW] : 0.f;
          }
        float *Ad = As + (k & 1) * A_FLOATS;
        float *Bd = Bs + (k & 1) * KC * PL;
#pragma unroll
        for (int i = 0; i < NA; ++i) *reinterpret_cast<avec_t *>(Ad + (tid + 256 * i) * VW) = avec[i];
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
          const int c = k * KC + kc;
          const bool on = bn && (c < p.Cin);
          const float sc = on ? p.in_scale[c] : 1.f, sh = on ? p.in_shift[c] : 0.f;
#pragma unroll
          for (int sl = 0; sl < BSLOTS; ++sl) {
            if (loff[sl] >= 0) {
              float v = breg[sl][kc];
              if (bn && gok[sl]) v = fmaxf(fmaf(v, sc, sh), 0.f);   // padding stays exactly zero
              Bd[kc * PL + loff[sl]] = v;
            }
          }
        }
      }
      __syncthreads();   // copy k&1 is complete; the MFMA waves have finished chunk k-1
    }
  } else {
    // ------------------------------------------------------------------ MFMA waves
    const int aoff = wm * (MB * 32) + l31 + lh * BM;
    __syncthreads();     // chunk 0 is staged
    for (int k = 0; k < nchunks; ++k) {
      const float *Ab = As + (k & 1) * A_FLOATS + aoff;
      const float *Bb = Bs + (k & 1) * KC * PL;
      float av[MB], bv[NB];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) av[mb] = Ab[32 * mb];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) bv[nb] = Bb[pixoff[nb]];
#pragma unroll
      for (int t = 0; t < T; ++t) {
        float nav[MB], nbv[NB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) nav[mb] = 0.f;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) nbv[nb] = 0.f;
        if (t + 1 < T) {
          const int tap = (t + 1) / (KC / 2), kk = 2 * ((t + 1) % (KC / 2));
          const int toff = (tap / 3) * IWS + (tap % 3);
#pragma unroll
          for (int mb = 0; mb < MB; ++mb) nav[mb] = Ab[(tap * KC + kk) * BM + 32 * mb];
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) nbv[nb] = Bb[kk * PL + pixoff[nb] + toff];
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
      __syncthreads();   // chunk k consumed: its LDS copy may be overwritten; copy (k+1)&1 is ready
    }
  }

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
        s1 = half32_sum(s1);
        s2 = half32_sum(s2);
        if (l31 == 0 && !loader) {
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
    if ((e = attr<9, KC9, 1>()) != hipSuccess) return e;
    if ((e = attr<9, KC9, 2>()) != hipSuccess) return e;
    if ((e = attr<9, KC9, 3>()) != hipSuccess) return e;
    if ((e = attr<9, KC9, 5>()) != hipSuccess) return e;
    return attr<9, KC9, 8>();
  }
  static hipError_t launch(int taps, const ConvArgs &a, hipStream_t s) {
    const dim3 grid(a.g.n_ptiles, a.g.mtiles), block(512);
    const int bs = conv_bslots_for(a.g.PLd);
    if (taps == 9) {
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

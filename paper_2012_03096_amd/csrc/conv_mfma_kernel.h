// Device code of the implicit-GEMM convolution on the fp32 matrix cores (see conv_mfma.hip for the
// overview).  Included by the translation units that instantiate one workgroup tile each.
#pragma once
#include <hip/hip_ext.h>

#include "pbkd_internal.h"

namespace pbkd {

typedef float floatx16 __attribute__((ext_vector_type(16)));


// Work split inside a workgroup of 8 waves: waves 0-3 do nothing but fetch MFMA operands from LDS and
// issue MFMAs (each owns a sub-tile of MB x NB blocks of 32 x 32); waves 4-7 are loaders: while the
// matrix cores work on chunk k (8 input channels x 9 taps) from LDS copy k&1 they fetch chunk k+1 from
// global memory (weights as contiguous 16-byte vectors of the pre-packed image, the input halo tile
// element by element), apply the producing layer's BatchNorm+ReLU, and write copy (k+1)&1.  One barrier per
// chunk hands over.  Keeping vector-memory instructions out of the MFMA waves matters: issuing them between
// MFMAs cost those waves about a quarter of their matrix throughput, whatever the data's latency.
//
// LDS layout: both operands keep the four channels 4h..4h+3 (h = half-wave) of a position adjacent, weights
// as [tap][h][row][4] and the halo tile as [h][pixel][4], so that an MFMA lane fetches the operands of the
// four K-steps of a tap with ONE 16-byte read each; step e pairs channels e and 4+e (a dot product does not
// care about the order of its terms).  Eight consecutive lanes read 128 consecutive bytes: no bank
// conflicts.  The operands of tap t+1 are fetched before the 4*MB*NB MFMAs of tap t issue, fenced so the
// compiler keeps it so.
template <int VW> struct VecOf;
template <> struct VecOf<4> { typedef float type __attribute__((ext_vector_type(4))); };
template <> struct VecOf<2> { typedef float type __attribute__((ext_vector_type(2))); };

// vector load through a buffer descriptor: descriptor base + scalar byte offset + lane byte offset
template <int VW> struct BufLoad;
template <> struct BufLoad<4> {
  typedef unsigned raw_t __attribute__((ext_vector_type(4)));
  static __device__ __forceinline__ VecOf<4>::type load(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
    return __builtin_bit_cast(VecOf<4>::type, __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0));
  }
};
template <> struct BufLoad<2> {
  typedef unsigned raw_t __attribute__((ext_vector_type(2)));
  static __device__ __forceinline__ VecOf<2>::type load(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
    return __builtin_bit_cast(VecOf<2>::type, __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0));
  }
};

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
  static_assert(KC == 8, "two half-waves x four channels per tap");
  static_assert(A_FLOATS % 256 == 0 && A_PT % VW == 0, "weight tile must divide evenly over the loader waves");
  typedef typename VecOf<VW>::type avec_t;
  typedef float f4 __attribute__((ext_vector_type(4)));
  extern __shared__ float smem[];
  const int PL = p.g.PL;
  float *As = smem;                    // [2][TAPS][2][BM][4]
  float *Bs = smem + 2 * A_FLOATS;     // [2][2][PL][4]

  const bool loader = threadIdx.x >= 256;
  const int tid = threadIdx.x & 255, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WGM, wn = wave / WGM;
  const int l31 = lane & 31, lh = lane >> 5;

  int pt = xcd_contiguous(blockIdx.x, gridDim.x);     // neighbouring pixel tiles (shared halo) on one die's L2
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
  // this workgroup's share of K: chunks [kb, kb + nk); the whole of it unless the launch splits K over gridDim.z
  const int kb = blockIdx.z * p.g.kchunks;
  const int nk = (nchunks - kb < p.g.kchunks) ? nchunks - kb : p.g.kchunks;
  float *const outp = (p.g.ksplit > 1) ? p.split_out + (size_t)blockIdx.z * ((size_t)p.N * p.Cout * HWo) : p.out;

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
    pixoff[nb] = img * IMS + (s * i) * IWS + s * j;
    const int n = n0 + img, y = y0 + i, x = x0 + j;
    pvalid[nb] = (n < p.N) && (y < p.Ho) && (x < p.Wo) && !loader;
    outoff[nb] = (size_t)n * p.Cout * HWo + (size_t)y * p.Wo + x;
  }

  if (loader) {
    // ------------------------------------------------------------------ loader waves
    // While the MFMA wave of a SIMD streams MFMAs, any other wave there gets roughly one instruction issued
    // per MFMA (measured: ~100 instructions took a whole chunk of 144 MFMAs, whatever the wave priority).
    // So the loader's budget is instructions, not bytes: every address is a wave-uniform 64-bit base (scalar
    // arithmetic) plus a per-lane 32-bit byte offset that never changes, nothing is predicated (positions
    // outside the image read element 0 and are zeroed by a select; channels past Cin are clamped, their
    // weights are zero), and BatchNorm's scale and shift come through scalar loads.
    const bool bn = (p.in_scale != nullptr);
    unsigned goff[BSLOTS];     // byte offset of the slot's pixel in channel 0 of its image (0 if outside)
    int loff[BSLOTS];          // where the element goes in the staged tile; -1: this slot is beyond the tile
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
      goff[sl] = gok[sl] ? (unsigned)((((size_t)n * p.Cin * HW) + (size_t)y * p.W + x) * sizeof(float)) : 0u;
      loff[sl] = in_tile ? img * IMS + iy * IWS + ix : -1;
    }
    // buffer addressing: 128-bit descriptor (base, size) in scalar registers + scalar byte offset + lane byte offset
    const __amdgpu_buffer_rsrc_t rin = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(p.in), 0, (int)((unsigned)p.N * p.Cin * HW * sizeof(float)), 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(p.wpk), 0, (int)((unsigned)gridDim.y * nchunks * A_FLOATS * sizeof(float)), 0x00020000);
    const unsigned aoff = (unsigned)(tid * VW * sizeof(float));
    const unsigned chb = (unsigned)(HW * sizeof(float));       // bytes between channels
    const float lo = bn ? 0.f : -__builtin_inff();             // ReLU only where there is a BatchNorm to apply
    // positions of the halo outside the image are zero for every chunk: write them once, in both copies
#pragma unroll
    for (int sl = 0; sl < BSLOTS; ++sl)
      if (loff[sl] >= 0 && !gok[sl]) {
        const f4 zero4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int cp = 0; cp < 2; ++cp)
#pragma unroll
          for (int h = 0; h < 2; ++h) *reinterpret_cast<f4 *>(Bs + cp * KC * PL + ((size_t)h * PL + loff[sl]) * 4) = zero4;
      }
    for (int kk = 0; kk <= nk; ++kk) {
      const int k = kb + kk;
      if (kk < nk) {
        avec_t avec[NA];
        float breg[BSLOTS][KC];
        float sc[KC], sh[KC];
        const unsigned wk = (unsigned)(((size_t)blockIdx.y * nchunks + k) * A_FLOATS * sizeof(float));
#pragma unroll
        for (int i = 0; i < NA; ++i)
          avec[i] = BufLoad<VW>::load(rw, aoff, wk + (unsigned)(i * 256 * VW * sizeof(float)));
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) {
          int c = k * KC + kc;
          if (c > p.Cin - 1) c = p.Cin - 1;
#pragma unroll
          for (int sl = 0; sl < BSLOTS; ++sl)
            breg[sl][kc] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rin, goff[sl], (unsigned)c * chb, 0));
        }
#pragma unroll
        for (int kc = 0; kc < KC; ++kc) sc[kc] = 1.f, sh[kc] = 0.f;
        if (bn) {
          if ((k + 1) * KC <= p.Cin) {           // all eight channels exist: consecutive scalar loads
            const float *ps = p.in_scale + k * KC, *pt = p.in_shift + k * KC;
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) sc[kc] = ps[kc], sh[kc] = pt[kc];
          } else {
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) {
              int c = k * KC + kc;
              if (c > p.Cin - 1) c = p.Cin - 1;
              sc[kc] = p.in_scale[c], sh[kc] = p.in_shift[c];
            }
          }
        }
        float *Ad = As + (kk & 1) * A_FLOATS;
        float *Bd = Bs + (kk & 1) * KC * PL;
#pragma unroll
        for (int i = 0; i < NA; ++i) *reinterpret_cast<avec_t *>(Ad + (tid + 256 * i) * VW) = avec[i];
#pragma unroll
        for (int sl = 0; sl < BSLOTS; ++sl) {
#pragma unroll
          for (int kc = 0; kc < KC; ++kc) breg[sl][kc] = fmaxf(fmaf(breg[sl][kc], sc[kc], sh[kc]), lo);
          if (gok[sl]) {                             // the padding was zeroed once and is never written again
#pragma unroll
            for (int h = 0; h < 2; ++h) {
              const f4 v = {breg[sl][4 * h + 0], breg[sl][4 * h + 1], breg[sl][4 * h + 2], breg[sl][4 * h + 3]};
              *reinterpret_cast<f4 *>(Bd + ((size_t)h * PL + loff[sl]) * 4) = v;
            }
          }
        }
      }
      __syncthreads();   // copy kk&1 is complete; the MFMA waves have finished chunk kk-1
    }
  } else {
    // ------------------------------------------------------------------ MFMA waves
    const int aoff = (lh * BM + wm * (MB * 32) + l31) * 4;
    __syncthreads();     // chunk 0 is staged
    for (int kk = 0; kk < nk; ++kk) {
      const float *Ab = As + (kk & 1) * A_FLOATS + aoff;
      const float *Bb = Bs + (kk & 1) * KC * PL + lh * (PL * 4);
      f4 av[MB], bv[NB];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) av[mb] = *reinterpret_cast<const f4 *>(Ab + mb * 128);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) bv[nb] = *reinterpret_cast<const f4 *>(Bb + pixoff[nb] * 4);
#pragma unroll
      for (int tap = 0; tap < TAPS; ++tap) {
        f4 nav[MB], nbv[NB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) nav[mb] = av[mb];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) nbv[nb] = bv[nb];
        if (tap + 1 < TAPS) {
          const int toff = ((tap + 1) / 3) * IWS + ((tap + 1) % 3);
#pragma unroll
          for (int mb = 0; mb < MB; ++mb) nav[mb] = *reinterpret_cast<const f4 *>(Ab + (tap + 1) * (2 * BM * 4) + mb * 128);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) nbv[nb] = *reinterpret_cast<const f4 *>(Bb + (pixoff[nb] + toff) * 4);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
              acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[mb][e], bv[nb][e], acc[mb][nb], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) av[mb] = nav[mb];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) bv[nb] = nbv[nb];
      }
      __syncthreads();   // chunk kk consumed: its LDS copy may be overwritten; copy (kk+1)&1 is ready
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
          if (pvalid[nb]) outp[outoff[nb] + (size_t)o * HWo] = acc[mb][nb][r];
      }
    }

  // ---- per-channel statistics partial of this pixel tile, for BatchNorm's batch statistics.  Every wave sums about
  // the value of its own first pixel column (valid whenever any of the wave's pixels is: a wave covers whole images or
  // a run of rows of one image, and validity only ends with growing row and image index); the WGN waves' sums are
  // then re-expressed about the first one's pivot and added.
  if (p.stat_partial && p.g.ksplit == 1) {
    StatPart *red = reinterpret_cast<StatPart *>(smem);   // [WGN][BM]; the last chunk's barrier has already passed
    float cnt = 0.f;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) cnt += pvalid[nb] ? 1.f : 0.f;
    cnt = half32_sum(cnt);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float pv = __shfl(acc[mb][0][r], lane & 32, 64);
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const float d = pvalid[nb] ? acc[mb][nb][r] - pv : 0.f;
          s1 += d;
          s2 += d * d;
        }
        s1 = half32_sum(s1);
        s2 = half32_sum(s2);
        if (l31 == 0 && !loader) {
          const int row = wm * (MB * 32) + mb * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
          StatPart sp;
          sp.pivot = pv; sp.s1 = s1; sp.s2 = s2; sp.n = cnt;
          red[wn * BM + row] = sp;
        }
      }
    __syncthreads();
    for (int e = tid; e < BM; e += 256) {
      const int o = m0 + e;
      if (o < p.Cout && !loader) {
        StatPart a = red[e];
#pragma unroll
        for (int w = 1; w < WGN; ++w) stat_rebase_add(a, red[w * BM + e]);
        stat_store(p.stat_partial, (size_t)o * gridDim.x + blockIdx.x, a);
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
  template <int BSLOTS>
  static void go(const dim3 &grid, const dim3 &block, const ConvArgs &a, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
    if (e0 && e1)
      hipExtLaunchKernelGGL((conv_mfma_kernel<9, KC9, WGM, MB, NB, BSLOTS>), grid, block, (unsigned)a.g.lds_bytes, s, e0, e1, 0, a);
    else
      hipLaunchKernelGGL((conv_mfma_kernel<9, KC9, WGM, MB, NB, BSLOTS>), grid, block, a.g.lds_bytes, s, a);
  }
  static hipError_t launch(int taps, const ConvArgs &a, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
    if (a.g.ksplit < 1 || a.g.kchunks < 1 || (long long)(a.g.ksplit - 1) * a.g.kchunks >= a.g.nchunks ||
        (long long)a.g.ksplit * a.g.kchunks < a.g.nchunks || (a.g.ksplit > 1 && !a.split_out))
      return hipErrorInvalidValue;   // every split needs at least one chunk, and together they cover K
    const dim3 grid(a.g.n_ptiles, a.g.mtiles, a.g.ksplit), block(512);
    const int bs = conv_bslots_for(a.g.PLd);
    if (taps == 9) {
      switch (bs) {
        case 1: go<1>(grid, block, a, s, e0, e1); break;
        case 2: go<2>(grid, block, a, s, e0, e1); break;
        case 3: go<3>(grid, block, a, s, e0, e1); break;
        case 5: go<5>(grid, block, a, s, e0, e1); break;
        case 8: go<8>(grid, block, a, s, e0, e1); break;
        default: return hipErrorInvalidValue;
      }
    } else {
      return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
};

// the bf16-split kernels (conv_split.hip)
hipError_t conv_split_init();
hipError_t launch_conv_split(const ConvArgs &a, hipStream_t s, hipEvent_t e0, hipEvent_t e1);

// tile ids (ConvGeom::tile): 0 = 128 ch x 128 px, 1 = 64 x 256, 2 = 64 x 128, 3 = 64 x 64
hipError_t conv_tile0_init();
hipError_t conv_tile1_init();
hipError_t conv_tile2_init();
hipError_t conv_tile3_init();
hipError_t conv_tile0_launch(int taps, const ConvArgs &a, hipStream_t s, hipEvent_t e0, hipEvent_t e1);
hipError_t conv_tile1_launch(int taps, const ConvArgs &a, hipStream_t s, hipEvent_t e0, hipEvent_t e1);
hipError_t conv_tile2_launch(int taps, const ConvArgs &a, hipStream_t s, hipEvent_t e0, hipEvent_t e1);
hipError_t conv_tile3_launch(int taps, const ConvArgs &a, hipStream_t s, hipEvent_t e0, hipEvent_t e1);

}  // namespace pbkd

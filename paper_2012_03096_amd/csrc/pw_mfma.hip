// 1x1 convolution (the student's pointwise conv, its data gradient, the projection shortcut) on the fp32
// matrix cores, written for what bounds it: HBM.  z[n,o,p] = sum_c A[o,c] * in[n,c,p].
//
// The weight matrix is small, the pixel dimension huge, and in NCHW consecutive pixels of one channel are
// contiguous bytes.  So the activations never touch LDS: every wave loads its B operands straight from
// global memory into registers, coalesced, through a ring of PW_D steps in flight, and only the weights
// (all K rows of the workgroup's channel tile, at most 128 x 128 floats per stage) are staged in LDS once
// per 128 input channels.  After that staging no barrier is needed: the four waves of a workgroup run
// independently.  Two kernels: pw_mfma_kernel (one pixel per lane and MFMA column, any stride and shape) and
// pw_mfma_vec_kernel (2 or 4 adjacent pixels per lane, stride 1 and even H*W; the one the benchmarks run).
#include <cstdlib>

#include "conv_mfma_kernel.h"

namespace pbkd {

#ifndef PBKD_PW_D
#define PBKD_PW_D 8
#endif
constexpr int PW_D = PBKD_PW_D;        // B-operand loads in flight per wave, in MFMA steps
constexpr int PW_KS = 128;     // input channels per LDS stage of the weights

template <int MB, int NB>
__global__ __launch_bounds__(256, 2) void pw_mfma_kernel(PwArgs p) {
  constexpr int BM = MB * 32;
  extern __shared__ float smem[];   // [PW_KS][BM]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l31 = lane & 31, lh = lane >> 5;
  // workgroup -> (pixel tile bxl, channel tile byl): the channel tiles of one pixel tile read the same activations, so
  // they are made neighbours on one die (channel tile fastest, a contiguous range of pixel tiles per die)
  const int lin = xcd_contiguous(blockIdx.x + gridDim.x * blockIdx.y, gridDim.x * gridDim.y);
  const int byl = lin % gridDim.y, bxl = lin / gridDim.y;
  const int m0 = byl * BM;
  const int HWo = p.Ho * p.Wo;
  const long long P = (long long)p.N * HWo;
  const int nsteps = p.nchunks * (KC1 / 2);    // MFMA steps over the zero-padded K

  ptrdiff_t inoff[NB];
  size_t outoff[NB];
  bool pvalid[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    long long g = ((long long)bxl * 4 + wave) * (NB * 32) + nb * 32 + l31;
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

  const float *wsrc = p.wpk + (size_t)byl * p.nchunks * (KC1 * BM);
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

  // ---- per-channel statistics partial over this workgroup's pixels, for BatchNorm: every wave sums about the value of
  // its first pixel (valid whenever any of its pixels is: validity ends with growing pixel index), then the four
  // waves' sums are re-expressed about the first one's pivot and added
  if (p.stat_partial) {
    __syncthreads();
    StatPart *red = reinterpret_cast<StatPart *>(smem);   // [4 waves][BM]
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
        if (l31 == 0) {
          const int row = mb * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
          StatPart sp;
          sp.pivot = pv; sp.s1 = s1; sp.s2 = s2; sp.n = cnt;
          red[wave * BM + row] = sp;
        }
      }
    __syncthreads();
    for (int e = tid; e < BM; e += 256) {
      const int o = m0 + e;
      if (o < p.Cout) {
        StatPart a = red[e];
#pragma unroll
        for (int w = 1; w < 4; ++w) stat_rebase_add(a, red[w * BM + e]);
        stat_store(p.stat_partial, (size_t)o * gridDim.x + bxl, a);
      }
    }
  }
}

// ---- stride 1 and H*W a multiple of VW (4 or 2): VW pixels per lane.
// The 32 columns of an MFMA need not be adjacent pixels: lane n of a half-wave loads pixels VW*n .. VW*n+VW-1
// of a channel row as one vector (a half-wave reads VW*128 contiguous bytes), and MFMA e of VW uses element e,
// so its column n is pixel VW*n + e; the VW accumulators of a lane then hold VW adjacent pixels of every
// output row and are stored as one vector.  A quarter of the load instructions for four times the bytes
// in flight.  The four waves of a workgroup are WM channel blocks of 32 x WP groups of VW*32 pixels;
// waves that share pixels fetch the same lines (L1 hits), waves that share channels the same weights.
template <int WM, int WP, int VW>
__global__ __launch_bounds__(256) void pw_mfma_vec_kernel(PwArgs p) {
  static_assert(WM * WP == 4 && (VW == 4 || VW == 2), "four waves; 2 or 4 pixels per lane");
  constexpr int BM = WM * 32;
  typedef float vec_t __attribute__((ext_vector_type(VW)));
  extern __shared__ float smem[];   // [PW_KS][BM]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l31 = lane & 31, lh = lane >> 5;
  const int wm = wave % WM, wp = wave / WM;
  // workgroup -> (pixel tile bxl, channel tile byl): the channel tiles of one pixel tile read the same activations, so
  // they are made neighbours on one die (channel tile fastest, a contiguous range of pixel tiles per die)
  const int lin = xcd_contiguous(blockIdx.x + gridDim.x * blockIdx.y, gridDim.x * gridDim.y);
  const int byl = lin % gridDim.y, bxl = lin / gridDim.y;
  const int m0 = byl * BM + wm * 32;
  const int HW = p.Ho * p.Wo;                  // == HWin (stride 1)
  const long long P = (long long)p.N * HW;
  const int tlast = (p.Cin + 1) / 2 - 1;       // last MFMA step (K = 2 each) that reads a real channel
  const int nsteps = (tlast / PW_D + 1) * PW_D;   // whole groups of PW_D steps; those past tlast meet zero weights
  const bool odd = p.Cin & 1;

  long long g = ((long long)bxl * WP + wp) * (VW * 32) + VW * l31;
  const bool pvalid = g < P;                   // P % VW == 0: the lane's pixels are valid together
  if (!pvalid) g = P - VW;                     // read real pixels, never store them
  const int n = (int)(g / HW);
  const int r0 = (int)(g - (long long)n * HW);
  float *dst = p.out + (size_t)n * p.Cout * HW + r0;
  // Step t reads channel 2t + lh: a base address that is the same for the whole wave (2t rows of H*W floats)
  // plus a per-lane byte offset that never changes (the input is smaller than 4 GiB, checked at launch).
  // With an odd channel count the upper half-wave repeats channel Cin-1 in the last step (zero weight).
  const unsigned off0 = (unsigned)(((size_t)n * p.Cin * HW + r0) * sizeof(float));
  const unsigned off1 = off0 + (unsigned)(lh * HW * sizeof(float));
  const char *inb = reinterpret_cast<const char *>(p.in);
  const size_t stepb = (size_t)2 * HW * sizeof(float);
  const char *const lastb = inb + (size_t)tlast * stepb;
  const unsigned offl = odd ? off0 : off1;     // lane offset in the last real step
  const char *nextb = inb;                     // base of the next step to fetch
  auto bload = [&]() -> vec_t {
    const bool tail = nextb >= lastb;          // wave-uniform
    const char *base = tail ? lastb : nextb;
    const unsigned off = tail ? offl : off1;
    nextb += stepb;
    return *reinterpret_cast<const vec_t *>(base + off);
  };

  floatx16 acc[VW];
#pragma unroll
  for (int e = 0; e < VW; ++e)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[e][r] = 0.f;

  // weights of one stage (up to PW_KS channels = 4 chunks of 16 steps): global -> registers -> LDS
  typedef float f4 __attribute__((ext_vector_type(4)));
  constexpr int WPT = BM / 32;                 // 16-byte vectors per thread and chunk
  const f4 *wsrc4 = reinterpret_cast<const f4 *>(p.wpk + (size_t)byl * p.nchunks * (KC1 * BM));
  f4 wreg[4][WPT];
  auto wfetch = [&](int s0, int steps) {
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (c * 16 < steps) {
#pragma unroll
        for (int jj = 0; jj < WPT; ++jj) wreg[c][jj] = wsrc4[(size_t)(s0 / 16 + c) * 8 * BM + tid + 256 * jj];
      }
  };
  auto wstash = [&](int steps) {
    f4 *wdst4 = reinterpret_cast<f4 *>(smem);
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (c * 16 < steps) {
#pragma unroll
        for (int jj = 0; jj < WPT; ++jj) wdst4[c * 8 * BM + tid + 256 * jj] = wreg[c][jj];
      }
  };

  // the (fast, L2-resident) weight loads go first: loads return in order, and the stash must not wait for
  // the activation loads behind them
  wfetch(0, nsteps < PW_KS / 2 ? nsteps : PW_KS / 2);
  vec_t ring[PW_D];
#pragma unroll
  for (int d = 0; d < PW_D; ++d) ring[d] = bload();

  const int aoff = wm * 32 + l31 + lh * BM;
  for (int s0 = 0; s0 < nsteps; s0 += PW_KS / 2) {
    const int steps = (nsteps - s0 < PW_KS / 2) ? nsteps - s0 : PW_KS / 2;   // multiple of PW_D
    if (s0 > 0) {
      __syncthreads();
      wfetch(s0, steps);
    }
    wstash(steps);
    __syncthreads();
    float av = smem[aoff];
    for (int tt = 0; tt < steps; tt += PW_D) {
      const float *arow = smem + (size_t)tt * 2 * BM + aoff;
#pragma unroll
      for (int d = 0; d < PW_D; ++d) {
        const vec_t bv = ring[d];
        ring[d] = bload();
        const float nav = arow[(d + 1) * 2 * BM];   // next step's weights; one row pair past the stage is allocated, unused
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int e = 0; e < VW; ++e) acc[e] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv[e], acc[e], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        av = nav;
      }
    }
  }

  // ---- store: accumulator register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4; column l%32 = pixels VW*(l%32)+e
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int o = m0 + 8 * (r / 4) + 4 * lh + (r % 4);
    if (o < p.Cout && pvalid) {
      vec_t v;
#pragma unroll
      for (int e = 0; e < VW; ++e) v[e] = acc[e][r];
      *reinterpret_cast<vec_t *>(dst + (size_t)o * HW) = v;
    }
  }

  // ---- per-channel statistics partial over this workgroup's pixels, for BatchNorm (as in pw_mfma_kernel: per-wave
  // sums about the wave's first pixel, re-expressed about one pivot and added).  On the vector ALU only: the pivot through two lane reads, the half-wave sums
  // by DPP with the total arriving in the half-wave's upper 16 lanes (LDS permutes made 48 dependent round trips of it).
  if (p.stat_partial) {
    __syncthreads();
    StatPart *red = reinterpret_cast<StatPart *>(smem);   // [WP][BM]
    const float cnt = half32_sum_upper(pvalid ? (float)VW : 0.f);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float a0 = acc[0][r];
      const float p0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a0), 0));
      const float p1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a0), 32));
      const float pv = lh ? p1 : p0;
      float s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int e = 0; e < VW; ++e) {
        const float d = pvalid ? acc[e][r] - pv : 0.f;
        s1 += d;
        s2 += d * d;
      }
      s1 = half32_sum_upper(s1);
      s2 = half32_sum_upper(s2);
      if (l31 == 16) {
        const int row = wm * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
        StatPart sp;
        sp.pivot = pv; sp.s1 = s1; sp.s2 = s2; sp.n = cnt;
        red[wp * BM + row] = sp;
      }
    }
    __syncthreads();
    for (int e = tid; e < BM; e += 256) {
      const int o = byl * BM + e;
      if (o < p.Cout) {
        StatPart a = red[e];
#pragma unroll
        for (int w = 1; w < WP; ++w) stat_rebase_add(a, red[w * BM + e]);
        stat_store(p.stat_partial, (size_t)o * gridDim.x + bxl, a);
      }
    }
  }
}


// ---- few pixels, many channels (4x4 and 2x2 feature maps with 256..512 channels): the tiles above would leave
// most of the chip idle and run a long K loop per wave.  Here a workgroup owns one block of 32 channels x VW*32
// pixels and its four waves split K in four contiguous parts; with 32-channel weight tiles the packed layout
// makes a step's A operand 64 consecutive floats, so both operands come straight from global memory through
// the ring and LDS only carries the final sum of the four partial accumulators (added in wave order).
template <int VW>
__global__ __launch_bounds__(256) void pw_mfma_ksplit_kernel(PwArgs p) {
  // operand loads in flight per wave, in MFMA steps: with one pixel per lane a step is a single MFMA and the short
  // K loop is bound by load latency, so the ring is deeper there (measured: 10 -> 8.5 us per launch at 2x2x512)
  constexpr int KS_D = (VW == 1) ? 16 : 8;
  static_assert(16 % KS_D == 0, "a wave's K range is a whole number of ring rounds");
  typedef float vec_t __attribute__((ext_vector_type(VW)));
  extern __shared__ float smem[];   // [4 waves][16*VW][64]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l31 = lane & 31, lh = lane >> 5;
  // workgroup -> (pixel tile bxl, channel tile byl): the channel tiles of one pixel tile read the same activations, so
  // they are made neighbours on one die (channel tile fastest, a contiguous range of pixel tiles per die)
  const int lin = xcd_contiguous(blockIdx.x + gridDim.x * blockIdx.y, gridDim.x * gridDim.y);
  const int byl = lin % gridDim.y, bxl = lin / gridDim.y;
  const int m0 = byl * 32;
  const int HW = p.Ho * p.Wo;
  const long long P = (long long)p.N * HW;
  const int total = p.nchunks * 16;                 // MFMA steps over the zero-padded K
  const int per_wave = ((total + 3) / 4 + KS_D - 1) / KS_D * KS_D;
  const int t_begin = wave * per_wave;
  const int t_end = (t_begin + per_wave < total) ? t_begin + per_wave : total;   // multiple of KS_D (total % 16 == 0)

  long long g = (long long)bxl * (VW * 32) + VW * l31;
  const bool pvalid = g < P;
  if (!pvalid) g = P - VW;                          // read real pixels, never store them
  const int n = (int)(g / HW);
  const int r0 = (int)(g - (long long)n * HW);
  const float *src = p.in + (size_t)n * p.Cin * HW + r0;
  const float *wsrc = p.wpk + (size_t)byl * p.nchunks * 1024 + lane;
  auto bload = [&](int t) -> vec_t {
    int k = 2 * t + lh;
    if (k > p.Cin - 1) k = p.Cin - 1;               // padded K: the weight rows are zero there
    return *reinterpret_cast<const vec_t *>(src + (size_t)k * HW);
  };

  floatx16 acc[VW];
#pragma unroll
  for (int e = 0; e < VW; ++e)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[e][r] = 0.f;

  if (t_begin < t_end) {
    vec_t rb[KS_D];
    float ra[KS_D];
#pragma unroll
    for (int d = 0; d < KS_D; ++d) {
      ra[d] = wsrc[(size_t)(t_begin + d) * 64];
      rb[d] = bload(t_begin + d);
    }
    for (int t = t_begin; t < t_end; t += KS_D) {
#pragma unroll
      for (int d = 0; d < KS_D; ++d) {
        const float av = ra[d];
        const vec_t bv = rb[d];
        int tn = t + d + KS_D;
        if (tn > total - 1) tn = total - 1;         // past the end: a valid address, the value is never used
        ra[d] = wsrc[(size_t)tn * 64];
        rb[d] = bload(tn);
#pragma unroll
        for (int e = 0; e < VW; ++e) acc[e] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv[e], acc[e], 0, 0, 0);
      }
    }
  }

  // ---- the four partial accumulators meet in LDS; wave w then finishes accumulator registers 4w..4w+3,
  // i.e. rows 8w + 4*(lane/32) + 0..3 of the channel block, for all of the tile's pixels
#pragma unroll
  for (int e = 0; e < VW; ++e)
#pragma unroll
    for (int r = 0; r < 16; ++r) smem[((wave * 16 + r) * VW + e) * 64 + lane] = acc[e][r];
  __syncthreads();
  float *dst = p.out + (size_t)n * p.Cout * HW + r0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int r = 4 * wave + j;
    const int o = m0 + 8 * wave + 4 * lh + j;
    vec_t v;
#pragma unroll
    for (int e = 0; e < VW; ++e) {
      float sum = smem[((0 * 16 + r) * VW + e) * 64 + lane];
#pragma unroll
      for (int w = 1; w < 4; ++w) sum += smem[((w * 16 + r) * VW + e) * 64 + lane];
      v[e] = sum;
    }
    if (o < p.Cout && pvalid) *reinterpret_cast<vec_t *>(dst + (size_t)o * HW) = v;
    if (p.stat_partial) {                           // per-channel statistics partial over this tile's pixels, about its first
      const float pv = __shfl(v[0], lane & 32, 64);
      float s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int e = 0; e < VW; ++e) {
        const float d = pvalid ? v[e] - pv : 0.f;
        s1 += d;
        s2 += d * d;
      }
      s1 = half32_sum(s1);
      s2 = half32_sum(s2);
      const float cnt = half32_sum(pvalid ? (float)VW : 0.f);
      if (l31 == 0 && o < p.Cout) {
        StatPart a;
        a.pivot = pv; a.s1 = s1; a.s2 = s2; a.n = cnt;
        stat_store(p.stat_partial, (size_t)o * gridDim.x + bxl, a);
      }
    }
  }
}

// Vector variants 4..9 = (WM, WP, VW): (4,1,4) (4,1,2) (2,2,4) (2,2,2) (1,4,4) (1,4,2)
static const int kVecWM[6] = {4, 4, 2, 2, 1, 1}, kVecWP[6] = {1, 1, 2, 2, 4, 4}, kVecVW[6] = {4, 2, 4, 2, 4, 2};

PwGeom pw_geom(int N, int Cin, int Cout, int Ho, int Wo, int stride) {
  const long long P = (long long)N * Ho * Wo;
  const int HW = Ho * Wo;
  int forced = -1;                                            // PBKD_PW_VARIANT=0..9: tuning aid
  if (const char *env = std::getenv("PBKD_PW_VARIANT")) forced = std::atoi(env);
  const bool small_in = (unsigned long long)N * Cin * HW * sizeof(float) < (1ull << 32);   // 32-bit lane offsets
  if (stride == 1 && HW % 2 == 0 && small_in && !(forced >= 0 && forced <= 3)) {
    const int wmi = Cout > 64 ? 0 : (Cout > 32 ? 2 : 4);     // index of the (WM, WP) pair with VW = 4
    auto blocks = [&](int i) {
      const long long px = (long long)kVecWP[i] * kVecVW[i] * 32;
      return (long long)cdiv(Cout, kVecWM[i] * 32) * ((P + px - 1) / px);
    };
    int i = wmi;
    // 33..64 output channels over a large map: two 32-channel tiles of 512 pixels (die-aware numbering puts them next to
    // each other on one die, so the second read of the input hits that die's L2) measured faster than one 64 x 256 tile
    // (ImageNet-sized block, 64 -> 64 at 224 x 224 x 32: forward 203 -> 194 us, data gradient 168 -> 164 us; CIFAR-sized
    // maps measured level, so the rule asks for a grid of several waves of workgroups)
    if (wmi == 2 && HW % 4 == 0 && blocks(4) >= 2048) i = 4;
    if (HW % 4 != 0 || blocks(i) < 256) i = wmi + 1;          // narrower vectors: twice the workgroups
    if (forced >= 4 && forced <= 9 && (kVecVW[forced - 4] == 2 || HW % 4 == 0)) i = forced - 4;
    // still fewer workgroups than compute units, or only the narrow vectors reach that many, and a K loop worth
    // splitting: 32 x VW*32 blocks, K over the waves
    const bool narrow = HW % 4 == 0 && i == wmi + 1 && Cin >= 256;   // (measured: at K = 128 the two are level)
    if ((forced < 0 && (blocks(i) < 256 || narrow) && Cin >= 128) || (forced >= 10 && forced <= 12)) {
      auto kblocks = [&](int vw) { return (long long)cdiv(Cout, 32) * ((P + 32 * vw - 1) / (32 * vw)); };
      int vw = (HW % 4 == 0 && kblocks(4) >= 256) ? 4 : (kblocks(2) >= 256 ? 2 : 1);
      if (forced == 10 && HW % 4 == 0) vw = 4;
      if (forced == 11) vw = 2;
      if (forced == 12) vw = 1;
      PwGeom g;
      g.variant = vw == 4 ? 10 : (vw == 2 ? 11 : 12);
      g.bm = 32;
      g.mtiles = cdiv(Cout, 32);
      g.nchunks = cdiv(Cin, KC1);
      g.a_floats = KC1 * g.bm;
      g.n_ptiles = (int)((P + 32 * vw - 1) / (32 * vw));
      g.lds_bytes = (size_t)4 * 16 * vw * 64 * sizeof(float);
      return g;
    }
    PwGeom g;
    g.variant = 4 + i;
    g.bm = kVecWM[i] * 32;
    g.mtiles = cdiv(Cout, g.bm);
    g.nchunks = cdiv(Cin, KC1);
    g.a_floats = KC1 * g.bm;
    const long long px = (long long)kVecWP[i] * kVecVW[i] * 32;
    g.n_ptiles = (int)((P + px - 1) / px);
    g.lds_bytes = (size_t)(PW_KS + 2) * g.bm * sizeof(float);
    return g;
  }
  // (MB, NB) = (channel blocks of 32 per workgroup, pixel blocks of 32 per wave).  Prefer the largest
  // tile that still gives two workgroups per compute unit; else the one with the most workgroups.
  static const int kMB[4] = {4, 4, 2, 2}, kNB[4] = {2, 1, 2, 1};
  auto blocks = [&](int v) { return (long long)cdiv(Cout, kMB[v] * 32) * ((P + 4 * kNB[v] * 32 - 1) / (4 * kNB[v] * 32)); };
  int v = 3;
  const int first = (Cout > 64) ? 0 : 2;
  for (int i = first; i < 4; ++i)
    if (blocks(i) >= 512) { v = i; break; }
  if (forced >= 0 && forced <= 3) v = forced;
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
#define PBKD_SETV(WM, WP, VW)                                                                               \
  e = hipFuncSetAttribute(reinterpret_cast<const void *>(&pw_mfma_vec_kernel<WM, WP, VW>),                  \
                          hipFuncAttributeMaxDynamicSharedMemorySize, MAX_LDS);                             \
  if (e != hipSuccess) return e;
  PBKD_SETV(4, 1, 4) PBKD_SETV(4, 1, 2) PBKD_SETV(2, 2, 4) PBKD_SETV(2, 2, 2) PBKD_SETV(1, 4, 4) PBKD_SETV(1, 4, 2)
#undef PBKD_SETV
#define PBKD_SETK(VW)                                                                                       \
  e = hipFuncSetAttribute(reinterpret_cast<const void *>(&pw_mfma_ksplit_kernel<VW>),                       \
                          hipFuncAttributeMaxDynamicSharedMemorySize, MAX_LDS);                             \
  if (e != hipSuccess) return e;
  PBKD_SETK(4) PBKD_SETK(2) PBKD_SETK(1)
#undef PBKD_SETK
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
    case 4: case 5: case 6: case 7: case 8: case 9: {
      const int vw = kVecVW[a.g.variant - 4];
      if (a.stride != 1 || (a.Ho * a.Wo) % vw || a.HWin != a.Ho * a.Wo || (size_t)a.N * a.Cin * a.HWin * sizeof(float) >= (1ull << 32) || (reinterpret_cast<uintptr_t>(a.in) & (4 * vw - 1)) ||
          (reinterpret_cast<uintptr_t>(a.out) & (4 * vw - 1)))
        return hipErrorInvalidValue;
      switch (a.g.variant) {
        case 4: hipLaunchKernelGGL((pw_mfma_vec_kernel<4, 1, 4>), grid, block, a.g.lds_bytes, s, a); break;
        case 5: hipLaunchKernelGGL((pw_mfma_vec_kernel<4, 1, 2>), grid, block, a.g.lds_bytes, s, a); break;
        case 6: hipLaunchKernelGGL((pw_mfma_vec_kernel<2, 2, 4>), grid, block, a.g.lds_bytes, s, a); break;
        case 7: hipLaunchKernelGGL((pw_mfma_vec_kernel<2, 2, 2>), grid, block, a.g.lds_bytes, s, a); break;
        case 8: hipLaunchKernelGGL((pw_mfma_vec_kernel<1, 4, 4>), grid, block, a.g.lds_bytes, s, a); break;
        default: hipLaunchKernelGGL((pw_mfma_vec_kernel<1, 4, 2>), grid, block, a.g.lds_bytes, s, a); break;
      }
      break;
    }
    case 10: case 11: case 12: {
      const int vw = a.g.variant == 10 ? 4 : (a.g.variant == 11 ? 2 : 1);
      if (a.stride != 1 || (a.Ho * a.Wo) % vw || a.HWin != a.Ho * a.Wo || a.g.bm != 32 || (reinterpret_cast<uintptr_t>(a.in) & (4 * vw - 1)) ||
          (reinterpret_cast<uintptr_t>(a.out) & (4 * vw - 1)))
        return hipErrorInvalidValue;
      if (vw == 4) hipLaunchKernelGGL((pw_mfma_ksplit_kernel<4>), grid, block, a.g.lds_bytes, s, a);
      else if (vw == 2) hipLaunchKernelGGL((pw_mfma_ksplit_kernel<2>), grid, block, a.g.lds_bytes, s, a);
      else hipLaunchKernelGGL((pw_mfma_ksplit_kernel<1>), grid, block, a.g.lds_bytes, s, a);
      break;
    }
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace pbkd

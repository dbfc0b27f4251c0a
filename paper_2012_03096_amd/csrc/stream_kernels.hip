// HBM-bound kernels of the per-block distillation step: depthwise 3x3 forward and fused backward
// (register windows with 16-byte loads for stride 1 and widths that are multiples of 4, LDS halo tiles
// otherwise), the weight gradient of a full 3x3 first layer, BatchNorm statistics, the block head (BN +
// shortcut add + ReLU + max-pool + local loss and its backward), the interior BatchNorm backward,
// SGD-momentum, fixed-order partial reductions, and the feature error of the reassembly check.
//
// BatchNorm is always applied as the single-rounding b = fmaf(z, scale, shift) (written out, not left to
// contraction), so that the ReLU and max-pool decisions every kernel takes from b are the same ones and
// can be reproduced bit for bit from z, scale and shift.
//
// Work is organised per channel (blockIdx.y = channel) wherever a per-channel reduction is needed, so
// that one workgroup's partial sums all belong to one channel; partials go to the workspace and are
// summed in a fixed order in fp64 -- results do not depend on scheduling.
#include <mutex>

#include "pbkd_internal.h"

namespace pbkd {

__device__ __forceinline__ float wave_sum(float v) { return wave64_sum(v); }
__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}

// sum_{t < n} a[t * stride] and the same for b, in fp64: lanes take t = lane, lane + 64, ..., then a fixed
// butterfly; every lane of the wave receives the results, and every wave that calls it gets the same bits
__device__ __forceinline__ void wave_strided_sum2(const float *a, const float *b, int n, size_t stride, double &sa, double &sb) {
  double x = 0.0, y = 0.0;
  for (int t = threadIdx.x & 63; t < n; t += 64) {
    const float va = a[(size_t)t * stride], vb = b[(size_t)t * stride];
    x += (double)va;
    y += (double)vb;
  }
  sa = wave_sum_d(x);
  sb = wave_sum_d(y);
}

// ------------------------------------------------------------------------------------------------ BatchNorm statistics
struct BnStat {
  float mean, rstd, scale, shift, var;
};

// Whole workgroup (256 threads) call: adds the statistics partials of channel c in a fixed order in fp64, every one
// re-expressed about the pivot of the channel's first partial (sum (z-P)^2 = sum (z-p)^2 + 2d sum (z-p) + n d^2 with
// d = p - P: no term is large against the result, whatever the channel's mean), and returns the same values to every
// thread.  sred: 8 doubles of shared memory.
__device__ __forceinline__ BnStat bn_finalize_block(const BnPending &b, int C, int c, double *sred) {
  typedef float f4 __attribute__((ext_vector_type(4)));
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  double s1 = 0.0, s2 = 0.0;
  const f4 *pc = reinterpret_cast<const f4 *>(b.partial) + (size_t)c * b.n_parts;   // contiguous per channel
  const double P = (double)pc[0][0];
  auto add = [&](const f4 &v) {
    const double d = (double)v[0] - P, n = (double)v[3], a = (double)v[1];
    s1 += a + n * d;
    s2 += (double)v[2] + d * (2.0 * a + n * d);
  };
  int t = tid;
  for (; t + 7 * 256 < b.n_parts; t += 8 * 256) {      // eight loads in flight, summed in index order
    f4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = pc[t + j * 256];
#pragma unroll
    for (int j = 0; j < 8; ++j) add(v[j]);
  }
  for (; t < b.n_parts; t += 256) add(pc[t]);
  s1 = wave_sum_d(s1);
  s2 = wave_sum_d(s2);
  __syncthreads();          // sred may still be read from an earlier call
  if (lane == 0) {
    sred[wave * 2 + 0] = s1;
    sred[wave * 2 + 1] = s2;
  }
  __syncthreads();
  s1 = (sred[0] + sred[2]) + (sred[4] + sred[6]);
  s2 = (sred[1] + sred[3]) + (sred[5] + sred[7]);
  const double dm = s1 / b.count;                      // mean - P
  const double mu = P + dm;
  double var = s2 / b.count - dm * dm;
  if (var < 0.0) var = 0.0;
  const double r = 1.0 / sqrt(var + (double)b.eps);
  const double sc = (double)b.gamma[c] * r;
  BnStat o;
  o.mean = (float)mu;
  o.rstd = (float)r;
  o.scale = (float)sc;
  o.shift = (float)((double)b.beta[c] - mu * sc);
  o.var = (float)var;
  return o;
}
// One thread per channel and forward pass calls this (so the running pair moves once per pass).
__device__ __forceinline__ void bn_store(const BnPending &b, int c, const BnStat &o) {
  b.mean[c] = o.mean;
  b.rstd[c] = o.rstd;
  b.scale[c] = o.scale;
  b.shift[c] = o.shift;
  if (b.rmean) {
    const double d = (double)b.decay;
    b.rmean[c] = (float)(d * (double)b.rmean[c] + (1.0 - d) * (double)o.mean);
    b.rvar[c] = (float)(d * (double)b.rvar[c] + (1.0 - d) * (double)o.var);
  }
}

__global__ __launch_bounds__(256) void bn_finalize_kernel(BnPending b, int C) {
  __shared__ double sred[8];
  const BnStat o = bn_finalize_block(b, C, blockIdx.x, sred);
  if (threadIdx.x == 0) bn_store(b, blockIdx.x, o);
}

hipError_t launch_bn_finalize(const BnPending &b, int C, hipStream_t s) {
  if (!b.partial || C < 1 || b.n_parts < 1) return hipErrorInvalidValue;
  hipLaunchKernelGGL(bn_finalize_kernel, dim3(C), dim3(256), 0, s, b, C);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void bn_running_kernel(const float *gamma, const float *beta, const float *rmean,
                                                         const float *rvar, float eps, float *mean, float *rstd,
                                                         float *scale, float *shift, int C) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= C) return;
  const double mu = (double)rmean[c];
  const double r = 1.0 / sqrt((double)rvar[c] + (double)eps);
  const double sc = (double)gamma[c] * r;
  mean[c] = (float)mu;
  rstd[c] = (float)r;
  scale[c] = (float)sc;
  shift[c] = (float)((double)beta[c] - mu * sc);
}

hipError_t launch_bn_running(const float *gamma, const float *beta, const float *rmean, const float *rvar, float eps,
                             float *mean, float *rstd, float *scale, float *shift, int C, hipStream_t s) {
  if (C < 1) return hipErrorInvalidValue;
  hipLaunchKernelGGL(bn_running_kernel, dim3(cdiv(C, 256)), dim3(256), 0, s, gamma, beta, rmean, rvar, eps, mean, rstd,
                     scale, shift, C);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------ depthwise
DwGeom dw_geom(int N, int Ho, int Wo, int stride, bool backward, int H, int W, bool first_layer, int C) {
  DwGeom g;
  g.fast = 0;
  g.rows = 2;
  if (stride == 2 && H > 0 && H % 2 == 0 && W % 8 == 0 && W > 0 && (!backward || first_layer)) {
    const long long strips = (long long)N * Ho * (Wo / 4);
    g.fast = 3;
    g.lTW = g.lTH = 0;
    g.nimg = 1;
    g.tiles_x = g.tiles_y = 1;
    g.tiles_n = g.n_tiles = (int)((strips + 255) / 256);
    g.lds_bytes = 0;
    return g;
  }
  if (stride == 1 && Ho == 2 && Wo == 2) {
    // 2x2 maps: one thread per (image, channel) map, 16 contiguous bytes; the backward kernel's threads each walk
    // nimg images of their channel, so there are at most 64 groups (= partials per channel)
    g.fast = 2;
    g.lTW = g.lTH = 0;
    g.nimg = backward ? cdiv(N, 64) : 1;
    g.tiles_x = g.tiles_y = 1;
    g.tiles_n = g.n_tiles = cdiv(N, g.nimg);
    g.lds_bytes = 0;
    return g;
  }
  if (stride == 1 && Wo % 4 == 0 && dw_fits_buffer(N, C, Ho, Wo)) {
    // register-window kernels: one thread per 2 rows x 4 columns, 256 threads per workgroup.  A thread reads the row
    // above and the row below its own as well, so every input row is read twice; on maps large enough to be bound by
    // bandwidth rather than latency a thread takes 4 rows (every row read 1.5 times)
    if (Ho % 4 == 0 && (long long)N * (Ho / 4) * (Wo / 4) >= 32768) g.rows = 4;
    const long long strips = (long long)N * cdiv(Ho, g.rows) * (Wo / 4);
    g.fast = 1;
    g.lTW = g.lTH = 0;
    g.nimg = 1;
    g.tiles_x = g.tiles_y = 1;
    g.tiles_n = g.n_tiles = (int)((strips + 255) / 256);
    g.lds_bytes = 0;
    return g;
  }
  const int tpmax = backward ? 1024 / (stride * stride) : 1024;
  int TW = pow2ceil(Wo);
  if (TW > 32) TW = 32;
  int TH = pow2ceil(Ho);
  if (TH > tpmax / TW) TH = tpmax / TW;
  int nimg = tpmax / (TW * TH);
  if (nimg < 1) nimg = 1;
  if (nimg > pow2ceil(N)) nimg = pow2ceil(N);
  g.lTW = ilog2(TW);
  g.lTH = ilog2(TH);
  g.nimg = nimg;
  g.tiles_x = cdiv(Wo, TW);
  g.tiles_y = cdiv(Ho, TH);
  g.tiles_n = cdiv(N, nimg);
  g.n_tiles = g.tiles_x * g.tiles_y * g.tiles_n;
  if (!backward) {
    const int IH = stride * (TH - 1) + 3, IW = stride * (TW - 1) + 3;
    g.lds_bytes = (size_t)nimg * IH * IW * sizeof(float);
  } else {
    g.lds_bytes = (size_t)nimg * ((TH + 2) * (TW + 2) + (stride * TH + 2) * (stride * TW + 2)) * sizeof(float);
  }
  return g;
}

__global__ __launch_bounds__(256) void dw_fwd_kernel(DwFwdArgs p) {
  extern __shared__ float tile[];
  const int tid = threadIdx.x;
  const int c = blockIdx.y;
  int pt = blockIdx.x;
  const int tx = pt % p.g.tiles_x;
  pt /= p.g.tiles_x;
  const int ty = pt % p.g.tiles_y;
  const int tn = pt / p.g.tiles_y;
  const int lTW = p.g.lTW, lTH = p.g.lTH, TW = 1 << lTW, TH = 1 << lTH, nimg = p.g.nimg;
  const int s = p.stride;
  const int x0 = tx * TW, y0 = ty * TH, n0 = tn * nimg;
  const int IH = s * (TH - 1) + 3, IW = s * (TW - 1) + 3, IHW = IH * IW;
  __shared__ double sred[8];
  const bool bn = p.in_scale != nullptr || p.pend.partial != nullptr;
  float sc = 1.f, sh = 0.f;
  if (p.pend.partial) {
    const BnStat o = bn_finalize_block(p.pend, p.C, c, sred);
    if (blockIdx.x == 0 && tid == 0) bn_store(p.pend, c, o);
    sc = o.scale, sh = o.shift;
  } else if (bn) {
    sc = p.in_scale[c], sh = p.in_shift[c];
  }
  float w[9];
#pragma unroll
  for (int k = 0; k < 9; ++k) w[k] = p.D[c * 9 + k];

  for (int q = tid; q < nimg * IHW; q += 256) {
    const int img = q / IHW;
    const int r = q - img * IHW;
    const int iy = r / IW, ix = r - iy * IW;
    const int n = n0 + img, y = y0 * s - 1 + iy, x = x0 * s - 1 + ix;
    float v = 0.f;
    if (n < p.N && y >= 0 && y < p.H && x >= 0 && x < p.W) {
      v = p.in[(((size_t)n * p.C + c) * p.H + y) * p.W + x];
      if (bn) v = fmaxf(fmaf(v, sc, sh), 0.f);
    }
    tile[q] = v;
  }
  __syncthreads();
  for (int e = tid; e < (nimg << (lTW + lTH)); e += 256) {
    const int img = e >> (lTW + lTH);
    const int i = (e >> lTW) & (TH - 1), j = e & (TW - 1);
    const int n = n0 + img, y = y0 + i, x = x0 + j;
    if (n < p.N && y < p.Ho && x < p.Wo) {
      const float *t = tile + (img * IH + s * i) * IW + s * j;
      float acc = 0.f;
#pragma unroll
      for (int ky = 0; ky < 3; ++ky)
#pragma unroll
        for (int kx = 0; kx < 3; ++kx) acc += w[ky * 3 + kx] * t[ky * IW + kx];
      p.out[(((size_t)n * p.C + c) * p.Ho + y) * p.Wo + x] = acc;
    }
  }
}


// ---- stride 1, width a multiple of 4: no LDS.  Workgroup b of a channel takes the strips of logical block
// xcd_contiguous(b): neighbouring row bands, which share a halo row, then run on one die and meet in its L2.
// A thread owns 2 (or 4) rows x 4 columns of one (image, channel)
// plane and reads the window around them straight from global memory (dw_load_row: one 16-byte load and two edge
// loads per row; neighbouring threads' windows overlap in L1), applying the producer's BatchNorm + ReLU to what it
// loads.  Padding stays an exact zero.
// strip index -> (image, first row, first column); false past the end
// (the launch checks that the strips are fewer than 2^31: 32-bit divisions, a fifth of the kernel's instructions otherwise)
template <int R>
__device__ __forceinline__ bool dw_strip(unsigned e, int N, int H, int W, int &n, int &y0, int &x) {
  const unsigned W4 = (unsigned)W >> 2, HG = (unsigned)(H + R - 1) / R;
  const unsigned total = (unsigned)N * HG * W4;
  const bool active = e < total;
  if (!active) e = total - 1;
  const unsigned q = e / W4;
  const unsigned xs = e - q * W4;
  const unsigned nn = q / HG;
  y0 = R * (int)(q - nn * HG);
  n = (int)nn;
  x = 4 * (int)xs;
  return active;
}

template <bool BN, int EDGE, int R>
__global__ __launch_bounds__(256) void dw_fwd_fast_kernel(DwFwdArgs p) {
  const int c = blockIdx.y;
  int n, y0, x;
  const bool active = dw_strip<R>((unsigned)xcd_contiguous(blockIdx.x, gridDim.x) * 256u + threadIdx.x, p.N, p.H, p.W, n, y0, x);
  float sc = 1.f, sh = 0.f;
  if (BN) {
    if (p.pend.partial) {
      __shared__ double sred[8];
      const BnStat o = bn_finalize_block(p.pend, p.C, c, sred);
      if (blockIdx.x == 0 && threadIdx.x == 0) bn_store(p.pend, c, o);
      sc = o.scale, sh = o.shift;
    } else {
      sc = p.in_scale[c], sh = p.in_shift[c];
    }
  }
  float w[9];
#pragma unroll
  for (int k = 0; k < 9; ++k) w[k] = p.D[c * 9 + k];
  const unsigned bytes = (unsigned)p.N * p.C * p.H * p.W * 4u;                      // (below 4 GiB: checked at launch)
  const __amdgpu_buffer_rsrc_t rin = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p.in), 0, (int)bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rout = __builtin_amdgcn_make_buffer_rsrc(p.out, 0, (int)bytes, 0x00020000);
  const unsigned pl = ((unsigned)n * p.C + c) * (unsigned)(p.H * p.W) * 4u;          // byte offset of the lane's plane
  float a[R + 2][6];
#pragma unroll
  for (int r = 0; r < R + 2; ++r) dw_load_row_buf<BN, EDGE>(rin, pl, y0 - 1, r, x, p.H, p.W, active, sc, sh, a[r]);
#pragma unroll
  for (int i = 0; i < R; ++i) {
    typedef unsigned u4 __attribute__((ext_vector_type(4)));
    u4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float acc = 0.f;
#pragma unroll
      for (int ky = 0; ky < 3; ++ky)
#pragma unroll
        for (int kx = 0; kx < 3; ++kx) acc += w[ky * 3 + kx] * a[i + ky][j + kx];
      o[j] = __builtin_bit_cast(unsigned, acc);
    }
    // (a row past the map, or an inactive lane's, is stored past the buffer: dropped)
    const unsigned off = (active && y0 + i < p.H) ? pl + (unsigned)((y0 + i) * p.W + x) * 4u : kPastBuffer;
    __builtin_amdgcn_raw_buffer_store_b128(o, rout, off, 0, 0);
  }
}

static bool aligned16(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; }
// strips of an image row in adjacent lanes of one 16-lane row: W/4 is 1, 2, 4, 8 or 16
// How the register-window kernels get a strip's two edge columns (dw_load_row_buf's EDGE): from the neighbouring lanes
// of a 16-lane row when the strips of an image row fill such rows exactly, else from the neighbouring lanes of the whole
// wave (measured at 224 x 224 x 64 against two more loads per row: forward 183 -> 176 us, backward 268 -> 239 us).
// PBKD_DW_EDGE=0 forces the loads (a measurement aid).
static int dw_edge_mode(int W) {
  const int w4 = W / 4;
  if (W % 4 == 0 && w4 <= 16 && (w4 & (w4 - 1)) == 0) return 1;
  if (const char *e = std::getenv("PBKD_DW_EDGE")) return std::atoi(e) == 0 ? 0 : 2;
  return 2;
}

// ---- stride 2, even H, W % 8 == 0: a thread owns outputs (i, j0..j0+3) and holds the 3 x 9 input window around
// them, columns 2*j0-1 .. 2*j0+7 (one scalar and two 16-byte loads per row), in registers.
__device__ __forceinline__ bool dw_strip_s2(long long e, int N, int Ho, int Wo, int &n, int &i, int &j0) {
  const int W4 = Wo >> 2;
  const long long total = (long long)N * Ho * W4;
  const bool active = e < total;
  if (!active) e = total - 1;
  j0 = 4 * (int)(e % W4);
  const long long q = e / W4;
  i = (int)(q % Ho);
  n = (int)(q / Ho);
  return active;
}

// row y of the window into r[0..8]; BN: relu(v*sc + sh) applied to what lies inside the image, zeros outside
template <bool BN>
__device__ __forceinline__ void dw_load_row_s2(const float *plane, int y, int x0, int H, int W, bool active, float sc, float sh,
                                               float (&r)[9]) {
#pragma unroll
  for (int k = 0; k < 9; ++k) r[k] = 0.f;
  if (active && y >= 0 && y < H) {
    const float *row = plane + (size_t)y * W + x0;
    const float4 a = *reinterpret_cast<const float4 *>(row), b = *reinterpret_cast<const float4 *>(row + 4);
    r[1] = a.x, r[2] = a.y, r[3] = a.z, r[4] = a.w, r[5] = b.x, r[6] = b.y, r[7] = b.z, r[8] = b.w;
    if (x0 > 0) r[0] = row[-1];
    if (BN) {
#pragma unroll
      for (int k = 1; k < 9; ++k) r[k] = fmaxf(fmaf(r[k], sc, sh), 0.f);
      if (x0 > 0) r[0] = fmaxf(fmaf(r[0], sc, sh), 0.f);
    }
  }
}

template <bool BN>
__global__ __launch_bounds__(256) void dw_fwd_s2_kernel(DwFwdArgs p) {
  const int c = blockIdx.y;
  int n, i, j0;
  const bool active = dw_strip_s2((long long)xcd_contiguous(blockIdx.x, gridDim.x) * 256 + threadIdx.x, p.N, p.Ho, p.Wo, n, i, j0);
  float sc = 1.f, sh = 0.f;
  if (BN) {
    if (p.pend.partial) {
      __shared__ double sred[8];
      const BnStat o = bn_finalize_block(p.pend, p.C, c, sred);
      if (blockIdx.x == 0 && threadIdx.x == 0) bn_store(p.pend, c, o);
      sc = o.scale, sh = o.shift;
    } else {
      sc = p.in_scale[c], sh = p.in_shift[c];
    }
  }
  float w[9];
#pragma unroll
  for (int k = 0; k < 9; ++k) w[k] = p.D[c * 9 + k];
  const float *plane = p.in + ((size_t)n * p.C + c) * p.H * p.W;
  float a[3][9];
#pragma unroll
  for (int r = 0; r < 3; ++r) dw_load_row_s2<BN>(plane, 2 * i - 1 + r, 2 * j0, p.H, p.W, active, sc, sh, a[r]);
  float o[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float acc = 0.f;
#pragma unroll
    for (int ky = 0; ky < 3; ++ky)
#pragma unroll
      for (int kx = 0; kx < 3; ++kx) acc += w[ky * 3 + kx] * a[ky][2 * j + kx];
    o[j] = acc;
  }
  if (active)
    *reinterpret_cast<float4 *>(p.out + (((size_t)n * p.C + c) * p.Ho + i) * p.Wo + j0) = make_float4(o[0], o[1], o[2], o[3]);
}

// backward of a first layer (weight gradient only): dD[ky][kx] += du[i][j] * in[2i+ky-1][2j+kx-1]
__global__ __launch_bounds__(256) void dw_bwd_s2_first_kernel(DwBwdArgs p) {
  __shared__ float red[4][11];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = blockIdx.y;
  int n, i, j0;
  const bool active = dw_strip_s2((long long)xcd_contiguous(blockIdx.x, gridDim.x) * 256 + tid, p.N, p.Ho, p.Wo, n, i, j0);
  const float *plane = p.in + ((size_t)n * p.C + c) * p.H * p.W;
  float a[3][9];
#pragma unroll
  for (int r = 0; r < 3; ++r) dw_load_row_s2<false>(plane, 2 * i - 1 + r, 2 * j0, p.H, p.W, active, 1.f, 0.f, a[r]);
  float d[4] = {0.f, 0.f, 0.f, 0.f};
  if (active) {
    const float4 v = *reinterpret_cast<const float4 *>(p.du + (((size_t)n * p.C + c) * p.Ho + i) * p.Wo + j0);
    d[0] = v.x, d[1] = v.y, d[2] = v.z, d[3] = v.w;
  }
  float acc[9];
#pragma unroll
  for (int k = 0; k < 9; ++k) acc[k] = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int ky = 0; ky < 3; ++ky)
#pragma unroll
      for (int kx = 0; kx < 3; ++kx) acc[ky * 3 + kx] += d[j] * a[ky][2 * j + kx];
#pragma unroll
  for (int k = 0; k < 9; ++k) {
    const float v = wave_sum(acc[k]);
    if (lane == 0) red[wave][k] = v;
  }
  __syncthreads();
  if (tid < 11) {
    const float v = tid < 9 ? (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]) : 0.f;
    p.partial[((size_t)blockIdx.x * p.C + c) * 11 + tid] = v;
  }
}

// 2x2 maps (the last VGG stage at CIFAR size): a 3x3 window with padding 1 sees the whole map from every position,
// and a map is one aligned float4.  The tile kernels above would give every workgroup one channel, whose maps lie
// 16 bytes each, 4*C*4 bytes apart; here consecutive threads take consecutive channels of one image instead.
// out[i][j] = sum_{y,x} D[(y-i+1)*3 + (x-j+1)] * a[y][x].
__global__ __launch_bounds__(256) void dw_fwd_2x2_kernel(DwFwdArgs p) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= (long long)p.N * p.C) return;
  const int c = (int)(t % p.C);
  float4 a = reinterpret_cast<const float4 *>(p.in)[t];
  if (p.in_scale) {
    const float sc = p.in_scale[c], sh = p.in_shift[c];
    a.x = fmaxf(fmaf(a.x, sc, sh), 0.f);
    a.y = fmaxf(fmaf(a.y, sc, sh), 0.f);
    a.z = fmaxf(fmaf(a.z, sc, sh), 0.f);
    a.w = fmaxf(fmaf(a.w, sc, sh), 0.f);
  }
  float w[9];
#pragma unroll
  for (int k = 0; k < 9; ++k) w[k] = p.D[c * 9 + k];
  float4 o;
  o.x = w[4] * a.x + w[5] * a.y + w[7] * a.z + w[8] * a.w;
  o.y = w[3] * a.x + w[4] * a.y + w[6] * a.z + w[7] * a.w;
  o.z = w[1] * a.x + w[2] * a.y + w[4] * a.z + w[5] * a.w;
  o.w = w[0] * a.x + w[1] * a.y + w[3] * a.z + w[4] * a.w;
  reinterpret_cast<float4 *>(p.out)[t] = o;
}

// Backward on 2x2 maps: thread (group g, channel c) walks images g*nimg .. of its channel and keeps the eleven sums
// (9 of dD, then sum g_prev, sum g_prev * xhat_prev) in registers: partial[g][c][11], no reduction across threads.
template <bool FIRST>
__global__ __launch_bounds__(256) void dw_bwd_2x2_kernel(DwBwdArgs p) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= (long long)p.g.n_tiles * p.C) return;
  const int c = (int)(t % p.C), grp = (int)(t / p.C);
  const float sc = FIRST ? 1.f : p.in_scale[c], sh = FIRST ? 0.f : p.in_shift[c];
  const float mean = FIRST ? 0.f : p.in_mean[c], rstd = FIRST ? 0.f : p.in_rstd[c];
  float w[9], acc[11];
#pragma unroll
  for (int k = 0; k < 9; ++k) w[k] = p.D[c * 9 + k];
#pragma unroll
  for (int k = 0; k < 11; ++k) acc[k] = 0.f;
  const int n_end = ((grp + 1) * p.g.nimg < p.N) ? (grp + 1) * p.g.nimg : p.N;
  for (int n = grp * p.g.nimg; n < n_end; ++n) {
    const size_t idx = (size_t)n * p.C + c;
    const float4 d4 = reinterpret_cast<const float4 *>(p.du)[idx];
    const float4 r4 = reinterpret_cast<const float4 *>(p.in)[idx];
    const float d[4] = {d4.x, d4.y, d4.z, d4.w}, raw[4] = {r4.x, r4.y, r4.z, r4.w};
    float a[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) a[q] = FIRST ? raw[q] : fmaxf(fmaf(raw[q], sc, sh), 0.f);
    // position q = 2*y + x; the tap that links output (i,j) to input (y,x) is (y-i+1, x-j+1)
#pragma unroll
    for (int o = 0; o < 4; ++o)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int ky = (q >> 1) - (o >> 1) + 1, kx = (q & 1) - (o & 1) + 1;
        acc[ky * 3 + kx] += d[o] * a[q];
      }
    if (!FIRST) {
      float g[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float da = 0.f;
#pragma unroll
        for (int o = 0; o < 4; ++o) {
          const int ky = (q >> 1) - (o >> 1) + 1, kx = (q & 1) - (o & 1) + 1;
          da += w[ky * 3 + kx] * d[o];
        }
        g[q] = a[q] > 0.f ? da : 0.f;
        acc[9] += g[q];
        acc[10] += g[q] * ((raw[q] - mean) * rstd);
      }
      reinterpret_cast<float4 *>(p.gout)[idx] = make_float4(g[0], g[1], g[2], g[3]);
    }
  }
  float *dst = p.partial + ((size_t)grp * p.C + c) * 11;
#pragma unroll
  for (int k = 0; k < 11; ++k) dst[k] = acc[k];
}

hipError_t launch_dw_fwd(const DwFwdArgs &a, hipStream_t s) {
  if (a.C > 65535) return hipErrorInvalidValue;
  if (a.g.fast == 2) {
    if (a.stride != 1 || a.H != 2 || a.W != 2 || a.Ho != 2 || a.Wo != 2 || a.pend.partial || !aligned16(a.in) || !aligned16(a.out))
      return hipErrorInvalidValue;
    const long long blocks = ((long long)a.N * a.C + 255) / 256;
    hipLaunchKernelGGL(dw_fwd_2x2_kernel, dim3((unsigned)blocks), dim3(256), 0, s, a);
    return hipGetLastError();
  }
  if (a.g.fast == 3) {
    if (a.stride != 2 || a.H % 2 || a.W % 8 || a.Ho != a.H / 2 || a.Wo != a.W / 2 || !aligned16(a.in) || !aligned16(a.out))
      return hipErrorInvalidValue;
    const dim3 grid(a.g.n_tiles, a.C);
    if (a.in_scale || a.pend.partial)
      hipLaunchKernelGGL(dw_fwd_s2_kernel<true>, grid, dim3(256), 0, s, a);
    else
      hipLaunchKernelGGL(dw_fwd_s2_kernel<false>, grid, dim3(256), 0, s, a);
    return hipGetLastError();
  }
  if (a.g.fast) {
    if (a.stride != 1 || a.W % 4 || a.H != a.Ho || a.W != a.Wo || !aligned16(a.in) || !aligned16(a.out) || !dw_fits_buffer(a.N, a.C, a.H, a.W))
      return hipErrorInvalidValue;
    const dim3 grid(a.g.n_tiles, a.C);
    const bool bn = a.in_scale || a.pend.partial;
    const int edge = dw_edge_mode(a.W);
    if (a.g.rows != 2 && !(a.g.rows == 4 && a.H % 4 == 0)) return hipErrorInvalidValue;
#define PBKD_GO1(BN, E, R) hipLaunchKernelGGL((dw_fwd_fast_kernel<BN, E, R>), grid, dim3(256), 0, s, a)
#define PBKD_GO(R)                                                                             \
    if (bn) {                                                                                  \
      if (edge == 1) PBKD_GO1(true, 1, R); else if (edge == 2) PBKD_GO1(true, 2, R); else PBKD_GO1(true, 0, R);      \
    } else {                                                                                   \
      if (edge == 1) PBKD_GO1(false, 1, R); else if (edge == 2) PBKD_GO1(false, 2, R); else PBKD_GO1(false, 0, R);   \
    }
    if (a.g.rows == 4) { PBKD_GO(4) } else { PBKD_GO(2) }
#undef PBKD_GO
#undef PBKD_GO1
    return hipGetLastError();
  }
  hipLaunchKernelGGL(dw_fwd_kernel, dim3(a.g.n_tiles, a.C), dim3(256), a.g.lds_bytes, s, a);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void dw_bwd_kernel(DwBwdArgs p) {
  extern __shared__ float sm[];
  __shared__ float red[4][11];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = blockIdx.y;
  int pt = blockIdx.x;
  const int tx = pt % p.g.tiles_x;
  pt /= p.g.tiles_x;
  const int ty = pt % p.g.tiles_y;
  const int tn = pt / p.g.tiles_y;
  const int lTW = p.g.lTW, lTH = p.g.lTH, TW = 1 << lTW, TH = 1 << lTH, nimg = p.g.nimg;
  const int s = p.stride, ls = (s == 2) ? 1 : 0;
  const int x0 = tx * TW, y0 = ty * TH, n0 = tn * nimg;
  const int DH = TH + 2, DWd = TW + 2, DHW = DH * DWd;
  const int AH = s * TH + 2, AW = s * TW + 2, AHW = AH * AW;
  float *dut = sm;                 // [nimg][DH][DWd]   du with a halo of 1, zero outside the map
  float *at = sm + nimg * DHW;     // [nimg][AH][AW]    layer input with a halo of 1, zero outside
  const bool bn = !p.first_layer;
  const float sc = bn ? p.in_scale[c] : 1.f, sh = bn ? p.in_shift[c] : 0.f;
  float w[9];
#pragma unroll
  for (int k = 0; k < 9; ++k) w[k] = p.D[c * 9 + k];

  for (int q = tid; q < nimg * DHW; q += 256) {
    const int img = q / DHW;
    const int r = q - img * DHW;
    const int iy = r / DWd, ix = r - iy * DWd;
    const int n = n0 + img, i = y0 - 1 + iy, j = x0 - 1 + ix;
    float v = 0.f;
    if (n < p.N && i >= 0 && i < p.Ho && j >= 0 && j < p.Wo) v = p.du[(((size_t)n * p.C + c) * p.Ho + i) * p.Wo + j];
    dut[q] = v;
  }
  for (int q = tid; q < nimg * AHW; q += 256) {
    const int img = q / AHW;
    const int r = q - img * AHW;
    const int iy = r / AW, ix = r - iy * AW;
    const int n = n0 + img, y = s * y0 - 1 + iy, x = s * x0 - 1 + ix;
    float v = 0.f;
    if (n < p.N && y >= 0 && y < p.H && x >= 0 && x < p.W) {
      v = p.in[(((size_t)n * p.C + c) * p.H + y) * p.W + x];
      if (bn) v = fmaxf(fmaf(v, sc, sh), 0.f);
    }
    at[q] = v;
  }
  __syncthreads();

  // weight gradient: every du position of the tile against the 3x3 window of the input around it
  float wacc[9];
#pragma unroll
  for (int k = 0; k < 9; ++k) wacc[k] = 0.f;
  for (int e = tid; e < (nimg << (lTW + lTH)); e += 256) {
    const int img = e >> (lTW + lTH);
    const int i = (e >> lTW) & (TH - 1), j = e & (TW - 1);
    const float g = dut[(img * DH + i + 1) * DWd + j + 1];
    const float *a = at + (img * AH + s * i) * AW + s * j;
#pragma unroll
    for (int ky = 0; ky < 3; ++ky)
#pragma unroll
      for (int kx = 0; kx < 3; ++kx) wacc[ky * 3 + kx] += g * a[ky * AW + kx];
  }

  // data gradient through the depthwise conv and the previous layer's ReLU; BN-backward sums
  float sb = 0.f, sg = 0.f;
  if (bn) {
    const float mean = p.in_mean[c], rstd = p.in_rstd[c];
    const int lSW = lTW + ls, lSH = lTH + ls;
    const int SW = 1 << lSW, SH = 1 << lSH;
    for (int e = tid; e < (nimg << (lSW + lSH)); e += 256) {
      const int img = e >> (lSW + lSH);
      const int yy = (e >> lSW) & (SH - 1), xx = e & (SW - 1);
      const int n = n0 + img, y = s * y0 + yy, x = s * x0 + xx;
      if (n < p.N && y < p.H && x < p.W) {
        float da = 0.f;
#pragma unroll
        for (int ky = 0; ky < 3; ++ky) {
          const int ty_ = yy + 1 - ky;
          if (ty_ & (s - 1)) continue;
          const int row = (ty_ >> ls) + 1;
#pragma unroll
          for (int kx = 0; kx < 3; ++kx) {
            const int tx_ = xx + 1 - kx;
            if (tx_ & (s - 1)) continue;
            const int col = (tx_ >> ls) + 1;
            da += w[ky * 3 + kx] * dut[(img * DH + row) * DWd + col];
          }
        }
        const float ac = at[(img * AH + yy + 1) * AW + xx + 1];
        const float g = (ac > 0.f) ? da : 0.f;
        const size_t off = (((size_t)n * p.C + c) * p.H + y) * p.W + x;
        p.gout[off] = g;
        const float xh = (p.in[off] - mean) * rstd;
        sb += g;
        sg += g * xh;
      }
    }
  }

#pragma unroll
  for (int k = 0; k < 9; ++k) {
    const float v = wave_sum(wacc[k]);
    if (lane == 0) red[wave][k] = v;
  }
  {
    const float v1 = wave_sum(sb), v2 = wave_sum(sg);
    if (lane == 0) {
      red[wave][9] = v1;
      red[wave][10] = v2;
    }
  }
  __syncthreads();
  if (tid < 11) {
    const float v = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
    p.partial[((size_t)blockIdx.x * p.C + c) * 11 + tid] = v;
  }
}


// Fused backward for stride 1 and width a multiple of 4, register windows as in the forward kernel: the
// thread's 2 x 4 positions take the weight gradient from (du centre) x (input window), the data gradient
// from (du window) x D, the previous layer's ReLU decision from the transformed centre, and the
// BatchNorm-backward sums from the raw centre.
template <bool FIRST, int EDGE, int R>
__global__ __launch_bounds__(256) void dw_bwd_fast_kernel(DwBwdArgs p) {
  __shared__ float red[4][11];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = blockIdx.y;
  int n, y0, x;
  const bool active = dw_strip<R>((unsigned)xcd_contiguous(blockIdx.x, gridDim.x) * 256u + tid, p.N, p.H, p.W, n, y0, x);
  const float sc = FIRST ? 1.f : p.in_scale[c], sh = FIRST ? 0.f : p.in_shift[c];
  float w[9];
#pragma unroll
  for (int k = 0; k < 9; ++k) w[k] = p.D[c * 9 + k];
  const unsigned bytes = (unsigned)p.N * p.C * p.H * p.W * 4u;                      // (below 4 GiB: checked at launch)
  const __amdgpu_buffer_rsrc_t rin = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p.in), 0, (int)bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rdu = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p.du), 0, (int)bytes, 0x00020000);
  const unsigned pl = ((unsigned)n * p.C + c) * (unsigned)(p.H * p.W) * 4u;          // byte offset of the lane's plane

  float a[R + 2][6], d[R + 2][6];
  float rawc[R][4];          // the centre rows of the input as stored (before BatchNorm + ReLU), for x-hat
#pragma unroll
  for (int r = 0; r < R + 2; ++r)
    dw_load_row_buf<!FIRST, EDGE>(rin, pl, y0 - 1, r, x, p.H, p.W, active, sc, sh, a[r], (!FIRST && r >= 1 && r <= R) ? rawc[r - 1] : nullptr);
#pragma unroll
  for (int r = 0; r < R + 2; ++r) dw_load_row_buf<false, EDGE>(rdu, pl, y0 - 1, r, x, p.H, p.W, active, 0.f, 0.f, d[r]);

  float acc[11];
#pragma unroll
  for (int k = 0; k < 11; ++k) acc[k] = 0.f;
  // rows past the map and inactive threads hold zeros in d, so they add nothing
#pragma unroll
  for (int i = 0; i < R; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float g = d[i + 1][j + 1];
#pragma unroll
      for (int ky = 0; ky < 3; ++ky)
#pragma unroll
        for (int kx = 0; kx < 3; ++kx) acc[ky * 3 + kx] += g * a[i + ky][j + kx];
    }

  if (!FIRST) {
    const float mean = p.in_mean[c], rstd = p.in_rstd[c];
    const __amdgpu_buffer_rsrc_t rg = __builtin_amdgcn_make_buffer_rsrc(p.gout, 0, (int)bytes, 0x00020000);
#pragma unroll
    for (int i = 0; i < R; ++i) {
      const bool rowok = active && y0 + i < p.H;
      typedef unsigned u4 __attribute__((ext_vector_type(4)));
      u4 o;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float da = 0.f;
#pragma unroll
        for (int ky = 0; ky < 3; ++ky)
#pragma unroll
          for (int kx = 0; kx < 3; ++kx) da += w[ky * 3 + kx] * d[i + 2 - ky][j + 2 - kx];
        // (a row that does not exist has zeros in a: nothing passes the ReLU's mask)
        const float g = (a[i + 1][j + 1] > 0.f) ? da : 0.f;
        o[j] = __builtin_bit_cast(unsigned, g);
        acc[9] += g;
        acc[10] += g * ((rawc[i][j] - mean) * rstd);
      }
      __builtin_amdgcn_raw_buffer_store_b128(o, rg, rowok ? pl + (unsigned)((y0 + i) * p.W + x) * 4u : kPastBuffer, 0, 0);
    }
  }

#pragma unroll
  for (int k = 0; k < 11; ++k) {
    const float v = wave_sum(acc[k]);
    if (lane == 0) red[wave][k] = v;
  }
  __syncthreads();
  if (tid < 11) p.partial[((size_t)blockIdx.x * p.C + c) * 11 + tid] = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
}

hipError_t launch_dw_bwd(const DwBwdArgs &a, hipStream_t s) {
  if (a.C > 65535) return hipErrorInvalidValue;
  if (a.g.fast == 2) {
    if (a.stride != 1 || a.H != 2 || a.W != 2 || a.Ho != 2 || a.Wo != 2 || a.g.nimg < 1 || a.g.n_tiles != cdiv(a.N, a.g.nimg) ||
        !aligned16(a.in) || !aligned16(a.du) || (!a.first_layer && !aligned16(a.gout)))
      return hipErrorInvalidValue;
    const long long blocks = ((long long)a.g.n_tiles * a.C + 255) / 256;
    if (a.first_layer)
      hipLaunchKernelGGL(dw_bwd_2x2_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, a);
    else
      hipLaunchKernelGGL(dw_bwd_2x2_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, a);
    return hipGetLastError();
  }
  if (a.g.fast == 3) {
    if (!a.first_layer || a.stride != 2 || a.H % 2 || a.W % 8 || a.Ho != a.H / 2 || a.Wo != a.W / 2 || !aligned16(a.in) ||
        !aligned16(a.du))
      return hipErrorInvalidValue;
    hipLaunchKernelGGL(dw_bwd_s2_first_kernel, dim3(a.g.n_tiles, a.C), dim3(256), 0, s, a);
    return hipGetLastError();
  }
  if (a.g.fast) {
    if (a.stride != 1 || a.W % 4 || a.H != a.Ho || a.W != a.Wo || !aligned16(a.in) || !aligned16(a.du) ||
        (!a.first_layer && !aligned16(a.gout)) || !dw_fits_buffer(a.N, a.C, a.H, a.W))
      return hipErrorInvalidValue;
    const dim3 grid(a.g.n_tiles, a.C);
    const int edge = dw_edge_mode(a.W);
    if (a.g.rows != 2 && !(a.g.rows == 4 && a.H % 4 == 0)) return hipErrorInvalidValue;
#define PBKD_GO1(F, E, R) hipLaunchKernelGGL((dw_bwd_fast_kernel<F, E, R>), grid, dim3(256), 0, s, a)
#define PBKD_GO(R)                                                                             \
    if (a.first_layer) {                                                                       \
      if (edge == 1) PBKD_GO1(true, 1, R); else if (edge == 2) PBKD_GO1(true, 2, R); else PBKD_GO1(true, 0, R);      \
    } else {                                                                                   \
      if (edge == 1) PBKD_GO1(false, 1, R); else if (edge == 2) PBKD_GO1(false, 2, R); else PBKD_GO1(false, 0, R);   \
    }
    if (a.g.rows == 4) { PBKD_GO(4) } else { PBKD_GO(2) }
#undef PBKD_GO
#undef PBKD_GO1
    return hipGetLastError();
  }
  hipLaunchKernelGGL(dw_bwd_kernel, dim3(a.g.n_tiles, a.C), dim3(256), a.g.lds_bytes, s, a);
  return hipGetLastError();
}

// one wave per (channel, k): sums the tiles in fp64
__global__ __launch_bounds__(256) void dw_bwd_finalize_kernel(const float *partial, int n_tiles, int C, float *dD,
                                                              float *dgamma_prev, float *dbeta_prev) {
  const int lane = threadIdx.x & 63;
  const int item = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= C * 11) return;
  const int c = item / 11, k = item - c * 11;
  double acc = 0.0;
  for (int t = lane; t < n_tiles; t += 64) acc += (double)partial[((size_t)t * C + c) * 11 + k];
  acc = wave_sum_d(acc);
  if (lane == 0) {
    if (k < 9) {
      if (dD) dD[c * 9 + k] = (float)acc;
    } else if (k == 9) {
      if (dbeta_prev) dbeta_prev[c] = (float)acc;
    } else {
      if (dgamma_prev) dgamma_prev[c] = (float)acc;
    }
  }
}

hipError_t launch_dw_bwd_finalize(const float *partial, int n_tiles, int C, float *dD, float *dgamma_prev,
                                  float *dbeta_prev, hipStream_t s) {
  hipLaunchKernelGGL(dw_bwd_finalize_kernel, dim3(cdiv(C * 11, 4)), dim3(256), 0, s, partial, n_tiles, C, dD,
                     dgamma_prev, dbeta_prev);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------ full 3x3 wgrad
// For a trainable full convolution that is a block's first layer (few input channels).  Lanes run along
// a row of 64 output pixels so dz loads coalesce; each wave keeps 4 output channels x 3 input channels x 9
// taps in registers, reads the input window from an LDS halo tile shared by the workgroup's 16 output
// channels, and reduces across lanes once per tile.
constexpr int CW_OB = 4;     // output channels per wave
constexpr int CW_CB = 3;     // input channels per pass

CwGeom cw_geom(int N, int Cin, int Ho, int Wo, int stride) {
  CwGeom g;
  g.TH = (stride == 1) ? 32 : 16;
  if (g.TH > Ho) g.TH = Ho;
  g.tiles_x = cdiv(Wo, 64);
  g.tiles_y = cdiv(Ho, g.TH);
  g.n_tiles = N * g.tiles_x * g.tiles_y;
  g.IH = stride * (g.TH - 1) + 3;
  g.IW = stride * 63 + 3;
  g.lds_bytes = (size_t)CW_CB * g.IH * g.IW * sizeof(float);
  (void)Cin;
  return g;
}

__global__ __launch_bounds__(256) void conv_wgrad_kernel(CwArgs p) {
  extern __shared__ float xt[];   // [CW_CB][IH][IW]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int pt = blockIdx.x;
  const int tx = pt % p.g.tiles_x;
  pt /= p.g.tiles_x;
  const int ty = pt % p.g.tiles_y;
  const int n = pt / p.g.tiles_y;
  const int s = p.stride;
  const int TH = p.g.TH, IH = p.g.IH, IW = p.g.IW, IHW = IH * IW;
  const int x0 = tx * 64, y0 = ty * TH;
  const int ob = blockIdx.y * (4 * CW_OB) + wave * CW_OB;
  const int j = x0 + lane;
  const bool jok = j < p.Wo;

  for (int cb = 0; cb < p.Cin; cb += CW_CB) {
    __syncthreads();
    for (int q = tid; q < CW_CB * IHW; q += 256) {
      const int cc = q / IHW;
      const int r = q - cc * IHW;
      const int iy = r / IW, ix = r - iy * IW;
      const int c = cb + cc, y = s * y0 - 1 + iy, x = s * x0 - 1 + ix;
      float v = 0.f;
      if (c < p.Cin && y >= 0 && y < p.H && x >= 0 && x < p.W) v = p.x[(((size_t)n * p.Cin + c) * p.H + y) * p.W + x];
      xt[q] = v;
    }
    __syncthreads();
    float acc[CW_OB][CW_CB][9];
#pragma unroll
    for (int a = 0; a < CW_OB; ++a)
#pragma unroll
      for (int b = 0; b < CW_CB; ++b)
#pragma unroll
        for (int k = 0; k < 9; ++k) acc[a][b][k] = 0.f;
    for (int i = 0; i < TH; ++i) {
      const int y = y0 + i;
      if (y >= p.Ho) break;
      float dzv[CW_OB];
#pragma unroll
      for (int a = 0; a < CW_OB; ++a) {
        const int o = ob + a;
        dzv[a] = (jok && o < p.Cout) ? p.dz[(((size_t)n * p.Cout + o) * p.Ho + y) * p.Wo + j] : 0.f;
      }
#pragma unroll
      for (int b = 0; b < CW_CB; ++b)
#pragma unroll
        for (int ky = 0; ky < 3; ++ky)
#pragma unroll
          for (int kx = 0; kx < 3; ++kx) {
            const float xv = xt[b * IHW + (s * i + ky) * IW + s * lane + kx];
#pragma unroll
            for (int a = 0; a < CW_OB; ++a) acc[a][b][ky * 3 + kx] += dzv[a] * xv;
          }
    }
#pragma unroll
    for (int a = 0; a < CW_OB; ++a)
#pragma unroll
      for (int b = 0; b < CW_CB; ++b)
#pragma unroll
        for (int k = 0; k < 9; ++k) {
          const float v = wave_sum(acc[a][b][k]);
          const int o = ob + a, c = cb + b;
          if (lane == 0 && o < p.Cout && c < p.Cin)
            p.partial[(((size_t)blockIdx.x * p.Cout + o) * p.Cin + c) * 9 + k] = v;
        }
  }
}

hipError_t launch_conv_wgrad(const CwArgs &a, hipStream_t s) {
  hipLaunchKernelGGL(conv_wgrad_kernel, dim3(a.g.n_tiles, cdiv(a.Cout, 4 * CW_OB)), dim3(256), a.g.lds_bytes, s, a);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------ reductions
constexpr int RP_SLICES = 16;   // waves per workgroup of the update kernel, each summing every 16th partial of the same 64 outputs


// ------------------------------------------------------------------------------------------------ block head
// MODE 0: out = pool(relu(bn(z) [+ bn_s(zs)]))
// MODE 1: loss partial sum (p-t)^2 and the BatchNorm-backward sums of g = dL/db:
//         g = gscale*(p-t) at the window's first maximum if that maximum is > 0, else 0
// MODE 2: dz = scale/m * (m*g - dbeta - xhat*dgamma) for every element
int head_blocks(int N, int H, int W, int pool) {
  const long long total = pool ? (long long)N * ((H + 1) / 2) * ((W + 1) / 2) : (long long)N * H * W;
  long long b = (total + 1023) / 1024;
  if (b < 1) b = 1;
  if (b > 64) b = 64;
  return (int)b;
}

// VEC: W % 4 == 0 (and H even under the pool): a thread takes 4 columns of one row (no pool) or of two rows (two
// pool windows) with 16-byte loads and stores; otherwise one element / one window per thread, any shape.
template <int MODE, bool POOL, bool VEC, bool HS>
__global__ __launch_bounds__(256) void head_kernel(HeadArgs p) {
  __shared__ float red[4][3];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = blockIdx.y;
  const int H = p.H, W = p.W;
  const int Hw = POOL ? (H + 1) / 2 : H, Ww = POOL ? (W + 1) / 2 : W;
  const int Hp = POOL ? H / 2 : H, Wp = POOL ? W / 2 : W;
  const int total = p.N * Hw * Ww;
  constexpr bool hs = HS;          // a second input (shortcut branch or identity skip) is added before the ReLU
  float sc, sh, scs = 0.f, shs = 0.f, mean = 0.f, rstd = 0.f;
  if (MODE != 2 && p.pend.partial) {
    __shared__ double sred[8];
    const BnStat o = bn_finalize_block(p.pend, p.C, c, sred);
    if (blockIdx.x == 0 && tid == 0) bn_store(p.pend, c, o);
    sc = o.scale, sh = o.shift, mean = o.mean, rstd = o.rstd;
    if (hs && !p.identity_skip) {
      const BnStat os = bn_finalize_block(p.pend_s, p.C, c, sred);
      if (blockIdx.x == 0 && tid == 0) bn_store(p.pend_s, c, os);
      scs = os.scale, shs = os.shift;
    }
  } else {
    sc = p.scale[c], sh = p.shift[c];
    if (hs && !p.identity_skip) scs = p.scale_s[c], shs = p.shift_s[c];
    if (MODE != 0) mean = p.mean[c], rstd = p.rstd[c];
  }
  if (p.identity_skip) scs = 1.f, shs = 0.f;      // fmaf(x, 1, 0) is x: the skip adds the block input itself
  const float m = (float)p.N * (float)H * (float)W;
  float dg = 0.f, db = 0.f;
  if (MODE == 2) {
    if (p.partial) {
      // the loss kernel's partials [n_blk][C][3] (loss, dbeta, dgamma) are still unsummed: every wave sums the
      // two of its channel; the first workgroup of a channel stores them, the very first one the loss
      const float *pc = p.partial + (size_t)c * 3;
      const size_t stride = (size_t)p.C * 3;
      double sb2, sg2;
      wave_strided_sum2(pc + 1, pc + 2, p.n_blk, stride, sb2, sg2);
      db = (float)sb2;
      dg = (float)sg2;
      if (blockIdx.x == 0 && tid == 0) {
        p.dbeta_out[c] = db;
        p.dgamma_out[c] = dg;
      }
      if (blockIdx.x == 0 && c == 0) {
        __shared__ double lred[4];
        double l = 0.0;
        for (int e = tid; e < p.n_blk * p.C; e += 256) l += (double)p.partial[(size_t)e * 3];
        l = wave_sum_d(l);
        if (lane == 0) lred[wave] = l;
        __syncthreads();
        if (tid == 0) p.loss_out[0] = (float)(((lred[0] + lred[1]) + (lred[2] + lred[3])) * (double)p.loss_scale);
      }
    } else {
      dg = p.dgamma[c], db = p.dbeta[c];
    }
  }
  const float f = sc / m;
  float loss = 0.f, sb = 0.f, sg = 0.f;

  if (VEC) {
    constexpr int ROWS = POOL ? 2 : 1;
    const int W4 = W >> 2, HR = POOL ? (H >> 1) : H;
    const int per_img = HR * W4;
    const int items = p.N * per_img;
    // an item = (image n, row group ri, quad q); the thread's first one by division, the later ones by carrying the
    // grid's stride along (two integer divisions per item were a third of this kernel's instructions)
    int it = blockIdx.x * 256 + tid;
    int n = it / per_img;
    int ri = (it - n * per_img) / W4;
    int q = it - n * per_img - ri * W4;
    const int S = gridDim.x * 256;
    const int dn = S / per_img, dri = (S - dn * per_img) / W4, dq = S - dn * per_img - dri * W4;
    for (; it < items; it += S) {
      const size_t plane = ((size_t)n * p.C + c);
      const size_t o0 = (plane * H + (size_t)ROWS * ri) * W + 4 * q;
      const size_t toff = POOL ? (plane * Hp + ri) * Wp + 2 * q : o0;
      // every load of the item first, then the arithmetic: with the loads spread through it each one had to land
      // before the next was issued
      float4 z4[ROWS], s4[ROWS];
#pragma unroll
      for (int rr = 0; rr < ROWS; ++rr) {
        z4[rr] = *reinterpret_cast<const float4 *>(p.z + o0 + (size_t)rr * W);
        if (hs) s4[rr] = *reinterpret_cast<const float4 *>(p.zs + o0 + (size_t)rr * W);
      }
      float4 t4 = make_float4(0.f, 0.f, 0.f, 0.f);
      float2 t2 = make_float2(0.f, 0.f);
      if (MODE != 0) {
        if (POOL)
          t2 = *reinterpret_cast<const float2 *>(p.t + toff);
        else
          t4 = *reinterpret_cast<const float4 *>(p.t + toff);
      }
      q += dq;
      const bool cq = q >= W4;
      q -= cq ? W4 : 0;
      ri += dri + (cq ? 1 : 0);
      const bool cr = ri >= HR;
      ri -= cr ? HR : 0;
      n += dn + (cr ? 1 : 0);
      float zv[ROWS][4], bv[ROWS][4];
#pragma unroll
      for (int rr = 0; rr < ROWS; ++rr) {
        zv[rr][0] = z4[rr].x, zv[rr][1] = z4[rr].y, zv[rr][2] = z4[rr].z, zv[rr][3] = z4[rr].w;
#pragma unroll
        for (int j = 0; j < 4; ++j) bv[rr][j] = fmaf(zv[rr][j], sc, sh);
        if (hs) {
          bv[rr][0] += fmaf(s4[rr].x, scs, shs);
          bv[rr][1] += fmaf(s4[rr].y, scs, shs);
          bv[rr][2] += fmaf(s4[rr].z, scs, shs);
          bv[rr][3] += fmaf(s4[rr].w, scs, shs);
        }
      }
      if (!POOL) {
        const float tv[4] = {t4.x, t4.y, t4.z, t4.w};
        float ov[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float y = fmaxf(bv[0][j], 0.f);
          if (MODE == 0) {
            ov[j] = y;
          } else {
            const float d = y - tv[j];
            const float g = (bv[0][j] > 0.f) ? p.gscale * d : 0.f;
            const float xh = (zv[0][j] - mean) * rstd;
            if (MODE == 1) {
              loss += d * d;
              sb += g;
              sg += g * xh;
            } else {
              ov[j] = f * (m * g - db - xh * dg);
            }
          }
        }
        if (MODE == 0) *reinterpret_cast<float4 *>(p.out + o0) = make_float4(ov[0], ov[1], ov[2], ov[3]);
        if (MODE == 2) *reinterpret_cast<float4 *>(p.dz + o0) = make_float4(ov[0], ov[1], ov[2], ov[3]);
      } else {
        const float tv[2] = {t2.x, t2.y};
        float pvv[2], dzv[2][4];
#pragma unroll
        for (int wv = 0; wv < 2; ++wv) {
          // window order (row, col): (0,0) (0,1) (1,0) (1,1); strict '>': the first maximum wins
          float pv = fmaxf(bv[0][2 * wv], 0.f);
          int best = 0;
#pragma unroll
          for (int k = 1; k < 4; ++k) {
            const float y = fmaxf(bv[k >> 1][2 * wv + (k & 1)], 0.f);
            if (y > pv) {
              pv = y;
              best = k;
            }
          }
          pvv[wv] = pv;
          if (MODE != 0) {
            const float d = pv - tv[wv];
            const float gk = (pv > 0.f) ? p.gscale * d : 0.f;
            if (MODE == 1) {
              loss += d * d;
              sb += gk;
              float xb = 0.f;
#pragma unroll
              for (int k = 0; k < 4; ++k)
                if (k == best) xb = (zv[k >> 1][2 * wv + (k & 1)] - mean) * rstd;
              sg += gk * xb;
            } else {
#pragma unroll
              for (int k = 0; k < 4; ++k) {
                const float g = (k == best) ? gk : 0.f;
                const float xh = (zv[k >> 1][2 * wv + (k & 1)] - mean) * rstd;
                dzv[k >> 1][2 * wv + (k & 1)] = f * (m * g - db - xh * dg);
              }
            }
          }
        }
        if (MODE == 0) *reinterpret_cast<float2 *>(p.out + toff) = make_float2(pvv[0], pvv[1]);
        if (MODE == 2) {
#pragma unroll
          for (int rr = 0; rr < 2; ++rr)
            *reinterpret_cast<float4 *>(p.dz + o0 + (size_t)rr * W) = make_float4(dzv[rr][0], dzv[rr][1], dzv[rr][2], dzv[rr][3]);
        }
      }
    }
  } else
  for (int idx = blockIdx.x * 256 + tid; idx < total; idx += gridDim.x * 256) {
    const int n = idx / (Hw * Ww);
    const int r = idx - n * (Hw * Ww);
    const int wi = r / Ww, wj = r - wi * Ww;
    const size_t plane = ((size_t)n * p.C + c);
    if (!POOL) {
      const size_t off = (plane * H + wi) * W + wj;
      const float z = p.z[off];
      float b = fmaf(z, sc, sh);
      if (hs) b = b + fmaf(p.zs[off], scs, shs);
      const float y = fmaxf(b, 0.f);
      if (MODE == 0) {
        p.out[off] = y;
      } else {
        const float d = y - p.t[off];
        const float g = (b > 0.f) ? p.gscale * d : 0.f;
        const float xh = (z - mean) * rstd;
        if (MODE == 1) {
          loss += d * d;
          sb += g;
          sg += g * xh;
        } else {
          p.dz[off] = f * (m * g - db - xh * dg);
        }
      }
    } else {
      float zv[4], bv[4];
      bool ok[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int yy = 2 * wi + (k >> 1), xx = 2 * wj + (k & 1);
        ok[k] = (yy < H) && (xx < W);
        zv[k] = 0.f;
        bv[k] = 0.f;
        if (ok[k]) {
          const size_t off = (plane * H + yy) * W + xx;
          zv[k] = p.z[off];
          float b = fmaf(zv[k], sc, sh);
          if (hs) b = b + fmaf(p.zs[off], scs, shs);
          bv[k] = b;
        }
      }
      const bool full = (wi < Hp) && (wj < Wp);
      int best = 0;
      float gk = 0.f, d = 0.f;
      if (full) {
        float pv = fmaxf(bv[0], 0.f);
#pragma unroll
        for (int k = 1; k < 4; ++k) {
          const float y = fmaxf(bv[k], 0.f);
          if (y > pv) {      // strict: the first maximum in row-major window order wins
            pv = y;
            best = k;
          }
        }
        const size_t toff = (plane * Hp + wi) * Wp + wj;
        if (MODE == 0) {
          p.out[toff] = pv;
        } else {
          d = pv - p.t[toff];
          gk = (pv > 0.f) ? p.gscale * d : 0.f;
        }
      }
      if (MODE == 1 && full) {
        loss += d * d;
        sb += gk;
        float xb = 0.f;
#pragma unroll
        for (int k = 0; k < 4; ++k)
          if (k == best) xb = (zv[k] - mean) * rstd;
        sg += gk * xb;
      }
      if (MODE == 2) {
#pragma unroll
        for (int k = 0; k < 4; ++k)
          if (ok[k]) {
            const int yy = 2 * wi + (k >> 1), xx = 2 * wj + (k & 1);
            const float g = (full && k == best) ? gk : 0.f;
            const float xh = (zv[k] - mean) * rstd;
            p.dz[(plane * H + yy) * W + xx] = f * (m * g - db - xh * dg);
          }
      }
    }
  }
  if (MODE == 1) {
    const float v0 = wave_sum(loss), v1 = wave_sum(sb), v2 = wave_sum(sg);
    if (lane == 0) {
      red[wave][0] = v0;
      red[wave][1] = v1;
      red[wave][2] = v2;
    }
    __syncthreads();
    if (tid < 3)
      p.partial[((size_t)blockIdx.x * p.C + c) * 3 + tid] = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
  }
}

hipError_t launch_head(int mode, const HeadArgs &a, hipStream_t s) {
  if (a.C > 65535 || a.n_blk < 1) return hipErrorInvalidValue;
  dim3 grid(a.n_blk, a.C), block(256);
  const bool pool = a.pool == 2;
  auto al16 = [](const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; };
  const bool vec = a.W % 4 == 0 && (!pool || a.H % 2 == 0) && al16(a.z) && al16(a.zs) && al16(a.t) && al16(a.out) && al16(a.dz);
#define PBKD_HEAD_HS(M, HS)                                                            \
  if (pool && vec)                                                                     \
    hipLaunchKernelGGL((head_kernel<M, true, true, HS>), grid, block, 0, s, a);        \
  else if (pool)                                                                       \
    hipLaunchKernelGGL((head_kernel<M, true, false, HS>), grid, block, 0, s, a);       \
  else if (vec)                                                                        \
    hipLaunchKernelGGL((head_kernel<M, false, true, HS>), grid, block, 0, s, a);       \
  else                                                                                 \
    hipLaunchKernelGGL((head_kernel<M, false, false, HS>), grid, block, 0, s, a);
#define PBKD_HEAD(M)       \
  if (a.zs != nullptr) {   \
    PBKD_HEAD_HS(M, true)  \
  } else {                 \
    PBKD_HEAD_HS(M, false) \
  }
  if (mode == 0) {
    PBKD_HEAD(0)
  } else if (mode == 1) {
    PBKD_HEAD(1)
  } else if (mode == 2) {
    PBKD_HEAD(2)
  } else {
    return hipErrorInvalidValue;
  }
#undef PBKD_HEAD
#undef PBKD_HEAD_HS
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void head_finalize_kernel(const float *partial, int n_blk, int C, float loss_scale,
                                                            float *dgamma, float *dbeta, float *loss) {
  __shared__ double red[256];
  const int tid = threadIdx.x;
  double lsum = 0.0;
  for (int c = tid; c < C; c += 256) {
    double l = 0.0, b = 0.0, g = 0.0;
    for (int t = 0; t < n_blk; ++t) {
      const float *q = partial + ((size_t)t * C + c) * 3;
      l += (double)q[0];
      b += (double)q[1];
      g += (double)q[2];
    }
    dbeta[c] = (float)b;
    dgamma[c] = (float)g;
    lsum += l;
  }
  red[tid] = lsum;
  __syncthreads();
  for (int d = 128; d >= 1; d >>= 1) {
    if (tid < d) red[tid] += red[tid + d];
    __syncthreads();
  }
  if (tid == 0) loss[0] = (float)(red[0] * (double)loss_scale);
}

hipError_t launch_head_finalize(const float *partial, int n_blk, int C, float loss_scale, float *dgamma, float *dbeta,
                                float *loss, hipStream_t s) {
  hipLaunchKernelGGL(head_finalize_kernel, dim3(1), dim3(256), 0, s, partial, n_blk, C, loss_scale, dgamma, dbeta, loss);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------ interior BN backward
template <bool VEC>
__global__ __launch_bounds__(256) void bn_bwd_apply_kernel(float *g, const float *z, const float *scale, const float *mean,
                                                           const float *rstd, float *dgamma, float *dbeta,
                                                           const float *__restrict__ dw_partial, int n_tiles, int N, int C,
                                                           int HW) {
  const int c = blockIdx.y;
  const float m = (float)N * (float)HW;
  float dg, db;
  if (dw_partial) {                            // at most 64 partials per channel: one per lane, then the same
    double sb = 0.0, sg = 0.0;                 // butterfly in every wave (same order, same bits)
    const int t = threadIdx.x & 63;
    if (t < n_tiles) {
      const float *q = dw_partial + ((size_t)t * C + c) * 11;
      sb = (double)q[9];
      sg = (double)q[10];
    }
    db = (float)wave_sum_d(sb);
    dg = (float)wave_sum_d(sg);
    if (blockIdx.x == 0 && threadIdx.x == 0) {
      dbeta[c] = db;
      dgamma[c] = dg;
    }
  } else {
    dg = dgamma[c];
    db = dbeta[c];
  }
  const float f = scale[c] / m, mu = mean[c], r = rstd[c];
  if (VEC) {                                   // HW % 4 == 0: 16 bytes per lane
    const int HW4 = HW >> 2, total = N * HW4;
    for (int idx = blockIdx.x * 256 + threadIdx.x; idx < total; idx += gridDim.x * 256) {
      const int n = idx / HW4;
      const int px = (idx - n * HW4) * 4;
      const size_t off = ((size_t)n * C + c) * HW + px;
      const float4 zv = *reinterpret_cast<const float4 *>(z + off);
      float4 gv = *reinterpret_cast<const float4 *>(g + off);
      gv.x = f * (m * gv.x - db - ((zv.x - mu) * r) * dg);
      gv.y = f * (m * gv.y - db - ((zv.y - mu) * r) * dg);
      gv.z = f * (m * gv.z - db - ((zv.z - mu) * r) * dg);
      gv.w = f * (m * gv.w - db - ((zv.w - mu) * r) * dg);
      *reinterpret_cast<float4 *>(g + off) = gv;
    }
  } else {
    const int total = N * HW;
    for (int idx = blockIdx.x * 256 + threadIdx.x; idx < total; idx += gridDim.x * 256) {
      const int n = idx / HW;
      const int px = idx - n * HW;
      const size_t off = ((size_t)n * C + c) * HW + px;
      const float xh = (z[off] - mu) * r;
      g[off] = f * (m * g[off] - db - xh * dg);
    }
  }
}

hipError_t launch_bn_bwd_apply(float *g, const float *z, const float *scale, const float *mean, const float *rstd,
                               float *dgamma, float *dbeta, const float *dw_partial, int n_tiles, int N, int C, int HW,
                               hipStream_t s) {
  if (C > 65535 || (dw_partial && (n_tiles < 1 || n_tiles > kBnBwdFoldMaxTiles))) return hipErrorInvalidValue;
  const bool vec = HW % 4 == 0 && (reinterpret_cast<uintptr_t>(g) & 15) == 0 && (reinterpret_cast<uintptr_t>(z) & 15) == 0;
  long long nb = ((long long)N * HW / (vec ? 4 : 1) + 1023) / 1024;
  if (nb < 1) nb = 1;
  if (nb > 64) nb = 64;
  if (vec)
    hipLaunchKernelGGL(bn_bwd_apply_kernel<true>, dim3((int)nb, C), dim3(256), 0, s, g, z, scale, mean, rstd, dgamma, dbeta, dw_partial, n_tiles, N, C, HW);
  else
    hipLaunchKernelGGL(bn_bwd_apply_kernel<false>, dim3((int)nb, C), dim3(256), 0, s, g, z, scale, mean, rstd, dgamma, dbeta, dw_partial, n_tiles, N, C, HW);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------ feature error
// mean((a - b)^2) in fp64, fixed order: 256 workgroups write one partial each, the last launch sums them
__global__ __launch_bounds__(256) void sqdiff_partial_kernel(const float *a, const float *b, size_t n, double *partial) {
  __shared__ double red[4];
  double acc = 0.0;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
    const double d = (double)a[i] - (double)b[i];
    acc += d * d;
  }
  acc = wave_sum_d(acc);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) partial[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}
__global__ __launch_bounds__(256) void sqdiff_final_kernel(const double *partial, int nparts, double inv_n, double *out) {
  __shared__ double red[4];
  double acc = threadIdx.x < nparts ? partial[threadIdx.x] : 0.0;
  acc = wave_sum_d(acc);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) out[0] = ((red[0] + red[1]) + (red[2] + red[3])) * inv_n;
}
hipError_t launch_feature_mse(const float *a, const float *b, size_t n, double *scratch257, hipStream_t s) {
  if (n == 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(sqdiff_partial_kernel, dim3(256), dim3(256), 0, s, a, b, n, scratch257);
  hipLaunchKernelGGL(sqdiff_final_kernel, dim3(1), dim3(256), 0, s, scratch257, 256, 1.0 / (double)n, scratch257 + 256);
  return hipGetLastError();
}

// The same two kernels for callers that may not allocate and hold no block workspace: the 256 partials and the result
// live in this array, of which every GPU the library runs on holds its own copy until the process ends (2056 bytes).
// In host code the array's name is only a stand-in; its device address on the current GPU comes from the runtime once
// per device and is what the kernels receive.
static __device__ __align__(256) double scratch[257];

hipError_t feature_mse_static_scratch(double **ptr_out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static double *ptr_of_device[kMaxDevices] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr_of_device[dev]) {
    double *p = nullptr;
    e = hipGetSymbolAddress(reinterpret_cast<void **>(&p), HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    ptr_of_device[dev] = p;
  }
  *ptr_out = ptr_of_device[dev];
  return hipSuccess;
}

// ------------------------------------------------------------------------------------------------ optimizer

// Gradient reduction and parameter update in one pass.  With many partials a workgroup serves 64 consecutive
// elements of one job's tensor: 16 waves each sum every 16th partial of those elements (fp64, index order, four loads in flight),
// wave 0 adds the 16 results in wave order, stores the gradient and updates the parameter.
__global__ __launch_bounds__(64 * RP_SLICES) void reduce_update_kernel(const GradJob *jobs, const int *job_of_block, float *theta,
                                                                       float *vel, float *grad, float lr, float mu,
                                                                       const int *map_f, const int *map_b, float *pk) {
  __shared__ double red[RP_SLICES][64];
  const GradJob jb = jobs[job_of_block[blockIdx.x]];
  if (jb.flat) {                               // block-uniform: one element per thread, its partials summed in index order
    const int i = (blockIdx.x - jb.first_block) * (64 * RP_SLICES) + threadIdx.x;
    if (i >= jb.count) return;
    const size_t a = (size_t)jb.arena_off + i;
    float gval;
    if (jb.kind == 2) {
      gval = grad[a];
    } else {
      size_t base, stride;
      if (jb.kind == 0) {
        base = (size_t)i;
        stride = (size_t)jb.count;
      } else {
        const int c = i / 9, k = i - c * 9;
        base = (size_t)c * 11 + k;
        stride = (size_t)jb.C * 11;
      }
      const float *src = jb.partial + base;
      double acc = 0.0;
      int t = 0;
      for (; t + 3 < jb.nparts; t += 4) {
        const float v0 = src[(size_t)t * stride], v1 = src[(size_t)(t + 1) * stride];
        const float v2 = src[(size_t)(t + 2) * stride], v3 = src[(size_t)(t + 3) * stride];
        acc += (double)v0;
        acc += (double)v1;
        acc += (double)v2;
        acc += (double)v3;
      }
      for (; t < jb.nparts; ++t) acc += (double)src[(size_t)t * stride];
      gval = (float)acc;
      grad[a] = gval;
    }
    const float v = mu * vel[a] + gval;
    vel[a] = v;
    const float th = theta[a] - lr * v;
    theta[a] = th;
    const int f = map_f[a], b = map_b[a];
    if (f >= 0) pk[f] = th;
    if (b >= 0) pk[b] = th;
    return;
  }
  const int o = threadIdx.x & 63, pl = threadIdx.x >> 6;
  const int i = (blockIdx.x - jb.first_block) * 64 + o;
  const bool ok = i < jb.count;
  if (jb.kind != 2) {                          // block-uniform
    double acc = 0.0;
    if (ok) {
      size_t base, stride;
      if (jb.kind == 0) {
        base = (size_t)i;
        stride = (size_t)jb.count;
      } else {
        const int c = i / 9, k = i - c * 9;
        base = (size_t)c * 11 + k;
        stride = (size_t)jb.C * 11;
      }
      const float *src = jb.partial + base;
      int t = pl;
      for (; t + 3 * RP_SLICES < jb.nparts; t += 4 * RP_SLICES) {   // four loads in flight, summed in index order
        const float v0 = src[(size_t)t * stride];
        const float v1 = src[(size_t)(t + RP_SLICES) * stride];
        const float v2 = src[(size_t)(t + 2 * RP_SLICES) * stride];
        const float v3 = src[(size_t)(t + 3 * RP_SLICES) * stride];
        acc += (double)v0;
        acc += (double)v1;
        acc += (double)v2;
        acc += (double)v3;
      }
      for (; t < jb.nparts; t += RP_SLICES) acc += (double)src[(size_t)t * stride];
    }
    red[pl][o] = acc;
    __syncthreads();
  }
  if (pl == 0 && ok) {
    const size_t a = (size_t)jb.arena_off + i;
    float gval;
    if (jb.kind != 2) {
      double v = red[0][o];
#pragma unroll
      for (int w = 1; w < RP_SLICES; ++w) v += red[w][o];
      gval = (float)v;
      grad[a] = gval;
    } else {
      gval = grad[a];
    }
    const float v = mu * vel[a] + gval;
    vel[a] = v;
    const float t = theta[a] - lr * v;
    theta[a] = t;
    const int f = map_f[a], b = map_b[a];
    if (f >= 0) pk[f] = t;
    if (b >= 0) pk[b] = t;
  }
}

hipError_t launch_reduce_update(const GradJob *jobs_dev, const int *job_of_block_dev, int n_blocks, float *theta, float *vel,
                                float *grad, float lr, float mu, const int *map_f, const int *map_b, float *pk, hipStream_t s) {
  if (n_blocks < 1) return hipSuccess;
  hipLaunchKernelGGL(reduce_update_kernel, dim3(n_blocks), dim3(64 * RP_SLICES), 0, s, jobs_dev, job_of_block_dev, theta, vel,
                     grad, lr, mu, map_f, map_b, pk);
  return hipGetLastError();
}

}  // namespace pbkd

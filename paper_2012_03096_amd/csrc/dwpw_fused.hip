// Depthwise 3x3 + pointwise 1x1 of one depthwise-separable layer in ONE kernel (stride 1): the depthwise output u
// is consumed as the matrix cores' B operand straight from LDS, so it is written once (the backward pass needs it)
// and never read back in the forward pass.  z[n,o,p] = sum_c P[o,c] * u[n,c,p],  u = D (*) act(in).
//
// A workgroup (4 waves) owns PX = WP*128 pixels -- nimg images x TH rows x TW columns, TW = 4, 8, 16 or 32, TH a
// multiple of 4 -- and BM = WM*32 output channels, and walks the input channels in stages of KC = 4096/PX channels:
//   phase A (all 256 threads): a thread computes the depthwise outputs of one channel on a 4 x 4 patch from the 6 x 6
//     window around it, read straight from global memory (one 16-byte and two edge loads per row) with the producing
//     layer's BatchNorm + ReLU applied on load; the 16 outputs go to LDS as [channel][pixel] (and to u in HBM, from
//     the first channel tile's workgroups only).  The window of chunk k+1 is fetched before the matrix phase of chunk
//     k, so its latency hides behind the MFMAs;
//   phase B: wave (wm, wp) multiplies its 32 channels x 128 pixels: lane n of a half-wave holds pixels 4n..4n+3 of the
//     wave's pixel group (one 16-byte LDS read per K-step), MFMA e of 4 uses element e, the half-waves take the two
//     channels of a K-step; the weights come from the packed image staged next to u.
// One barrier per chunk (two LDS copies).  Epilogue as in the pointwise kernel: vector stores of z and per-channel
// statistics partials.
#include "conv_mfma_kernel.h"

namespace pbkd {

constexpr int DP_UPAD = 4;         // floats of padding per LDS row of u
constexpr int dp_kc(int wp) { return 32 / wp; }   // input channels per stage: one 4 x 4 patch per thread

bool dwpw_ok(int N, int Cin, int Cout, int H, int W, int stride) {
  if (stride != 1 || H % 4 || W % 4) return false;
  if (!(W % 32 == 0 || W == 16 || W == 8 || W == 4)) return false;
  if ((unsigned long long)N * Cin * H * W * sizeof(float) >= (1ull << 32)) return false;
  (void)Cout;
  return true;
}

DwPwGeom dwpw_geom(int N, int Cin, int Cout, int H, int W) {
  DwPwGeom g{};
  g.wide = Cout <= 64 ? 1 : 0;                 // (WM, WP) = (2, 2): 64 channels x 256 pixels; else (4, 1): 128 x 128
  const int PX = g.wide ? 256 : 128;
  g.bm = g.wide ? 64 : 128;
  g.TW = W % 32 == 0 ? 32 : W;
  const int rows = PX / g.TW;                  // stacked rows of a tile
  g.TH = H < rows ? H : rows;
  // a tile holds whole images when an image has fewer rows than the tile (H a power of two then), else TH | H is needed
  g.ok = dwpw_ok(N, Cin, Cout, H, W, 1) && rows % g.TH == 0 && H % g.TH == 0 && g.TH % 4 == 0;
  g.nimg = rows / (g.TH > 0 ? g.TH : 1);
  g.tiles_x = W / g.TW;
  g.tiles_y = g.TH > 0 ? H / g.TH : 1;
  g.tiles_n = cdiv(N, g.nimg > 0 ? g.nimg : 1);
  g.n_ptiles = g.tiles_x * g.tiles_y * g.tiles_n;
  g.mtiles = cdiv(Cout, g.bm);
  g.nchunks = cdiv(Cin, KC1);
  g.lds_bytes = (size_t)2 * dp_kc(g.wide ? 2 : 1) * ((PX + DP_UPAD) + g.bm) * sizeof(float);
  const size_t red = (size_t)4 * g.bm * kStatFloats * sizeof(float);
  if (g.lds_bytes < red) g.lds_bytes = red;
  return g;
}

template <int WM, int WP>
__global__ __launch_bounds__(256, 2) void dwpw_fwd_kernel(DwPwArgs p) {
  static_assert(WM * WP == 4, "four waves");
  constexpr int BM = WM * 32;
  constexpr int PX = WP * 128;
  constexpr int USTR = PX + DP_UPAD;
  constexpr int PATCHES = PX / 16;              // 4 x 4 patches per channel
  constexpr int DP_KC = dp_kc(WP);              // = 256 / PATCHES: every thread computes one patch per stage
  constexpr int APT = DP_KC * BM / 256 / 4;     // 16-byte vectors of packed weights per thread and stage
  static_assert(DP_KC * PATCHES == 256 && APT >= 1, "one patch per thread and stage");
  typedef float f4 __attribute__((ext_vector_type(4)));
  extern __shared__ float smem[];
  float *Us = smem;                             // [2][DP_KC][USTR]
  float *As = smem + 2 * DP_KC * USTR;          // [2][DP_KC][BM]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l31 = lane & 31, lh = lane >> 5;
  const int wm = wave % WM, wp = wave / WM;
  const int TW = p.g.TW, TH = p.g.TH, TW4 = TW >> 2;
  const int H = p.H, W = p.W, HW = H * W;
  int pt = blockIdx.x;
  const int tx = pt % p.g.tiles_x;
  pt /= p.g.tiles_x;
  const int ty = pt % p.g.tiles_y;
  const int tn = pt / p.g.tiles_y;
  const int x0 = tx * TW, y0 = ty * TH, n0 = tn * p.g.nimg;
  const bool bn = p.in_scale != nullptr;
  const bool write_u = blockIdx.y == 0;

  // ---- phase A geometry: this thread's patch (the same for every chunk) and channel within a pass
  const int q = tid % PATCHES, cl = tid / PATCHES;
  const int qx = q % TW4, qy = q / TW4;
  const int prow = 4 * qy;                       // first stacked row of the patch
  const int pimg = prow / TH, py = y0 + prow % TH, px = x0 + 4 * qx;
  const int pn = n0 + pimg;
  const bool pact = pn < p.N;                    // (py, px) lie inside the map by construction
  const int ustrip = prow * TW4 + qx;            // strip index of the patch's first row; + TW4 per row

  // ---- phase B geometry: this lane's strip of 4 pixels
  const int s = wp * 32 + l31;
  const int srow = s / TW4, sx = s - srow * TW4;
  const int simg = srow / TH;
  const int sn = n0 + simg, sy = y0 + srow % TH, sxx = x0 + 4 * sx;
  const bool pvalid = sn < p.N;

  floatx16 acc[4];
#pragma unroll
  for (int e = 0; e < 4; ++e)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[e][r] = 0.f;

  float win[6][6];
  f4 areg[APT];
  // packed weights of this channel tile: [chunk of 32 channels][k][BM], i.e. [k][BM] over the zero-padded K
  const f4 *wsrc4 = reinterpret_cast<const f4 *>(p.wpk + (size_t)blockIdx.y * p.g.nchunks * (KC1 * BM));
  const int nstages = p.g.nchunks * (KC1 / DP_KC);

  auto fetch = [&](int k) {
#pragma unroll
    for (int j = 0; j < APT; ++j) areg[j] = wsrc4[(size_t)k * (DP_KC * BM / 4) + tid + 256 * j];
    const int c = k * DP_KC + cl;
    const bool act = pact && c < p.Cin;
    const int cc = c < p.Cin ? c : p.Cin - 1;
    float sc = 1.f, sh = 0.f;
    if (bn) sc = p.in_scale[cc], sh = p.in_shift[cc];
    const float *plane = p.in + ((size_t)(pact ? pn : 0) * p.Cin + cc) * HW;
    if (bn) {
#pragma unroll
      for (int r = 0; r < 6; ++r) dw_load_row<true>(plane, py - 1, r, px, H, W, act, sc, sh, win[r]);
    } else {
#pragma unroll
      for (int r = 0; r < 6; ++r) dw_load_row<false>(plane, py - 1, r, px, H, W, act, sc, sh, win[r]);
    }
  };

  fetch(0);
  for (int k = 0; k < nstages; ++k) {
    float *Ub = Us + (k & 1) * DP_KC * USTR;
    float *Ab = As + (k & 1) * DP_KC * BM;
    // ---- phase A: depthwise outputs of chunk k from the fetched windows
#pragma unroll
    for (int j = 0; j < APT; ++j) reinterpret_cast<f4 *>(Ab)[tid + 256 * j] = areg[j];
    {
      const int c = k * DP_KC + cl;
      const int cc = c < p.Cin ? c : p.Cin - 1;
      float w[9];
#pragma unroll
      for (int t = 0; t < 9; ++t) w[t] = p.D[cc * 9 + t];
      float *urow = Ub + cl * USTR + 4 * ustrip;
      float *ug = p.u_out + ((size_t)(pact ? pn : 0) * p.Cin + cc) * HW + (size_t)py * W + px;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        f4 o;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float a = 0.f;
#pragma unroll
          for (int ky = 0; ky < 3; ++ky)
#pragma unroll
            for (int kx = 0; kx < 3; ++kx) a += w[ky * 3 + kx] * win[i + ky][j + kx];
          o[j] = a;
        }
        *reinterpret_cast<f4 *>(urow + i * (4 * TW4)) = o;      // zeros where the window was inactive
        if (write_u && pact && c < p.Cin) *reinterpret_cast<f4 *>(ug + (size_t)i * W) = o;
      }
    }
    if (k + 1 < nstages) fetch(k + 1);            // in flight during the matrix phase
    __syncthreads();                              // copy k&1 is complete; every wave has finished chunk k-1
    // ---- phase B: 16 K-steps of 2 channels
    const float *Ap = Ab + lh * BM + wm * 32 + l31;
    const float *Bp = Ub + lh * USTR + 4 * s;
    float av = Ap[0];
    f4 bv = *reinterpret_cast<const f4 *>(Bp);
#pragma unroll
    for (int t = 0; t < DP_KC / 2; ++t) {
      float nav = av;
      f4 nbv = bv;
      if (t + 1 < DP_KC / 2) {
        nav = Ap[(2 * t + 2) * BM];
        nbv = *reinterpret_cast<const f4 *>(Bp + (2 * t + 2) * USTR);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[e] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv[e], acc[e], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      av = nav;
      bv = nbv;
    }
  }

  // ---- store: accumulator register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4; column l%32 = pixels 4*(l%32)+e
  const int mrow0 = blockIdx.y * BM + wm * 32;
  float *dst = p.z_out + (size_t)(pvalid ? sn : 0) * p.Cout * HW + (size_t)sy * W + sxx;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int o = mrow0 + 8 * (r / 4) + 4 * lh + (r % 4);
    if (o < p.Cout && pvalid) {
      f4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = acc[e][r];
      *reinterpret_cast<f4 *>(dst + (size_t)o * HW) = v;
    }
  }

  // ---- per-channel statistics partial over this workgroup's pixels (per-wave sums about the wave's first pixel,
  // re-expressed about one pivot and added).  A wave's first strip is valid whenever any of its strips is: validity
  // ends with growing image index, and strips are ordered by image.
  if (p.stat_partial) {
    __syncthreads();
    StatPart *red = reinterpret_cast<StatPart *>(smem);   // [WP][BM]
    const float cnt = half32_sum(pvalid ? 4.f : 0.f);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float pv = __shfl(acc[0][r], lane & 32, 64);
      float s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float d = pvalid ? acc[e][r] - pv : 0.f;
        s1 += d;
        s2 += d * d;
      }
      s1 = half32_sum(s1);
      s2 = half32_sum(s2);
      if (l31 == 0) {
        const int row = wm * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
        StatPart sp;
        sp.pivot = pv; sp.s1 = s1; sp.s2 = s2; sp.n = cnt;
        red[wp * BM + row] = sp;
      }
    }
    __syncthreads();
    for (int e = tid; e < BM; e += 256) {
      const int o = blockIdx.y * BM + e;
      if (o < p.Cout) {
        StatPart a = red[e];
#pragma unroll
        for (int w = 1; w < WP; ++w) stat_rebase_add(a, red[w * BM + e]);
        stat_store(p.stat_partial, (size_t)o * gridDim.x + blockIdx.x, a);
      }
    }
  }
}

hipError_t init_dwpw_attributes() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&dwpw_fwd_kernel<4, 1>), hipFuncAttributeMaxDynamicSharedMemorySize, MAX_LDS);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void *>(&dwpw_fwd_kernel<2, 2>), hipFuncAttributeMaxDynamicSharedMemorySize, MAX_LDS);
}

hipError_t launch_dwpw_fwd(const DwPwArgs &a, hipStream_t s) {
  const DwPwGeom &g = a.g;
  if (!g.ok || a.N <= 0 || a.Cin <= 0 || a.Cout <= 0 || g.mtiles > 65535 || !a.u_out || !a.z_out || !a.wpk) return hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(a.in) | reinterpret_cast<uintptr_t>(a.u_out) | reinterpret_cast<uintptr_t>(a.z_out)) & 15)
    return hipErrorInvalidValue;
  const dim3 grid(g.n_ptiles, g.mtiles), block(256);
  if (g.wide)
    hipLaunchKernelGGL((dwpw_fwd_kernel<2, 2>), grid, block, g.lds_bytes, s, a);
  else
    hipLaunchKernelGGL((dwpw_fwd_kernel<4, 1>), grid, block, g.lds_bytes, s, a);
  return hipGetLastError();
}

}  // namespace pbkd

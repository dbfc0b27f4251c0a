// 3x3 convolution of a block's FIRST layer when it has at most three input channels (the image itself):
// K = 9*Cin <= 27 is far too short for the general kernel, which pads every chunk to 8 channels x 9 taps = 72 and
// stages weights per chunk.  Here the K (channel, tap) terms are taken two at a time in NS = ceil(K/2) MFMA steps:
//   * a wave owns 32 of the workgroup's 64 output channels (waves 0/2: the first 32, waves 1/3: the second) and keeps
//     their whole weight matrix in NS registers for the kernel's lifetime, straight from the canonical OIHW tensor;
//   * a workgroup stages one halo tile of the input ([Cin][TH+2][TW+2], a few KB), fetched into registers while the
//     tile before it is computed (wave w fetches tile rows w, w+4, ...: all index arithmetic is scalar), and every
//     wave walks rows of 32 pixels: lane n fetches B[k][n] = tile[c][row + dy][n + dx] with one LDS read per step.
//     The two terms of a step (one per half-wave) are paired so that their tile offsets differ by 1, by a tile row
//     or by a tile plane: three lane address registers and a compile-time offset per step serve all steps;
//   * no input BatchNorm (a block input is raw), stride 1, zero padding 1.
// The layer writes 64 output values per 27 multiply-adds: it is bound by HBM writes (a kernel that does nothing but
// this kernel's stores takes three quarters of its time), with the MFMA time (K padded from 27 to 28, the matrix
// cores at the fp32 rate: about half of it) and the per-value statistics arithmetic behind.  A wave needs few
// registers (one accumulator block, 16 triples of pivot and sums), so four workgroups share a compute unit and one
// wave's MFMAs run under the others' stores, statistics and staging.  Workgroups are persistent (each walking tiles
// blockIdx.x, blockIdx.x + gridDim.x, ...), so the weights are set up once.  Epilogue: z, and per WORKGROUP one
// statistics partial of every channel over all its tiles.
#include <hip/hip_ext.h>

#include <cstdlib>

#include "conv_mfma_kernel.h"

namespace pbkd {

constexpr int CF_TW = 32;      // tile width = pixels of one MFMA column block
constexpr int CF_OCC = 4;      // workgroups per compute unit

// Tile height TH (TH/2 rows per wave): finer tiles leave a shorter last round of the persistent loop, at the price of
// more halo rows staged per output row.  PBKD_CF_TH (4 or 8) and PBKD_CF_OCC (workgroups per compute unit the grid is
// sized for) are tuning aids.
ConvFirstGeom conv_first_geom(int N, int Cin, int Cout, int H, int W) {
  ConvFirstGeom g;
  g.th = 8;
  if (const char *e = std::getenv("PBKD_CF_TH")) {
    const int v = std::atoi(e);
    if (v == 4 || v == 8) g.th = v;
  }
  g.tiles_x = cdiv(W, CF_TW);
  g.tiles_y = cdiv(H, g.th);
  g.n_tiles = N * g.tiles_x * g.tiles_y;
  // every workgroup walks the same number of tiles (up to one): as many workgroups as spread the rounds evenly
  int occ = CF_OCC;
  if (const char *e = std::getenv("PBKD_CF_OCC")) occ = std::atoi(e) >= 1 && std::atoi(e) <= 8 ? std::atoi(e) : CF_OCC;
  const int slots = 256 * occ;
  const int rounds = cdiv(g.n_tiles, slots);
  g.n_wgs = cdiv(g.n_tiles, rounds);
  g.mtiles = cdiv(Cout, 64);
  (void)Cin;
  return g;
}

// Step s of CIN input channels pairs the terms (channel, tap) first(s) [lanes 0-31] and second(s) [lanes 32-63]:
//   s = 4c + j, j < 4: taps (0,1) (3,4) (6,7) (2,5) of channel c;  then tap 8 of channels 0 and 1 (of channel 0 alone
//   if there is one channel);  then, with three channels, tap 8 of channel 2 alone.  A missing second term has weight 0.
// PLAIN: the output channels are a multiple of 64 and the width a multiple of the tile's: every value is stored and counted
template <int TH, int CIN, bool PLAIN>
__global__ __launch_bounds__(256, CF_OCC) void conv_first_kernel(ConvArgs p, ConvFirstGeom g) {
  constexpr int XS = CF_TW + 2, YS = TH + 2, CHS = XS * YS;
  constexpr int RPW = TH / 2;                       // rows per wave and tile
  constexpr int K = 9 * CIN, NS = (K + 1) / 2;
  constexpr int NLD = (CIN * YS + 3) / 4;           // halo rows per wave and tile
  __shared__ float xt[CIN * CHS];
  __shared__ StatPart red[4][32];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l31 = lane & 31, lh = lane >> 5;
  const int mbw = wave & 1, rw = wave >> 1;         // this wave's channel block and its first row in a tile
  const int m0 = blockIdx.y * 64;
  const int mw = m0 + mbw * 32;                     // the wave's first output channel
  const int HW = p.H * p.W;

  // ---- the terms of every step: channel and tap of the two half-waves, and which address register serves it
  struct Step { int c0, t0, c1, t1; };     // c1 < 0: no second term
  auto step_terms = [](int s) {
    constexpr int TA[4] = {0, 3, 6, 2}, TB[4] = {1, 4, 7, 5};
    if (s < 4 * CIN) return Step{s / 4, TA[s % 4], s / 4, TB[s % 4]};
    if (s == 4 * CIN) return Step{0, 8, CIN >= 2 ? 1 : -1, 8};
    return Step{2, 8, -1, 8};
  };
  auto tile_offset = [](int c, int tap) { return c * CHS + (tap / 3) * XS + (tap % 3); };
  // this lane's weights: row l31 of the wave's channel block, the term of its half-wave
  float wa[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    const Step st = step_terms(s);
    const int k = lh ? st.c1 * 9 + st.t1 : st.c0 * 9 + st.t0;
    const bool kok = lh ? st.c1 >= 0 : true;
    const int o = mw + l31;
    wa[s] = (kok && o < p.Cout) ? p.w_canon[(size_t)o * K + k] : 0.f;
  }
  // the lane's pixel in the staged tile, plus the second half-wave's distance to its term of a step
  const int lbase = rw * XS + l31;
  const int lb1 = lbase + (lh ? 1 : 0), lbx = lbase + (lh ? XS : 0), lbc = lbase + (lh ? CHS : 0);

  // the halo tile [CIN][YS][XS] of `tile` into registers: wave w fetches tile rows w, w + 4, ... (a row = one channel's
  // XS values of one image row), lane l < XS column l.  No load is under a condition: what lies outside the image (or
  // the tile) is read from the nearest real element and replaced by a zero, by `okm` bit i, when the values go to LDS.
  // The loads stay in flight while the caller goes on, and because none of them hides behind a branch the compiler
  // knows their number and waits for them, not for every store issued after them.
  auto fetch = [&](int tile, float (&v)[NLD], int &okm) {
    int t = tile;
    const int tx = t % g.tiles_x;
    t /= g.tiles_x;
    const int ty = t % g.tiles_y;
    const int n = t / g.tiles_y;
    const int x0 = tx * CF_TW, y0 = ty * TH;
    const float *src = p.in + (size_t)n * CIN * HW;
    const int x = x0 - 1 + lane;
    const bool colok = lane < XS && x >= 0 && x < p.W;
    const int xc = x < 0 ? 0 : (x >= p.W ? p.W - 1 : x);
    okm = 0;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int R = wave + 4 * i;                    // wave-uniform
      const int Rc = R < CIN * YS ? R : CIN * YS - 1;
      const int c = (Rc >= YS) + (Rc >= 2 * YS);
      const int y = y0 - 1 + (Rc - c * YS);
      const int yc = y < 0 ? 0 : (y >= p.H ? p.H - 1 : y);
      v[i] = src[(size_t)c * HW + (size_t)yc * p.W + xc];
      okm |= (colok && R < CIN * YS && y >= 0 && y < p.H) ? (1 << i) : 0;
    }
  };

  const __amdgpu_buffer_rsrc_t rout = __builtin_amdgcn_make_buffer_rsrc(
      p.out, 0, (int)((unsigned)p.N * p.Cout * HW * sizeof(float)), 0x00020000);
  const unsigned planeb = (unsigned)(HW * sizeof(float));
  constexpr unsigned kPastBuffer = 0xffffffffu;        // a lane offset the buffer's range check always rejects
  const int chlim = p.Cout - mw - 4 * lh;              // register r's channel row exists iff 8*(r/4) + r%4 < chlim

  // statistics: a lane sums its pixel column of every channel row about the value of the first pixel the wave computes
  // for that row (x = x0 of a row inside the image, held by lanes 0 and 32)
  float pv[16], s1[16], s2[16];
  float cnt = 0.f;
  bool have_pivot = false;                             // wave-uniform
#pragma unroll
  for (int r = 0; r < 16; ++r) pv[r] = s1[r] = s2[r] = 0.f;

  float nx[NLD];                                       // the next tile's halo, fetched while this one is computed
  int nok = 0;
  fetch((int)blockIdx.x < g.n_tiles ? blockIdx.x : 0, nx, nok);
  for (int tile = blockIdx.x; tile < g.n_tiles; tile += gridDim.x) {
    int t = tile;
    const int tx = t % g.tiles_x;
    t /= g.tiles_x;
    const int ty = t % g.tiles_y;
    const int n = t / g.tiles_y;
    const int x0 = tx * CF_TW, y0 = ty * TH;
    __syncthreads();                                   // the previous tile has been consumed
#pragma unroll
    for (int i = 0; i < NLD; ++i)
      if (lane < XS && wave + 4 * i < CIN * YS) xt[(wave + 4 * i) * XS + lane] = ((nok >> i) & 1) ? nx[i] : 0.f;
    __syncthreads();
    {
      const int next = tile + (int)gridDim.x;        // (the last tile fetches itself again: no condition, see fetch)
      fetch(next < g.n_tiles ? next : tile, nx, nok);
    }
    const int x = x0 + l31;
    const bool xok = PLAIN || x < p.W;
#pragma unroll
    for (int jr = 0; jr < RPW; ++jr) {
      const int i = rw + 2 * jr;
      const int y = y0 + i;
      if (y >= p.H) break;                             // wave-uniform
      floatx16 acc;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.f;
      float bv[NS];
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        const Step st = step_terms(s);
        const int o0 = tile_offset(st.c0, st.t0) + jr * (2 * XS);
        const int d = st.c1 < 0 ? 0 : tile_offset(st.c1, st.t1) - tile_offset(st.c0, st.t0);
        bv[s] = xt[(d == 0 ? lbase : d == 1 ? lb1 : d == XS ? lbx : lbc) + o0];
      }
#pragma unroll
      for (int s = 0; s < NS; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(wa[s], bv[s], acc, 0, 0, 0);
      // accumulator register r of lane l holds channel row 8*(r/4) + 4*(l/32) + r%4, pixel column l%32
      if (!have_pivot) {
#pragma unroll
        for (int r = 0; r < 16; ++r) pv[r] = __shfl(acc[r], lane & 32, 64);
        have_pivot = true;
      }
      // one buffer store per value: the channel's plane offset a scalar, the lane's pixel a vector offset; lanes past
      // the image's right edge, or whose channel does not exist, get an offset past the buffer: the store is dropped
      const unsigned vo = xok ? (unsigned)((((size_t)n * p.Cout + m0 + 4 * lh) * HW + (size_t)y * p.W + x) * sizeof(float)) : kPastBuffer;
      if (PLAIN) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const unsigned so = (unsigned)(mbw * 32 + 8 * (r / 4) + (r % 4)) * planeb;
          const float v = acc[r];              // (a bit cast applied to the vector element itself reads element 0)
          __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), rout, vo, so, 0);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float d = acc[r] - pv[r];
          s1[r] += d;
          s2[r] += d * d;
        }
        cnt += 1.f;
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const unsigned so = (unsigned)(mbw * 32 + 8 * (r / 4) + (r % 4)) * planeb;
          const float v = acc[r];
          const unsigned vor = (8 * (r / 4) + (r % 4) < chlim) ? vo : kPastBuffer;
          __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), rout, vor, so, 0);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float d = xok ? acc[r] - pv[r] : 0.f;            // (channels past Cout: their sums are never stored)
          s1[r] += d;
          s2[r] += d * d;
        }
        cnt += xok ? 1.f : 0.f;
      }
    }
  }

  // ---- per-channel statistics partial over this workgroup's tiles, for BatchNorm's batch statistics: the sums of the
  // two waves of a channel block re-expressed about one pivot and added
  if (p.stat_partial) {
    cnt = half32_sum(cnt);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float a = half32_sum(s1[r]), b = half32_sum(s2[r]);
      if (l31 == 0) {
        const int rowi = 8 * (r / 4) + 4 * lh + (r % 4);
        StatPart sp;
        sp.pivot = pv[r]; sp.s1 = a; sp.s2 = b; sp.n = cnt;
        red[wave][rowi] = sp;
      }
    }
    __syncthreads();
    if (tid < 64 && m0 + tid < p.Cout) {
      StatPart a = red[tid >> 5][tid & 31];
      stat_rebase_add(a, red[2 + (tid >> 5)][tid & 31]);
      stat_store(p.stat_partial, (size_t)(m0 + tid) * gridDim.x + blockIdx.x, a);
    }
  }
}

hipError_t launch_conv_first(const ConvArgs &a, const ConvFirstGeom &g, hipStream_t s, hipEvent_t ev_start, hipEvent_t ev_stop) {
  if ((unsigned long long)a.N * a.Cout * a.H * a.W * sizeof(float) >= (1ull << 32)) return hipErrorInvalidValue;   // 32-bit store offsets
  if (!conv_first_ok(a.Cin, a.stride) || a.Cin < 1 || a.Cin > 3 || a.in_scale || !a.w_canon || a.H != a.Ho || a.W != a.Wo || g.mtiles > 65535 || g.n_tiles < 1 || g.n_wgs < 1 || g.n_wgs > g.n_tiles ||
      (g.th != 4 && g.th != 8) || g.tiles_y != cdiv(a.H, g.th))
    return hipErrorInvalidValue;
  const dim3 grid(g.n_wgs, g.mtiles), block(256);
  const bool plain = a.Cout % 64 == 0 && a.W % CF_TW == 0;
#define PBKD_CF1(TH, CIN, PLAIN)                                                                                   \
  if (g.th == TH && a.Cin == CIN && plain == PLAIN) {                                                              \
    if (ev_start && ev_stop)                                                                                       \
      hipExtLaunchKernelGGL((conv_first_kernel<TH, CIN, PLAIN>), grid, block, 0, s, ev_start, ev_stop, 0, a, g);   \
    else                                                                                                           \
      hipLaunchKernelGGL((conv_first_kernel<TH, CIN, PLAIN>), grid, block, 0, s, a, g);                            \
  }
#define PBKD_CF(TH, CIN) PBKD_CF1(TH, CIN, true) PBKD_CF1(TH, CIN, false)
  PBKD_CF(8, 3) PBKD_CF(8, 2) PBKD_CF(8, 1) PBKD_CF(4, 3) PBKD_CF(4, 2) PBKD_CF(4, 1)
#undef PBKD_CF
#undef PBKD_CF1
  return hipGetLastError();
}

}  // namespace pbkd

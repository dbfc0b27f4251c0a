// 3x3 convolution of a block's FIRST layer when it has at most three input channels (the image itself):
// K = 9*Cin <= 27 is far too short for the general kernel, which pads every chunk to 8 channels x 9 taps = 72 and
// stages weights per chunk.  Here K is the flattened (channel, tap) index padded to 32 = 16 MFMA steps:
//   * the whole weight matrix of a wave's 64 output channels lives in 32 registers for the kernel's lifetime
//     (A[m][k] = W[o][k] straight from the canonical OIHW tensor, k = c*9 + tap);
//   * a workgroup stages one halo tile of the input ([Cin][TH+2][TW+2], a few KB) and every wave walks rows of
//     32 pixels: lane n fetches B[k][n] = tile[c][row + dy][n + dx] with one LDS read per step, the offset of
//     step t being a per-lane constant (the half-waves hold the two k of a step);
//   * no input BatchNorm (a block input is raw), stride 1, zero padding 1.
// What remains is writing the output: the layer is bound by HBM writes.  Workgroups are persistent (two per compute
// unit, each walking tiles blockIdx.x, blockIdx.x + gridDim.x, ...), so the weights and tap offsets are set up once
// and two workgroups hide each other's staging and stores.  Epilogue: z, and per WORKGROUP one statistics partial
// of every channel over all its tiles.
#include <hip/hip_ext.h>

#include "conv_mfma_kernel.h"

namespace pbkd {

constexpr int CF_TW = 32;      // tile width = pixels of one MFMA column block
constexpr int CF_TH = 16;      // tile height: four rows per wave

ConvFirstGeom conv_first_geom(int N, int Cin, int Cout, int H, int W) {
  ConvFirstGeom g;
  g.tiles_x = cdiv(W, CF_TW);
  g.tiles_y = cdiv(H, CF_TH);
  g.n_tiles = N * g.tiles_x * g.tiles_y;
  g.n_wgs = g.n_tiles < 512 ? g.n_tiles : 512;
  g.mtiles = cdiv(Cout, 64);
  (void)Cin;
  return g;
}

__global__ __launch_bounds__(256, 2) void conv_first_kernel(ConvArgs p, ConvFirstGeom g) {
  constexpr int XS = CF_TW + 2, YS = CF_TH + 2, CHS = XS * YS;
  __shared__ float xt[3 * CHS];
  __shared__ StatPart red[4][64];
  __shared__ __attribute__((aligned(16))) float pivs[4][64];   // per wave: the statistics pivot of every channel row
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l31 = lane & 31, lh = lane >> 5;
  const int m0 = blockIdx.y * 64;
  const int K = 9 * p.Cin;
  const int HW = p.H * p.W;

  // ---- this lane's weights (rows l31 and 32 + l31 of the channel block, k = 2*step + half-wave) and tap offsets
  float wa[2][16];
  int kofw[16];            // where step s finds its input value for the wave's first row and this lane's column
#pragma unroll
  for (int s = 0; s < 16; ++s) {
    const int k = 2 * s + lh;
    const bool kok = k < K;
    const int c = kok ? k / 9 : 0, tap = kok ? k - c * 9 : 0;
    kofw[s] = c * CHS + (tap / 3) * XS + (tap % 3) + wave * XS + l31;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
      const int o = m0 + mb * 32 + l31;
      wa[mb][s] = (kok && o < p.Cout) ? p.w_canon[(size_t)o * K + k] : 0.f;
    }
  }

  const bool full = m0 + 64 <= p.Cout;                 // workgroup-uniform
  const __amdgpu_buffer_rsrc_t rout = __builtin_amdgcn_make_buffer_rsrc(
      p.out, 0, (int)((unsigned)p.N * p.Cout * HW * sizeof(float)), 0x00020000);
  const unsigned planeb = (unsigned)(HW * sizeof(float));

  // statistics: every wave sums about the values of the first pixel it computes (x = x0 of a row inside the image).
  // Those 64 pivots live in LDS, written and read by this wave only, and are fetched again for every row of pixels:
  // kept in registers they would cost the second workgroup per compute unit.
  float s1[2][16], s2[2][16];
  float cnt = 0.f;
  bool have_pivot = false;                             // wave-uniform
#pragma unroll
  for (int mb = 0; mb < 2; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) s1[mb][r] = s2[mb][r] = 0.f;
  if (lane < 64) pivs[wave][lane] = 0.f;

  for (int tile = blockIdx.x; tile < g.n_tiles; tile += gridDim.x) {
    int t = tile;
    const int tx = t % g.tiles_x;
    t /= g.tiles_x;
    const int ty = t % g.tiles_y;
    const int n = t / g.tiles_y;
    const int x0 = tx * CF_TW, y0 = ty * CF_TH;
    __syncthreads();                                   // the previous tile has been consumed
    // ---- the input halo tile (zero outside the image)
    for (int q = tid; q < p.Cin * CHS; q += 256) {
      const int c = q / CHS, r = q - c * CHS;
      const int iy = r / XS, ix = r - iy * XS;
      const int y = y0 - 1 + iy, x = x0 - 1 + ix;
      float v = 0.f;
      if (y >= 0 && y < p.H && x >= 0 && x < p.W) v = p.in[((size_t)n * p.Cin + c) * HW + (size_t)y * p.W + x];
      xt[q] = v;
    }
    __syncthreads();
    const int x = x0 + l31;
    const bool xok = x < p.W;
#pragma unroll
    for (int jr = 0; jr < CF_TH / 4; ++jr) {
      const int i = wave + 4 * jr;
      const int y = y0 + i;
      if (y >= p.H) break;                             // wave-uniform
      floatx16 acc[2];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mb][r] = 0.f;
      float bv[16];
#pragma unroll
      for (int s = 0; s < 16; ++s) bv[s] = xt[kofw[s] + jr * (4 * XS)];   // lane address + a constant per row
#pragma unroll
      for (int s = 0; s < 16; ++s)
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) acc[mb] = __builtin_amdgcn_mfma_f32_32x32x2f32(wa[mb][s], bv[s], acc[mb], 0, 0, 0);
      // accumulator register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32
      if (!have_pivot) {                               // lanes 0 and 32 hold pixel x0 (inside the image) of their rows
        if (l31 == 0) {
#pragma unroll
          for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r) pivs[wave][mb * 32 + 8 * (r / 4) + 4 * lh + (r % 4)] = acc[mb][r];
        }
        have_pivot = true;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // same wave reads them back: order only
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      }
      cnt += xok ? 1.f : 0.f;
      if (full) {
        // all 64 channels exist: one buffer store per value, the channel's plane offset a scalar, the lane's pixel a
        // vector offset (lanes past the image's right edge get an offset past the buffer: the store is dropped)
        const unsigned vo = xok ? (unsigned)((((size_t)n * p.Cout + m0 + 4 * lh) * HW + (size_t)y * p.W + x) * sizeof(float)) : 0xffffffffu;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const unsigned so = (unsigned)(mb * 32 + 8 * (r / 4) + (r % 4)) * planeb;
            const float v = acc[mb][r];        // (a bit cast applied to the vector element itself reads element 0)
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), rout, vo, so, 0);
          }
      } else {
        float *dst = p.out + (size_t)n * p.Cout * HW + (size_t)y * p.W + x;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int o = m0 + mb * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
            if (xok && o < p.Cout) dst[(size_t)o * HW] = acc[mb][r];
          }
      }
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          typedef float f4 __attribute__((ext_vector_type(4)));
          const f4 pv = *reinterpret_cast<const f4 *>(&pivs[wave][mb * 32 + 8 * q + 4 * lh]);
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int r = 4 * q + j;
            const float d = xok ? acc[mb][r] - pv[j] : 0.f;     // (channels past Cout: their sums are never stored)
            s1[mb][r] += d;
            s2[mb][r] += d * d;
          }
        }
    }
  }

  // ---- per-channel statistics partial over this workgroup's tiles, for BatchNorm's batch statistics: the four
  // waves' sums re-expressed about one pivot and added
  if (p.stat_partial) {
    cnt = half32_sum(cnt);
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float a = half32_sum(s1[mb][r]), b = half32_sum(s2[mb][r]);
        if (l31 == 0) {
          const int rowi = mb * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
          StatPart sp;
          sp.pivot = pivs[wave][rowi]; sp.s1 = a; sp.s2 = b; sp.n = cnt;
          red[wave][rowi] = sp;
        }
      }
    __syncthreads();
    if (tid < 64 && m0 + tid < p.Cout) {
      StatPart a = red[0][tid];
#pragma unroll
      for (int w = 1; w < 4; ++w) stat_rebase_add(a, red[w][tid]);
      stat_store(p.stat_partial, (size_t)(m0 + tid) * gridDim.x + blockIdx.x, a);
    }
  }
}

hipError_t launch_conv_first(const ConvArgs &a, const ConvFirstGeom &g, hipStream_t s, hipEvent_t ev_start, hipEvent_t ev_stop) {
  if ((unsigned long long)a.N * a.Cout * a.H * a.W * sizeof(float) >= (1ull << 32)) return hipErrorInvalidValue;   // 32-bit store offsets
  if (!conv_first_ok(a.Cin, a.stride) || a.in_scale || !a.w_canon || a.H != a.Ho || a.W != a.Wo || g.mtiles > 65535 || g.n_tiles < 1 || g.n_wgs < 1 || g.n_wgs > g.n_tiles)
    return hipErrorInvalidValue;
  if (ev_start && ev_stop)
    hipExtLaunchKernelGGL(conv_first_kernel, dim3(g.n_wgs, g.mtiles), dim3(256), 0, s, ev_start, ev_stop, 0, a, g);
  else
    hipLaunchKernelGGL(conv_first_kernel, dim3(g.n_wgs, g.mtiles), dim3(256), 0, s, a, g);
  return hipGetLastError();
}

}  // namespace pbkd

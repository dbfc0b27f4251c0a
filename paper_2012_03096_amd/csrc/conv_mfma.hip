// Implicit-GEMM 3x3 convolution on the fp32 matrix cores of gfx950 (v_mfma_f32_32x32x2_f32), staged
// through LDS: host side (tile choice, geometry, launch).  Serves the teacher's 3x3 convolutions and a
// trainable full 3x3 first layer of a student.  The device code is in conv_mfma_kernel.h.
//
// GEMM view: M = Cout, N = output pixels, K = 9*Cin.  A = weights, B = activations, so that the 32
// MFMA columns held by 32 consecutive lanes are 32 consecutive pixels and stores to NCHW coalesce.
// A workgroup (4 MFMA waves + 4 loader waves) owns a tile of 128x128, 64x256, 64x128 or 64x64 (channels x
// pixels); a pixel tile is nimg whole images x TH x TW (powers of two), so small feature maps pack several
// images per tile.  Per chunk of 8 input channels the loaders stage the packed weights and ONE halo tile of
// the input; the nine taps are read from that halo tile with a constant offset, no im2col is materialised.
#include <cstdlib>

#include "conv_mfma_kernel.h"

namespace pbkd {

// Tile choice.  Large tiles reuse staged operands best, so take the largest tile that still gives every
// one of the 256 compute units a workgroup, else the smallest (measured on the VGG/ResNet shapes: 128x128
// for 16x16 maps with 128 channels, 64x128 for 8x8 maps, 64x64 for 4x4 and 2x2 maps, 64x256 when there
// are only 64 output channels).  PBKD_CONV_TILE=0..3 overrides the choice (tuning aid).
static const int kBM[4] = {128, 64, 64, 64}, kBN[4] = {128, 256, 128, 64};
static ConvGeom conv_geom_for_tile(int tile, int taps, int N, int Cin, int Cout, int Ho, int Wo, int stride, bool want_split);

ConvGeom conv_geom(int taps, int N, int Cin, int Cout, int Ho, int Wo, int stride, bool want_split) {
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
    if (t >= 0 && t < 4) return conv_geom_for_tile(t, taps, N, Cin, Cout, Ho, Wo, stride, want_split);
  }
  // (For the bf16-split kernel larger tiles with K split over workgroups were measured on the small maps: 512 channels
  // on 4x4 maps 72 -> 58 + 6.5 us for the finishing kernel with 64x128 tiles and two splits, 256 channels on 8x8 maps
  // level; the all-block step got 3 % slower with either (1.14 -> 1.18 ms, three runs each on one box): not taken.)
  return conv_geom_for_tile(tile, taps, N, Cin, Cout, Ho, Wo, stride, want_split);
}

static ConvGeom conv_geom_for_tile(int tile, int taps, int N, int Cin, int Cout, int Ho, int Wo, int stride, bool want_split) {
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
  // LDS strides, in pixels of 16 bytes (4 banks): 8 consecutive lanes of a 16-byte read must fall into 8
  // different groups of 4 banks for every tap.  Within a row they do; where 8 lanes span several rows
  // (TW < 8) or images (TH*TW < 8) the row / image stride is made congruent to TW / TH*TW modulo 8
  // (stride-1 convolutions; with stride 2 a two-way conflict remains)
  g.IWS = g.IW;
  if (TW < 8) while (g.IWS % 8 != TW % 8) ++g.IWS;
  g.IMS = g.IH * g.IWS;
  if (TH * TW < 8) while (g.IMS % 8 != (TH * TW) % 8) ++g.IMS;
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
  const size_t red = (size_t)4 * g.bm * kStatFloats;   // the statistics epilogue's [waves][bm] partials
  if (fl < red) fl = red;
  g.lds_bytes = fl * sizeof(float);
  // Small maps with many channels (2x2 x 512) leave even the smallest tile with far fewer workgroups than compute
  // units while K = 9*Cin is long: split K over gridDim.z, up to one workgroup per compute unit and at least four
  // chunks per split; a second kernel adds the partial outputs.  Only where a pixel tile is whole images (the second
  // kernel's statistics partials are per group of nimg images).  PBKD_CONV_KSPLIT=n overrides (tuning aid).
  g.ksplit = 1;
  if (g.tiles_x == 1 && g.tiles_y == 1) {
    const long long wgs = (long long)g.mtiles * g.n_ptiles;
    long long want = 256 / wgs;
    if (want > g.nchunks / 4) want = g.nchunks / 4;
    if (want > 8) want = 8;
    if (const char *env = std::getenv("PBKD_CONV_KSPLIT")) want = std::atoi(env);
    if (want > g.nchunks) want = g.nchunks;
    if (want > 1) g.ksplit = (int)want;
  }
  g.kchunks = cdiv(g.nchunks, g.ksplit);
  g.ksplit = cdiv(g.nchunks, g.kchunks);          // no empty split
  // bf16-split kernel where its staging fits.  A tile must have at least two chunks wherever statistics are taken (its
  // statistics exchange has one copy).
  g.split = false;
  // a raw row: from four columns left of the tile (three spare + the halo) to its right halo column; where one tile
  // spans the map's width (both halo columns outside the image), just the map's columns (stride*Wo of them: the input
  // width is a multiple of 4 wherever this kernel runs)
  g.raw_lead = (g.tiles_x == 1) ? 0 : 4;
  g.raw_w = (g.tiles_x == 1) ? 4 * cdiv(stride * Wo, 4) : 4 * cdiv(g.IW + 3, 4);
  // a tile of whole images (stride 1): the unit is the channel plane, H*W contiguous values, whatever the width (2x2,
  // 6x6, 14x14 maps: H*W a multiple of 4 where the width is not)
  g.raw_plane = (g.tiles_x == 1 && g.tiles_y == 1 && stride == 1 && (Ho * Wo) % 4 == 0) ? 1 : 0;
  if (g.raw_plane) g.raw_w = Ho * Wo;
  g.raw_bytes = 8 * g.nimg * (g.raw_plane ? 1 : g.IH) * g.raw_w * (int)sizeof(float);
  g.raw_rounds = cdiv(g.raw_bytes / 16, 256);
  if (want_split && taps == 9) {
    static const int kWGN[4] = {2, 4, 4, 2};          // waves along the pixels of tiles 0..3
    const size_t need = conv_split_lds_bytes(g.bm, kWGN[tile], g.PL, g.raw_bytes);
    const int slots = conv_bslots_for(g.PLd);
    // the two large tiles keep every register busy: with more than two halo slots per thread they would spill
    if (need <= (size_t)MAX_LDS && slots != 0 && g.raw_rounds <= conv_split_rounds_max(slots) && (tile >= 2 || slots <= 2) &&
        g.IH < 256 && g.IW < 256 && (g.ksplit > 1 || g.nchunks >= 2)) {
      g.split = true;
      g.lds_bytes = need;
    }
  }
  return g;
}

// One wave per (group of nimg images, channel): adds the splits' partial outputs in split order, stores the sum and
// leaves the statistics partial of the group's pixels (summed about the group's first value) where the unsplit
// kernel's epilogue would.
__global__ __launch_bounds__(64) void conv_ksplit_finish_kernel(const float *part, int ksplit, size_t split_stride, float *out,
                                                                float *stat_partial, int N, int C, int HW, int nimg) {
  const int t = blockIdx.x, c = blockIdx.y, lane = threadIdx.x;
  const int n_first = t * nimg;
  const int n_imgs = (N - n_first < nimg) ? N - n_first : nimg;
  float s1 = 0.f, s2 = 0.f, pv = 0.f;
  for (int e0 = 0; e0 < n_imgs * HW; e0 += 64) {      // wave-uniform trip count
    const int e = e0 + lane;
    float v = 0.f;
    if (e < n_imgs * HW) {
      const int img = e / HW, px = e - img * HW;
      const size_t off = ((size_t)(n_first + img) * C + c) * HW + px;
      v = part[off];
      for (int s = 1; s < ksplit; ++s) v += part[(size_t)s * split_stride + off];
      out[off] = v;
    }
    if (e0 == 0) pv = __shfl(v, 0, 64);               // element 0 always exists
    if (e < n_imgs * HW) {
      const float d = v - pv;
      s1 += d;
      s2 += d * d;
    }
  }
  if (stat_partial) {
    s1 = wave64_sum(s1);
    s2 = wave64_sum(s2);
    if (lane == 0) {
      StatPart a;
      a.pivot = pv; a.s1 = s1; a.s2 = s2; a.n = (float)(n_imgs * HW);
      stat_store(stat_partial, (size_t)c * gridDim.x + t, a);
    }
  }
}

hipError_t launch_conv_ksplit_finish(const ConvArgs &a, hipStream_t s) {
  if (a.g.ksplit < 2 || !a.split_out || a.g.tiles_x != 1 || a.g.tiles_y != 1 || a.Cout > 65535) return hipErrorInvalidValue;
  hipLaunchKernelGGL(conv_ksplit_finish_kernel, dim3(a.g.n_ptiles, a.Cout), dim3(64), 0, s, a.split_out, a.g.ksplit,
                     (size_t)a.N * a.Cout * a.Ho * a.Wo, a.out, a.stat_partial, a.N, a.Cout, a.Ho * a.Wo, a.g.nimg);
  return hipGetLastError();
}

hipError_t init_conv_attributes() {
  hipError_t e;
  if ((e = conv_tile0_init()) != hipSuccess) return e;
  if ((e = conv_tile1_init()) != hipSuccess) return e;
  if ((e = conv_tile2_init()) != hipSuccess) return e;
  if ((e = conv_tile3_init()) != hipSuccess) return e;
  return conv_split_init();
}

hipError_t launch_conv(int taps, const ConvArgs &a, hipStream_t s, hipEvent_t ev_start, hipEvent_t ev_stop) {
  if (a.g.lds_bytes > (size_t)MAX_LDS) return hipErrorInvalidValue;
  if (a.N <= 0 || a.Cout <= 0 || a.Cin <= 0) return hipErrorInvalidValue;
  if (a.g.split) return launch_conv_split(a, s, ev_start, ev_stop);
  switch (a.g.tile) {
    case 0: return conv_tile0_launch(taps, a, s, ev_start, ev_stop);
    case 1: return conv_tile1_launch(taps, a, s, ev_start, ev_stop);
    case 2: return conv_tile2_launch(taps, a, s, ev_start, ev_stop);
    case 3: return conv_tile3_launch(taps, a, s, ev_start, ev_stop);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace pbkd

// Internal declarations shared by the kernel file and the host runtime of libpbkd.so.
// Nothing here is part of the public C ABI (see include/pbkd.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace pbkd {

inline int pow2ceil(int v) {
  int p = 1;
  while (p < v) p <<= 1;
  return p;
}
inline int ilog2(int v) {
  int l = 0;
  while ((1 << l) < v) ++l;
  return l;
}
inline int cdiv(int a, int b) { return (a + b - 1) / b; }
inline int out_dim(int in, int s) { return (in - 1) / s + 1; }

#if defined(__HIPCC__)
// Cross-lane sums on the VALU's data-parallel-primitive path instead of LDS permutes.
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
// every lane receives the sum over its row of 16 lanes
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_mov<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_mov<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_mov<0x141>(v);   // row_half_mirror
  v += dpp_mov<0x140>(v);   // row_mirror
  return v;
}
// every lane receives the sum over its half-wave (lanes 0-31 or 32-63)
__device__ __forceinline__ float half32_sum(float v) {
  v = row16_sum(v);
  v += __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F));   // lane ^ 16
  return v;
}
// the sum over a half-wave, valid only in that half-wave's lanes 16-31: no LDS permute
__device__ __forceinline__ float half32_sum_upper(float v) {
  v = row16_sum(v);
  return v + dpp_mov<0x142>(v);    // row_bcast:15: lane 15 of the row below
}
__device__ __forceinline__ float wave64_sum(float v) {
  v = half32_sum(v);
  return v + __shfl_xor(v, 32, 64);
}
#endif

#if defined(__HIPCC__)
// Workgroups are handed to the chip's 8 accelerator dies (XCDs, each with an L2 of its own) round robin by their
// linear index, so neighbouring indices never share an L2.  This maps workgroup `b` of `n` to a logical tile such that
// die k works through one contiguous range of tiles: tiles that overlap (halo rows and columns, shared operand rows)
// then meet in one L2 instead of being fetched once per die.  A bijection on [0, n).
__device__ __forceinline__ int xcd_contiguous(int b, int n) {
  const int per = n >> 3, rem = n & 7, k = b & 7, j = b >> 3;
  return k * per + (k < rem ? k : rem) + j;
}
#endif

// ------------------------------------------------------------------ BatchNorm statistics partials
// A convolution leaves, per output channel and pixel tile, the sums of (z - pivot) and (z - pivot)^2 over the tile's
// n values, where pivot is one of those values.  Sums about a value inside the data do not cancel when a channel's
// |mean| is many standard deviations (a one-pass E[z^2] - mean^2 loses (mean/sigma)^2 times the rounding error of its
// sums); whoever finishes the statistics re-expresses every partial about one common pivot in fp64 and adds them.
// A partial with n == 0 is all zeros.
struct __attribute__((aligned(16))) StatPart {
  float pivot, s1, s2, n;
};
#if defined(__HIPCC__)
// acc += w, with w's sums re-expressed about acc's pivot: sum (z-P)^2 = sum (z-p)^2 + 2d sum (z-p) + n d^2, d = p - P
__device__ __forceinline__ void stat_rebase_add(StatPart &acc, const StatPart &w) {
  if (w.n > 0.f) {
    if (!(acc.n > 0.f)) {
      acc = w;
    } else {
      const float d = w.pivot - acc.pivot;
      acc.s1 += w.s1 + w.n * d;
      acc.s2 += w.s2 + d * (2.f * w.s1 + w.n * d);
      acc.n += w.n;
    }
  }
}
__device__ __forceinline__ void stat_store(float *stat_partial, size_t index, StatPart a) {
  typedef float f4 __attribute__((ext_vector_type(4)));
  if (!(a.n > 0.f)) a.pivot = a.s1 = a.s2 = a.n = 0.f;
  const f4 v = {a.pivot, a.s1, a.s2, a.n};
  reinterpret_cast<f4 *>(stat_partial)[index] = v;
}
#endif
constexpr int kStatFloats = 4;   // floats per partial

#if defined(__HIPCC__)
// One row of a depthwise window: the six input values x-1 .. x+4 of row y = ybase + dr of one (image, channel) plane,
// the producer's BatchNorm + ReLU applied (BN), zeros outside the map.  One 16-byte load and two edge loads through
// plain pointers (any tensor size).  Nothing here branches: a row outside the map (or an inactive lane, whose strip the
// caller has clamped to a real one) loads from the nearest real row and discards what it got, an edge column outside
// the map loads the strip's own first / last element, so the loads of all the rows of a window can be issued back to
// back and waited for once.
template <bool BN>
__device__ __forceinline__ void dw_load_row(const float *plane, int ybase, int dr, int x, int H, int W, bool active,
                                            float sc, float sh, float (&r)[6]) {
  const int y = ybase + dr;
  const bool rowok = active && y >= 0 && y < H;
  const bool left = x > 0, right = x + 4 < W;
  const int yc = y < 0 ? 0 : (y >= H ? H - 1 : y);
  const float *row = plane + ((size_t)yc * W + x);
  const float4 c = *reinterpret_cast<const float4 *>(row);
  r[0] = row[left ? -1 : 0];
  r[5] = row[right ? 4 : 3];
  r[1] = c.x, r[2] = c.y, r[3] = c.z, r[4] = c.w;
  if (BN) {
#pragma unroll
    for (int k = 0; k < 6; ++k) r[k] = fmaxf(fmaf(r[k], sc, sh), 0.f);
  }
  if (!rowok) {
#pragma unroll
    for (int k = 0; k < 6; ++k) r[k] = 0.f;
  }
  r[0] = left ? r[0] : 0.f;
  r[5] = right ? r[5] : 0.f;
}

// The same row through a buffer descriptor (tensors below 4 GiB), with three ways to the two edge columns:
//   EDGE 0  two more loads;
//   EDGE 1  the strips of an image row sit in adjacent lanes of one 16-lane DPP row (W/4 a power of two <= 16): the
//           edges come from the neighbouring lanes' vectors (row_shr:1 / row_shl:1);
//   EDGE 2  consecutive lanes of the wave hold consecutive strips (of one row, continuing into the next row of strips):
//           the edges come from the neighbouring lanes across the whole wave (wave_shr:1 / wave_shl:1, which gfx950 has),
//           and only the values next to the wave's first and last lane, which sit in other waves, are loaded (by every
//           lane, from one offset each).
// With EDGE 1 and 2 all 64 lanes must call it.  `raw`, if given, receives the row's four centre values as loaded.
// `plane_off` is the byte offset of the lane's (image,
// channel) plane, every address is 32-bit arithmetic, and what does not exist is not selected away afterwards but never
// read: a row outside the map (or an inactive lane) gets a lane offset past the buffer, which reads zeros; the
// producer's BatchNorm + ReLU then runs with scale and shift zeroed for that row, so the zeros stay zeros.  No branch
// and no select per value: a window's loads are issued back to back, and the kernels that use this are bound as much
// by the vector instructions they issue as by their bytes.
constexpr unsigned kPastBuffer = 0xffffffffu;
template <bool BN, int EDGE>
__device__ __forceinline__ void dw_load_row_buf(__amdgpu_buffer_rsrc_t rs, unsigned plane_off, int ybase, int dr, int x, int H,
                                                int W, bool active, float sc, float sh, float (&r)[6], float *raw = nullptr) {
  typedef float f4 __attribute__((ext_vector_type(4)));
  const int y = ybase + dr;
  const bool rowok = active && y >= 0 && y < H;
  const bool left = x > 0, right = x + 4 < W;
  // byte offset of the row's column x; the edge columns one element before and four after it, where they exist (else
  // the strip's own first element again: in range, its value discarded below).  All three are past the buffer, and read
  // zeros, for a row that does not exist (the buffer is at least 32 bytes short of 4 GiB: checked at launch).
  const unsigned off = rowok ? plane_off + (unsigned)(y * W + x) * 4u : kPastBuffer - 16u;
  const unsigned offl = off - (left ? 4u : 0u), offr = off + (right ? 16u : 0u);
  const f4 c = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0));
  float e0 = 0.f, e5 = 0.f;
  if (EDGE == 0) {
    e0 = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, offl, 0, 0));
    e5 = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, offr, 0, 0));
  }
  if (EDGE == 2) {
    // the two values that sit in other waves: every lane reads them from the same (wave-uniform) offset
    const unsigned o0 = (unsigned)__builtin_amdgcn_readfirstlane((int)offl);
    const unsigned o63 = (unsigned)__builtin_amdgcn_readlane((int)offr, 63);
    e0 = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, o0, 0, 0));
    e5 = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, o63, 0, 0));
  }
  if (raw) raw[0] = c[0], raw[1] = c[1], raw[2] = c[2], raw[3] = c[3];
  r[1] = c[0], r[2] = c[1], r[3] = c[2], r[4] = c[3];
  r[0] = e0, r[5] = e5;
  if (BN) {
    const float scr = rowok ? sc : 0.f, shr = rowok ? sh : 0.f;
#pragma unroll
    for (int k = 0; k < 6; ++k) r[k] = fmaxf(fmaf(r[k], scr, shr), 0.f);
  }
  if (EDGE == 0) {
    r[0] = left ? r[0] : 0.f;
    r[5] = right ? r[5] : 0.f;
  }
  if (EDGE == 1) {
    const float fromleft = dpp_mov<0x111>(r[4]);    // row_shr:1: lane i receives lane i-1
    const float fromright = dpp_mov<0x101>(r[1]);   // row_shl:1: lane i receives lane i+1
    r[0] = left ? fromleft : 0.f;
    r[5] = right ? fromright : 0.f;
  }
  if (EDGE == 2) {
    const float fromleft = dpp_mov<0x138>(r[4]);    // wave_shr:1: lane i receives lane i-1, lane 0 a zero
    const float fromright = dpp_mov<0x130>(r[1]);   // wave_shl:1: lane i receives lane i+1, lane 63 a zero
    const int lane = threadIdx.x & 63;
    r[0] = left ? (lane == 0 ? r[0] : fromleft) : 0.f;
    r[5] = right ? (lane == 63 ? r[5] : fromright) : 0.f;
  }
}

#endif

// ------------------------------------------------------------------ implicit-GEMM convolution (MFMA)
// z[n,o,i,j] = sum_{c,tap} wgt[o,c,tap] * act(in)[n,c,s*i+ky-pad,s*j+kx-pad], taps = 9 (pad 1) or 1 (pad 0).
// act = identity, or relu(in*scale[c]+shift[c]) when in_scale != nullptr (BatchNorm+ReLU of the producer
// applied on load).  Optional epilogue: per-channel (sum z, sum z^2) partials of this block's pixel tile.
struct ConvGeom {
  int tile;                // workgroup tile id: 0 = 128 ch x 128 px, 1 = 64 x 256, 2 = 64 x 128, 3 = 64 x 64
  int bm;                  // output channels per workgroup
  int mtiles, nchunks;     // ceil(Cout/bm), ceil(Cin/kc)
  int a_floats;            // taps*kc*bm: weights staged per (mtile, chunk)
  int lTW, lTH;            // log2 of the output tile width / height
  int nimg;                // images per pixel tile
  int IH, IW;              // staged input rows / cols per image
  int IWS, IMS;            // row and image stride of the staged tile in LDS, in pixels (padded against bank conflicts)
  int PLd;                 // staged pixels per channel = nimg*IH*IW
  int PL;                  // pixels per staged plane = nimg*IMS; LDS holds [2 halves][PL][4 channels] per chunk
  int tiles_x, tiles_y, tiles_n;
  int n_ptiles;            // tiles_x*tiles_y*tiles_n
  int kc;                  // input channels staged per step
  int ksplit, kchunks;     // K split over gridDim.z workgroups of kchunks chunks each (1, nchunks: no split)
  bool split;              // products on the bf16 matrix cores from operands split three ways (conv_split_kernel.h)
  int raw_w, raw_rounds;   // split kernel: columns of a staged raw row (a multiple of 4); rounds of 256 16-byte groups per raw copy
  int raw_bytes;           // bytes of a raw copy: 8 channels x staged rows x raw_w columns of fp32
  int raw_lead;            // columns a raw row starts left of the tile's first column: 4, or 0 where a tile is as wide as the map
  int raw_plane;           // 1: a tile is whole images (stride 1) and a raw "row" is a whole channel plane of raw_w = H*W values
  size_t lds_bytes;
};
// want_split: take the bf16-split kernel where its staging fits the LDS (frozen weights only: they are split once, on
// the host); g.split tells whether it was taken.
ConvGeom conv_geom(int taps, int N, int Cin, int Cout, int Ho, int Wo, int stride, bool want_split = false);
// The split kernel fetches its input in aligned groups of four columns: input width and the tiles' first input column
// must be multiples of 4.
// Where a tile is whole images the unit is the channel plane instead of the row: then H*W must be a multiple of 4.
inline bool conv_split_fits_width(const ConvGeom &g, int H, int W, int stride) {
  if (g.raw_plane) return stride == 1 && (H * W) % 4 == 0 && H * W == g.raw_w;
  return W % 4 == 0 && ((1 << g.lTW) * stride) % 4 == 0;
}
// The bf16-split kernel's weights: per (channel tile, chunk of 8 input channels) the exact LDS image
// [slot 0..2][tap pair j 0..4][h 0..1][bm rows][8 channels] of bf16, padded to a multiple of 4096 bytes so that 256
// loader threads copy it in whole rounds of 16 bytes each.  For the tap pairs 0..3, slot = piece and half-wave h holds
// tap 2j+h.  The ninth tap has no partner; its six products are paired by piece instead, three MFMAs for six:
// slot c of "pair" 4 holds piece kSplitLastW[c][h] of tap 8 and meets piece kSplitLastX[c][h] of the activations
// (w0x0 + w1x0, w0x1 + w0x2, w1x1 + w2x0).
constexpr int kSplitLastW[3][2] = {{0, 1}, {0, 0}, {1, 2}};
constexpr int kSplitLastX[3][2] = {{0, 0}, {1, 2}, {1, 0}};
constexpr int conv_split_a_stride(int bm) { return (480 * bm + 4095) & ~4095; }
// LDS of the bf16-split kernel: two copies each of the pre-split weights, of the three bf16 planes (48 bytes a staged
// position, one spare position) and of the raw fp32 halo tile; the statistics exchange (wgn waves along the pixels x bm
// partials of 16 bytes); the table of the workgroup's tiles (48 x 32 bytes)
inline size_t conv_split_lds_bytes(int bm, int wgn, int PL, int raw_bytes) {
  return 2 * (size_t)conv_split_a_stride(bm) + (size_t)96 * (PL + 1) + 2 * (size_t)raw_bytes + (size_t)16 * wgn * bm + 1536;
}
// 16-byte groups of activations a loader thread fetches per chunk, at most, in the kernel built for `slots` halo slots
// per thread (a raw copy has 8 channels x staged rows x groups per row of them; shapes that need more take the fp32 kernel)
constexpr int conv_split_rounds_max(int slots) { return slots == 1 ? 3 : slots == 2 ? 4 : slots == 3 ? 6 : 0; }
inline size_t conv_split_pack_floats(const ConvGeom &g) { return (size_t)g.mtiles * g.nchunks * conv_split_a_stride(g.bm) / sizeof(float); }
// index, in 2-byte units, of weight (output channel m, input channel k) in slot `slot` of tap pair j, half-wave h
inline size_t conv_split_pack_index(const ConvGeom &g, int m, int k, int slot, int j, int h) {
  const int mt = m / g.bm, mi = m % g.bm, ch = k / 8, ki = k % 8;
  return ((size_t)(mt * g.nchunks + ch) * conv_split_a_stride(g.bm)) / 2 + ((size_t)(((slot * 5 + j) * 2 + h) * g.bm + mi)) * 8 + ki;
}
// Weights are handed to the kernel re-packed as the exact LDS image of every (channel tile, chunk of 8
// input channels): wpk[mtile][chunk][tap][half][bm][4], zero padded, so that staging them is a contiguous
// vector copy and an MFMA lane (row m, half-wave h) reads the four channels 4h..4h+3 of a tap as one
// 16-byte vector.  (The order of the terms of a dot product is free: MFMA step e of a tap pairs channels
// e and 4+e.)
inline size_t conv_pack_floats(const ConvGeom &g) { return (size_t)g.mtiles * g.nchunks * g.a_floats; }
inline size_t conv_pack_index(const ConvGeom &g, int m, int k, int tap) {
  const int mt = m / g.bm, mi = m % g.bm, ch = k / g.kc, ki = k % g.kc;   // kc == 8
  return ((size_t)(mt * g.nchunks + ch) * g.a_floats) + ((size_t)((tap * 2 + ki / 4) * g.bm + mi)) * 4 + ki % 4;
}

struct ConvArgs {
  const float *in;         // [N,Cin,H,W]
  const float *wpk;        // packed weights, see conv_pack_index
  float *out;              // [N,Cout,Ho,Wo]
  const float *in_scale;   // [Cin] or nullptr
  const float *in_shift;
  float *stat_partial;     // [Cout][n_ptiles] StatPart (one per pixel tile) or nullptr
  int N, Cin, Cout, H, W, Ho, Wo, stride;
  ConvGeom g;
  float *split_out;        // g.ksplit > 1: [ksplit][N,Cout,Ho,Wo] partial outputs, summed by launch_conv_ksplit_finish
  const float *w_canon;    // launch_conv_first only: the canonical OIHW weights
};
// With g.ksplit > 1 the kernel writes partial outputs into split_out (out and stat_partial are left alone).
// ev_start / ev_stop (both or neither): the launch itself carries the two events, which then hold the dispatch's own
// begin and end time stamps (what a kernel trace shows), instead of a pair of event records around it.
hipError_t launch_conv(int taps, const ConvArgs &a, hipStream_t s, hipEvent_t ev_start = nullptr, hipEvent_t ev_stop = nullptr);
// out = sum over the splits, in split order; stat_partial as the unsplit kernel leaves it (one entry per channel and
// pixel tile; a split convolution's pixel tiles are groups of g.nimg whole images).
hipError_t launch_conv_ksplit_finish(const ConvArgs &a, hipStream_t s);

// A block's first 3x3 convolution with at most three input channels (stride 1, no BatchNorm on its input): the 9*Cin
// (channel, tap) terms two per MFMA step, weights in registers, see conv_first.hip.  Statistics partials:
// [Cout][n_wgs] StatPart.
struct ConvFirstGeom {
  int tiles_x, tiles_y, n_tiles, mtiles;
  int n_wgs;               // persistent workgroups per channel block = statistics partials per channel
  int th;                  // tile height: 4 or 8 rows
};
inline bool conv_first_ok(int Cin, int stride) { return stride == 1 && 9 * Cin <= 32; }
ConvFirstGeom conv_first_geom(int N, int Cin, int Cout, int H, int W);
hipError_t launch_conv_first(const ConvArgs &a, const ConvFirstGeom &g, hipStream_t s, hipEvent_t ev_start = nullptr,
                             hipEvent_t ev_stop = nullptr);

// ------------------------------------------------------------------ 1x1 convolution (MFMA, activations straight from HBM)
// z[n,o,i,j] = sum_c A[o,c] * in[n,c,s*i,s*j]  (pointwise forward, pointwise data gradient with A = P^T,
// projection shortcut).  Weights packed like the 3x3 kernel's with one tap and 32 channels per chunk.
struct PwGeom {
  int variant;             // 0..3: scalar kernel, (channel blocks per workgroup, pixel blocks per wave) (4,2) (4,1) (2,2) (2,1);
                           // 4..9: vector kernel (stride 1, even H*W), see pw_mfma.hip
  int bm, mtiles, nchunks, a_floats, n_ptiles;
  size_t lds_bytes;
};
PwGeom pw_geom(int N, int Cin, int Cout, int Ho, int Wo, int stride);
inline size_t pw_pack_floats(const PwGeom &g) { return (size_t)g.mtiles * g.nchunks * g.a_floats; }
inline size_t pw_pack_index(const PwGeom &g, int m, int k) {
  const int mt = m / g.bm, mi = m % g.bm, ch = k / 32, ki = k % 32;
  return ((size_t)(mt * g.nchunks + ch) * g.a_floats) + (size_t)ki * g.bm + mi;
}
struct PwArgs {
  const float *in;         // [N,Cin,H,W]
  const float *wpk;        // packed weights
  float *out;              // [N,Cout,Ho,Wo]
  float *stat_partial;     // [Cout][n_ptiles] StatPart (one per pixel tile) or nullptr
  int N, Cin, Cout, HWin, Win, Ho, Wo, stride, nchunks;
  PwGeom g;
};
hipError_t launch_pw(const PwArgs &a, hipStream_t s);
hipError_t init_pw_attributes();

// ------------------------------------------------------------------ pointwise weight gradient (MFMA, split-K)
// dP[o,c] = sum_{n,p} dz[n,o,p] * u[n,c,p];  partial[split][Co][Ci], summed by the update kernel (launch_reduce_update).
struct WgradGeom {
  int variant;             // bit 1: 64 (else 128) rows of dP per workgroup; bit 0: 64 (else 128) columns
  int vec;                 // 2: H*W % 32 == 0, buffer addressing; 1: H*W % 4 == 0, 16-byte vectors; 0: scalar loads;
                           // 3: the columns are the 3x3 taps of a few input channels (wgrad_taps_geom)
  int tiles_m, tiles_n, splits, chunks_per_split;   // chunks of 32 pixels
  int slabs;               // partial[slab][Co][Ci] slabs written: = splits, or 2 * splits (wgrad_taps_bn_geom)
  size_t lds_bytes;
};
WgradGeom wgrad_geom(int N, int Co, int Ci, int HW);
// Weight gradient of a full 3x3 convolution (stride 1, padding 1) with few input channels, as the same product:
// column c*9 + tap of "u" is input channel c shifted by that tap (zero outside the image), so dP[o][c*9 + tap] is
// dW[o][c][tap] in its own layout.  Needs 9*Cin <= 64 and W % 4 == 0 (wgrad_taps_ok).
inline bool wgrad_taps_ok(int Cin, int W, int stride) { return stride == 1 && 9 * Cin <= 64 && W % 4 == 0; }
// ... and both tensors of at most 2 GiB: the kernel addresses them with 32-bit offsets, 2 GiB and beyond meaning "zero"
inline bool wgrad_taps_small(int N, int Co, int Cin, int HW) {
  return (unsigned long long)N * Co * HW * sizeof(float) <= (1ull << 31) && (unsigned long long)N * Cin * HW * sizeof(float) <= (1ull << 31);
}
WgradGeom wgrad_taps_geom(int N, int Co, int Cin, int HW);
// The same with the BatchNorm backward of the convolution's output folded in (g.vec == 4; 9*Cin <= 32): the kernel
// reads g = dL/d(BatchNorm output, masked by the ReLU) and the stored pre-BatchNorm z instead of dz, which is never
// formed.  dz = scale*g - scale/m*dbeta - scale/m*dgamma*rstd*(z - mean) is linear in g and z, so
//   dW[o][k] = scale_o * sum g*x_k  -  scale_o/m*dgamma_o*rstd_o * sum (z - mean_o)*x_k  -  scale_o/m*dbeta_o * sum x_k:
// two matrix products over the pixels (one per pair of MFMA waves) and the column sums of the shifted input.
inline bool wgrad_taps_bn_ok(int Cin, int W, int stride) { return wgrad_taps_ok(Cin, W, stride) && 9 * Cin <= 32; }
WgradGeom wgrad_taps_bn_geom(int N, int Co, int Cin, int HW);
struct WgradArgs {
  const float *dz, *u;     // g.vec >= 3: u is the convolution's input [N,Cin,H,W] and Ci = 9*Cin; g.vec == 4: dz is g
  const float *z, *scale, *mean, *rstd, *dgamma, *dbeta;   // g.vec == 4 only: the convolution's output and its BatchNorm
  float *partial;
  int N, Co, Ci, HW;
  WgradGeom g;
  int W;                   // g.vec == 3 only: image width (H = HW / W)
};
hipError_t launch_pw_wgrad(const WgradArgs &a, hipStream_t s);
hipError_t init_pw_wgrad_attributes();

// ------------------------------------------------------------------ BatchNorm statistics
// A convolution leaves the statistics of its output as per-tile partial sums.  Either launch_bn_finalize
// turns them into (mean, rstd, scale = gamma*rstd, shift = beta - mean*scale), or the first kernel that
// reads the layer does so in its prologue (every workgroup for its own channel, in the same fixed order, so
// all of them get the same bits; the first workgroup of a channel also stores the four values).
struct BnPending {
  const float *partial;    // [C][n_parts] StatPart; nullptr: nothing pending
  int n_parts;
  double count;            // elements per channel
  float eps;
  const float *gamma, *beta;
  float *mean, *rstd, *scale, *shift;
  // running statistics, moved by whoever stores the finished ones: r <- decay*r + (1-decay)*batch value
  // (batch mean, biased batch variance); nullptr: left alone
  float *rmean, *rvar;
  float decay;
};
hipError_t launch_bn_finalize(const BnPending &b, int C, hipStream_t s);
// inference mode: scale = gamma/sqrt(rvar+eps), shift = beta - rmean*scale (mean <- rmean, rstd <- 1/sqrt(rvar+eps))
hipError_t launch_bn_running(const float *gamma, const float *beta, const float *rmean, const float *rvar, float eps,
                             float *mean, float *rstd, float *scale, float *shift, int C, hipStream_t s);

// ------------------------------------------------------------------ depthwise 3x3
struct DwGeom {
  int rows;                // fast == 1: output rows per thread, 2 or 4
  int fast;                // 1: stride 1 and width % 4 == 0 -> register-window kernels, n_tiles workgroups of 256 strips;
                           // 2: 2x2 maps, stride 1 -> one thread per map; backward: n_tiles groups of nimg images;
                           // 3: stride 2, even H, W % 8 == 0 -> register windows, one thread per 1 x 4 outputs (forward, and
                           //    the backward pass of a first layer)
  int lTW, lTH, nimg;      // LDS kernels: tile = nimg images (same channel) x TH x TW outputs
  int tiles_x, tiles_y, tiles_n, n_tiles;
  size_t lds_bytes;
};
// H, W: the layer's input size (0: unknown); first_layer: the backward pass needs no data gradient.
DwGeom dw_geom(int N, int Ho, int Wo, int stride, bool backward, int H = 0, int W = 0, bool first_layer = false, int C = 1);
// the register-window kernels (DwGeom::fast == 1) address their tensors through buffer descriptors with 32-bit offsets
inline bool dw_fits_buffer(int N, int C, int H, int W) {
  return (unsigned long long)N * C * H * W * sizeof(float) <= (1ull << 32) - 32;
}

struct DwFwdArgs {
  const float *in;         // [N,C,H,W]
  const float *D;          // [C][9]
  float *out;              // [N,C,Ho,Wo]
  const float *in_scale, *in_shift;   // [C] or nullptr (BN+ReLU of the producer applied on load)
  BnPending pend;          // the producer's statistics, if nobody has finished them yet (then in_scale/in_shift are unused)
  int N, C, H, W, Ho, Wo, stride;
  DwGeom g;
};
hipError_t launch_dw_fwd(const DwFwdArgs &a, hipStream_t s);

// Fused depthwise backward: dD partials (9 per channel) from (du, act(in)); and, unless first_layer,
// g_prev = (du (*)^T D) * 1[act>0] written to gout plus (sum g_prev, sum g_prev*xhat_prev) partials.
// partial[n_tiles][C][11] = 9 taps, dbeta_prev, dgamma_prev.
struct DwBwdArgs {
  const float *du;         // [N,C,Ho,Wo]
  const float *in;         // [N,C,H,W]: block input x (first layer) or previous layer's pre-BN z
  const float *D;          // [C][9]
  float *gout;             // [N,C,H,W] (unused for the first layer)
  const float *in_scale, *in_shift, *in_mean, *in_rstd;   // previous layer's BN (nullptr for first layer)
  float *partial;
  int N, C, H, W, Ho, Wo, stride, first_layer;
  DwGeom g;
};
hipError_t launch_dw_bwd(const DwBwdArgs &a, hipStream_t s);
// dD[c][9] (skipped if dD is null) and (dgamma_prev[c], dbeta_prev[c]) (skipped if null) from the partials above
hipError_t launch_dw_bwd_finalize(const float *partial, int n_tiles, int C, float *dD, float *dgamma_prev,
                                  float *dbeta_prev, hipStream_t s);

// ------------------------------------------------------------------ depthwise 3x3 + pointwise 1x1 in one kernel (forward)
struct DwPwGeom {
  int ok;                  // the layer's shape fits the kernel (stride 1, H % 4 == 0, W a multiple of 32 or 16, 8, 4, ...)
  int wide;                // 1: 64 output channels x 256 pixels per workgroup (Cout <= 64); 0: 128 x 128
  int bm;                  // output channels per workgroup = the packed weights' tile (pw_pack_index with this bm)
  int TW, TH, nimg;        // pixel tile: nimg images x TH rows x TW columns
  int tiles_x, tiles_y, tiles_n, n_ptiles, mtiles;
  int nchunks;             // chunks of 32 input channels in the packed weights
  size_t lds_bytes;
};
bool dwpw_ok(int N, int Cin, int Cout, int H, int W, int stride);
DwPwGeom dwpw_geom(int N, int Cin, int Cout, int H, int W);
struct DwPwArgs {
  const float *in;         // [N,Cin,H,W]
  const float *D;          // [Cin][9]
  const float *wpk;        // pointwise weights packed with bm = g.bm
  const float *in_scale, *in_shift;   // [Cin] finished BatchNorm of the producer (applied with ReLU on load), or nullptr
  float *u_out;            // [N,Cin,H,W] depthwise output (kept for the backward pass)
  float *z_out;            // [N,Cout,H,W]
  float *stat_partial;     // [Cout][n_ptiles] StatPart or nullptr
  int N, Cin, Cout, H, W;
  DwPwGeom g;
};
hipError_t launch_dwpw_fwd(const DwPwArgs &a, hipStream_t s);
hipError_t init_dwpw_attributes();

// ------------------------------------------------------------------ full 3x3 weight gradient (first layer)
// dW[o,c,tap] = sum dz[n,o,i,j] * x[n,c,s*i+ky-1,s*j+kx-1]; partial[n_tiles][Cout][Cin][9]
struct CwGeom {
  int TH, tiles_x, tiles_y, n_tiles, IH, IW;
  size_t lds_bytes;
};
CwGeom cw_geom(int N, int Cin, int Ho, int Wo, int stride);
struct CwArgs {
  const float *dz, *x;
  float *partial;
  int N, Cin, Cout, H, W, Ho, Wo, stride;
  CwGeom g;
};
hipError_t launch_conv_wgrad(const CwArgs &a, hipStream_t s);

// ------------------------------------------------------------------ block head: BN + (shortcut add) + ReLU + (pool) + loss
struct HeadArgs {
  const float *z;          // [N,C,H,W] last layer pre-BN output
  const float *zs;         // [N,C,H,W] shortcut pre-BN output, or the block input (identity_skip), or nullptr
  int identity_skip;       // zs is added as it is (no BatchNorm of its own)
  const float *t;          // target [N,C,Hp,Wp] (modes 1, 2)
  float *out;              // mode 0: block output [N,C,Hp,Wp]
  float *dz;               // mode 2: [N,C,H,W]
  const float *scale, *shift, *mean, *rstd;
  const float *scale_s, *shift_s;
  BnPending pend, pend_s;  // statistics of the last layer / the shortcut still pending (modes 0 and 1)
  const float *dgamma, *dbeta;   // mode 2 with partial == nullptr: finished per-channel sums
  float *partial;          // mode 1: written, [n_blk][C][3] = loss, dbeta, dgamma.  Mode 2: if set, the sums are still
                           // these partials; the kernel sums them itself and stores dgamma_out, dbeta_out, loss_out
  float *dgamma_out, *dbeta_out, *loss_out;
  float loss_scale;
  int N, C, H, W, pool;
  float gscale;            // 2 / cnt
  int n_blk;               // blocks per channel
};
int head_blocks(int N, int H, int W, int pool);
hipError_t launch_head(int mode, const HeadArgs &a, hipStream_t s);
// sums the mode-1 partials: dgamma[c], dbeta[c], and loss = loss_scale * sum
hipError_t launch_head_finalize(const float *partial, int n_blk, int C, float loss_scale, float *dgamma, float *dbeta,
                                float *loss, hipStream_t s);

// interior BN backward, in place: g <- scale/m * (m*g - dbeta - xhat*dgamma).  With dw_partial (the depthwise
// backward kernel's [n_tiles][C][11] partials, entries 9 and 10) every wave first sums its channel's dbeta and
// dgamma itself, in a fixed order in fp64, and the channel's first thread stores them; else both are read.
hipError_t launch_bn_bwd_apply(float *g, const float *z, const float *scale, const float *mean, const float *rstd,
                               float *dgamma, float *dbeta, const float *dw_partial, int n_tiles, int N, int C, int HW,
                               hipStream_t s);
constexpr int kBnBwdFoldMaxTiles = 64;   // beyond this many partials per channel a kernel of its own sums them

// One gradient tensor of the student's arena and where its value comes from.
//   kind 0: grad[i] = sum_t partial[t*count + i]                               (split-K / per-tile partials)
//   kind 1: grad[c*9 + k] = sum_t partial[(t*C + c)*11 + k], count = 9*C       (depthwise backward partials)
//   kind 2: grad[i] already holds the value
struct GradJob {
  const float *partial;
  unsigned arena_off;      // index of the tensor's first element in the parameter / gradient / momentum arenas
  int count, nparts, kind, C;
  int flat;                // 1: few partials, one thread sums them all and a workgroup serves 1024 elements;
                           // 0: a workgroup serves 64 elements, 16 waves share the partials
  int first_block;         // the job's first workgroup
};
constexpr int kGradJobFlatMaxParts = 16;
inline int grad_job_blocks(const GradJob &j) { return (j.count + (j.flat ? 1023 : 63)) / (j.flat ? 1024 : 64); }
// Finishes every gradient (fixed order, fp64) and applies SGD-momentum to it in one launch:
// v <- mu*v + g ; theta <- theta - lr*v; the updated value is also written into the packed
// copies the MFMA kernels read: pk[map_f[i]] and pk[map_b[i]] (entries < 0: no copy).
hipError_t launch_reduce_update(const GradJob *jobs_dev, const int *job_of_block_dev, int n_blocks, float *theta, float *vel,
                                float *grad, float lr, float mu, const int *map_f, const int *map_b, float *pk, hipStream_t s);


// scratch257[0..255]: partial sums, scratch257[256] <- mean((a-b)^2) over n elements (fp64, fixed order)
hipError_t launch_feature_mse(const float *a, const float *b, size_t n, double *scratch257, hipStream_t s);
// device address, on the current GPU, of the library's own 257-double array for the same purpose (no allocation)
hipError_t feature_mse_static_scratch(double **ptr_out);

hipError_t init_kernel_attributes();

}  // namespace pbkd

// Device code of the 3x3 implicit-GEMM convolution that forms its fp32 products on the bf16 matrix cores
// (v_mfma_f32_32x32x16_bf16, sixteen times the fp32 MFMA rate of gfx950).  Host side: conv_split.hip.
//
// Arithmetic.  Every fp32 operand is written exactly as the sum of three bf16 terms, x = x0 + x1 + x2
// (x0 = bf16 nearest x, x1 = bf16 nearest x - x0, x2 = x - x0 - x1: eight significant bits each, so nothing is left
// over), and a product x*w is formed as the six terms x0w0 + x0w1 + x1w0 + x1w1 + x0w2 + x2w0, every one exact in
// the fp32 accumulator's product width.  |x1| <= 2^-8 |x| and |x2| <= 2^-17 |x|, so the three terms left out (x1w2,
// x2w1, x2w2) are at most 2^-24 |x w| (2^-27 rms, no bias): no more than the rounding of one fp32 operation.
// Accumulation is fp32, as in the fp32-MFMA kernel.
//
// GEMM view as in conv_mfma_kernel.h (M = Cout, N = pixels, A = weights, B = activations); K is walked in chunks of
// 8 input channels, and one MFMA (K = 16) takes two taps of a chunk: half-wave h supplies tap 2j+h, its eight
// k-values are the chunk's eight channels.  Nine taps fill four such pairs; the ninth tap's six products are paired by
// piece instead (the half-waves supply two different pieces of tap 8: w0x0 + w1x0, w0x1 + w0x2, w1x1 + w2x0), three
// MFMAs for six, so that no MFMA slot is left empty: 27 MFMAs per output block and chunk.
//
// A workgroup is 4 MFMA waves + 4 loader waves.  Its staging (two copies each of the weights, the bf16 planes and the
// raw tile) fills most of a compute unit's LDS, so there is one workgroup per compute unit and nothing else to hide
// its start-up and its output stores behind: the kernel is persistent instead.  Workgroup w walks the tiles
// w, w + G, w + 2G, ... (G = workgroups launched) as ONE sequence of chunks through a three-stage pipeline, one
// barrier per stage shift, so that the loaders are already fetching the next tile while the MFMA waves finish and
// store the current one:
//   loader waves chunk i    global -> LDS "raw" fp32 halo tile (plus the pre-split weights of chunk i-1, a plain copy)
//   loader waves chunk i-1  raw -> BatchNorm+ReLU of the producing layer -> three bf16 planes in LDS
//   MFMA waves   chunk i-2  MFMAs from the bf16 planes
// The split costs about 10 vector instructions per element.  A wave that shares its SIMD with a wave streaming MFMAs
// still issues a vector instruction every 6 cycles or so without slowing the MFMA wave (the MFMA wave's own vector
// instructions cost it 6 cycles and more per MFMA they follow), so the loader waves do the split, between issuing their
// copies and waiting for them, and the MFMA waves do nothing but fetch operands and multiply.
#pragma once
#include <hip/hip_ext.h>

#include "pbkd_internal.h"

namespace pbkd {

typedef float sfloatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef unsigned uintx2 __attribute__((ext_vector_type(2)));

// two floats -> their nearest bf16, packed (low half = a)
__device__ __forceinline__ unsigned pack_bf16_rn(float a, float b) {
  const floatx2 v = {a, b};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}

// One tile of a workgroup's list: where it is, and which chunks of K it takes.
struct __attribute__((aligned(16))) SplitTile {
  int x0, y0, n0;      // first output column, row and image
  int mt;              // channel tile
  int kb, nk;          // first chunk and number of chunks
  int kz;              // K split the tile belongs to
  int pt;              // pixel tile index (statistics partial)
};
constexpr int kSplitMaxTiles = 48;   // tiles per workgroup that the table in LDS holds
// A table entry is the same for every lane: say so, or what is computed from it (scalar offsets of buffer loads, LDS
// base addresses) is taken for lane-dependent and the compiler loops over its values.
__device__ __forceinline__ SplitTile uniform_tile(const SplitTile &d) {
  SplitTile u;
  u.x0 = __builtin_amdgcn_readfirstlane(d.x0); u.y0 = __builtin_amdgcn_readfirstlane(d.y0); u.n0 = __builtin_amdgcn_readfirstlane(d.n0);
  u.mt = __builtin_amdgcn_readfirstlane(d.mt); u.kb = __builtin_amdgcn_readfirstlane(d.kb); u.nk = __builtin_amdgcn_readfirstlane(d.nk);
  u.kz = __builtin_amdgcn_readfirstlane(d.kz); u.pt = __builtin_amdgcn_readfirstlane(d.pt);
  return u;
}

// 16 bytes per lane from a buffer straight into LDS: lane l lands 16 l bytes behind `lds`, which must be the same for
// the whole wave; soff likewise.  Completion counts as a vector-memory load's.
__device__ __forceinline__ void load16_to_lds(__amdgpu_buffer_rsrc_t r, char *lds, unsigned voff, unsigned soff) {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (__attribute__((address_space(3))) void *)lds, 16, voff, soff, 0, 0);
#endif
}

template <int WGM, int MB, int NB, int BSLOTS>
__global__ __launch_bounds__(512) void conv_split_kernel(ConvArgs p) {
  constexpr int WGN = 4 / WGM;
  constexpr int BM = WGM * MB * 32;     // output channels per workgroup
  constexpr int WN = NB * 32;           // pixels per wave
  constexpr int A_STRIDE = conv_split_a_stride(BM);   // bytes of pre-split weights per (channel tile, chunk)
  constexpr int NA = A_STRIDE / 4096;                 // 16-byte loads of weights per loader thread and chunk
  constexpr int NI = conv_split_rounds_max(BSLOTS);   // 16-byte loads of activations per loader thread and chunk, at most
  extern __shared__ float smem[];
  const int PL = p.g.PL + 1;                               // staged positions per plane + one that is never read
  char *const As = reinterpret_cast<char *>(smem);        // [2][A_STRIDE]: [piece][tap pair][h][BM][8 bf16]
  char *const Ss = As + 2 * A_STRIDE;                      // [2][PL][3 pieces][8 bf16]: the pieces of a position side by side,
                                                           // 48 bytes apart 16 lanes' 16-byte reads still cover all banks once
  // raw fp32 halo tile: [2][staged row][8 channels][RW columns], RW = the staged width in whole 16-byte groups
  char *const Rs = Ss + (size_t)2 * 3 * PL * 16;
  const int RW = p.g.raw_w, RAWB = p.g.raw_bytes;
  // statistics exchange [WGN][BM]: written by the MFMA waves when a tile ends, read by the loader waves in the next stage;
  // a tile has at least two chunks wherever statistics are taken (the host checks), so the next write is a barrier later
  StatPart *const red = reinterpret_cast<StatPart *>(Rs + (size_t)2 * RAWB);
  SplitTile *const tiles = reinterpret_cast<SplitTile *>(red + WGN * BM);          // [kSplitMaxTiles]

  const bool loader = threadIdx.x >= 256;
  const int tid = threadIdx.x & 255, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WGM, wn = wave / WGM;
  const int l31 = lane & 31, lh = lane >> 5;
  const int lTW = p.g.lTW, lTH = p.g.lTH;
  const int TW = 1 << lTW, TH = 1 << lTH;
  const int IH = p.g.IH, IW = p.g.IW, IWS = p.g.IWS, IMS = p.g.IMS;
  const int s = p.stride;
  const int HWo = p.Ho * p.Wo;
  const int HW = p.H * p.W;
  const int IHW = IH * IW;
  const int nchunks = p.g.nchunks;

  // ---- this workgroup's tiles.  In every round of G tiles a die (workgroup index modulo 8) takes a contiguous run,
  // so that tiles sharing halo rows meet in one L2.
  const int G = gridDim.x;
  const int items = p.g.n_ptiles * p.g.mtiles * p.g.ksplit;
  const int first = xcd_contiguous(blockIdx.x, G);
  const int n_mine = (items - first + G - 1) / G;          // the host launches G <= items, and G*kSplitMaxTiles >= items
  if ((int)threadIdx.x < n_mine) {
    const int L = first + (int)threadIdx.x * G;
    SplitTile d;
    d.pt = L % p.g.n_ptiles;
    const int r = L / p.g.n_ptiles;
    d.mt = r % p.g.mtiles;
    d.kz = r / p.g.mtiles;
    int q = d.pt;
    d.x0 = (q % p.g.tiles_x) * TW;
    q /= p.g.tiles_x;
    d.y0 = (q % p.g.tiles_y) * TH;
    d.n0 = (q / p.g.tiles_y) * p.g.nimg;
    d.kb = d.kz * p.g.kchunks;
    d.nk = (nchunks - d.kb < p.g.kchunks) ? nchunks - d.kb : p.g.kchunks;
    tiles[threadIdx.x] = d;
  }
  __syncthreads();
  int TC = 0;                                              // chunks in all of this workgroup's tiles
  for (int t = 0; t < n_mine; ++t) TC += tiles[t].nk;
  TC = __builtin_amdgcn_readfirstlane(TC);

  // After the barrier that follows a tile's end: the WGN MFMA waves' statistics partials (in red), re-expressed about the
  // first one's pivot and added.  The loader waves do it: they have nothing else to do while they wait for their copies.
  auto finish_stats = [&](const SplitTile &d) {
    if (p.stat_partial && p.g.ksplit == 1) {
      for (int e = tid; e < BM; e += 256) {
        const int o = d.mt * BM + e;
        if (o < p.Cout) {
          StatPart a = red[e];
#pragma unroll
          for (int w = 1; w < WGN; ++w) stat_rebase_add(a, red[w * BM + e]);
          stat_store(p.stat_partial, (size_t)o * p.g.n_ptiles + d.pt, a);
        }
      }
    }
  };

  if (loader) {
    // ------------------------------------------------------------------ loader waves: copies, and the statistics' last step
    const __amdgpu_buffer_rsrc_t rin = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(p.in), 0, (int)((unsigned)p.N * p.Cin * HW * sizeof(float)), 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(p.wpk), 0, (int)((unsigned)p.g.mtiles * nchunks * A_STRIDE), 0x00020000);
    const unsigned aoff = (unsigned)(tid * 16);
    const unsigned chunkb = (unsigned)(8 * HW * sizeof(float));       // bytes between chunks of 8 channels
    // Activations travel in groups of four columns of one channel's row (16 bytes): group t of a raw copy is
    // (staged row t / (8 G), channel t / G % 8, columns 4 (t % G) ..), G = RW / 4, so that a wave's 64 groups are
    // contiguous in LDS and, channel by channel, in memory.  Where a row of tiles spans the map a staged row starts
    // FOUR columns left of the tile (the halo needs one), else, the tile being as wide as the map, at the map's first
    // column and ends at its last (both halo columns are outside the image: zeros, never fetched).  With the width and
    // the tile's first column multiples of 4 (the host checks) every group is 16-byte aligned within its row and lies
    // wholly inside the tensor or wholly outside it.  A group's address is a constant of the thread plus one number
    // per tile; what a group holds beyond the image is never used (the split selects by position).  The whole
    // byte offset goes into the lane offset, which the buffer descriptor checks: a group before the tensor's start or
    // past its end (a halo row above the first or below the last channel, channels past Cin in a ragged last chunk)
    // reads zeros instead of memory.  Where a tile is whole images (stride 1) the unit is the channel plane instead of
    // the row: H*W contiguous values, 16-byte aligned when H*W is a multiple of 4 whatever the width.
    const int rows_img = p.g.raw_plane ? 1 : IH;             // raw rows per image: staged rows, or the one channel plane
    const int G4 = RW >> 2, n_groups = p.g.nimg * rows_img * 8 * G4;
    int kit[NI];               // element offset of the group relative to the tile's first halo element
    bool git[NI];              // the group exists
#pragma unroll
    for (int r = 0; r < NI; ++r) {
      const int t = tid + 256 * r;
      const int row = t / (8 * G4), rem = t - row * (8 * G4);
      const int ch = rem / G4, g = rem - ch * G4;
      const int img = row / rows_img, iy = row - img * rows_img;
      git[r] = t < n_groups;
      kit[r] = ((img * p.Cin + ch) * p.H + iy) * p.W + 4 * g;
    }
    unsigned goff[NI];
    auto enter = [&](const SplitTile &d) {
      const int tb = p.g.raw_plane ? d.n0 * p.Cin * p.H * p.W : (d.n0 * p.Cin * p.H + d.y0 * s - 1) * p.W + d.x0 * s - p.g.raw_lead;
#pragma unroll
      for (int r = 0; r < NI; ++r) goff[r] = git[r] ? (unsigned)(kit[r] + tb) * 4u : kPastBuffer - 15u;
    };
    // Both copies go from memory straight into LDS (buffer loads with the LDS bit: lane l of a wave lands 16 l bytes
    // behind a wave-uniform LDS address), so a loader thread issues one instruction per 16 bytes and holds no data.
    auto copy_b = [&](int k, int buf) {
      char *Rd = Rs + buf * RAWB + __builtin_amdgcn_readfirstlane(wave) * 1024;
#pragma unroll
      for (int r = 0; r < NI; ++r)
        if (git[r])       // a group past the raw copy must not be written: it would land in the next LDS region
          load16_to_lds(rin, Rd + r * 4096, goff[r] + (unsigned)k * chunkb, 0);
    };
    auto copy_a = [&](int mt, int k, int buf) {
      const unsigned wk = (unsigned)(((size_t)mt * nchunks + k) * A_STRIDE);
      char *Ad = As + buf * A_STRIDE + __builtin_amdgcn_readfirstlane(wave) * 1024;
#pragma unroll
      for (int i = 0; i < NA; ++i) load16_to_lds(rw, Ad + i * 4096, aoff, wk + (unsigned)(i * 4096));
    };
    // the halo-tile slots this thread splits.  Where a slot sits in the staged tile does not depend on the tile.
    unsigned spos[BSLOTS];     // image (bits 16..), row (8..15) and column (0..7) of the slot within the staged tile
    int loff[BSLOTS];          // the slot's position in the bf16 planes; slots past the tile work on the spare position
    int roff[BSLOTS];          // byte offset of the slot's channel 0 in a raw copy
#pragma unroll
    for (int sl = 0; sl < BSLOTS; ++sl) {
      const int q = tid + 256 * sl;
      const bool in_tile = q < p.g.PLd;
      const int img = q / IHW;
      const int r = q - img * IHW;
      const int iy = r / IW;
      const int ix = r - iy * IW;
      loff[sl] = in_tile ? img * IMS + iy * IWS + ix : PL - 1;
      // a raw row starts raw_lead columns left of the tile's first column: the staged column ix (the halo column first)
      // is raw column ix - 1 + raw_lead; with no lead the left halo column is outside the image and never used
      // (where a tile is whole images a raw "row" is a channel plane: the position is (iy - 1) * W + ix - 1 within it)
      const int rcol = p.g.raw_plane ? (iy - 1) * p.W + ix - 1 : ix - 1 + p.g.raw_lead;
      const int rrow = p.g.raw_plane ? img : img * IH + iy;
      const bool rin_plane = !p.g.raw_plane || (iy >= 1 && iy <= p.H && ix >= 1 && ix <= p.W);
      roff[sl] = (in_tile && rin_plane) ? ((rrow * 8) * RW + (rcol > 0 ? rcol : 0)) * 4 : 0;
      spos[sl] = in_tile ? ((unsigned)img << 16 | (unsigned)iy << 8 | (unsigned)ix) : 0x7fff0000u;   // beyond every batch
    }

    // The split of chunk kc, raw copy rc -> bf16 copy rc, this thread's slots.  Nothing is conditional but the
    // BatchNorm: positions outside the image become zeros by a select, slots past the tile write the spare position.
    const bool bn = (p.in_scale != nullptr);
    const float lo = bn ? 0.f : -__builtin_inff();             // ReLU only where there is a BatchNorm to apply
    bool gok[BSLOTS];          // the slot is inside the tile and inside the image (elsewhere the bf16 planes hold zeros)
    auto enter_split = [&](const SplitTile &d) {
#pragma unroll
      for (int sl = 0; sl < BSLOTS; ++sl) {
        const int n = d.n0 + (int)(spos[sl] >> 16), y = d.y0 * s - 1 + (int)(spos[sl] >> 8 & 255), x = d.x0 * s - 1 + (int)(spos[sl] & 255);
        gok[sl] = (n < p.N) && (y >= 0) && (y < p.H) && (x >= 0) && (x < p.W);
      }
    };
    // the producing layer's scale and shift for a chunk's channels, through the scalar cache (the constant address
    // space: an earlier kernel wrote them): two loads of eight for a whole chunk instead of sixteen vector loads
    typedef const float __attribute__((address_space(4))) *ConstFloats;
    const ConstFloats cscale = (ConstFloats)(p.in_scale), cshift = (ConstFloats)(p.in_shift);
    float sc[8], sh[8];
    auto fetch_bn = [&](int kc) {
#pragma unroll
      for (int e = 0; e < 8; ++e) sc[e] = 1.f, sh[e] = 0.f;
      if (bn) {
        if (kc * 8 + 8 <= p.Cin) {
          typedef float Floats8 __attribute__((ext_vector_type(8), aligned(4)));
          typedef const Floats8 __attribute__((address_space(4))) *ConstFloats8;
          const Floats8 a = *(ConstFloats8)(cscale + kc * 8), b = *(ConstFloats8)(cshift + kc * 8);
#pragma unroll
          for (int e = 0; e < 8; ++e) sc[e] = a[e], sh[e] = b[e];
        } else {                         // a ragged last chunk: its missing channels take the last one's (their weights are zero)
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            int c = kc * 8 + e;
            if (c > p.Cin - 1) c = p.Cin - 1;
            sc[e] = cscale[c], sh[e] = cshift[c];
          }
        }
      }
    };
    auto split = [&](int rc) {
      const char *Rb = Rs + rc * RAWB;
      char *Sd = Ss + (size_t)rc * 3 * PL * 16;
      float raw[BSLOTS][8];
#pragma unroll
      for (int sl = 0; sl < BSLOTS; ++sl)
#pragma unroll
        for (int e = 0; e < 8; ++e) raw[sl][e] = *reinterpret_cast<const float *>(Rb + roff[sl] + e * RW * 4);
#pragma unroll
      for (int sl = 0; sl < BSLOTS; ++sl) {
        uintx4 pp[3];
#pragma unroll
        for (int t = 0; t < 4; ++t) {              // channels 2t, 2t+1
          const float x0 = gok[sl] ? fmaxf(fmaf(raw[sl][2 * t], sc[2 * t], sh[2 * t]), lo) : 0.f;
          const float x1 = gok[sl] ? fmaxf(fmaf(raw[sl][2 * t + 1], sc[2 * t + 1], sh[2 * t + 1]), lo) : 0.f;
          const unsigned a = pack_bf16_rn(x0, x1);
          const float r0 = x0 - __builtin_bit_cast(float, a << 16);
          const float r1 = x1 - __builtin_bit_cast(float, a & 0xffff0000u);
          const unsigned b = pack_bf16_rn(r0, r1);
          const float s0 = r0 - __builtin_bit_cast(float, b << 16);
          const float s1 = r1 - __builtin_bit_cast(float, b & 0xffff0000u);
          pp[0][t] = a;
          pp[1][t] = b;
          pp[2][t] = pack_bf16_rn(s0, s1);
        }
#pragma unroll
        for (int pc = 0; pc < 3; ++pc) *reinterpret_cast<uintx4 *>(Sd + loff[sl] * 48 + pc * 16) = pp[pc];
      }
    };
    // Stage i: copies the activations of chunk i and the weights of chunk i-1 and, while those are on their way, splits
    // chunk i-1; all of it is needed when the barrier that ends the stage has passed (the barrier's wait covers the
    // copies: they count as vector-memory loads).
    int lt = 0, lc = 0, a_mt = 0, a_k = 0;
    SplitTile ld = uniform_tile(tiles[0]);
    enter(ld);
    enter_split(ld);
    if (n_mine == 1) {
      // One tile only (the small maps: as many tiles as compute units): the same stages without the bookkeeping of
      // which tile a chunk belongs to.  On those tiles a stage of the MFMA waves is short (1 100 cycles for 64
      // channels x 64 pixels), and what the barrier waits for is the loaders' instruction count per stage, not memory.
      for (int i = 0; i <= TC + 1; ++i) {
        const bool splits = i >= 1 && i <= TC;
        if (splits) fetch_bn(ld.kb + i - 1);
        if (i < TC) copy_b(ld.kb + i, i & 1);
        if (splits) {
          copy_a(ld.mt, ld.kb + i - 1, (i - 1) & 1);
          split((i - 1) & 1);
        }
        __syncthreads();
      }
      finish_stats(ld);
      return;
    }
    int st = 0;                         // the tile of the chunk being split (chunk i-1 in stage i)
    int ft = 0, fc = 0;                 // the multiplying side's tile and chunk (it is at chunk i-2 in stage i)
    bool pending = false;
    SplitTile fd = ld, pd = ld;
    for (int i = 0; i <= TC + 1; ++i) {
      const bool splits = i >= 1 && i <= TC;
      if (splits) fetch_bn(a_k);        // ahead of the copies: vector-memory loads complete in the order issued
      if (i < TC) copy_b(ld.kb + lc, i & 1);
      if (splits) copy_a(a_mt, a_k, (i - 1) & 1);
      if (pending) {                    // the tile that ended in the stage before this one
        finish_stats(pd);
        pending = false;
      }
      if (splits) split((i - 1) & 1);
      if (i >= 2) {
        if (++fc == fd.nk) {
          pd = fd;
          pending = true;
          fc = 0;
          if (ft + 1 < n_mine) fd = uniform_tile(tiles[++ft]);
        }
      }
      a_mt = ld.mt;
      a_k = ld.kb + lc;
      if (st != lt) {                   // the chunk split next (the one just fetched) belongs to the tile entered last
        st = lt;
        enter_split(ld);
      }
      if (i + 1 < TC) {
        if (++lc == ld.nk) {
          lc = 0;
          ld = uniform_tile(tiles[++lt]);
          enter(ld);
        }
      }
      __syncthreads();
    }
    if (pending) finish_stats(pd);
  } else {
    // ------------------------------------------------------------------ MFMA waves
    sfloatx16 acc[MB][NB];
#pragma unroll
    for (int a = 0; a < MB; ++a)
#pragma unroll
      for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
    // where this lane's pixel columns sit in the staged tile
    int pixoff[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int pn = wn * WN + nb * 32 + l31;
      const int img = pn >> (lTW + lTH);
      const int rem = pn & (TH * TW - 1);
      pixoff[nb] = img * IMS + (s * (rem >> lTW)) * IWS + s * (rem & (TW - 1));
    }
    // tap 2j+h of this half-wave as an offset in the staged tile (in the last step both half-waves read tap 8)
    int toff[5];
#pragma unroll
    for (int j = 0; j < 5; ++j) {
      const int tap = (2 * j + lh < 9) ? 2 * j + lh : 8;
      toff[j] = (tap / 3) * IWS + (tap % 3);
    }
    const int arow = (wm * (MB * 32) + l31) * 16;      // byte offset of this lane's weight row within a [BM][8] slab

    // One pipeline stage of the MFMA waves: multiplies the chunk whose weights and bf16 planes are in copy mc.
    //
    // The six products of a tap pair run in the order (weight piece, activation piece) = 10 11 20 00 01 02.  Every
    // operand piece then falls free at least two products (eight MFMAs) before the next tap pair needs it again, so
    // the next tap pair's pieces are fetched into the same registers: no second set of operand registers.  The ninth
    // tap's three products (operand slot c with operand slot c) follow in the order 1 0 2, the order their operands
    // arrive in.  The fences keep the compiler from moving the LDS reads down to their first use.
    auto stage = [&](int mc) {
      const char *Ab = As + mc * A_STRIDE + arow;
      const char *Sb = Ss + (size_t)mc * 3 * PL * 16;
      auto lda = [&](int pc, int j, int mb) {
        return *reinterpret_cast<const uintx4 *>(Ab + ((pc * 5 + j) * 2 + lh) * (BM * 16) + mb * 512);
      };
      auto ldb = [&](int pc, int j, int nb) {
        // operand slot pc is piece pc, but for the ninth tap, where the half-waves read two different pieces of it
        const int piece = j < 4 ? pc : kSplitLastX[pc][0] + lh * (kSplitLastX[pc][1] - kSplitLastX[pc][0]);
        return *reinterpret_cast<const uintx4 *>(Sb + (pixoff[nb] + toff[j]) * 48 + piece * 16);
      };
      uintx4 av[3][MB], bv[3][NB];
      auto fill_a = [&](int pc, int j) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) av[pc][mb] = lda(pc, j, mb);
      };
      auto fill_b = [&](int pc, int j) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) bv[pc][nb] = ldb(pc, j, nb);
      };
      // tap pair 0, in the order of first use
      fill_a(1, 0); fill_b(0, 0); fill_b(1, 0); fill_a(2, 0); fill_a(0, 0); fill_b(2, 0);
#pragma unroll
      for (int j = 0; j < 5; ++j) {
        __builtin_amdgcn_sched_barrier(0);
        constexpr int PA[6] = {1, 1, 2, 0, 0, 0}, PB[6] = {0, 1, 0, 0, 1, 2}, PL4[3] = {1, 0, 2};
#pragma unroll
        for (int q = 0; q < (j < 4 ? 6 : 3); ++q) {
          const int qa = j < 4 ? PA[q] : PL4[q], qb = j < 4 ? PB[q] : PL4[q];
#pragma unroll
          for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
              acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av[qa][mb]),
                                                                    __builtin_bit_cast(bf16x8, bv[qb][nb]), acc[mb][nb], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          if (j + 1 < 5) {          // the next tap pair's pieces, into the registers that have just fallen free
            if (q == 1) fill_a(1, j + 1);
            if (q == 2) fill_a(2, j + 1);
            if (q == 3) fill_b(0, j + 1);
            if (q == 4) fill_b(1, j + 1);
            if (q == 5) { fill_a(0, j + 1); fill_b(2, j + 1); }
          }
        }
      }
    };
    // the multiplying side leaves a tile: leaves every wave's statistics partial in red, stores the tile, clears
    // the accumulators.  Accumulator register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32.  The stores
    // go through a buffer descriptor: a wave-uniform byte offset for the channel (rows 8*(r/4) + r%4 of the block), a
    // lane offset for the pixel and the half-wave's four channels, and pixels or channels that do not exist get an
    // offset past the buffer, which drops the store; no branch, no 64-bit address arithmetic.
    const __amdgpu_buffer_rsrc_t rout = __builtin_amdgcn_make_buffer_rsrc(
        p.g.ksplit > 1 ? p.split_out : p.out, 0, (int)((unsigned)p.g.ksplit * p.N * p.Cout * HWo * sizeof(float)), 0x00020000);
    auto leave = [&](const SplitTile &d) {
      const int m0 = d.mt * BM + wm * (MB * 32);      // first channel of this wave
      bool pvalid[NB];
      unsigned voff[NB];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const int pn = wn * WN + nb * 32 + l31;
        const int img = pn >> (lTW + lTH);
        const int rem = pn & (TH * TW - 1);
        const int n = d.n0 + img, y = d.y0 + (rem >> lTW), x = d.x0 + (rem & (TW - 1));
        pvalid[nb] = (n < p.N) && (y < p.Ho) && (x < p.Wo);
        voff[nb] = (unsigned)(((d.kz * p.N + n) * p.Cout + 4 * lh) * HWo + y * p.Wo + x) * 4u;
      }
      // per-channel statistics partial of this pixel tile (as in the fp32-MFMA kernel): every wave sums about the value
      // of its own first pixel column
      // (all of it on the vector ALU: the pivot through two lane reads, the half-wave sums through DPP with the
      // total arriving in the half-wave's upper 16 lanes; LDS permutes would make 64 dependent round trips of it)
      if (p.stat_partial && p.g.ksplit == 1) {
        float cnt = 0.f;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) cnt += pvalid[nb] ? 1.f : 0.f;
        cnt = half32_sum_upper(cnt);
        StatPart *const rw = red + wn * BM + wm * (MB * 32) + 4 * lh;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float a0 = acc[mb][0][r];
            const float p0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a0), 0));
            const float p1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a0), 32));
            const float pv = lh ? p1 : p0;
            float s1 = 0.f, s2 = 0.f;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
              const float dv = pvalid[nb] ? acc[mb][nb][r] - pv : 0.f;
              s1 += dv;
              s2 += dv * dv;
            }
            s1 = half32_sum_upper(s1);
            s2 = half32_sum_upper(s2);
            if (l31 == 16) {
              StatPart sp;
              sp.pivot = pv; sp.s1 = s1; sp.s2 = s2; sp.n = cnt;
              rw[mb * 32 + 8 * (r / 4) + (r % 4)] = sp;
            }
          }
      }
      const bool whole8 = (p.Cout & 7) == 0;          // then the eight channels of an accumulator row group exist or do not together
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int ou = m0 + mb * 32 + 8 * (r / 4) + (r % 4);     // wave-uniform part of the channel
          const unsigned soff = (unsigned)ou * (unsigned)HWo * 4u;
          const bool ch_ok = whole8 ? (ou < p.Cout) : (ou + 4 * lh < p.Cout);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            const float v = acc[mb][nb][r];       // (a bit cast applied to the vector element itself reads element 0)
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), rout,
                                                  (pvalid[nb] && ch_ok) ? voff[nb] + soff : kPastBuffer, 0, 0);
          }
        }
#pragma unroll
      for (int a = 0; a < MB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;
    };
    int mt = 0, mc = 0;
    SplitTile md = uniform_tile(tiles[0]);
    __syncthreads();                              // stage 0: the loaders fetch chunk 0
    __syncthreads();                              // stage 1: ... and split it
    for (int i = 2; i <= TC + 1; ++i) {           // stage i: multiplies chunk i-2
      stage(i & 1);
      if (++mc == md.nk) {
        leave(md);
        mc = 0;
        if (mt + 1 < n_mine) md = uniform_tile(tiles[++mt]);
      }
      __syncthreads();
    }
  }
}

}  // namespace pbkd

// Weight gradient of the student's pointwise convolution on the fp32 matrix cores:
//   dP[o,c] = sum_q dz[o,q] * u[c,q],   q = (image, pixel):   M = Cout, N = Cin, K = N*H*W  (split-K).
//
// Both operands are contiguous along the reduction index q (NCHW rows), the opposite of what an MFMA
// operand wants (32 lanes = 32 different rows at the same q).  Loading them in operand order straight from
// global memory makes every lane of a load touch another 128-byte line; so they are transposed through LDS
// instead: four loader waves read whole 128-byte row segments (8 lanes x 16 bytes per row, 32 pixels per
// chunk) and write them into a [row][36]-float image, and four MFMA waves read their operands back as
// 16-byte vectors along q.  A sum does not care about the order of its terms: lanes 0..31 take pixels
// 8g..8g+3 of their row and lanes 32..63 pixels 8g+4..8g+7, and the four MFMA steps that follow pair
// element e of the A vector with element e of the B vector.  The row stride of 36 floats keeps both the
// 16-byte writes (8 lanes = one row) and the 16-byte reads (8 lanes = 8 rows, 4 banks each) conflict free.
//
// A workgroup owns a tile of dP (128 or 64 rows by 128 or 64 columns, a quarter per MFMA wave) and a
// contiguous range of q; the chunks are double buffered with one barrier each and the loader fetches two
// chunks ahead.  Every workgroup writes its tile to partial[split], summed afterwards in a fixed order.
#include <cstdlib>

#include "conv_mfma_kernel.h"

namespace pbkd {

constexpr int WG_KC = 32;           // pixels per staged chunk
constexpr int WG_LS = WG_KC + 4;    // LDS row stride in floats

// MODE 2: H*W a multiple of 32 (a chunk lies inside one image) and operands below 4 GiB: the loaders address
// through buffer descriptors, wave-uniform scalar offset per chunk + constant lane offset, no vector ALU work
// at all (every instruction a loader wave issues while the matrix pipe streams is expensive).
// MODE 1: H*W a multiple of 4 (16-byte loads, per-lane index arithmetic).  MODE 0: any shape, scalar loads.
// MODE 3: the weight gradient of a full 3x3 convolution with few input channels: dz rows as in MODE 1; the "u"
// row c*9 + tap is input channel c shifted by the tap, four pixels of one image row per lane, each checked
// against the image border (W % 4 == 0).  That kernel is bound by reading dz, the loaders' arithmetic is free.
template <int MBW, int NBW, int MODE>
__global__ __launch_bounds__(512) void pw_wgrad_kernel(WgradArgs p) {
  constexpr bool VEC = MODE >= 1;
  constexpr int BM = 2 * MBW * 32, BN = 2 * NBW * 32;
  constexpr int BUF = (BM + BN) * WG_LS;
  constexpr int NA = BM / 32, NBL = BN / 32, NR = NA + NBL;   // 16-byte loads per loader thread and chunk
  typedef float f4 __attribute__((ext_vector_type(4)));
  extern __shared__ float smem[];   // [2][BM + BN][WG_LS]

  const bool loader = threadIdx.x >= 256;
  const int tid = threadIdx.x & 255, lane = tid & 63, wave = tid >> 6;
  const int l31 = lane & 31, lh = lane >> 5;
  const int wm = wave & 1, wn = wave >> 1;
  // the tiles of one split read the same rows of dz and u: the workgroups are renumbered so that they are neighbours
  // on one die (tile index fastest inside a split, a contiguous range of splits per die)
  const int lin = xcd_contiguous(blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z), gridDim.x * gridDim.y * gridDim.z);
  const int bx = lin % gridDim.x, by = (lin / gridDim.x) % gridDim.y;
  const int m0 = by * BM, c0 = bx * BN;
  const int split = lin / (gridDim.x * gridDim.y);
  const int HW = p.HW;
  const long long K = (long long)p.N * HW;
  const int nch = p.g.chunks_per_split;
  const long long q_base = (long long)split * nch * WG_KC;

  floatx16 acc[MBW][NBW];
#pragma unroll
  for (int a = 0; a < MBW; ++a)
#pragma unroll
    for (int b = 0; b < NBW; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  if (loader) {
    // ------------------------------------------------------------------ loader waves
    const int kq = tid & 7, r0 = tid >> 3;    // which 4 pixels of the chunk; first row (then every 32nd)
    size_t rowoff[NR];
    bool rok[NR];
    int tdy[NR], tdx[NR];     // MODE 3: the tap of a "u" row
#pragma unroll
    for (int j = 0; j < NR; ++j) {
      const bool isa = j < NA;
      int row = (isa ? m0 + 32 * j : c0 + 32 * (j - NA)) + r0;
      const int lim = isa ? p.Co : p.Ci;
      rok[j] = row < lim;
      if (!rok[j]) row = lim - 1;
      rowoff[j] = (size_t)row * HW;
      tdy[j] = tdx[j] = 0;
      if (MODE == 3 && !isa) {
        const int c = row / 9, tap = row - c * 9;
        tdy[j] = tap / 3 - 1;
        tdx[j] = tap % 3 - 1;
        rowoff[j] = (size_t)c * HW;
      }
    }
    const f4 zero4 = {0.f, 0.f, 0.f, 0.f};
    // MODE 3 state: image, row and first column of this lane's four pixels of the next chunk to fetch, moved on by
    // a chunk's 32 pixels after every fetch (W % 4 == 0: the four pixels stay inside one image row)
    int tn = 0, ty = 0, tx = 0;
    const int H3 = MODE == 3 ? HW / p.W : 1;
    const int adv_n = MODE == 3 ? WG_KC / HW : 0, adv_y = MODE == 3 ? (WG_KC % HW) / p.W : 0, adv_x = MODE == 3 ? (WG_KC % HW) % p.W : 0;
    if (MODE == 3) {
      const long long q = q_base + 4 * kq;
      tn = (int)(q / HW);
      const int px = (int)(q - (long long)tn * HW);
      ty = px / p.W;
      tx = px - ty * p.W;
    }
    constexpr unsigned kPast = 0x80000000u;
    unsigned voff3[NR];        // MODE 3: byte offset of the lane's row (A: dz channel, B: input channel of the tap row)
#pragma unroll
    for (int j = 0; j < NR; ++j) voff3[j] = (unsigned)(rowoff[j] * sizeof(float));   // (a row past the last repeats it)
    // MODE 2 state: image and pixel of the next chunk's first reduction index (wave-uniform), lane offsets
    int fn = (int)(q_base / HW), fpx = (int)(q_base - (long long)fn * HW);
    unsigned voff[NR];
#pragma unroll
    for (int j = 0; j < NR; ++j) voff[j] = (unsigned)((rowoff[j] + 4 * kq) * sizeof(float));
    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(p.dz), 0, (int)((unsigned)p.N * p.Co * HW * sizeof(float)), 0x00020000);
    const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(p.u), 0, (int)((unsigned)p.N * (MODE == 3 ? p.Ci / 9 : p.Ci) * HW * sizeof(float)), 0x00020000);
    const __amdgpu_buffer_rsrc_t ra_none = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p.dz), 0, 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t rb_none = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(p.u), 0, 0, 0x00020000);
    // issues the loads of chunk k (any k >= 0, also past the split's last chunk: what lies past K reads zeros or a
    // valid address whose value stash() discards); what lies past K or past the last row is replaced by zeros in stash()
    auto fetch = [&](int k, f4 (&v)[NR], int &okmask) {
      const long long q = q_base + (long long)k * WG_KC + 4 * kq;
      if (MODE == 2) {
        // K is a multiple of the chunk: a chunk is valid or not as a whole.  One past K is read through descriptors of
        // length zero, which deliver zeros without touching memory: no branch around the loads, so the loader knows
        // how many are in flight and waits for the older chunk's only
        const bool ok = fn < p.N;
        okmask = ok ? 15 : 0;
        const __amdgpu_buffer_rsrc_t qa = ok ? ra : ra_none, qb = ok ? rb : rb_none;
        const unsigned sa = (unsigned)(((size_t)fn * p.Co * HW + fpx) * sizeof(float));
        const unsigned sb = (unsigned)(((size_t)fn * p.Ci * HW + fpx) * sizeof(float));
#pragma unroll
        for (int j = 0; j < NR; ++j)
          v[j] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(j < NA ? qa : qb, voff[j], j < NA ? sa : sb, 0));
        fpx += WG_KC;
        if (fpx >= HW) fpx -= HW, ++fn;
      } else if (MODE == 3) {
        // this lane's four pixels of the chunk: image tn, row ty, first column tx, kept from chunk to chunk.  All
        // addresses are 32-bit byte offsets into buffers (both tensors at most 2 GiB); an offset of 2 GiB or more is
        // past either buffer and reads zeros, which is how pixels past K and taps that
        // fall outside the image get theirs (rows past the last channel repeat it: their products are never stored).
        const bool ok = tn < p.N;
        const unsigned pxo = (unsigned)(ty * p.W + tx);
        const unsigned basea = ok ? (unsigned)(((unsigned)tn * (unsigned)p.Co * (unsigned)HW + pxo) * 4u) : kPast;
        okmask = 0;
#pragma unroll
        for (int j = 0; j < NR; ++j) {
          if (j < NA) {
            v[j] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(ra, basea + voff3[j], 0, 0));
          } else {
            // the four input values under the tap: one 16-byte load at x + dx (4-byte aligned); at the left / right
            // border the load starts at the row's first / last group and stash() moves the values over by one.  No
            // branch around any load (a group of 32 rows with no tap row in it loads zeros like everything else that
            // does not exist): the loader then knows how many loads are in flight and waits for the older chunk only.
            const int yy = ty + tdy[j];
            const bool yok = ok && yy >= 0 && yy < H3 && c0 + 32 * (j - NA) < p.Ci;
            const int xs = tx + tdx[j];
            const bool le = xs < 0, re = xs + 4 > p.W;
            const unsigned off = ((unsigned)tn * (unsigned)(p.Ci / 9) * (unsigned)HW + (unsigned)(yy * p.W + (le ? 0 : (re ? p.W - 4 : xs)))) * 4u;
            v[j] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rb, (yok ? off : kPast) + voff3[j], 0, 0));
            okmask |= (le ? 1 : (re ? 2 : 0)) << (2 * (j - NA));
          }
        }
        // on by a chunk's 32 pixels = adv_n images + adv_y rows + adv_x columns, each carry at most one (no loop, no
        // branch: see the note at the loader's main loop)
        tx += adv_x;
        const bool cx = tx >= p.W;
        tx -= cx ? p.W : 0;
        ty += adv_y + (cx ? 1 : 0);
        const bool cy = ty >= H3;
        ty -= cy ? H3 : 0;
        tn += adv_n + (cy ? 1 : 0);
      } else if (VEC) {                       // HW % 4 == 0: the four pixels share an image and are 16-byte aligned
        okmask = (q < K) ? 15 : 0;
        const long long qq = (q < K) ? q : 0;
        const int n = (int)(qq / HW);
        const int px = (int)(qq - (long long)n * HW);
        const float *pa = p.dz + (size_t)n * p.Co * HW + px;
        const float *pb = p.u + (size_t)n * p.Ci * HW + px;
#pragma unroll
        for (int j = 0; j < NR; ++j) v[j] = *reinterpret_cast<const f4 *>((j < NA ? pa : pb) + rowoff[j]);
      } else {
        okmask = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const bool ok = q + e < K;
          okmask |= ok ? (1 << e) : 0;
          const long long qq = ok ? q + e : 0;
          const int n = (int)(qq / HW);
          const int px = (int)(qq - (long long)n * HW);
          const float *pa = p.dz + (size_t)n * p.Co * HW + px;
          const float *pb = p.u + (size_t)n * p.Ci * HW + px;
#pragma unroll
          for (int j = 0; j < NR; ++j) v[j][e] = (j < NA ? pa : pb)[rowoff[j]];
        }
      }
    };
    auto stash = [&](int k, const f4 (&v)[NR], int okmask) {
      float *dst = smem + (k & 1) * BUF + r0 * WG_LS + 4 * kq;
#pragma unroll
      for (int j = 0; j < NR; ++j) {
        f4 w = v[j];
        if (MODE == 2) {
          // rows past the last channel repeat the last one: their products land in rows/columns never stored
        } else if (MODE == 3) {
          // whatever must be zero was read as zero; a tap row at the image's left / right border moves over by one
          if (j >= NA) {
            const int sf = (okmask >> (2 * (j - NA))) & 3;
            const f4 t = w;
            w[0] = sf == 1 ? 0.f : (sf == 2 ? t[1] : t[0]);
            w[1] = sf == 1 ? t[0] : (sf == 2 ? t[2] : t[1]);
            w[2] = sf == 1 ? t[1] : (sf == 2 ? t[3] : t[2]);
            w[3] = sf == 1 ? t[2] : (sf == 2 ? 0.f : t[3]);
          }
        } else if (VEC) {
          if (!(okmask && rok[j])) w = zero4;
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (!(((okmask >> e) & 1) && rok[j])) w[e] = 0.f;
        }
        *reinterpret_cast<f4 *>(dst + (size_t)(32 * j) * WG_LS) = w;    // A rows first, B rows follow at BM
      }
    };
    // two register sets take turns (no copies: vector ALU work is what the loaders cannot afford); every
    // __syncthreads below says "copy k&1 is complete, the MFMA waves have finished chunk k-1"
    f4 ra4[NR], rb4[NR];
    int oka = 0, okb = 0;
    // (the fetch after the split's last chunk is issued like any other and never stashed: a fetch under a condition
    // would make the compiler wait for all loads before every stash, not knowing how many are in flight)
    fetch(0, ra4, oka);
    int k = 0;
    while (k < nch) {
      fetch(k + 1, rb4, okb);
      stash(k, ra4, oka);
      __syncthreads();
      if (++k >= nch) break;
      fetch(k + 1, ra4, oka);
      stash(k, rb4, okb);
      __syncthreads();
      ++k;
    }
    __syncthreads();
  } else {
    // ------------------------------------------------------------------ MFMA waves
    const float *A0 = smem + (wm * (MBW * 32) + l31) * WG_LS + 4 * lh;
    const float *B0 = smem + (BM + wn * (NBW * 32) + l31) * WG_LS + 4 * lh;
    // MODE 3: the tap rows fill only the first 9*Cin columns of the tile; a wave whose columns all lie past them has
    // nothing to multiply (it still keeps the barriers' count)
    const bool idle = MODE == 3 && c0 + wn * (NBW * 32) >= p.Ci;
    __syncthreads();     // chunk 0 is staged
    for (int k = 0; k < nch; ++k) {
      if (idle) {
        __syncthreads();
        continue;
      }
      const float *Ab = A0 + (k & 1) * BUF, *Bb = B0 + (k & 1) * BUF;
      f4 av[MBW], bv[NBW];
#pragma unroll
      for (int mb = 0; mb < MBW; ++mb) av[mb] = *reinterpret_cast<const f4 *>(Ab + mb * 32 * WG_LS);
#pragma unroll
      for (int nb = 0; nb < NBW; ++nb) bv[nb] = *reinterpret_cast<const f4 *>(Bb + nb * 32 * WG_LS);
#pragma unroll
      for (int g = 0; g < WG_KC / 8; ++g) {
        f4 nav[MBW], nbv[NBW];
#pragma unroll
        for (int mb = 0; mb < MBW; ++mb) nav[mb] = av[mb];
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) nbv[nb] = bv[nb];
        if (g + 1 < WG_KC / 8) {
#pragma unroll
          for (int mb = 0; mb < MBW; ++mb) nav[mb] = *reinterpret_cast<const f4 *>(Ab + mb * 32 * WG_LS + 8 * (g + 1));
#pragma unroll
          for (int nb = 0; nb < NBW; ++nb) nbv[nb] = *reinterpret_cast<const f4 *>(Bb + nb * 32 * WG_LS + 8 * (g + 1));
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb)
              acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[mb][e], bv[nb][e], acc[mb][nb], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int mb = 0; mb < MBW; ++mb) av[mb] = nav[mb];
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) bv[nb] = nbv[nb];
      }
      __syncthreads();   // chunk k consumed: its LDS copy may be overwritten; copy (k+1)&1 is ready
    }

    // ---- accumulator register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32
    float *dst = p.partial + (size_t)split * p.Co * p.Ci;
#pragma unroll
    for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int o = m0 + (wm * MBW + mb) * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
        if (o < p.Co) {
#pragma unroll
          for (int nb = 0; nb < NBW; ++nb) {
            const int c = c0 + (wn * NBW + nb) * 32 + l31;
            if (c < p.Ci) dst[(size_t)o * p.Ci + c] = acc[mb][nb][r];
          }
        }
      }
  }
}

// ---- weight gradient of a full 3x3 first layer with its BatchNorm backward folded in (WgradArgs, g.vec == 4).
// LDS per chunk of 32 pixels: 64 rows of g, 64 rows of z, 32 tap rows of the shifted input, transposed as above.
// MFMA wave (wm, wn): output channels 32*wm .. +31; wn = 0 multiplies g, wn = 1 multiplies z - mean, both with the
// same 32 tap columns.  A wave writes its product, scaled by its per-channel factor (wn = 0: plus the column-sum
// term), as a partial slab of its own: slab 2*split + wn; the update kernel adds the slabs.  Loaders as in MODE 3.
__global__ __launch_bounds__(512) void wgrad_taps_bn_kernel(WgradArgs p) {
  constexpr int BM = 64, AROWS = 2 * BM, BROWS = 32;
  constexpr int BUF = (AROWS + BROWS) * WG_LS;
  constexpr int NR = 5;                          // loads per loader thread and chunk: g, g, z, z, tap row
  typedef float f4 __attribute__((ext_vector_type(4)));
  extern __shared__ float smem[];                // [2][AROWS + BROWS][WG_LS]

  const bool loader = threadIdx.x >= 256;
  const int tid = threadIdx.x & 255, lane = tid & 63, wave = tid >> 6;
  const int l31 = lane & 31, lh = lane >> 5;
  const int wm = wave & 1, wn = wave >> 1;
  const int lin = xcd_contiguous(blockIdx.y + gridDim.y * blockIdx.z, gridDim.y * gridDim.z);
  const int by = lin % gridDim.y, split = lin / gridDim.y;
  const int m0 = by * BM;
  const int HW = p.HW;
  const int nch = p.g.chunks_per_split;
  const long long q_base = (long long)split * nch * WG_KC;

  floatx16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  float ssum = 0.f;                              // wn = 0: this lane's share of its tap column's sum

  if (loader) {
    const int kq = tid & 7, r0 = tid >> 3;       // which 4 pixels of the chunk; row within a group of 32
    constexpr unsigned kPast = 0x80000000u;      // offsets from here on are past either buffer: they read zeros
    unsigned voff[NR];
    int tdy, tdx;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int row = m0 + 32 * (j & 1) + r0;
      if (row > p.Co - 1) row = p.Co - 1;        // a row past the last channel repeats it: its products are never stored
      voff[j] = (unsigned)row * (unsigned)HW * 4u;
    }
    {
      const int row = r0 < p.Ci ? r0 : p.Ci - 1;
      const int c = row / 9, tap = row - c * 9;
      tdy = tap / 3 - 1;
      tdx = tap % 3 - 1;
      voff[4] = (unsigned)c * (unsigned)HW * 4u;
    }
    const __amdgpu_buffer_rsrc_t rg = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(p.dz), 0, (int)((unsigned)p.N * p.Co * HW * sizeof(float)), 0x00020000);
    const __amdgpu_buffer_rsrc_t rz = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(p.z), 0, (int)((unsigned)p.N * p.Co * HW * sizeof(float)), 0x00020000);
    const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(p.u), 0, (int)((unsigned)p.N * (p.Ci / 9) * HW * sizeof(float)), 0x00020000);
    // image, row and first column of this lane's four pixels of the next chunk to fetch (W % 4 == 0: they stay inside
    // one image row), moved on by a chunk's 32 pixels after every fetch
    const int H3 = HW / p.W;
    const int adv_n = WG_KC / HW, adv_y = (WG_KC % HW) / p.W, adv_x = (WG_KC % HW) % p.W;
    int tn, ty, tx;
    {
      const long long q = q_base + 4 * kq;
      tn = (int)(q / HW);
      const int px = (int)(q - (long long)tn * HW);
      ty = px / p.W;
      tx = px - ty * p.W;
    }
    // no load is issued under a condition (what does not exist reads zeros through its offset): the compiler then
    // knows how many loads are in flight and lets the newer chunk's stay there while the older one is staged
    auto fetch = [&](f4 (&v)[NR], int &sf) {
      const bool ok = tn < p.N;
      const unsigned pxo = (unsigned)(ty * p.W + tx);
      const unsigned basea = ok ? ((unsigned)tn * (unsigned)p.Co * (unsigned)HW + pxo) * 4u : kPast;
      v[0] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rg, basea + voff[0], 0, 0));
      v[1] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rg, basea + voff[1], 0, 0));
      v[2] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rz, basea + voff[2], 0, 0));
      v[3] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rz, basea + voff[3], 0, 0));
      // the four input values under the tap: one 16-byte load at x + dx (4-byte aligned); at the left / right border
      // the load starts at the row's first / last group and stash() moves the values over by one
      const int yy = ty + tdy;
      const bool yok = ok && r0 < p.Ci && yy >= 0 && yy < H3;
      const int xs = tx + tdx;
      const bool le = xs < 0, re = xs + 4 > p.W;
      const unsigned off = ((unsigned)tn * (unsigned)(p.Ci / 9) * (unsigned)HW + (unsigned)(yy * p.W + (le ? 0 : (re ? p.W - 4 : xs)))) * 4u;
      v[4] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rb, (yok ? off : kPast) + voff[4], 0, 0));
      sf = le ? 1 : (re ? 2 : 0);
      tx += adv_x;
      const bool cx = tx >= p.W;
      tx -= cx ? p.W : 0;
      ty += adv_y + (cx ? 1 : 0);
      const bool cy = ty >= H3;
      ty -= cy ? H3 : 0;
      tn += adv_n + (cy ? 1 : 0);
    };
    auto stash = [&](int k, const f4 (&v)[NR], int sf) {
      float *dst = smem + (k & 1) * BUF + r0 * WG_LS + 4 * kq;
#pragma unroll
      for (int j = 0; j < 4; ++j) *reinterpret_cast<f4 *>(dst + (size_t)(32 * j) * WG_LS) = v[j];   // g rows, then z rows
      const f4 t = v[4];
      f4 w;
      w[0] = sf == 1 ? 0.f : (sf == 2 ? t[1] : t[0]);
      w[1] = sf == 1 ? t[0] : (sf == 2 ? t[2] : t[1]);
      w[2] = sf == 1 ? t[1] : (sf == 2 ? t[3] : t[2]);
      w[3] = sf == 1 ? t[2] : (sf == 2 ? 0.f : t[3]);
      *reinterpret_cast<f4 *>(dst + (size_t)AROWS * WG_LS) = w;
    };
    f4 ra4[NR], rb4[NR];
    int sfa = 0, sfb = 0;
    fetch(ra4, sfa);
    int k = 0;
    while (k < nch) {          // (the fetch after the last chunk is issued like any other and never staged)
      fetch(rb4, sfb);
      stash(k, ra4, sfa);
      __syncthreads();
      if (++k >= nch) break;
      fetch(ra4, sfa);
      stash(k, rb4, sfb);
      __syncthreads();
      ++k;
    }
    __syncthreads();
  } else {
    const float *A0 = smem + (wn * BM + wm * 32 + l31) * WG_LS + 4 * lh;
    const float *B0 = smem + (AROWS + l31) * WG_LS + 4 * lh;
    const int orow = m0 + wm * 32 + l31;
    const float mean = wn ? p.mean[orow < p.Co ? orow : p.Co - 1] : 0.f;
    __syncthreads();     // chunk 0 is staged
    for (int k = 0; k < nch; ++k) {
      const float *Ab = A0 + (k & 1) * BUF, *Bb = B0 + (k & 1) * BUF;
#pragma unroll
      for (int g = 0; g < WG_KC / 8; ++g) {
        f4 av = *reinterpret_cast<const f4 *>(Ab + 8 * g);
        const f4 bv = *reinterpret_cast<const f4 *>(Bb + 8 * g);
        if (wn) {
#pragma unroll
          for (int e = 0; e < 4; ++e) av[e] -= mean;
        } else {
          ssum += (bv[0] + bv[1]) + (bv[2] + bv[3]);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av[e], bv[e], acc, 0, 0, 0);
      }
      __syncthreads();   // chunk k consumed: its LDS copy may be overwritten; copy (k+1)&1 is ready
    }
    // ---- accumulator register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32
    const float colsum = ssum + __shfl_xor(ssum, 32, 64);       // sum of tap column l%32 over the split's pixels
    const float invm = 1.f / ((float)p.N * (float)HW);
    float *dst = p.partial + (size_t)(2 * split + wn) * p.Co * p.Ci;
    const int c = l31;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int o = m0 + wm * 32 + 8 * (r / 4) + 4 * lh + (r % 4);
      if (o < p.Co && c < p.Ci) {
        const float sc = p.scale[o];
        float v;
        if (wn)
          v = -(sc * invm) * p.dgamma[o] * p.rstd[o] * acc[r];
        else
          v = sc * acc[r] - (sc * invm) * p.dbeta[o] * colsum;
        dst[(size_t)o * p.Ci + c] = v;
      }
    }
  }
}

WgradGeom wgrad_taps_bn_geom(int N, int Co, int Cin, int HW) {
  WgradGeom g{};
  g.variant = 3;
  g.vec = 4;
  g.tiles_m = cdiv(Co, 64);
  g.tiles_n = 1;
  const long long K = (long long)N * HW;
  const int nchunks = (int)((K + WG_KC - 1) / WG_KC);
  g.lds_bytes = (size_t)2 * (2 * 64 + 32) * WG_LS * sizeof(float);
  // three workgroups per compute unit (their LDS allows no more): the kernel is bound by the bytes its loaders keep in flight
  int want = 768 / g.tiles_m;
  if (want < 1) want = 1;
  if (want > nchunks) want = nchunks;
  g.chunks_per_split = cdiv(nchunks, want);
  g.splits = cdiv(nchunks, g.chunks_per_split);
  g.slabs = 2 * g.splits;
  (void)Cin;
  return g;
}

static inline int wg_bm(int variant) { return (variant & 2) ? 64 : 128; }
static inline int wg_bn(int variant) { return (variant & 1) ? 64 : 128; }

WgradGeom wgrad_taps_geom(int N, int Co, int Cin, int HW) {
  WgradGeom g = wgrad_geom(N, Co, 9 * Cin, HW);
  g.vec = 3;
  // Only dz comes from HBM here (the input has few channels and stays in cache) and the tile of dW is tiny, so the
  // kernel is bound by the bytes its loaders keep in flight: four workgroups per compute unit instead of one.
  const long long K = (long long)N * HW;
  const int nchunks = (int)((K + WG_KC - 1) / WG_KC);
  int want = 1024 / (g.tiles_m * g.tiles_n);
  if (want < 1) want = 1;
  if (want > nchunks) want = nchunks;
  g.chunks_per_split = cdiv(nchunks, want);
  g.splits = cdiv(nchunks, g.chunks_per_split);
  g.slabs = g.splits;
  return g;
}

WgradGeom wgrad_geom(int N, int Co, int Ci, int HW) {
  WgradGeom g;
  // 64x64 tiles: every split costs a whole tile of partial-sum traffic, written and read again, so more tiles
  // with fewer splits beat larger tiles (measured, 128x128 weights at K = 32768: 27 us against 36 us for both
  // layers of the default workload), although each operand row is then read by two workgroups (L2 hits)
  g.variant = 3;
  (void)Co; (void)Ci;
  if (const char *env = std::getenv("PBKD_WGRAD_VARIANT")) {   // tuning aid: bit 1 = 64 rows, bit 0 = 64 columns
    const int v = std::atoi(env);
    if (v >= 0 && v <= 3) g.variant = v;
  }
  const bool small = (unsigned long long)N * Co * HW * sizeof(float) < (1ull << 32) &&
                     (unsigned long long)N * Ci * HW * sizeof(float) < (1ull << 32);
  g.vec = (HW % WG_KC == 0 && small) ? 2 : (HW % 4 == 0) ? 1 : 0;
  g.tiles_m = cdiv(Co, wg_bm(g.variant));
  g.tiles_n = cdiv(Ci, wg_bn(g.variant));
  const long long K = (long long)N * HW;
  const int nchunks = (int)((K + WG_KC - 1) / WG_KC);
  // one workgroup per compute unit: every further split costs a whole tile of partial-sum traffic
  int want = 256 / (g.tiles_m * g.tiles_n);
  if (want < 1) want = 1;
  if (want > nchunks) want = nchunks;
  g.chunks_per_split = cdiv(nchunks, want);
  g.splits = cdiv(nchunks, g.chunks_per_split);
  g.slabs = g.splits;
  g.lds_bytes = (size_t)2 * (wg_bm(g.variant) + wg_bn(g.variant)) * WG_LS * sizeof(float);
  return g;
}

hipError_t init_pw_wgrad_attributes() {
  hipError_t e;
#define PBKD_SET(MBW, NBW, MODE)                                                                            \
  e = hipFuncSetAttribute(reinterpret_cast<const void *>(&pw_wgrad_kernel<MBW, NBW, MODE>),                 \
                          hipFuncAttributeMaxDynamicSharedMemorySize, MAX_LDS);                             \
  if (e != hipSuccess) return e;
#define PBKD_SET3(MBW, NBW) PBKD_SET(MBW, NBW, 0) PBKD_SET(MBW, NBW, 1) PBKD_SET(MBW, NBW, 2) PBKD_SET(MBW, NBW, 3)
  PBKD_SET3(2, 2) PBKD_SET3(2, 1) PBKD_SET3(1, 2) PBKD_SET3(1, 1)
#undef PBKD_SET3
#undef PBKD_SET
  return hipFuncSetAttribute(reinterpret_cast<const void *>(&wgrad_taps_bn_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, MAX_LDS);
}

hipError_t launch_pw_wgrad(const WgradArgs &a, hipStream_t s) {
  if (a.g.splits <= 0 || a.g.splits > 65535 || a.g.tiles_m > 65535 || a.N <= 0 || a.HW <= 0) return hipErrorInvalidValue;
  if (a.g.vec && (a.HW % 4 || (reinterpret_cast<uintptr_t>(a.dz) & 15) || (reinterpret_cast<uintptr_t>(a.u) & 15)))
    return hipErrorInvalidValue;
  if (a.g.vec == 2 && a.HW % WG_KC) return hipErrorInvalidValue;
  if (a.g.vec == 3 && (a.W < 4 || a.W % 4 || a.HW % a.W || a.Ci % 9 || a.Ci > 64 || !wgrad_taps_small(a.N, a.Co, a.Ci / 9, a.HW)))
    return hipErrorInvalidValue;
  if (a.g.vec == 4) {
    if (a.W < 4 || a.W % 4 || a.HW % a.W || a.Ci % 9 || a.Ci > 32 || !wgrad_taps_small(a.N, a.Co, a.Ci / 9, a.HW) || a.g.tiles_n != 1 ||
        a.g.slabs != 2 * a.g.splits || !a.z || !a.scale || !a.mean || !a.rstd || !a.dgamma || !a.dbeta || (reinterpret_cast<uintptr_t>(a.z) & 15))
      return hipErrorInvalidValue;
    hipLaunchKernelGGL(wgrad_taps_bn_kernel, dim3(1, a.g.tiles_m, a.g.splits), dim3(512), a.g.lds_bytes, s, a);
    return hipGetLastError();
  }
  const dim3 grid(a.g.tiles_n, a.g.tiles_m, a.g.splits), block(512);
#define PBKD_GO(MBW, NBW)                                                                                   \
  if (a.g.vec == 3)                                                                                         \
    hipLaunchKernelGGL((pw_wgrad_kernel<MBW, NBW, 3>), grid, block, a.g.lds_bytes, s, a);                   \
  else if (a.g.vec == 2)                                                                                    \
    hipLaunchKernelGGL((pw_wgrad_kernel<MBW, NBW, 2>), grid, block, a.g.lds_bytes, s, a);                   \
  else if (a.g.vec == 1)                                                                                    \
    hipLaunchKernelGGL((pw_wgrad_kernel<MBW, NBW, 1>), grid, block, a.g.lds_bytes, s, a);                   \
  else                                                                                                      \
    hipLaunchKernelGGL((pw_wgrad_kernel<MBW, NBW, 0>), grid, block, a.g.lds_bytes, s, a);
  switch (a.g.variant) {
    case 0: PBKD_GO(2, 2) break;
    case 1: PBKD_GO(2, 1) break;
    case 2: PBKD_GO(1, 2) break;
    case 3: PBKD_GO(1, 1) break;
    default: return hipErrorInvalidValue;
  }
#undef PBKD_GO
  return hipGetLastError();
}

}  // namespace pbkd

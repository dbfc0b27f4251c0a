// 3x3 convolution with frozen weights on the bf16 matrix cores, fp32 operands split three ways (device code and the
// arithmetic: conv_split_kernel.h).  Same workgroup tiles and pixel-tile geometry as the fp32-MFMA kernel, launched as
// a persistent grid; this file instantiates the tiles and launches.
#include <cstdlib>
#include <type_traits>

#include "conv_mfma_kernel.h"
#include "conv_split_kernel.h"

namespace pbkd {

namespace {
int compute_units() {
  static const int n = [] {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 1) v = 256;
    return v;
  }();
  return n;
}

template <int WGM, int MB, int NB>
struct SplitLaunch {
  template <int BSLOTS>
  static hipError_t attr() {
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_split_kernel<WGM, MB, NB, BSLOTS>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, MAX_LDS);
  }
  static hipError_t init() {
    hipError_t e;
    if ((e = attr<1>()) != hipSuccess) return e;
    if ((e = attr<2>()) != hipSuccess) return e;
    if constexpr (WGM * MB * NB >= 4) return hipSuccess;      // the two large tiles stop at two halo slots per thread
    else return attr<3>();
  }
  template <int BSLOTS>
  static void go(const dim3 &grid, const dim3 &block, const ConvArgs &a, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
    if (e0 && e1)
      hipExtLaunchKernelGGL((conv_split_kernel<WGM, MB, NB, BSLOTS>), grid, block, (unsigned)a.g.lds_bytes, s, e0, e1, 0, a);
    else
      hipLaunchKernelGGL((conv_split_kernel<WGM, MB, NB, BSLOTS>), grid, block, a.g.lds_bytes, s, a);
  }
  static hipError_t launch(const ConvArgs &a, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
    // persistent: one workgroup per compute unit (their LDS allows no more), each walking every G-th tile; more
    // workgroups only where a workgroup's tile table would overflow
    const long long items = (long long)a.g.n_ptiles * a.g.mtiles * a.g.ksplit;
    long long cus = compute_units();
    if (const char *env = std::getenv("PBKD_SPLIT_WGS")) {
      const int v = std::atoi(env);
      if (v >= 1 && v < cus) cus = v;
    }
    long long G = items < cus ? items : cus;
    if (G * kSplitMaxTiles < items) G = (items + kSplitMaxTiles - 1) / kSplitMaxTiles;
    if (items < 1 || items > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)G), block(512);
    switch (conv_bslots_for(a.g.PLd)) {
      case 1: go<1>(grid, block, a, s, e0, e1); break;
      case 2: go<2>(grid, block, a, s, e0, e1); break;
      case 3:
        if constexpr (WGM * MB * NB >= 4) return hipErrorInvalidValue;
        else go<3>(grid, block, a, s, e0, e1);
        break;
      default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
};
}  // namespace

hipError_t conv_split_init() {
  hipError_t e;
  if ((e = SplitLaunch<2, 2, 2>::init()) != hipSuccess) return e;
  if ((e = SplitLaunch<1, 2, 2>::init()) != hipSuccess) return e;
  if ((e = SplitLaunch<1, 2, 1>::init()) != hipSuccess) return e;
  return SplitLaunch<2, 1, 1>::init();
}

hipError_t launch_conv_split(const ConvArgs &a, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  if (!a.g.split || !conv_split_fits_width(a.g, a.H, a.W, a.stride) || a.g.lds_bytes > (size_t)MAX_LDS || a.g.raw_rounds > conv_split_rounds_max(conv_bslots_for(a.g.PLd)) || a.g.raw_w % 4 != 0)
    return hipErrorInvalidValue;
  if (a.g.ksplit < 1 || a.g.kchunks < 1 || (long long)(a.g.ksplit - 1) * a.g.kchunks >= a.g.nchunks ||
      (long long)a.g.ksplit * a.g.kchunks < a.g.nchunks || (a.g.ksplit > 1 && !a.split_out))
    return hipErrorInvalidValue;
  // the output (all K splits of it) and the weight image are addressed through buffer descriptors with 32-bit offsets
  if ((unsigned long long)a.g.ksplit * a.N * a.Cout * a.Ho * a.Wo * sizeof(float) >= (1ull << 32)) return hipErrorInvalidValue;
  if ((unsigned long long)a.g.mtiles * a.g.nchunks * conv_split_a_stride(a.g.bm) >= (1ull << 32)) return hipErrorInvalidValue;
  switch (a.g.tile) {
    case 0: return SplitLaunch<2, 2, 2>::launch(a, s, e0, e1);
    case 1: return SplitLaunch<1, 2, 2>::launch(a, s, e0, e1);
    case 2: return SplitLaunch<1, 2, 1>::launch(a, s, e0, e1);
    case 3: return SplitLaunch<2, 1, 1>::launch(a, s, e0, e1);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace pbkd

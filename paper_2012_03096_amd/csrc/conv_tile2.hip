// Workgroup tile 2 of the MFMA convolution: 64 output channels x 128 pixels (4 waves of 64 x 32).
#include "conv_mfma_kernel.h"

namespace pbkd {
hipError_t conv_tile2_init() { return ConvTile<1, 2, 1>::init(); }
hipError_t conv_tile2_launch(int taps, const ConvArgs &a, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  return ConvTile<1, 2, 1>::launch(taps, a, s, e0, e1);
}
}  // namespace pbkd

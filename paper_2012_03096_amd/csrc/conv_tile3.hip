// Workgroup tile 3 of the MFMA convolution: 64 output channels x 64 pixels (4 waves of 32 x 32).
#include "conv_mfma_kernel.h"

namespace pbkd {
hipError_t conv_tile3_init() { return ConvTile<2, 1, 1>::init(); }
hipError_t conv_tile3_launch(int taps, const ConvArgs &a, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  return ConvTile<2, 1, 1>::launch(taps, a, s, e0, e1);
}
}  // namespace pbkd

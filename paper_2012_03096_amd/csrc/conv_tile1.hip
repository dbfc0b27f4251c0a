// Workgroup tile 1 of the MFMA convolution: 64 output channels x 256 pixels (4 waves of 64 x 64).
#include "conv_mfma_kernel.h"

namespace pbkd {
hipError_t conv_tile1_init() { return ConvTile<1, 2, 2>::init(); }
hipError_t conv_tile1_launch(int taps, const ConvArgs &a, hipStream_t s, hipEvent_t e0, hipEvent_t e1) {
  return ConvTile<1, 2, 2>::launch(taps, a, s, e0, e1);
}
}  // namespace pbkd

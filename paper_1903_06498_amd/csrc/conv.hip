// Nested-tile convolution-shaped contraction on the gfx950 matrix cores.
#include <hip/hip_runtime.h>

#include "kernels.hpp"

namespace stripe {

bool conv_select(const Conv2dShape&, int, ConvLaunch*, stripe_block_info_t*) { return false; }

hipError_t launch_conv(const Conv2dShape&, const ConvLaunch&, const void*, const void*, void*, hipStream_t) {
  return hipErrorNotSupported;
}

}  // namespace stripe

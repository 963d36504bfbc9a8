// Stride-1 convolution with the input patch resident in LDS (schedule variant 1): channel count
// equal to the k-tile, RSCK weights.
#include "alcop_instantiate.hip.h"
namespace alcop {
void register_conv_patch(std::vector<KernelEntry>& t)
{
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 256, 64, 64, 64, 0, 3)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 128, 64, 64, 32, 0, 3)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 128, 128, 64, 64, 0, 3)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 256, 128, 128, 64, 0, 3)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 64, 64, 32, 32, 0, 3)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 1, 256, 64, 64, 64, 0, 3)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 1, 128, 64, 64, 32, 0, 3)
}
}  // namespace alcop

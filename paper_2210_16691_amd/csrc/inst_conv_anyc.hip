// Implicit-GEMM convolution for channel counts that the k-tile does not divide (any multiple of
// 8): every lane tracks the filter tap of its own 8-channel chunk.  Weights RSCK and KRSC.
#include "alcop_instantiate.hip.h"
namespace alcop {
void register_conv_anyc(std::vector<KernelEntry>& t)
{
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 128, 64, 64, 32, 0, 2)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 64, 64, 32, 32, 0, 2)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 128, 128, 64, 64, 0, 2)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 256, 64, 64, 64, 0, 2)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 1, 128, 64, 64, 32, 0, 2)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 128, 64, 64, 32, 1, 2)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 64, 64, 32, 32, 1, 2)
}
}  // namespace alcop

// Implicit-GEMM convolution with KRSC weights (B stored N x K, k-contiguous).
#include "alcop_instantiate.hip.h"
namespace alcop {
void register_conv_krsc(std::vector<KernelEntry>& t)
{
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 128, 64, 64, 32, 1, 1)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 256, 64, 64, 64, 1, 1)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 64, 64, 32, 32, 1, 1)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 128, 128, 64, 64, 1, 1)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 1, 128, 64, 64, 32, 1, 1)
}
}  // namespace alcop

// Implicit-GEMM convolution (gathering A loader), weights RSCK = B stored K x N.
#include "alcop_instantiate.hip.h"
namespace alcop {
void register_conv(std::vector<KernelEntry>& t)
{
  ALCOP_BOTH_BK(ALCOP_ALL_PIPES, t, 0, 128, 64, 64, 32, 0, 1)
  ALCOP_BOTH_BK(ALCOP_ALL_PIPES, t, 0, 256, 64, 64, 64, 0, 1)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 64, 64, 32, 32, 0, 1)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 128, 128, 64, 64, 0, 1)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 64, 128, 32, 64, 0, 1)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 256, 128, 128, 64, 0, 1)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 1, 128, 64, 64, 32, 0, 1)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 1, 128, 128, 64, 64, 0, 1)
}
}  // namespace alcop

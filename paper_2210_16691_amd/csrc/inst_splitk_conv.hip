// Split-K variants of the implicit-GEMM convolution (long reduction axis R*S*C, few output tiles).
#include "alcop_instantiate.hip.h"
namespace alcop {
void register_splitk_conv(std::vector<KernelEntry>& t)
{
  ALCOP_SPLITK_PIPES(t, 0, 128, 128, 64, 64, 64, 0, 1)
  ALCOP_SPLITK_PIPES(t, 0, 128, 64, 64, 64, 32, 0, 1)
  ALCOP_SPLITK_PIPES(t, 0, 64, 128, 64, 32, 64, 0, 1)
  ALCOP_SPLITK_PIPES(t, 0, 64, 64, 64, 32, 32, 0, 1)
  ALCOP_SPLITK_PIPES(t, 1, 128, 64, 64, 64, 32, 0, 1)
}
}  // namespace alcop

// B stored N x K (the Q.K^T layout), fp16 and bf16.
#include "alcop_instantiate.hip.h"
namespace alcop {
void register_nk(std::vector<KernelEntry>& t)
{
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 256, 256, 128, 128, 1, 0)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 256, 128, 128, 64, 1, 0)
  ALCOP_BOTH_BK(ALCOP_ALL_PIPES, t, 0, 128, 128, 64, 64, 1, 0)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 128, 64, 64, 32, 1, 0)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 64, 64, 32, 32, 1, 0)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 1, 256, 256, 128, 128, 1, 0)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 1, 128, 128, 64, 64, 1, 0)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 1, 64, 64, 32, 32, 1, 0)
}
}  // namespace alcop

// fp16, B stored K x N: tiles with a 64-wide side.
#include "alcop_instantiate.hip.h"
namespace alcop {
void register_f16_kn_small(std::vector<KernelEntry>& t)
{
  ALCOP_BOTH_BK(ALCOP_ALL_PIPES, t, 0, 64, 64, 32, 32, 0, 0)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 128, 64, 64, 32, 0, 0)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 256, 64, 64, 64, 0, 0)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 64, 128, 32, 64, 0, 0)
}
}  // namespace alcop

// fp16, B stored K x N: 256-wide tiles.
#include "alcop_instantiate.hip.h"
namespace alcop {
void register_f16_kn_big(std::vector<KernelEntry>& t)
{
  ALCOP_BOTH_BK(ALCOP_ALL_PIPES, t, 0, 256, 256, 128, 128, 0, 0)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 256, 256, 128, 64, 0, 0)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 256, 128, 128, 64, 0, 0)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 0, 128, 256, 64, 128, 0, 0)
}
}  // namespace alcop

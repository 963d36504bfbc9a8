// bf16, B stored K x N.
#include "alcop_instantiate.hip.h"
namespace alcop {
void register_bf16_kn(std::vector<KernelEntry>& t)
{
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 1, 256, 256, 128, 128, 0, 0)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 1, 256, 256, 128, 64, 0, 0)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 1, 256, 128, 128, 64, 0, 0)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 1, 128, 256, 64, 128, 0, 0)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 1, 128, 128, 64, 64, 0, 0)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 1, 128, 64, 64, 32, 0, 0)
  ALCOP_BOTH_BK(ALCOP_KEY_PIPES, t, 1, 64, 64, 32, 32, 0, 0)
}
}  // namespace alcop

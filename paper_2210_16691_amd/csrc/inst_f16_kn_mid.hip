// fp16, B stored K x N: 128 x 128 tiles.
#include "alcop_instantiate.hip.h"
namespace alcop {
void register_f16_kn_mid(std::vector<KernelEntry>& t)
{
  ALCOP_BOTH_BK(ALCOP_ALL_PIPES, t, 0, 128, 128, 64, 64, 0, 0)
}
}  // namespace alcop

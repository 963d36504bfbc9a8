// Kernels with the third pipeline level (HBM -> L2 touches): one more load per wave and k-tile.
// A few fused pipelines of the main tiles; schedules with l2_prefetch > 0 resolve to these.
#include "alcop_instantiate.hip.h"
namespace alcop {
#define ALCOP_PF_PIPES(T, DT, BM, BN, BK, WM, WN, BL)                   \
  add_instance<DT, BM, BN, BK, WM, WN, 3, 2, 1, BL, 0, 0, 0, 1>(T);      \
  add_instance<DT, BM, BN, BK, WM, WN, 4, 2, 1, BL, 0, 0, 0, 1>(T);
void register_pf(std::vector<KernelEntry>& t)
{
  ALCOP_PF_PIPES(t, 0, 128, 128, 64, 64, 64, 0)
  ALCOP_PF_PIPES(t, 0, 128, 128, 32, 64, 64, 0)
  ALCOP_PF_PIPES(t, 0, 256, 256, 32, 128, 64, 0)
  ALCOP_PF_PIPES(t, 0, 64, 64, 32, 32, 32, 0)
  ALCOP_PF_PIPES(t, 1, 128, 128, 64, 64, 64, 0)
  ALCOP_PF_PIPES(t, 1, 256, 256, 32, 128, 64, 0)
  ALCOP_PF_PIPES(t, 0, 128, 128, 64, 64, 64, 1)
}
}  // namespace alcop

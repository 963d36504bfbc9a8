// k-tile of 128: half as many block-wide synchronisations per unit of work; two stages of a
// 128 x 128 tile fill 128 KB of LDS.
#include "alcop_instantiate.hip.h"
namespace alcop {
#define BK128_PIPES(T, DT, BM, BN, WM, WN, BL)                    \
  add_instance<DT, BM, BN, 128, WM, WN, 1, 1, 0, BL, 0>(T);        \
  add_instance<DT, BM, BN, 128, WM, WN, 2, 1, 0, BL, 0>(T);        \
  add_instance<DT, BM, BN, 128, WM, WN, 2, 2, 0, BL, 0>(T);        \
  add_instance<DT, BM, BN, 128, WM, WN, 2, 2, 1, BL, 0>(T);        \
  add_instance<DT, BM, BN, 128, WM, WN, 3, 2, 1, BL, 0>(T);        \
  add_instance<DT, BM, BN, 128, WM, WN, 4, 2, 1, BL, 0>(T);
void register_bk128(std::vector<KernelEntry>& t)
{
  BK128_PIPES(t, 0, 128, 128, 64, 64, 0)
  BK128_PIPES(t, 0, 128, 64, 64, 32, 0)
  BK128_PIPES(t, 0, 64, 64, 32, 32, 0)
  BK128_PIPES(t, 1, 128, 128, 64, 64, 0)
  BK128_PIPES(t, 1, 64, 64, 32, 32, 0)
  BK128_PIPES(t, 0, 128, 128, 64, 64, 1)
  BK128_PIPES(t, 0, 64, 64, 32, 32, 1)
  BK128_PIPES(t, 1, 128, 128, 64, 64, 1)
}
}  // namespace alcop

// Register pipelines deeper than two stages (R = 3, 4; fused only): R - 1 fragments are being
// read from LDS ahead of the one the matrix cores consume.
#include "alcop_instantiate.hip.h"
namespace alcop {
#define ALCOP_DEEP_PIPES(T, DT, BM, BN, BK, WM, WN, BL, AM)      \
  add_instance<DT, BM, BN, BK, WM, WN, 2, 3, 1, BL, AM>(T);       \
  add_instance<DT, BM, BN, BK, WM, WN, 3, 3, 1, BL, AM>(T);       \
  add_instance<DT, BM, BN, BK, WM, WN, 4, 3, 1, BL, AM>(T);       \
  add_instance<DT, BM, BN, BK, WM, WN, 2, 4, 1, BL, AM>(T);       \
  add_instance<DT, BM, BN, BK, WM, WN, 3, 4, 1, BL, AM>(T);       \
  add_instance<DT, BM, BN, BK, WM, WN, 4, 4, 1, BL, AM>(T);
void register_deep(std::vector<KernelEntry>& t)
{
  ALCOP_BOTH_BK(ALCOP_DEEP_PIPES, t, 0, 128, 128, 64, 64, 0, 0)
  ALCOP_BOTH_BK(ALCOP_DEEP_PIPES, t, 0, 256, 256, 128, 128, 0, 0)
  ALCOP_BOTH_BK(ALCOP_DEEP_PIPES, t, 0, 256, 256, 128, 64, 0, 0)
  ALCOP_BOTH_BK(ALCOP_DEEP_PIPES, t, 0, 256, 128, 128, 64, 0, 0)
  ALCOP_BOTH_BK(ALCOP_DEEP_PIPES, t, 0, 64, 64, 32, 32, 0, 0)
  ALCOP_BOTH_BK(ALCOP_DEEP_PIPES, t, 1, 128, 128, 64, 64, 0, 0)
  ALCOP_BOTH_BK(ALCOP_DEEP_PIPES, t, 1, 256, 256, 128, 128, 0, 0)
  ALCOP_BOTH_BK(ALCOP_DEEP_PIPES, t, 1, 256, 256, 128, 64, 0, 0)
  ALCOP_BOTH_BK(ALCOP_DEEP_PIPES, t, 0, 128, 128, 64, 64, 1, 0)
}
}  // namespace alcop

// A stored K x M (transA): both operands can use the transposing LDS read when B is K x N.
#include "alcop_instantiate.hip.h"
namespace alcop {
#define TA_BOTH_BK(T, DT, BM, BN, WM, WN, BL)       \
  ALCOP_KEY_PIPES_TA(T, DT, BM, BN, 32, WM, WN, BL) \
  ALCOP_KEY_PIPES_TA(T, DT, BM, BN, 64, WM, WN, BL)
void register_ta(std::vector<KernelEntry>& t)
{
  // fp16 / bf16, B stored K x N
  TA_BOTH_BK(t, 0, 256, 256, 128, 128, 0)
  TA_BOTH_BK(t, 0, 256, 256, 128, 64, 0)
  TA_BOTH_BK(t, 0, 128, 128, 64, 64, 0)
  TA_BOTH_BK(t, 0, 64, 64, 32, 32, 0)
  TA_BOTH_BK(t, 1, 256, 256, 128, 64, 0)
  TA_BOTH_BK(t, 1, 128, 128, 64, 64, 0)
  TA_BOTH_BK(t, 1, 64, 64, 32, 32, 0)
  // B stored N x K
  TA_BOTH_BK(t, 0, 256, 256, 128, 64, 1)
  TA_BOTH_BK(t, 0, 128, 128, 64, 64, 1)
  TA_BOTH_BK(t, 0, 64, 64, 32, 32, 1)
  TA_BOTH_BK(t, 1, 128, 128, 64, 64, 1)
}
}  // namespace alcop

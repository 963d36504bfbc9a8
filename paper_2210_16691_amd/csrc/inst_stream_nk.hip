// Persistent producer / consumer kernels: fp16 with B stored N x K (Q.K^T), bf16, and the tiles 192
// wide along n.
#include "alcop_instantiate_stream.hip.h"
namespace alcop {
void register_stream_nk(std::vector<KernelEntry>& t)
{
  // fp16, B stored N x K
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 128, 128, 64, 64, 1, 0)
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 128, 64, 64, 32, 1, 0)
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 64, 64, 32, 32, 1, 0)
  ALCOP_STREAM_DEEP(t, 0, 128, 128, 64, 64, 1, 0)
  // bf16
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 1, 128, 128, 64, 64, 0, 0)
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 1, 64, 64, 32, 32, 0, 0)
  ALCOP_STREAM_DEEP(t, 1, 128, 128, 64, 64, 0, 0)
  // tiles 192 wide along n (three 64-column LDS images; one producer load per image needs bk = 32)
  ALCOP_STREAM_STAGES(t, 1, 128, 192, 32, 64, 96, 0, 0)
  ALCOP_STREAM_STAGES(t, 0, 128, 192, 32, 64, 96, 0, 0)
}
}  // namespace alcop

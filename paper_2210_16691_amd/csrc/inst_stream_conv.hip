// Persistent producer / consumer kernels: the convolution gather with one filter tap per k-tile,
// RSCK weights.
#include "alcop_instantiate_stream.hip.h"
namespace alcop {
void register_stream_conv(std::vector<KernelEntry>& t)
{
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 128, 64, 64, 32, 0, 1)
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 64, 64, 32, 32, 0, 1)
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 256, 64, 64, 64, 0, 1)
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 128, 128, 64, 64, 0, 1)
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 64, 128, 32, 64, 0, 1)
  ALCOP_STREAM_DEEP(t, 0, 64, 128, 32, 64, 0, 1)
}
}  // namespace alcop

// Persistent producer / consumer kernels (schedule variant 2): tiles with four consumer waves,
// two to four ring stages.  This shard: fp16 with B stored K x N; the other layouts, bf16, the
// wide tiles and the convolution gather are in inst_stream_nk.hip and inst_stream_conv.hip.
#include "alcop_instantiate_stream.hip.h"
namespace alcop {
void register_stream_nk(std::vector<KernelEntry>& t);
void register_stream_conv(std::vector<KernelEntry>& t);
void register_stream(std::vector<KernelEntry>& t)
{
  // fp16, B stored K x N
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 128, 128, 64, 64, 0, 0)
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 128, 64, 64, 32, 0, 0)
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 64, 64, 32, 32, 0, 0)
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 256, 64, 64, 64, 0, 0)
  ALCOP_STREAM_DEEP(t, 0, 128, 128, 64, 64, 0, 0)
  ALCOP_STREAM_DEEP(t, 0, 128, 64, 64, 32, 0, 0)
  register_stream_nk(t);
  register_stream_conv(t);
}
}  // namespace alcop

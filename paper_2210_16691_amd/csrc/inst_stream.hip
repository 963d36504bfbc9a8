// Persistent producer / consumer kernels (schedule variant 2): tiles with four consumer waves,
// two to four ring stages; fp16 and bf16; matrix operands in both layouts of B, and the
// convolution gather with one filter tap per k-tile.
#include "alcop_instantiate_stream.hip.h"
namespace alcop {
// every ring depth, the consumers' register pipeline fused across k-tiles and not
#define ALCOP_STREAM_STAGES(T, DT, BM, BN, BK, WM, WN, BL, AM)   \
  add_stream<DT, BM, BN, BK, WM, WN, 2, BL, AM, 0, 1>(T);        \
  add_stream<DT, BM, BN, BK, WM, WN, 3, BL, AM, 0, 1>(T);        \
  add_stream<DT, BM, BN, BK, WM, WN, 4, BL, AM, 0, 1>(T);        \
  add_stream<DT, BM, BN, BK, WM, WN, 2, BL, AM, 0, 0>(T);        \
  add_stream<DT, BM, BN, BK, WM, WN, 3, BL, AM, 0, 0>(T);        \
  add_stream<DT, BM, BN, BK, WM, WN, 4, BL, AM, 0, 0>(T);
// the consumers' deep register pipeline (k-tile 64): measured no faster than the two above on any
// configuration, so these stay outside the default schedule space (alcop_sched_variants)
#define ALCOP_STREAM_DEEP(T, DT, BM, BN, WM, WN, BL, AM)         \
  add_stream<DT, BM, BN, 64, WM, WN, 2, BL, AM, 0, 2>(T);        \
  add_stream<DT, BM, BN, 64, WM, WN, 3, BL, AM, 0, 2>(T);
void register_stream(std::vector<KernelEntry>& t)
{
  // fp16, B stored K x N
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 128, 128, 64, 64, 0, 0)
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 128, 64, 64, 32, 0, 0)
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 64, 64, 32, 32, 0, 0)
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 256, 64, 64, 64, 0, 0)
  // fp16, B stored N x K (Q.K^T)
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 128, 128, 64, 64, 1, 0)
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 128, 64, 64, 32, 1, 0)
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 64, 64, 32, 32, 1, 0)
  // bf16
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 1, 128, 128, 64, 64, 0, 0)
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 1, 64, 64, 32, 32, 0, 0)
  ALCOP_STREAM_DEEP(t, 0, 128, 128, 64, 64, 0, 0)
  ALCOP_STREAM_DEEP(t, 0, 128, 64, 64, 32, 0, 0)
  ALCOP_STREAM_DEEP(t, 0, 128, 128, 64, 64, 1, 0)
  ALCOP_STREAM_DEEP(t, 1, 128, 128, 64, 64, 0, 0)
  ALCOP_STREAM_DEEP(t, 0, 64, 128, 32, 64, 0, 1)
  // tiles 192 wide along n (three 64-column LDS images; one producer load per image needs bk = 32)
  ALCOP_STREAM_STAGES(t, 1, 128, 192, 32, 64, 96, 0, 0)
  ALCOP_STREAM_STAGES(t, 0, 128, 192, 32, 64, 96, 0, 0)
  // convolution gather, RSCK weights
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 128, 64, 64, 32, 0, 1)
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 64, 64, 32, 32, 0, 1)
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 256, 64, 64, 64, 0, 1)
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 128, 128, 64, 64, 0, 1)
  ALCOP_BOTH_BK(ALCOP_STREAM_STAGES, t, 0, 64, 128, 32, 64, 0, 1)
}
}  // namespace alcop

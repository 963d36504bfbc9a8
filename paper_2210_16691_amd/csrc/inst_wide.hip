// Tiles 192 wide along n (three 64-column LDS images, alcop_kernel.hip.h): 4096 x 3072 outputs
// split into exactly 256 tiles of 256 x 192, one per compute unit, at 0.6 of the L2 -> LDS bytes
// per flop of a 128 x 128 tile.
#include "alcop_instantiate.hip.h"
namespace alcop {
void register_wide(std::vector<KernelEntry>& t)
{
  // 4 waves of 128 x 96 (k-tile 32) and 8 waves of 64 x 96 (k-tile 64): one block-wide load per image
  ALCOP_KEY_PIPES(t, 1, 256, 192, 32, 128, 96, 0, 0)
  ALCOP_KEY_PIPES(t, 0, 256, 192, 32, 128, 96, 0, 0)
  ALCOP_KEY_PIPES(t, 1, 256, 192, 64, 64, 96, 0, 0)
  ALCOP_KEY_PIPES(t, 0, 256, 192, 64, 64, 96, 0, 0)
  add_instance<1, 256, 192, 32, 128, 96, 3, 3, 1, 0, 0>(t);
  add_instance<1, 256, 192, 32, 128, 96, 4, 3, 1, 0, 0>(t);
  // 128 x 192 with 4 waves of 64 x 96: the tile of the persistent kernels of this width
  ALCOP_KEY_PIPES(t, 1, 128, 192, 32, 64, 96, 0, 0)
  ALCOP_KEY_PIPES(t, 0, 128, 192, 32, 64, 96, 0, 0)
  // B stored N x K: plain rows
  ALCOP_KEY_PIPES(t, 1, 256, 192, 32, 128, 96, 1, 0)
  ALCOP_KEY_PIPES(t, 0, 256, 192, 32, 128, 96, 1, 0)
}
}  // namespace alcop

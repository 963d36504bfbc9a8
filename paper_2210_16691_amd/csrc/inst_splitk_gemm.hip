// Split-K variants for GEMM / batched matmul (A stored M x K or K x M; B stored K x N or N x K), and the
// launcher of the reduction step.
#include "alcop_instantiate.hip.h"
namespace alcop {
void register_splitk_gemm(std::vector<KernelEntry>& t)
{
  ALCOP_SPLITK_PIPES(t, 0, 128, 128, 64, 64, 64, 0, 0)
  ALCOP_SPLITK_PIPES(t, 0, 128, 64, 64, 64, 32, 0, 0)
  ALCOP_SPLITK_PIPES(t, 0, 64, 64, 64, 32, 32, 0, 0)
  ALCOP_SPLITK_PIPES(t, 0, 256, 128, 64, 128, 64, 0, 0)
  ALCOP_SPLITK_PIPES(t, 1, 128, 128, 64, 64, 64, 0, 0)
  ALCOP_SPLITK_PIPES(t, 1, 64, 64, 64, 32, 32, 0, 0)
  ALCOP_SPLITK_PIPES(t, 1, 256, 128, 64, 128, 64, 0, 0)
  ALCOP_SPLITK_PIPES(t, 0, 128, 128, 64, 64, 64, 1, 0)
  ALCOP_SPLITK_PIPES(t, 0, 64, 64, 64, 32, 32, 1, 0)
  ALCOP_SPLITK_PIPES(t, 1, 128, 128, 64, 64, 64, 1, 0)
  // A stored K x M, B stored K x N
  ALCOP_SPLITK_PIPES_TA(t, 0, 128, 128, 64, 64, 64, 0)
  ALCOP_SPLITK_PIPES_TA(t, 0, 64, 64, 64, 32, 32, 0)
  ALCOP_SPLITK_PIPES_TA(t, 1, 128, 128, 64, 64, 64, 0)
  ALCOP_SPLITK_PIPES_TA(t, 1, 64, 64, 64, 32, 32, 0)
}

hipError_t launch_splitk_reduce(const ReduceParams& p, dim3 grid, hipStream_t st)
{
  alcop_splitk_reduce<Gfx950><<<grid, dim3(REDUCE_THREADS), 0, st>>>(p);
  return hipGetLastError();
}
}  // namespace alcop

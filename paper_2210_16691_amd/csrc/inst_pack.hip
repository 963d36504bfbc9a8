// Launchers of the pack / unpack kernels behind the entry points for unaligned operands.
#include "alcop_gfx950.hip.h"
#include "alcop_registry.h"
namespace alcop {

hipError_t launch_pack(const PackParams& p, int batch, hipStream_t st)
{
  const long threads = (long)p.rows_d * (p.cols_d / (16 / p.esize));
  const dim3 grid((unsigned)((threads + PACK_THREADS - 1) / PACK_THREADS), (unsigned)batch, 1);
  alcop_pack<Gfx950><<<grid, dim3(PACK_THREADS), 0, st>>>(p);
  return hipGetLastError();
}

hipError_t launch_unpack(const PackParams& p, int batch, hipStream_t st)
{
  const long threads = (long)p.rows * (p.cols_d / (16 / p.esize));
  const dim3 grid((unsigned)((threads + PACK_THREADS - 1) / PACK_THREADS), (unsigned)batch, 1);
  alcop_unpack<Gfx950><<<grid, dim3(PACK_THREADS), 0, st>>>(p);
  return hipGetLastError();
}

}  // namespace alcop

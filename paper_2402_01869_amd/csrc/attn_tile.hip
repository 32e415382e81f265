// Tile kernel: recomputation spans on the matrix cores (see tile_body.h).
#include "tile_body.h"

namespace ic {

namespace {

using namespace tilep;

template <int D>
__global__ __launch_bounds__(TW<D>::kThreads, (D <= 128 ? 2 : 1)) void tile_attn_kernel(AttnParams p) {
  __shared__ __attribute__((aligned(16))) uint16_t lds[tile_lds_bytes<D>() / 2];
  const int H = p.num_heads;
  const uint32_t wg = blockIdx.x;
  const int item_idx = wg / H;
  const int head = wg - item_idx * H;
  const TileItem it = p.tile_items[item_idx];
  tile_body<D>(p, it, head, lds);
}

}  // namespace

hipError_t launch_tile_kernel(const AttnParams& p, int head_dim, hipStream_t st) {
  if (p.n_tile_items <= 0) return hipSuccess;
  const uint64_t grid = (uint64_t)p.n_tile_items * p.num_heads;
  if (grid > 0x7fffffffull) return hipErrorInvalidValue;
  const dim3 g((uint32_t)grid);
  switch (head_dim) {
    case 64: hipLaunchKernelGGL(tile_attn_kernel<64>, g, dim3(TW<64>::kThreads), 0, st, p); break;
    case 128: hipLaunchKernelGGL(tile_attn_kernel<128>, g, dim3(TW<128>::kThreads), 0, st, p); break;
    case 256: hipLaunchKernelGGL(tile_attn_kernel<256>, g, dim3(TW<256>::kThreads), 0, st, p); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace ic

// Fused mixed-batch kernel: decode rows and span tiles of one iteration in ONE launch.
//
// Section 4.2 batches decoding with recomputation because the two are complementary: decode rows
// are bound by HBM reads, span tiles by the matrix cores and the vector ALU.  Two separate
// launches cannot exploit that (measured: the hardware dispatcher lets whichever kernel fits
// first crowd out the other and the pair runs no faster than back to back), so this kernel gives
// every workgroup the same footprint (256 threads, the tile path's registers and LDS, two
// workgroups per CU; head_dim 256 needs the whole register file for one tile workgroup and keeps
// the two single-role kernels) and keeps exactly that many workgroups resident.  They
// pull work from queues with atomic counters:
//   - one tile queue per XCD (L2 domain).  Workgroups are dealt round-robin to the 8 XCDs by block
//     index, so XCD x = index % 8 owns the tile items of the heads h = x (mod 8), in head-major
//     order: the query tiles of one (sequence, head), which read the same keys, run on one L2 at
//     the same time, and rocprof shows the fused kernel fetching each span's keys about once;
//   - one global row queue.
// Half of the workgroups prefer tiles and half prefer rows; each switches to the other kind when
// its own queue runs dry, so every CU keeps both kinds of work for as long as both exist and
// nothing idles at the end.  Measured on MI355X: four row-path waves per CU already saturate HBM,
// which leaves the other half of each CU to the tile path.
#include "row_body.h"
#include "tile_body.h"

#ifndef IC_FUSED_PF
#define IC_FUSED_PF 1  // row-role tiles prefetched ahead inside the fused kernel
#endif

#ifdef IC_TRACE2
extern "C" int ic_debug_dump_phase(long long* host) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(ic::tilep::g_phase), 64, 0, hipMemcpyDeviceToHost);
}
#endif
#ifdef IC_TRACE
// Debug build only: per-workgroup log of (kind, start, end) in 100 MHz ticks.
__device__ long long g_trace[512 * 128 * 3];
extern "C" int ic_debug_dump_trace(long long* host, size_t bytes) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_trace), bytes, 0, hipMemcpyDeviceToHost);
}
#endif

namespace ic {

namespace {

template <int D>
constexpr int fused_lds_bytes() {
  return tilep::tile_lds_bytes<D>() > rowp::row_lds_bytes<D>() ? tilep::tile_lds_bytes<D>()
                                                               : rowp::row_lds_bytes<D>();
}

// counters: [0..7] next tile of XCD x, [8] next row item; zeroed by the descriptor upload.
template <int D, int PF>
__global__ __launch_bounds__(256, 2) void fused_persist_kernel(AttnParams p) {
  static_assert(D <= 128, "head_dim 256 does not fit two workgroups per CU: it uses the two single-role kernels");
  __shared__ __attribute__((aligned(16))) uint16_t lds[fused_lds_bytes<D>() / 2];
  __shared__ int s_next;
  const int H = p.num_heads;
  const uint32_t x = blockIdx.x & 7u, j = blockIdx.x >> 3;
  const uint32_t heads_x = (uint32_t)(H - (int)x + 7) / 8u;
  const uint32_t n_t = (uint32_t)p.n_tile_items * heads_x;
  const uint32_t n_r = (uint32_t)p.n_row_items * (uint32_t)H;
  int* ctr = p.counters;
  const bool prefer_tile = j >= (gridDim.x >> 4);  // second half of every XCD's workgroups
  bool tile_done = n_t == 0, row_done = n_r == 0;
#ifdef IC_TRACE
  int n_ev = 0;
#endif
  while (!(tile_done && row_done)) {
#ifdef IC_TRACE
    const long long t_begin = wall_clock64();
#endif
    const bool do_tile = tile_done ? false : (row_done ? true : prefer_tile);
    if (threadIdx.x == 0) s_next = atomicAdd(do_tile ? &ctr[x] : &ctr[8], 1);
    __syncthreads();
    const uint32_t idx = (uint32_t)s_next;
    __syncthreads();  // s_next is rewritten at the top of the next round
    if (do_tile) {
      if (idx >= n_t) { tile_done = true; continue; }
      const uint32_t hsel = idx / (uint32_t)p.n_tile_items;
      const uint32_t item = idx - hsel * (uint32_t)p.n_tile_items;
      const TileItem it = p.tile_items[item];
      tilep::tile_body<D>(p, it, (int)(x + 8u * hsel), lds);
    } else {
      if (idx >= n_r) { row_done = true; continue; }
      const uint32_t item = idx / (uint32_t)H;
      const RowItem it = p.row_items[item];
      rowp::row_body<D, PF, true>(p, it, (int)(idx - item * (uint32_t)H), (float*)lds);
    }
    __syncthreads();  // the bodies leave LDS in use until every wave is through
#ifdef IC_TRACE
    if (threadIdx.x == 0 && n_ev < 127) {
      long long* e = g_trace + ((size_t)blockIdx.x * 128 + n_ev) * 3;
      e[0] = do_tile ? 1 : 2; e[1] = t_begin; e[2] = wall_clock64();
      ++n_ev;
    }
#endif
  }
#ifdef IC_TRACE
  if (threadIdx.x == 0) { long long* e = g_trace + ((size_t)blockIdx.x * 128 + n_ev) * 3; e[0] = 0; e[1] = 0; e[2] = 0; }
#endif
}

}  // namespace

hipError_t launch_fused_kernel(const AttnParams& p, int head_dim, hipStream_t st) {
  if (p.n_tile_items <= 0 || p.n_row_items <= 0 || !p.counters) return hipErrorInvalidValue;
  const int slots = p.persist_slots - p.persist_slots % 16;  // a whole number of pairs per XCD
  if (slots < 16) return hipErrorInvalidValue;
  const dim3 g((uint32_t)slots), b(256);
  switch (head_dim) {
    case 64: hipLaunchKernelGGL((fused_persist_kernel<64, IC_FUSED_PF>), g, b, 0, st, p); break;
    case 128: hipLaunchKernelGGL((fused_persist_kernel<128, IC_FUSED_PF>), g, b, 0, st, p); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace ic

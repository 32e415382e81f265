// Tile kernels: recomputation spans on the matrix cores.  head_dim <= 128: 32 query rows per wave (tile_body.h);
// head_dim 256: 16 rows per wave (tile16_body.h).  Either way a workgroup is 8 waves, two per SIMD.
#include "tile_body.h"
#include "tile16_body.h"

namespace ic {

namespace {

using namespace tilep;

// What a workgroup of the tile kernels is for head_dim D.
template <int D, bool k16 = (D > 128)>
struct Impl {
  static constexpr int kThreads = TW<D>::kThreads;
  static constexpr int kLdsBytes = tile_lds_bytes<D>();
  template <bool kAlone>
  static __device__ __forceinline__ void body(const AttnParams& p, const TileItem& it, int th, uint16_t* lds) {
    tile_body<D>(p, it, th, lds);
  }
};
template <int D>
struct Impl<D, true> {
  static constexpr int kThreads = tile16::G16<D>::kThreads;
  static constexpr int kLdsBytes = tile16::tile16_lds_bytes<D>();
  template <bool kAlone>  // a kernel with its SIMDs to itself has registers for the pinned operand prefetch
  static __device__ __forceinline__ void body(const AttnParams& p, const TileItem& it, int th, uint16_t* lds) {
    tile16::tile16_body<D, kAlone>(p, it, th, lds);
  }
};

template <int D>
__global__ __launch_bounds__(Impl<D>::kThreads, 2) void tile_attn_kernel(AttnParams p) {
  __shared__ __attribute__((aligned(16))) uint16_t lds[Impl<D>::kLdsBytes / 2];
  const int n_th = p.num_heads >> p.tile_g_shift;  // head groups, each served by one workgroup per item
  const uint32_t wg = blockIdx.x;
  const int item_idx = wg / n_th;
  const int th = wg - item_idx * n_th;
  const TileItem it = p.tile_items[item_idx];
  Impl<D>::template body<true>(p, it, th, lds);
}

// Persistent launch of the same body, for running beside the row kernel: `slots` workgroups (one
// per CU; two do not fit) pull tile items from one queue per XCD with atomic counters
// (counters[0..7], zeroed by the descriptor upload).  Workgroups are dealt round-robin to the 8 XCDs
// (L2 domains) by block index, so XCD x = index % 8 owns the tile items of the heads h = x (mod 8),
// in head-major order: the query tiles of one (sequence, head), which read the same keys, run on
// one L2 at the same time, and each span's keys are fetched from HBM about once.
// Register budget: at most 216 per lane for head_dim <= 128, 208 for head_dim 256 (checked by the test-suite
// from the compiler's resource report).  Two waves of this kernel and one of the slim row kernel (80, head_dim
// 256: 96) or of the slim group kernel (96) fill the 512 of a SIMD, which is what lets one workgroup of each
// share a CU.
// kBeside only names the build (side by side with a row or group kernel, or on its own), so that a kernel trace
// tells the two uses apart; the code is the same.
// amdgpu_num_vgpr: on this target vector and accumulation registers share one file and the compiler doubles the
// figure it is given, so 104 caps the kernel at 208 registers (launch bounds alone would allow 256).
template <int D, bool kBeside>
__global__ __launch_bounds__(Impl<D>::kThreads, 2) __attribute__((amdgpu_num_vgpr(104))) void tile_persist_kernel(AttnParams p) {
  __shared__ __attribute__((aligned(16))) uint16_t lds[Impl<D>::kLdsBytes / 2];
  __shared__ int s_next;
  if (p.tile_first) __builtin_amdgcn_s_setprio(3);
  const int H = p.num_heads >> p.tile_g_shift;               // head groups
  const bool per_xcd = H >= 8;   // with fewer head groups than XCDs, one shared queue instead
  const uint32_t x = blockIdx.x & 7u;
  const uint32_t heads_x = (uint32_t)(H - (int)x + 7) / 8u;  // head groups congruent to x mod 8
  const uint32_t n_t = (uint32_t)p.n_tile_items * (per_xcd ? heads_x : (uint32_t)H);
  for (;;) {
    if (threadIdx.x == 0) s_next = atomicAdd(&p.counters[per_xcd ? x : (uint32_t)kCtrTileShared], 1);
    __syncthreads();
    const uint32_t idx = (uint32_t)s_next;
    __syncthreads();  // s_next is rewritten at the top of the next round
    if (idx >= n_t) break;
    uint32_t item, th;
    if (per_xcd) {
      const uint32_t hsel = idx / (uint32_t)p.n_tile_items;
      item = idx - hsel * (uint32_t)p.n_tile_items;
      th = x + 8u * hsel;
    } else {
      item = idx / (uint32_t)H;
      th = idx - item * (uint32_t)H;
    }
    const TileItem it = p.tile_items[item];
    Impl<D>::template body<false>(p, it, (int)th, lds);
    __syncthreads();  // the body leaves LDS in use until every wave is through
  }
  queue_leave(p.counters, 0, 8, kCtrTileShared, kCtrTileLeft);
}

}  // namespace

hipError_t launch_tile_kernel(const AttnParams& p, int head_dim, hipStream_t st) {
  if (p.n_tile_items <= 0) return hipSuccess;
  const uint64_t grid = (uint64_t)p.n_tile_items * (uint64_t)(p.num_heads >> p.tile_g_shift);
  if (grid > 0x7fffffffull) return hipErrorInvalidValue;
  const dim3 g((uint32_t)grid);
  switch (head_dim) {
    case 64: hipLaunchKernelGGL(tile_attn_kernel<64>, g, dim3(Impl<64>::kThreads), 0, st, p); break;
    case 128: hipLaunchKernelGGL(tile_attn_kernel<128>, g, dim3(Impl<128>::kThreads), 0, st, p); break;
    case 256: hipLaunchKernelGGL(tile_attn_kernel<256>, g, dim3(Impl<256>::kThreads), 0, st, p); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// slots is rounded down to a multiple of 8 so that every XCD gets the same number of workgroups.
hipError_t launch_tile_persist(const AttnParams& p, int head_dim, int slots, bool beside, hipStream_t st) {
  if (p.n_tile_items <= 0) return hipSuccess;
  if (!p.counters || slots < 8) return hipErrorInvalidValue;
  const dim3 g((uint32_t)(slots - slots % 8));
#define IC_TILE_CASE(DD)                                                                                          \
  case DD:                                                                                                        \
    if (beside) hipLaunchKernelGGL((tile_persist_kernel<DD, true>), g, dim3(Impl<DD>::kThreads), 0, st, p);        \
    else hipLaunchKernelGGL((tile_persist_kernel<DD, false>), g, dim3(Impl<DD>::kThreads), 0, st, p);              \
    break;
  switch (head_dim) {
    IC_TILE_CASE(64)
    IC_TILE_CASE(128)
    IC_TILE_CASE(256)
    default: return hipErrorInvalidValue;
  }
#undef IC_TILE_CASE
  return hipGetLastError();
}

}  // namespace ic

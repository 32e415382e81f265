// Row kernel (decode rows, and spans row by row when asked) and the split-KV merge.
#include "row_body.h"

namespace ic {

namespace {

using namespace rowp;

template <int D, int PF, bool NT>
__global__ __launch_bounds__(kRowWaves * 64) void row_attn_kernel(AttnParams p) {
  __shared__ __attribute__((aligned(16))) float lds[row_lds_bytes<D>() / sizeof(float)];
  const int H = p.num_heads;
  const uint32_t wg = blockIdx.x;
  const int item_idx = wg / H;
  const int head = wg - item_idx * H;
  const RowItem it = p.row_items[item_idx];
  row_body<D, PF, NT>(p, it, head, lds);
}

// Persistent launch of the same body: `slots` workgroups (one per CU) pull (item, head) pairs from a
// queue with an atomic counter (counters[8], zeroed by the descriptor upload).  Measured on MI355X:
// 256 resident workgroups read 6.65 TB/s, 4 % more than one workgroup per work item, because no
// workgroup launch or drain sits between two items.
template <int D, int PF>
__global__ __launch_bounds__(kRowWaves * 64) void row_persist_kernel(AttnParams p) {
  __shared__ __attribute__((aligned(16))) float lds[row_lds_bytes<D>() / sizeof(float)];
  __shared__ int s_next;
  const int H = p.num_heads;
  const uint32_t n_r = (uint32_t)p.n_vec_items * (uint32_t)H;
  for (;;) {
    if (threadIdx.x == 0) s_next = atomicAdd(&p.counters[8], 1);
    __syncthreads();
    const uint32_t idx = (uint32_t)s_next;
    __syncthreads();  // s_next is rewritten at the top of the next round
    if (idx >= n_r) break;
    const uint32_t item = idx / (uint32_t)H;  // head fastest: neighbours read adjacent tiles of a block
    const RowItem it = p.row_items[item];
    row_body<D, PF, true>(p, it, (int)(idx - item * (uint32_t)H), lds);
    __syncthreads();  // the body leaves LDS in use until every wave is through
  }
  queue_leave(p.counters, kCtrRowQueue, 1, -1, kCtrRowLeft);
}

// Split-KV merge: out = sum_p o_p 2^(m_p - m) / sum_p l_p 2^(m_p - m), m = max_p m_p.
// One workgroup of D threads per (row, head); partials are read coalesced over d.
template <int D>
__global__ __launch_bounds__(D) void merge_kernel(AttnParams p) {
  const int H = p.num_heads;
  const uint32_t wg = blockIdx.x;
  const int mi = wg / H;
  const int head = wg - mi * H;
  const MergeItem it = p.merge_items[mi];
  const int d = threadIdx.x;
  float M = kNegBig;
  for (int k = 0; k < it.nparts; ++k)
    M = __builtin_fmaxf(M, p.part_ml[((int64_t)(it.slot0 + k) * H + head) * 2]);
  float L = 0.f, O = 0.f;
  for (int k = 0; k < it.nparts; ++k) {
    const int64_t ps = (int64_t)(it.slot0 + k) * H + head;
    const float wgt = __builtin_amdgcn_exp2f(p.part_ml[ps * 2] - M);
    L = __builtin_fmaf(p.part_ml[ps * 2 + 1], wgt, L);
    O = __builtin_fmaf(p.part_o[ps * D + d], wgt, O);
  }
  p.out[((int64_t)it.qrow * H + head) * D + d] = (uint16_t)f32_to_bf16(O / L);
}

}  // namespace

hipError_t launch_row_kernel(const AttnParams& p, int head_dim, hipStream_t st) {
  if (p.n_vec_items <= 0) return hipSuccess;
  const uint64_t grid = (uint64_t)p.n_vec_items * p.num_heads;
  if (grid > 0x7fffffffull) return hipErrorInvalidValue;
  const dim3 g((uint32_t)grid), b(kRowWaves * 64);
#define IC_ROW_CASE(DD)                                                                       \
  case DD:                                                                                    \
    switch (p.row_variant & 3) {                                                              \
      case 0: hipLaunchKernelGGL((row_attn_kernel<DD, 1, true>), g, b, 0, st, p); break;       \
      case 1: hipLaunchKernelGGL((row_attn_kernel<DD, 2, true>), g, b, 0, st, p); break;       \
      case 2: hipLaunchKernelGGL((row_attn_kernel<DD, 1, false>), g, b, 0, st, p); break;      \
      default: hipLaunchKernelGGL((row_attn_kernel<DD, 2, false>), g, b, 0, st, p); break;     \
    }                                                                                         \
    break;
  switch (head_dim) {
    IC_ROW_CASE(64)
    IC_ROW_CASE(128)
    IC_ROW_CASE(256)
    default: return hipErrorInvalidValue;
  }
#undef IC_ROW_CASE
  return hipGetLastError();
}

// Slim build of the persistent row kernel for running BESIDE the tile kernel: no register prefetch
// (measured not to matter there: the CU's memory pipe, not the wave, holds the loads in flight)
// and at most 80 VGPRs (head_dim 256: 96, with blocks taken in two halves), so that one of these workgroups fits
// on a CU next to a tile workgroup.
template <int D>
__global__ __launch_bounds__(kRowWaves * 64, (D <= 128 ? 6 : 5)) void row_persist_slim_kernel(AttnParams p) {
  __shared__ __attribute__((aligned(16))) float lds[row_lds_bytes<D>() / sizeof(float)];
  __shared__ int s_next;
  const int H = p.num_heads;
  const uint32_t n_r = (uint32_t)p.n_vec_items * (uint32_t)H;
  for (;;) {
    if (threadIdx.x == 0) s_next = atomicAdd(&p.counters[8], 1);
    __syncthreads();
    const uint32_t idx = (uint32_t)s_next;
    __syncthreads();
    if (idx >= n_r) break;
    const uint32_t item = idx / (uint32_t)H;
    const RowItem it = p.row_items[item];
    row_body<D, 0, true, (D > 128)>(p, it, (int)(idx - item * (uint32_t)H), lds);
    __syncthreads();
  }
  queue_leave(p.counters, kCtrRowQueue, 1, -1, kCtrRowLeft);
}

hipError_t launch_row_persist(const AttnParams& p, int head_dim, int slots, hipStream_t st) {
  if (p.n_vec_items <= 0) return hipSuccess;
  if (!p.counters || slots < 1) return hipErrorInvalidValue;
  const dim3 g((uint32_t)slots), b(kRowWaves * 64);
  switch (head_dim) {
    case 64: hipLaunchKernelGGL((row_persist_kernel<64, 1>), g, b, 0, st, p); break;
    case 128: hipLaunchKernelGGL((row_persist_kernel<128, 1>), g, b, 0, st, p); break;
    case 256: hipLaunchKernelGGL((row_persist_kernel<256, 1>), g, b, 0, st, p); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_row_persist_slim(const AttnParams& p, int head_dim, int slots, hipStream_t st) {
  if (p.n_vec_items <= 0) return hipSuccess;
  if (!p.counters || slots < 1) return hipErrorInvalidValue;
  const dim3 g((uint32_t)slots), b(kRowWaves * 64);
  switch (head_dim) {
    case 64: hipLaunchKernelGGL(row_persist_slim_kernel<64>, g, b, 0, st, p); break;
    case 128: hipLaunchKernelGGL(row_persist_slim_kernel<128>, g, b, 0, st, p); break;
    case 256: hipLaunchKernelGGL(row_persist_slim_kernel<256>, g, b, 0, st, p); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_merge_kernel(const AttnParams& p, int head_dim, hipStream_t st) {
  if (p.n_merge_items <= 0) return hipSuccess;
  const uint64_t grid = (uint64_t)p.n_merge_items * p.num_heads;
  if (grid > 0x7fffffffull) return hipErrorInvalidValue;
  const dim3 g((uint32_t)grid);
  switch (head_dim) {
    case 64: hipLaunchKernelGGL(merge_kernel<64>, g, dim3(64), 0, st, p); break;
    case 128: hipLaunchKernelGGL(merge_kernel<128>, g, dim3(128), 0, st, p); break;
    case 256: hipLaunchKernelGGL(merge_kernel<256>, g, dim3(256), 0, st, p); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace ic

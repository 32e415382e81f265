// Measurement aid, not part of the method: what an MFMA-only loop reaches on this GPU with the caller's operand
// data.  With realistic (random) operands the power limit lowers the shader clock well below the nominal one, so
// this figure, not the vendor peak, is what a perfectly fed matrix pipe could deliver; reports price the tile
// kernel against both.
#include "ic_internal.h"

namespace ic {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kCeilBlocks = 256, kCeilThreads = 512;   // one 8-wave workgroup per CU
constexpr size_t kCeilOperandBytes = 1u << 20;          // 65536 16-byte operands
constexpr size_t kCeilSinkBytes = (size_t)kCeilBlocks * kCeilThreads * 4 + (size_t)kCeilBlocks * 16;

__global__ __launch_bounds__(kCeilThreads, 2) void mfma_ceiling_kernel(const u32x4* operands, float* sink,
                                                                       long long* clocks, int iters) {
  const int tid = threadIdx.x + blockIdx.x * kCeilThreads;
  u32x4 ra = operands[(tid * 2) & 0xffff], rb = operands[(tid * 2 + 1) & 0xffff];
  const bf16x8 a = *(bf16x8*)&ra, b = *(bf16x8*)&rb;
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
  const long long c0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j], 0, 0, 0);
  }
  const long long c1 = clock64(), w1 = wall_clock64();
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[j][i];
  sink[tid] = s;
  if (threadIdx.x == 0) {
    clocks[blockIdx.x * 2] = c1 - c0;       // shader clock ticks
    clocks[blockIdx.x * 2 + 1] = w1 - w0;   // constant 100 MHz ticks
  }
}

// Streaming read (mode 0: every 16-byte chunk of src is loaded once and folded into one word per lane) and plain
// copy (mode 1: src -> dst) by one-wave workgroups, non-temporal loads and stores.  A copy workgroup moves 1 KiB,
// the launch shape of the block gather / scatter kernel without its indirection; a read workgroup takes 8 KiB,
// because one-wave workgroups that only load 1 KiB finish faster than the dispatcher can start them.
constexpr int kReadChunks = 8;

__global__ __launch_bounds__(64) void hbm_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst) {
  const size_t i = (size_t)blockIdx.x * 64 + threadIdx.x;
  __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

__global__ __launch_bounds__(64) void hbm_read_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst) {
  const size_t i = (size_t)blockIdx.x * (64 * kReadChunks) + threadIdx.x;
  u32x4 v[kReadChunks];
#pragma unroll
  for (int c = 0; c < kReadChunks; ++c) v[c] = __builtin_nontemporal_load(src + i + 64 * c);
  u32x4 x = v[0];
#pragma unroll
  for (int c = 1; c < kReadChunks; ++c) x ^= v[c];
  if ((x[0] ^ x[1] ^ x[2] ^ x[3]) == 0x9e3779b9u) dst[0] = x;  // keeps the loads alive; true about once in 2^32
}

// The decode kernels' access pattern with the arithmetic taken out: one one-wave workgroup per (listed block, K/V
// head) loads that head's K tile and V tile (block_size x head_dim bf16 each) and folds them into one word.
template <int LOADS>  // 16-byte loads per lane and tile: tile bytes / 1024
__global__ __launch_bounds__(64) void paged_read_kernel(const char* __restrict__ pool, const int32_t* __restrict__ ids,
                                                        int Hk, size_t tile_bytes, u32x4* __restrict__ sink) {
  const int b = blockIdx.x / Hk, h = blockIdx.x - b * Hk;
  const char* k = pool + (size_t)ids[b] * (2 * (size_t)Hk * tile_bytes) + (size_t)h * tile_bytes + threadIdx.x * 16;
  const char* v = k + (size_t)Hk * tile_bytes;
  u32x4 x = {0u, 0u, 0u, 0u};
  u32x4 a[LOADS], c[LOADS];
#pragma unroll
  for (int i = 0; i < LOADS; ++i) a[i] = __builtin_nontemporal_load((const u32x4*)(k + i * 1024));
#pragma unroll
  for (int i = 0; i < LOADS; ++i) c[i] = __builtin_nontemporal_load((const u32x4*)(v + i * 1024));
#pragma unroll
  for (int i = 0; i < LOADS; ++i) x ^= a[i] ^ c[i];
  if ((x[0] ^ x[1] ^ x[2] ^ x[3]) == 0x9e3779b9u) sink[0] = x;  // keeps the loads alive
}

}  // namespace
}  // namespace ic

extern "C" int ic_paged_read_ceiling(const ic_pool* pool, const int32_t* host_ids, int32_t n, void* dev_sink,
                                     int32_t reps, void* hip_stream, double* gbps) {
  using namespace ic;
  if (!pool || !host_ids || !dev_sink || !gbps) return IC_ENULL;
  const PoolView pv = pool_view(pool);
  if (n < 1 || reps < 1 || reps > 10000 || (uint64_t)n * (uint64_t)pv.cfg.num_kv_heads > 0x7fffffffull) return IC_EINVAL;
  const int rc0 = ic_check_ids(&pv.cfg, host_ids, n, 0);
  if (rc0 != IC_OK) return rc0;
  if ((uintptr_t)dev_sink & 15) return IC_EALIGN;
  hipStream_t st = (hipStream_t)hip_stream;
  int32_t* dev_ids = nullptr;
  if (hipMalloc((void**)&dev_ids, sizeof(int32_t) * (size_t)n) != hipSuccess) return IC_EHIP;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int rc = IC_OK;
  float ms = 0.f;
  if (hipMemcpy(dev_ids, host_ids, sizeof(int32_t) * (size_t)n, hipMemcpyHostToDevice) != hipSuccess ||
      hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess || hipEventRecord(e0, st) != hipSuccess)
    rc = IC_EHIP;
  const int Hk = pv.cfg.num_kv_heads;
  const size_t tile_bytes = (size_t)pv.cfg.block_size * pv.cfg.head_dim * 2;
  const dim3 grid((uint32_t)n * (uint32_t)Hk), block(64);
  for (int r = 0; rc == IC_OK && r < reps; ++r) {
    switch (pv.cfg.head_dim) {
      case 64: hipLaunchKernelGGL(paged_read_kernel<2>, grid, block, 0, st, pv.base, dev_ids, Hk, tile_bytes, (u32x4*)dev_sink); break;
      case 128: hipLaunchKernelGGL(paged_read_kernel<4>, grid, block, 0, st, pv.base, dev_ids, Hk, tile_bytes, (u32x4*)dev_sink); break;
      default: hipLaunchKernelGGL(paged_read_kernel<8>, grid, block, 0, st, pv.base, dev_ids, Hk, tile_bytes, (u32x4*)dev_sink); break;
    }
    if (hipGetLastError() != hipSuccess) rc = IC_EHIP;
  }
  if (rc == IC_OK && (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                      hipEventElapsedTime(&ms, e0, e1) != hipSuccess))
    rc = IC_EHIP;
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  (void)hipFree(dev_ids);
  if (rc != IC_OK) return rc;
  *gbps = ms > 0.f ? (double)n * (double)pv.block_bytes * reps / ((double)ms * 1e-3) / 1e9 : 0.0;
  return IC_OK;
}

extern "C" int ic_hbm_ceiling(const void* dev_src, void* dev_dst, size_t bytes, int32_t mode, int32_t reps,
                              void* hip_stream, double* gbps) {
  using namespace ic;
  if (!dev_src || !dev_dst || !gbps) return IC_ENULL;
  if ((mode != 0 && mode != 1) || reps < 1 || reps > 10000 || bytes < 8192 || bytes % 8192 != 0 ||
      bytes / 1024 > 0x7fffffffull)
    return IC_EINVAL;
  if (((uintptr_t)dev_src | (uintptr_t)dev_dst) & 15) return IC_EALIGN;
  {
    const char* a = (const char*)dev_src;
    const char* b = (const char*)dev_dst;
    const size_t dst_bytes = mode == 1 ? bytes : 16;
    if (a < b + dst_bytes && b < a + bytes) return IC_EINVAL;  // the two ranges overlap
  }
  hipStream_t st = (hipStream_t)hip_stream;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
    if (e0) (void)hipEventDestroy(e0);
    return IC_EHIP;
  }
  const dim3 grid((uint32_t)(bytes / (mode == 1 ? 1024 : 1024 * kReadChunks))), block(64);
  int rc = IC_OK;
  float ms = 0.f;
  if (hipEventRecord(e0, st) != hipSuccess) rc = IC_EHIP;
  for (int r = 0; rc == IC_OK && r < reps; ++r) {
    if (mode == 1)
      hipLaunchKernelGGL(hbm_copy_kernel, grid, block, 0, st, (const u32x4*)dev_src, (u32x4*)dev_dst);
    else
      hipLaunchKernelGGL(hbm_read_kernel, grid, block, 0, st, (const u32x4*)dev_src, (u32x4*)dev_dst);
    if (hipGetLastError() != hipSuccess) rc = IC_EHIP;
  }
  if (rc == IC_OK && (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                      hipEventElapsedTime(&ms, e0, e1) != hipSuccess))
    rc = IC_EHIP;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc != IC_OK) return rc;
  const double moved = (mode == 1 ? 2.0 : 1.0) * (double)bytes * reps;
  *gbps = ms > 0.f ? moved / ((double)ms * 1e-3) / 1e9 : 0.0;
  return IC_OK;
}

extern "C" int ic_mfma_ceiling(const void* dev_operands, size_t operand_bytes, void* dev_sink, size_t sink_bytes,
                               int32_t iters, void* hip_stream, double* tflops, double* shader_ghz) {
  using namespace ic;
  if (!dev_operands || !dev_sink || !tflops || !shader_ghz) return IC_ENULL;
  if (iters <= 0 || iters > (1 << 24)) return IC_EINVAL;
  if (operand_bytes < kCeilOperandBytes || sink_bytes < kCeilSinkBytes) return IC_ESIZE;
  if (((uintptr_t)dev_operands | (uintptr_t)dev_sink) & 15) return IC_EALIGN;
  hipStream_t st = (hipStream_t)hip_stream;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) {
    if (e0) (void)hipEventDestroy(e0);
    return IC_EHIP;
  }
  long long* clocks = (long long*)((char*)dev_sink + (size_t)kCeilBlocks * kCeilThreads * 4);
  int rc = IC_OK;
  float ms = 0.f;
  long long host_clk[2] = {0, 0};
  if (hipEventRecord(e0, st) != hipSuccess) rc = IC_EHIP;
  if (rc == IC_OK) {
    hipLaunchKernelGGL(mfma_ceiling_kernel, dim3(kCeilBlocks), dim3(kCeilThreads), 0, st, (const u32x4*)dev_operands,
                       (float*)dev_sink, clocks, (int)iters);
    if (hipGetLastError() != hipSuccess || hipEventRecord(e1, st) != hipSuccess ||
        hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess ||
        hipMemcpy(host_clk, clocks, sizeof host_clk, hipMemcpyDeviceToHost) != hipSuccess)
      rc = IC_EHIP;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc != IC_OK) return rc;
  const double flops = (double)kCeilBlocks * (kCeilThreads / 64) * (double)iters * 4.0 * 2.0 * 32 * 32 * 16;
  *tflops = ms > 0.f ? flops / ((double)ms * 1e-3) / 1e12 : 0.0;
  *shader_ghz = host_clk[1] > 0 ? (double)host_clk[0] / (double)host_clk[1] * 0.1 : 0.0;
  return IC_OK;
}

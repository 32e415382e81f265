// Gather / scatter of whole KV blocks between the paged pool and a contiguous staging buffer:
// the device half of the swap of Section 3.2 / 4.1, done in one launch for any number of
// scattered blocks instead of one launch per discontinuous region.
//
// Pure byte movement, HBM-bound.  Every lane moves 16 bytes with non-temporal loads and stores;
// the grid is (blocks in the list) x (chunks per block), hundreds of thousands of workgroups.
#include <cstring>
#include <mutex>

#include "ic_internal.h"

namespace ic {

namespace {

// Measured on MI355X: one-wave workgroups moving 1 KiB each beat every larger shape tried
// (more bytes per lane or more waves per group lose 5-35 %): the dispatcher keeps far more
// independent, short-lived waves in flight than any unrolled loop does.
constexpr int kThreads = 64;
constexpr int kUnroll = 1;
constexpr int kChunk = kThreads * 16 * kUnroll;  // 1 KiB per workgroup

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// PACK: staging[i] <- pool[ids[i]];  !PACK: pool[ids[i]] <- staging[i].
template <bool PACK>
__global__ __launch_bounds__(kThreads) void swap_blocks_kernel(char* __restrict__ pool,
                                                               char* __restrict__ staging,
                                                               const int32_t* __restrict__ ids,
                                                               uint32_t block_bytes,
                                                               uint32_t chunks_per_block, uint32_t n_blocks) {
  // Workgroups are dealt to the 8 XCDs round-robin by index.  Within every full group of 8 listed blocks, XCD x
  // (index = x mod 8) takes block 8 g + x whole, so that one block's bytes go through one XCD's L2 and address
  // translation; the last n % 8 blocks are dealt chunk by chunk.
  const uint32_t wg = blockIdx.x;
  const uint32_t group_wgs = 8u * chunks_per_block;
  const uint32_t g = wg / group_wgs, r = wg - g * group_wgs;
  uint32_t i, c;
  if ((g + 1u) * 8u <= n_blocks) {
    i = g * 8u + (r & 7u);
    c = r >> 3;
  } else {
    i = g * 8u + r / chunks_per_block;
    c = r % chunks_per_block;
  }
  const int64_t id = ids[i];
  const char* src;
  char* dst;
  if (PACK) {
    src = pool + id * (int64_t)block_bytes;
    dst = staging + (int64_t)i * block_bytes;
  } else {
    src = staging + (int64_t)i * block_bytes;
    dst = pool + id * (int64_t)block_bytes;
  }
  const uint32_t off0 = c * kChunk + threadIdx.x * 16;
  u32x4 v[kUnroll];
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint32_t off = off0 + u * (kThreads * 16);
    if (off < block_bytes) v[u] = __builtin_nontemporal_load((const u32x4*)(src + off));
  }
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint32_t off = off0 + u * (kThreads * 16);
    if (off < block_bytes) __builtin_nontemporal_store(v[u], (u32x4*)(dst + off));
  }
}

template <bool PACK>
hipError_t launch_swap(char* pool, char* staging, const int32_t* dev_ids, int32_t n,
                       size_t block_bytes, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  const uint32_t chunks = (uint32_t)((block_bytes + kChunk - 1) / kChunk);
  const uint64_t grid = (uint64_t)n * chunks;
  if (grid > 0x7fffffffull || block_bytes > 0xffffffffull) return hipErrorInvalidValue;
  hipLaunchKernelGGL(swap_blocks_kernel<PACK>, dim3((uint32_t)grid), dim3(kThreads), 0, st, pool,
                     staging, dev_ids, (uint32_t)block_bytes, chunks, (uint32_t)n);
  return hipGetLastError();
}

// Descriptor upload: pinned host memory -> device, 16 bytes per lane, read over the host link by
// the kernel itself.  Used instead of a DMA copy so that a call's small descriptor never queues
// behind a bulk transfer on a copy engine (a layer of a swap occupies one for milliseconds) and the
// kernels that follow need no cross-engine synchronisation.
__global__ __launch_bounds__(256) void upload_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src,
                                                     uint32_t n16) {
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (i < n16) dst[i] = __builtin_nontemporal_load(src + i);
}

// KV append: the keys and values a chunk (or a decode token) has just computed for its own positions
// enter the paged cache (Sections 4.2, 4.3).  One lane moves 16 bytes; consecutive lanes read
// consecutive bytes of a row of k_new (then v_new) and write D * 2 contiguous bytes per head into
// the (block, K/V, head) tile at the row's slot.
template <int D>
__global__ __launch_bounds__(kThreads) void kv_append_kernel(char* __restrict__ pool, const char* __restrict__ k_new,
                                                        const char* __restrict__ v_new,
                                                        const int32_t* __restrict__ dst, uint32_t rows,
                                                        uint32_t num_heads) {
  constexpr uint32_t kChunksPerHead = D / 8;                  // 16-byte chunks of one head's vector
  const uint32_t per_plane = num_heads * kChunksPerHead;      // chunks of one row of K (or V)
  const uint64_t idx = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  const uint32_t row = (uint32_t)(idx / (2u * per_plane));
  if (row >= rows) return;
  const uint32_t rem = (uint32_t)(idx - (uint64_t)row * (2u * per_plane));
  const uint32_t kv = rem / per_plane;
  const uint32_t c = rem - kv * per_plane;
  const uint32_t h = c / kChunksPerHead, cc = c % kChunksPerHead;
  const int32_t d = dst[row];
  if (d < 0) return;
  const uint32_t blk = (uint32_t)d / (uint32_t)kBlockSize, slot = (uint32_t)d % (uint32_t)kBlockSize;
  const char* src = (kv ? v_new : k_new) + ((uint64_t)row * per_plane + c) * 16u;
  char* out = pool + ((((uint64_t)blk * 2u + kv) * num_heads + h) * kBlockSize + slot) * (D * 2) + cc * 16u;
  __builtin_nontemporal_store(__builtin_nontemporal_load((const u32x4*)src), (u32x4*)out);
}

}  // namespace

hipError_t launch_append(void* pool, const void* k_new, const void* v_new, const int32_t* dev_dst, int32_t rows,
                         int num_heads, int head_dim, hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  const uint64_t lanes = (uint64_t)rows * 2u * (uint64_t)num_heads * (uint64_t)(head_dim / 8);
  const uint64_t grid = (lanes + kThreads - 1) / kThreads;  // one-wave workgroups, as for the block moves
  if (grid > 0x7fffffffull) return hipErrorInvalidValue;
  const dim3 g((uint32_t)grid), b(kThreads);
  switch (head_dim) {
    case 64: hipLaunchKernelGGL(kv_append_kernel<64>, g, b, 0, st, (char*)pool, (const char*)k_new, (const char*)v_new, dev_dst, (uint32_t)rows, (uint32_t)num_heads); break;
    case 128: hipLaunchKernelGGL(kv_append_kernel<128>, g, b, 0, st, (char*)pool, (const char*)k_new, (const char*)v_new, dev_dst, (uint32_t)rows, (uint32_t)num_heads); break;
    case 256: hipLaunchKernelGGL(kv_append_kernel<256>, g, b, 0, st, (char*)pool, (const char*)k_new, (const char*)v_new, dev_dst, (uint32_t)rows, (uint32_t)num_heads); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_upload(void* dev_dst, const void* pinned_src, size_t bytes, hipStream_t st) {
  if (bytes == 0) return hipSuccess;
  if ((bytes & 15u) || bytes > ((size_t)1 << 31)) return hipErrorInvalidValue;
  const uint32_t n16 = (uint32_t)(bytes / 16);
  hipLaunchKernelGGL(upload_kernel, dim3((n16 + 255u) / 256u), dim3(256), 0, st, (u32x4*)dev_dst,
                     (const u32x4*)pinned_src, n16);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// kv_pack_blocks for callers that cannot allocate: the device-side id list, which kv_pack_blocks
// keeps in a buffer the library allocates, lives in a fixed array of this library's image instead,
// and the ids travel to it as kernel arguments, so that the call needs no pinned host buffer either.
// ---------------------------------------------------------------------------------------------
namespace {

static __device__ __align__(256) int32_t scratch[IC_STATIC_PACK_MAX_BLOCKS];  // one copy per GPU, held until the process ends

struct IdChunk {
  int32_t v[960];  // with the other arguments: under the 4 KiB a launch may carry
};

__global__ __launch_bounds__(64) void ids_from_args_kernel(IdChunk chunk, int32_t* __restrict__ dst, int32_t count) {
  const int32_t i = (int32_t)(blockIdx.x * 64u + threadIdx.x);
  if (i < count) dst[i] = chunk.v[i];
}

// Device address of `scratch` on the current device.  In host code the array's name is only a handle
// for hipGetSymbolAddress; every GPU holds its own copy at its own address, looked up once.
int static_ids(int32_t** out) {
  static std::mutex mu;
  static int32_t* ptr[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return IC_EHIP;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return IC_EHIP;
    ptr[dev] = (int32_t*)p;
  }
  *out = ptr[dev];
  return IC_OK;
}

}  // namespace

}  // namespace ic

extern "C" int kv_pack_blocks_static(ic_pool* pool, const int32_t* host_ids, int32_t n, void* dev_staging,
                                     size_t staging_bytes, void* hip_stream) {
  using namespace ic;
  if (!pool) return IC_ENULL;
  if (n < 0) return IC_EINVAL;
  if (n == 0) return IC_OK;
  if (!host_ids || !dev_staging) return IC_ENULL;
  if (n > IC_STATIC_PACK_MAX_BLOCKS) return IC_ELIMIT;
  const PoolView pv = pool_view(pool);
  for (int32_t i = 0; i < n; ++i)
    if (host_ids[i] < 0 || host_ids[i] >= pv.cfg.num_blocks) return IC_ERANGE;
  if ((uintptr_t)dev_staging & 15u) return IC_EALIGN;
  if (staging_bytes / pv.block_bytes < (size_t)n) return IC_ESIZE;
  {
    const char* s0 = (const char*)dev_staging;
    const char* s1 = s0 + (size_t)n * pv.block_bytes;
    if (s0 < pv.base + pv.bytes && pv.base < s1) return IC_EINVAL;  // staging must not overlap the pool
  }
  int32_t* ids = nullptr;
  const int rc = static_ids(&ids);
  if (rc != IC_OK) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  IdChunk chunk;
  constexpr int32_t kPer = (int32_t)(sizeof(chunk.v) / sizeof(chunk.v[0]));
  for (int32_t off = 0; off < n; off += kPer) {
    const int32_t count = n - off < kPer ? n - off : kPer;
    std::memcpy(chunk.v, host_ids + off, sizeof(int32_t) * (size_t)count);
    hipLaunchKernelGGL(ids_from_args_kernel, dim3((uint32_t)(count + 63) / 64u), dim3(64), 0, st, chunk, ids + off, count);
    if (hipGetLastError() != hipSuccess) return IC_EHIP;
  }
  return launch_pack(pv.base, dev_staging, ids, n, pv.block_bytes, st) == hipSuccess ? IC_OK : IC_EHIP;
}

namespace ic {

hipError_t launch_pack(const void* pool, void* staging, const int32_t* dev_ids, int32_t n,
                       size_t block_bytes, hipStream_t st) {
  return launch_swap<true>((char*)pool, (char*)staging, dev_ids, n, block_bytes, st);
}

hipError_t launch_unpack(void* pool, const void* staging, const int32_t* dev_ids, int32_t n,
                         size_t block_bytes, hipStream_t st) {
  return launch_swap<false>((char*)pool, (char*)staging, dev_ids, n, block_bytes, st);
}

}  // namespace ic

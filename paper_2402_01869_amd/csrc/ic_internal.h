// Internal declarations shared by the host-side planner and the gfx950 kernels.
// Nothing here is part of the C ABI (include/infercept_hot.h is).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/infercept_hot.h"
#include "../../include/infercept_measure.h"

namespace ic {

// What other translation units may know of a pool (the struct itself lives with the C ABI).
struct PoolView {
  ic_pool_cfg cfg;
  char* base;          // device address of block 0
  size_t bytes;        // bytes the caller said are behind base
  size_t block_bytes;  // K and V of one block
};
PoolView pool_view(const ic_pool* pool);

constexpr int kBlockSize = 16;  // tokens per cache block (the only size built)
constexpr int kRowWaves = 4;    // waves per workgroup of the row kernel
constexpr int kMaxRowPart = 4096;  // keys per row-kernel work item: 64 block ids per wave

// Query rows per work item of the MFMA tile kernel (planner and kernel must agree).
constexpr int tile_rows(int head_dim) { return head_dim <= 128 ? 256 : 128; }

// One work item of the row kernel: one query row against keys [k_begin, k_end) of its sequence,
// for every head (the head is a grid dimension).  32 bytes so a wave reads it with scalar loads.
struct RowItem {
  int32_t seq;      // index into bt_off
  int32_t qrow;     // row in packed q / out
  int32_t k_begin;  // first key, multiple of 16
  int32_t k_end;    // one past the last visible key of this item
  int32_t slot;     // partial-result slot, or -1: the item is the whole row, write bf16 out
  int32_t pad[3];
};

// One work item of the MFMA tile kernel: up to tile_rows(D) >> tile_g_shift consecutive query rows of one
// sequence, for the 1 << tile_g_shift query heads that share a K/V head, against keys [k_begin, k_end)
// (k_end is a bound for the LAST row; earlier rows see fewer keys).
struct TileItem {
  int32_t seq;
  int32_t qrow0;    // first row of the tile in packed q / out
  int32_t n_rows;   // rows in this tile (<= tile height)
  int32_t pos0;     // absolute position of the tile's first row: it sees keys 0..pos0
  int32_t k_begin;  // first key of this partition, multiple of 64
  int32_t k_end;    // one past the last key of this partition (<= pos0 + n_rows)
  int32_t slot0;    // partial slot of (row 0, this partition) or -1 for direct output
  int32_t nparts;   // partitions of this tile: slot(row r) = slot0 + r * nparts
};

// One row whose partial results must be merged.
struct MergeItem {
  int32_t qrow;
  int32_t slot0;
  int32_t nparts;
  int32_t pad;
};

struct AttnParams {
  const uint16_t* pool;
  const uint16_t* q;
  uint16_t* out;
  const int32_t* bt_off;   // [num_seqs] offset of each sequence's ids in bt_flat
  const int32_t* bt_flat;  // compacted block tables
  const RowItem* row_items;
  const TileItem* tile_items;
  const MergeItem* merge_items;
  float* part_o;           // [slots][H][D] unnormalised partial outputs
  float* part_ml;          // [slots][H][2] (running max in log2 units, normaliser)
  int32_t num_heads;       // query heads H
  int32_t num_kv_heads;    // key/value heads in the pool; query head h reads K/V head h / group
  int32_t group;           // H / num_kv_heads
  int32_t tile_g_shift;    // log2 of the query heads one tile workgroup serves (they share K/V): a tile's
                           // row r is query row r >> shift, head (first head of the workgroup) + (r & mask)
  int32_t n_row_items;
  int32_t n_vec_items;     // row items [0, n_vec_items) belong to the vector row kernel, the rest to the group kernel
  int32_t n_tile_items;
  int32_t n_merge_items;
  float scale_log2e;       // scale * log2(e): scores are kept in log2 units
  int32_t row_variant;     // row-kernel build: bit0 = prefetch depth 2, bit1 = plain (cached) loads
  int32_t tile_first;      // persistent tile kernel: its waves ask for issue priority over the kernel beside it
  int32_t* counters;       // 16 work-queue counters, zero when the kernel starts
};

// Work-queue counters of the persistent kernels (16 ints at the head of the descriptor image):
//   [0..7] tile queue of each XCD, [9] shared tile queue, [8] row queue, [10] queue of the slim group kernel,
//   [12] / [13] / [14] workgroups of the row / tile / slim group kernel that have left.
// A persistent kernel's workgroups leave through queue_leave: the last one out (every other has made
// its final, failing pull by then) puts the kernel's counters back to zero, so that a descriptor
// image already in device memory serves the next launch as it is.
constexpr int kCtrRowQueue = 8, kCtrTileShared = 9, kCtrGroupQueue = 10, kCtrRowLeft = 12, kCtrTileLeft = 13, kCtrGroupLeft = 14;
__device__ __forceinline__ void queue_leave(int32_t* counters, int first, int count, int extra, int left_slot) {
  if (threadIdx.x == 0) {
    const int gone = atomicAdd(&counters[left_slot], 1);
    if (gone == (int)gridDim.x - 1) {
      for (int i = 0; i < count; ++i) atomicExch(&counters[first + i], 0);
      if (extra >= 0) atomicExch(&counters[extra], 0);
      atomicExch(&counters[left_slot], 0);
    }
  }
}

// Launchers (defined next to their kernels).  Each returns a hipError_t.
hipError_t launch_row_kernel(const AttnParams& p, int head_dim, hipStream_t st);
hipError_t launch_row_persist(const AttnParams& p, int head_dim, int slots, hipStream_t st);
hipError_t launch_row_persist_slim(const AttnParams& p, int head_dim, int slots, hipStream_t st);
hipError_t launch_tile_persist(const AttnParams& p, int head_dim, int slots, bool beside, hipStream_t st);
hipError_t launch_tile_kernel(const AttnParams& p, int head_dim, hipStream_t st);
hipError_t launch_merge_kernel(const AttnParams& p, int head_dim, hipStream_t st);
hipError_t launch_group_kernel(const AttnParams& p, int head_dim, hipStream_t st);  // row items x K/V heads
// The same items from a queue, built to share a CU with a tile workgroup: head_dim 128 and groups of 2..16 heads only.
hipError_t launch_group_slim(const AttnParams& p, int head_dim, int slots, hipStream_t st);
// Rows of k_new / v_new ([rows][H][D] bf16) into the pool at slot dst[row] (block * 16 + slot; < 0: skip).
hipError_t launch_append(void* pool, const void* k_new, const void* v_new, const int32_t* dev_dst, int32_t rows,
                         int num_heads, int head_dim, hipStream_t st);
// bytes: multiple of 16; pinned_src: pinned host memory (device-visible); dev_dst: device, 16-byte aligned.
hipError_t launch_upload(void* dev_dst, const void* pinned_src, size_t bytes, hipStream_t st);
hipError_t launch_pack(const void* pool, void* staging, const int32_t* dev_ids, int32_t n,
                       size_t block_bytes, hipStream_t st);
hipError_t launch_unpack(void* pool, const void* staging, const int32_t* dev_ids, int32_t n,
                         size_t block_bytes, hipStream_t st);

}  // namespace ic

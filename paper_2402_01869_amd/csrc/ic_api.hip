// C ABI, host-side validation and launch planning for the intercept hot path.
// See include/infercept_hot.h for the contract of every entry point.
#include <algorithm>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <vector>

#include "ic_internal.h"

using namespace ic;

namespace {

constexpr int kStagingSlots = 4;       // pinned host buffers cycled by successive calls
// Keys per decode work item: 4096 (the most a row item can hold).  Measured on the 13B-shaped batches: contexts up to
// 4096 keys as ONE item each (no partial results, no merge pass) are 1 % faster than 2048-key items, alone and beside
// the tile kernel; 512- and 1024-key items are 1-5 % slower (head_dim 256, GPT-J-shaped decode: 6 % slower at 512).
constexpr int kDefaultRowPart = 4096;
constexpr int kDefaultSpanPart = 8192; // keys per span-tile work item (partials of 256 rows are costly)
constexpr int kUnsplitWorkgroups = 1024;  // tile workgroups (4 per CU) from which spans are not split at all
// Rows that see fewer keys than this stay off the matrix cores.  There the weights are rounded to bf16
// before the PV product; with a handful of keys a single weight's rounding (2^-9 relative) shows in the
// output, with dozens the roundings average out.  The vector path keeps the weights in fp32.
constexpr int kShareKeys = 8192;  // sequences at least this long keep their tile items side by side
constexpr int kMfmaMinKeys = 64;

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct StagingSlot {
  void* host = nullptr;
  size_t cap = 0;
  hipEvent_t ev = nullptr;
  bool pending = false;
};

struct ProfState {
  bool on = false;
  std::vector<hipEvent_t> ev;       // pairs
  std::vector<int> kind;            // per pair
  int used = 0;                     // pairs recorded
};

}  // namespace

struct ic_pool {
  ic_pool_cfg cfg;
  char* base;
  size_t bytes;
  size_t block_bytes;
  ic_tuning tune;
  // library-owned runtime state (created lazily by the first GPU call)
  StagingSlot slots[kStagingSlots];
  int next_slot;
  // Device-side int32 lists, one per use (block ids of a pack, of an unpack, row destinations of an append), each
  // with the host copy of what it holds: a call whose list equals the previous one's (the same blocks moved for
  // every layer of a model, say) skips the upload and the checks that list already passed.
  struct DevList {
    int32_t* dev = nullptr;
    size_t cap = 0;
    std::vector<int32_t> held;  // contents of dev (from the last upload queued), empty = nothing usable
    bool checked = false;       // ... which have passed the host checks (false: uploaded under IC_FLAG_TRUSTED)
  };
  DevList lists[3];
  std::vector<void*> retired_dev;   // id lists that were outgrown: earlier launches may still read them, freed at destroy
  std::vector<void*> retired_host;  // the same for pinned descriptor buffers
  int num_cus;           // compute units of the pool's device (0 until the first attention call)
  hipStream_t side;      // second stream: the tile kernel runs beside the row kernel
  hipEvent_t ev_fork, ev_join;
  ProfState prof;
};

namespace ic {
PoolView pool_view(const ic_pool* pool) { return PoolView{pool->cfg, pool->base, pool->bytes, pool->block_bytes}; }
}  // namespace ic

namespace {

int check_cfg(const ic_pool_cfg* c) {
  if (!c) return IC_ENULL;
  if (c->num_blocks < 1 || c->num_heads < 1 || c->num_kv_heads < 1 || c->head_dim < 1 ||
      c->block_size < 1)
    return IC_EINVAL;
  if (c->dtype != 0 || c->layout != 0) return IC_EUNSUPPORTED;
  if (c->block_size != kBlockSize) return IC_EUNSUPPORTED;
  if (c->num_kv_heads > c->num_heads || c->num_heads % c->num_kv_heads != 0) return IC_EINVAL;
  if (c->head_dim != 64 && c->head_dim != 128 && c->head_dim != 256) return IC_EUNSUPPORTED;
  if (c->num_heads > 4096) return IC_EINVAL;
  return IC_OK;
}

size_t cfg_block_bytes(const ic_pool_cfg& c) {
  return (size_t)c.block_size * 2 * c.num_kv_heads * c.head_dim * 2;
}

// Structural checks (always done) and content checks (skipped when trusted).
int check_batch(const ic_pool_cfg& cfg, const ic_batch_desc* d, bool trusted) {
  if (!d) return IC_ENULL;
  if (!d->ctx_len || !d->q_len || !d->q_start || !d->block_tables) return IC_ENULL;
  if (d->num_seqs < 1 || d->max_blocks_per_seq < 1 || d->total_q_rows < 1) return IC_EINVAL;
  if (!(d->scale > 0.f) || d->scale > 3.0e38f) return IC_EINVAL;  // NaN fails the first comparison
  int64_t rows = 0;
  for (int s = 0; s < d->num_seqs; ++s) {
    const int32_t c = d->ctx_len[s], n = d->q_len[s];
    if (c < 1 || n < 1 || n > c) return IC_EINVAL;
    if ((c + kBlockSize - 1) / kBlockSize > d->max_blocks_per_seq) return IC_ESIZE;
    const int64_t r0 = d->q_start[s];
    if (r0 < 0 || r0 + n > d->total_q_rows) return IC_EOVERLAP;
    rows += n;
  }
  if (rows > d->total_q_rows) return IC_EOVERLAP;
  if (trusted) return IC_OK;
  std::vector<uint8_t> taken((size_t)d->total_q_rows, 0);
  for (int s = 0; s < d->num_seqs; ++s) {
    for (int32_t r = d->q_start[s]; r < d->q_start[s] + d->q_len[s]; ++r) {
      if (taken[r]) return IC_EOVERLAP;
      taken[r] = 1;
    }
    const int nb = (d->ctx_len[s] + kBlockSize - 1) / kBlockSize;
    const int32_t* row = d->block_tables + (int64_t)s * d->max_blocks_per_seq;
    for (int j = 0; j < nb; ++j)
      if (row[j] < 0 || row[j] >= cfg.num_blocks) return IC_ERANGE;
  }
  return IC_OK;
}

int check_ids(const ic_pool_cfg& cfg, const int32_t* ids, int32_t n, bool distinct) {
  if (n < 0) return IC_EINVAL;
  if (n == 0) return IC_OK;
  if (!ids) return IC_ENULL;
  for (int32_t i = 0; i < n; ++i)
    if (ids[i] < 0 || ids[i] >= cfg.num_blocks) return IC_ERANGE;
  if (distinct) {
    std::vector<uint8_t> seen((size_t)cfg.num_blocks, 0);
    for (int32_t i = 0; i < n; ++i) {
      if (seen[ids[i]]) return IC_EDUP;
      seen[ids[i]] = 1;
    }
  }
  return IC_OK;
}

// Destination of every query row's new K/V: block * block_size + slot (rows no sequence owns keep -1).
void append_destinations(const ic_batch_desc* desc, int32_t* dst) {
  for (int s = 0; s < desc->num_seqs; ++s) {
    const int32_t* table = desc->block_tables + (int64_t)s * desc->max_blocks_per_seq;
    const int t0 = desc->ctx_len[s] - desc->q_len[s];
    for (int i = 0; i < desc->q_len[s]; ++i) {
      const int t = t0 + i;
      dst[desc->q_start[s] + i] = table[t / kBlockSize] * kBlockSize + t % kBlockSize;
    }
  }
}

// Two rows on one slot would make the result depend on the order of the writes.
bool destinations_distinct(const ic_pool_cfg& cfg, const int32_t* dst, size_t rows) {
  std::vector<uint8_t> seen((size_t)cfg.num_blocks * kBlockSize, 0);
  for (size_t r = 0; r < rows; ++r) {
    if (dst[r] < 0) continue;
    if (seen[dst[r]]) return false;
    seen[dst[r]] = 1;
  }
  return true;
}

// ---------------------------------------------------------------------------------------
// Launch plan.  Sizes only (plan_sizes) or the filled descriptor image (plan_fill).
// Device image layout (all sections 256-byte aligned, in this order):
//   counters[16] | bt_off[num_seqs] | bt_flat[table_entries] | row_items | tile_items | merge_items
// followed in the workspace by part_o[slots][H][D] and part_ml[slots][H][2].
// ---------------------------------------------------------------------------------------
struct PlanSizes {
  ic_plan_info info;
  int row_part, span_part, tile_rows;  // tile_rows: QUERY rows per tile item
  int min_keys;                        // rows that see fewer keys are vector row items whatever their kind
  int vec_items;                       // row items [0, vec_items) run on the vector kernel, the rest on the group kernel
  int tile_g_shift;                    // log2 of the query heads one tile workgroup serves
  bool spans_as_rows;
  bool decode_as_tiles;                // grouped pools, span_kernel = 2: decode rows as one-row tile items
  bool decode_as_group;                // grouped pools: decode rows stay row items, run by the group kernel
  bool tile_leads;                     // the tile items are expected to take longer than the row items
  size_t off_ctr, off_bt_off, off_bt_flat, off_row, off_tile, off_merge, off_row_dst, image_bytes;
  size_t off_part_o, off_part_ml, total_bytes;
};

int round64(int x) { return (x + 63) / 64 * 64; }

}  // namespace

struct ic_plan {
  PlanSizes ps;
  ic_pool_cfg cfg;   // shape the plan was made for
  ic_tuning tune;    // launch knobs it was made with
  float scale;
  char* ws;          // the caller's workspace: descriptor image + partial results
  int32_t total_q_rows;
  bool append_checked;  // the rows' cache slots were found distinct (or the descriptor was trusted)
};

namespace {

// Where the rows of one sequence go.  Rows [0, n_few) see fewer than min_keys keys and are vector row
// items whatever their kind; the rest are row items (vector or group kernel) or tile items.
struct SeqRoute {
  int n_few;        // leading rows of the sequence that stay off the matrix cores
  bool rest_rows;   // the other rows are row items (else: tile items)
  bool rest_group;  // ... run by the group kernel
};

SeqRoute route(const PlanSizes& ps, int c, int n) {
  SeqRoute r;
  r.n_few = std::min(n, std::max(0, ps.min_keys - 1 - (c - n)));
  r.rest_rows = n == 1 ? !ps.decode_as_tiles : ps.spans_as_rows;
  r.rest_group = r.rest_rows && n == 1 && ps.decode_as_group;
  return r;
}

void plan_sizes(const ic_pool* pool, const ic_batch_desc* d, PlanSizes& ps) {
  std::memset(&ps, 0, sizeof ps);
  // Grouped-query attention: the G = H / Hkv query heads of a group read the same keys.  When G is a
  // power of two up to 32, a tile workgroup takes all of them (G rows per query row), so keys are
  // staged once per group, and decode rows (G rows of one query token) go to the matrix cores too:
  // as row items run by the group kernel, or (span_kernel = 2) as one-row tile items.
  const int G = pool->cfg.num_heads / pool->cfg.num_kv_heads;
  ps.tile_g_shift = 0;
  if (G >= 2 && G <= 32 && (G & (G - 1)) == 0)
    while ((1 << ps.tile_g_shift) < G) ++ps.tile_g_shift;
  const int kTileRows = tile_rows(pool->cfg.head_dim) >> ps.tile_g_shift;
  ps.tile_rows = kTileRows;
  const ic_tuning& t = pool->tune;
  ps.row_part = t.decode_part_tokens > 0 ? round64(t.decode_part_tokens) : kDefaultRowPart;
  ps.row_part = std::min(ps.row_part, kMaxRowPart);
  ps.span_part = t.span_part_tokens > 0 ? round64(t.span_part_tokens) : kDefaultSpanPart;
  ps.min_keys = t.mfma_min_keys > 0 ? std::min(t.mfma_min_keys, 64) : kMfmaMinKeys;  // <= the smallest partition
  ps.spans_as_rows = (t.span_kernel == 1);  // default: MFMA tiles
  ps.decode_as_tiles = ps.tile_g_shift > 0 && t.span_kernel == 2;
  ps.decode_as_group = ps.tile_g_shift > 0 && t.span_kernel == 0;
  if (t.span_part_tokens == 0) {
    // Splitting a span's keys buys parallelism at the price of fp32 partial results for every row
    // and a merge pass (measured on the long-context shape: 7 % of the call).  When the unsplit query
    // tiles already give every CU several workgroups, do not split.
    int64_t tiles = 0;
    for (int s = 0; s < d->num_seqs; ++s)
      if (d->q_len[s] > 1) {
        const int rest = d->q_len[s] - route(ps, d->ctx_len[s], d->q_len[s]).n_few;
        tiles += (rest + kTileRows - 1) / kTileRows;
      }
    const int64_t head_groups = pool->cfg.num_heads >> ps.tile_g_shift;
    if (tiles * head_groups >= kUnsplitWorkgroups) ps.span_part = 1 << 30;
  }
  ic_plan_info& in = ps.info;
  double tile_pairs = 0, row_keys = 0;  // (query row, key) pairs of the tile items; keys of the row items
  for (int s = 0; s < d->num_seqs; ++s) {
    const int c = d->ctx_len[s], n = d->q_len[s];
    in.table_entries += (c + kBlockSize - 1) / kBlockSize;
    if (n == 1) in.decode_rows += 1; else in.span_rows += n;
    const SeqRoute rt = route(ps, c, n);
    const int n_as_rows = rt.rest_rows ? n : rt.n_few;
    for (int i = 0; i < n_as_rows; ++i) {
      const int klen = c - n + i + 1;
      const int parts = (klen + ps.row_part - 1) / ps.row_part;
      in.row_items += parts;
      row_keys += klen;
      if (i < rt.n_few || !rt.rest_group) ps.vec_items += parts;
      if (parts > 1) { in.partial_slots += parts; in.merge_rows += 1; }
    }
    if (!rt.rest_rows) {
      const int part = n == 1 ? ps.row_part : ps.span_part;
      for (int r0 = rt.n_few; r0 < n; r0 += kTileRows) {
        const int nr = std::min(kTileRows, n - r0);
        const int klen = c - n + r0 + nr;  // keys visible to the tile's last row
        const int parts = (klen + part - 1) / part;
        in.tile_items += parts;
        tile_pairs += (double)nr * (klen - 0.5 * nr);
        if (parts > 1) { in.partial_slots += parts * nr; in.merge_rows += nr; }
      }
    }
  }
  const int H = pool->cfg.num_heads, D = pool->cfg.head_dim;
  // Which of the two kernels of a side-by-side launch ends last, from the rates they reach there (tile kernel
  // 0.9 PFLOP/s at 4 D flop per pair and head, row kernels 5.5 TB/s at 4 D bytes per key and K/V head): that one
  // goes on the caller's stream, the other through the fork and join of the second stream.  (head_dim 256: 0.5 PFLOP/s.)
  ps.tile_leads = tile_pairs * H * (4.0 * D / (D > 128 ? 0.5e15 : 0.9e15)) > row_keys * pool->cfg.num_kv_heads * (4.0 * D / 5.5e12);
  size_t o = 0;
  ps.off_ctr = o;     o = align_up(o + sizeof(int32_t) * 16, 256);
  ps.off_bt_off = o;  o = align_up(o + sizeof(int32_t) * (size_t)d->num_seqs, 256);
  ps.off_bt_flat = o; o = align_up(o + sizeof(int32_t) * (size_t)in.table_entries, 256);
  ps.off_row = o;     o = align_up(o + sizeof(RowItem) * (size_t)in.row_items, 256);
  ps.off_tile = o;    o = align_up(o + sizeof(TileItem) * (size_t)in.tile_items, 256);
  ps.off_merge = o;   o = align_up(o + sizeof(MergeItem) * (size_t)in.merge_rows, 256);
  ps.off_row_dst = o; o = align_up(o + sizeof(int32_t) * (size_t)d->total_q_rows, 256);  // for kv_write_span_planned
  ps.image_bytes = o;
  ps.off_part_o = o;  o = align_up(o + sizeof(float) * (size_t)in.partial_slots * H * D, 256);
  ps.off_part_ml = o; o = align_up(o + sizeof(float) * (size_t)in.partial_slots * H * 2, 256);
  ps.total_bytes = o;
}

// May throw std::bad_alloc (per-sequence scratch vectors); callers at the ABI catch it.
void plan_fill(const ic_batch_desc* d, const PlanSizes& ps, char* img) {
  const int kTileRows = ps.tile_rows;
  std::memset(img + ps.off_ctr, 0, sizeof(int32_t) * 16);  // work-queue counters start at zero
  int32_t* bt_off = (int32_t*)(img + ps.off_bt_off);
  int32_t* bt_flat = (int32_t*)(img + ps.off_bt_flat);
  RowItem* rows = (RowItem*)(img + ps.off_row);
  TileItem* tiles = (TileItem*)(img + ps.off_tile);
  MergeItem* merges = (MergeItem*)(img + ps.off_merge);
  {
    int32_t* row_dst = (int32_t*)(img + ps.off_row_dst);
    std::fill(row_dst, row_dst + (ps.image_bytes - ps.off_row_dst) / sizeof(int32_t), -1);
    append_destinations(d, row_dst);
  }
  int64_t nbt = 0;
  int nvec = 0, ngrp = ps.vec_items;  // vector items first, group-kernel items after them
  int ntiles = 0, nmerge = 0, slot = 0;
  std::vector<int> tile_slot0, tile_parts;
  for (int s = 0; s < d->num_seqs; ++s) {
    const int c = d->ctx_len[s], n = d->q_len[s];
    const int nb = (c + kBlockSize - 1) / kBlockSize;
    bt_off[s] = (int32_t)nbt;
    std::memcpy(bt_flat + nbt, d->block_tables + (int64_t)s * d->max_blocks_per_seq,
                sizeof(int32_t) * (size_t)nb);
    nbt += nb;
    const SeqRoute rt = route(ps, c, n);
    const int n_as_rows = rt.rest_rows ? n : rt.n_few;
    for (int i = 0; i < n_as_rows; ++i) {
      const int klen = c - n + i + 1;
      const int parts = (klen + ps.row_part - 1) / ps.row_part;
      const int qrow = d->q_start[s] + i;
      const bool vec = i < rt.n_few || !rt.rest_group;
      if (parts > 1) merges[nmerge++] = MergeItem{qrow, slot, parts, 0};
      for (int k = 0; k < parts; ++k) {
        RowItem& it = rows[vec ? nvec++ : ngrp++];
        it.seq = s;
        it.qrow = qrow;
        it.k_begin = k * ps.row_part;
        it.k_end = std::min(klen, (k + 1) * ps.row_part);
        it.slot = parts > 1 ? slot++ : -1;
        it.pad[0] = it.pad[1] = it.pad[2] = 0;
      }
    }
    if (!rt.rest_rows && rt.n_few < n) {
      // slots first (per tile: rows x partitions), then items ordered partition-major so that the
      // query tiles which read the same keys are dispatched next to each other
      const int first = rt.n_few;
      const int ntile = (n - first + kTileRows - 1) / kTileRows;
      const int part = n == 1 ? ps.row_part : ps.span_part;
      int max_parts = 0;
      tile_slot0.assign((size_t)ntile, -1);
      tile_parts.assign((size_t)ntile, 0);
      for (int ti = 0; ti < ntile; ++ti) {
        const int r0 = first + ti * kTileRows;
        const int nr = std::min(kTileRows, n - r0);
        const int klen = c - n + r0 + nr;
        const int parts = (klen + part - 1) / part;
        tile_parts[ti] = parts;
        max_parts = std::max(max_parts, parts);
        if (parts > 1) {
          tile_slot0[ti] = slot;
          for (int r = 0; r < nr; ++r)
            merges[nmerge++] = MergeItem{d->q_start[s] + r0 + r, slot + r * parts, parts, 0};
          slot += parts * nr;
        }
      }
      for (int k = 0; k < max_parts; ++k)
        for (int ti = 0; ti < ntile; ++ti) {
          if (k >= tile_parts[ti]) continue;
          const int r0 = first + ti * kTileRows;
          const int nr = std::min(kTileRows, n - r0);
          const int pos0 = c - n + r0;
          const int klen = pos0 + nr;
          TileItem& it = tiles[ntiles++];
          it.seq = s;
          it.qrow0 = d->q_start[s] + r0;
          it.n_rows = nr;
          it.pos0 = pos0;
          it.k_begin = k * part;
          it.k_end = std::min(klen, (k + 1) * part);
          it.slot0 = tile_parts[ti] > 1 ? tile_slot0[ti] + k : -1;
          it.nparts = tile_parts[ti];
        }
    }
  }
  // Longest tile items first: workgroups are handed out in item order (per head), and a few hundred items of
  // unequal length (contexts differ 3 : 1) over 256 CUs otherwise end with the longest ones running alone.
  // The items of one long sequence count as equally long (the stable sort then leaves them side by side, in
  // the order made above): they read the same keys, which no longer stay in an L2 from one item to the next
  // (8192 keys of one head are 4 MiB), so they have to run at the same time to share them.  Measured on one
  // box: 2048-row chunks on 16384-token prefixes 3 % faster side by side than longest-item-first, 512-row
  // chunks on prefixes of 512..2048 tokens 2 % slower.
  const auto weight = [d](const TileItem& t) {
    return d->ctx_len[t.seq] >= kShareKeys ? (int64_t)d->ctx_len[t.seq] * 256 : (int64_t)(t.k_end - t.k_begin) * t.n_rows;
  };
  std::stable_sort(tiles, tiles + ntiles, [&](const TileItem& a, const TileItem& b) { return weight(a) > weight(b); });
  // The same for row items, within the vector kernel's and the group kernel's share: decode contexts differ 16 : 1.
  const auto longer = [](const RowItem& a, const RowItem& b) { return a.k_end - a.k_begin > b.k_end - b.k_begin; };
  std::stable_sort(rows, rows + ps.vec_items, longer);
  std::stable_sort(rows + ps.vec_items, rows + ps.info.row_items, longer);
}

// ---------------------------------------------------------------------------------------
// Runtime helpers
// ---------------------------------------------------------------------------------------
// The second stream of the side-by-side launch.  ONE per device for the whole process, shared by all
// pools (a model has one pool per layer): a process gets few hardware queues (four by default), streams
// are dealt onto them round-robin, and two streams on one queue run in order; a side stream per pool
// would sooner or later share the caller's queue and silently serialise the two kernels.  Lives until
// the process ends.
hipStream_t shared_side_stream() {
  static std::mutex mu;
  static hipStream_t side[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  std::lock_guard<std::mutex> lock(mu);
  if (!side[dev] && hipStreamCreateWithFlags(&side[dev], hipStreamNonBlocking) != hipSuccess) side[dev] = nullptr;
  return side[dev];
}

// Sizes of the pool's own buffers, fixed at the first GPU call from the pool's shape so that later calls
// allocate nothing: a descriptor image is block tables (at most one entry per block while sequences
// share none), work items and one int per query row; an id list is at most one entry per block (a
// swap, one list each for packs and unpacks) or per cache slot (an append).  Only a call beyond these sizes grows a buffer, and then the
// old one is kept until kv_pool_destroy (launches in flight may still read it) instead of being
// freed behind a device-wide wait.
size_t pinned_slot_bytes(const ic_pool* pool) { return align_up(((size_t)256 << 10) + 8 * (size_t)pool->cfg.num_blocks, 4096); }
enum { kListPack = 0, kListUnpack = 1, kListAppend = 2 };
size_t dev_list_bytes(const ic_pool* pool, int which) {
  const size_t entries = (size_t)pool->cfg.num_blocks * (which == kListAppend ? (size_t)kBlockSize : 1);
  return align_up(std::max((size_t)1 << 16, sizeof(int32_t) * entries), 4096);
}

int acquire_slot(ic_pool* pool, size_t bytes, StagingSlot** out) {
  StagingSlot& s = pool->slots[pool->next_slot];
  pool->next_slot = (pool->next_slot + 1) % kStagingSlots;
  if (s.pending) {
    if (hipEventSynchronize(s.ev) != hipSuccess) return IC_EHIP;
    s.pending = false;
  }
  if (!s.ev && hipEventCreateWithFlags(&s.ev, hipEventDisableTiming) != hipSuccess) return IC_EHIP;
  if (s.cap < bytes) {
    const size_t cap = std::max(align_up(bytes, 4096), pinned_slot_bytes(pool));
    void* fresh = nullptr;
    if (hipHostMalloc(&fresh, cap, hipHostMallocDefault) != hipSuccess) return IC_EHIP;
    if (s.host) pool->retired_host.push_back(s.host);
    s.host = fresh;
    s.cap = cap;
  }
  *out = &s;
  return IC_OK;
}

struct ProfScope {
  ic_pool* pool;
  hipStream_t st;
  int idx;
  ProfScope(ic_pool* p, int kind, hipStream_t s) : pool(p), st(s), idx(-1) {
    ProfState& pr = p->prof;
    if (pr.on && (size_t)(pr.used + 1) * 2 <= pr.ev.size()) {
      idx = pr.used++;
      pr.kind[idx] = kind;
      (void)hipEventRecord(pr.ev[2 * idx], st);
    }
  }
  ~ProfScope() {
    if (idx >= 0) (void)hipEventRecord(pool->prof.ev[2 * idx + 1], st);
  }
};

bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

// Nothing may be thrown through the C ABI: the host-side checks and the planner use std::vector.
template <class F>
int guarded(F&& body) noexcept {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    return IC_ENOMEM;
  } catch (...) {
    return IC_EINVAL;
  }
}

}  // namespace

// =========================================================================================
extern "C" {

const char* ic_strerror(int code) {
  switch (code) {
    case IC_OK: return "ok";
    case IC_ENULL: return "null pointer argument";
    case IC_EINVAL: return "size, length or count out of range";
    case IC_ERANGE: return "block id outside the pool";
    case IC_ESIZE: return "caller buffer too small";
    case IC_EALIGN: return "device pointer not 16-byte aligned";
    case IC_EDUP: return "duplicate destination block id";
    case IC_EUNSUPPORTED: return "configuration not supported by this build";
    case IC_EOVERLAP: return "query-row ranges overlap or leave the packed array";
    case IC_EHIP: return "HIP runtime error";
    case IC_ENOMEM: return "host allocation failed";
    case IC_ELIMIT: return "more than the fixed capacity of this allocation-free entry point";
    default: return "unknown error code";
  }
}

int kv_pool_init(const ic_pool_cfg* cfg, void* dev_pool_base, size_t pool_bytes, ic_pool** out) {
  if (!cfg || !dev_pool_base || !out) return IC_ENULL;
  const int rc = check_cfg(cfg);
  if (rc != IC_OK) return rc;
  if (misaligned(dev_pool_base)) return IC_EALIGN;
  const size_t bb = cfg_block_bytes(*cfg);
  if (pool_bytes / bb < (size_t)cfg->num_blocks) return IC_ESIZE;
  ic_pool* p = new (std::nothrow) ic_pool();
  if (!p) return IC_ENOMEM;
  p->cfg = *cfg;
  p->base = (char*)dev_pool_base;
  p->bytes = pool_bytes;
  p->block_bytes = bb;
  std::memset(&p->tune, 0, sizeof p->tune);
  p->next_slot = 0;
  p->num_cus = 0;
  p->side = nullptr;
  p->ev_fork = p->ev_join = nullptr;
  *out = p;
  return IC_OK;
}

int kv_pool_destroy(ic_pool* pool) {
  if (!pool) return IC_ENULL;
  int rc = IC_OK;
  for (StagingSlot& s : pool->slots) {
    if (s.pending && hipEventSynchronize(s.ev) != hipSuccess) rc = IC_EHIP;
    if (s.ev) (void)hipEventDestroy(s.ev);
    if (s.host) (void)hipHostFree(s.host);
  }
  for (hipEvent_t e : pool->prof.ev) (void)hipEventDestroy(e);
  for (ic_pool::DevList& dl : pool->lists)
    if (dl.dev) (void)hipFree(dl.dev);
  for (void* p : pool->retired_dev) (void)hipFree(p);
  for (void* p : pool->retired_host) (void)hipHostFree(p);
  if (pool->side && hipStreamSynchronize(pool->side) != hipSuccess) rc = IC_EHIP;  // shared: never destroyed
  if (pool->ev_fork) (void)hipEventDestroy(pool->ev_fork);
  if (pool->ev_join) (void)hipEventDestroy(pool->ev_join);
  delete pool;
  return rc;
}

size_t kv_block_bytes(const ic_pool* pool) { return pool ? pool->block_bytes : 0; }

int ic_check_batch(const ic_pool_cfg* cfg, const ic_batch_desc* desc) {
  const int rc = check_cfg(cfg);
  if (rc != IC_OK) return rc;
  return guarded([&] { return check_batch(*cfg, desc, false); });
}

int ic_check_ids(const ic_pool_cfg* cfg, const int32_t* host_ids, int32_t n, int require_distinct) {
  const int rc = check_cfg(cfg);
  if (rc != IC_OK) return rc;
  return guarded([&] { return check_ids(*cfg, host_ids, n, require_distinct != 0); });
}

int ic_pool_set_tuning(ic_pool* pool, const ic_tuning* tuning) {
  if (!pool || !tuning) return IC_ENULL;
  if (tuning->decode_part_tokens < 0 || tuning->span_part_tokens < 0 || tuning->span_kernel < 0 ||
      tuning->span_kernel > 2 || tuning->row_variant < 0 || tuning->row_variant > 3 ||
      tuning->serial_spans < 0 || tuning->serial_spans > 1 || tuning->row_launch < 0 || tuning->row_launch > 3 ||
      tuning->row_slots < 0 || tuning->row_slots > 65536 || tuning->mfma_min_keys < 0 ||
      tuning->mfma_min_keys > 64 || tuning->reserved[0])
    return IC_EINVAL;
  pool->tune = *tuning;
  return IC_OK;
}

int ic_plan_query(const ic_pool* pool, const ic_batch_desc* desc, ic_plan_info* out) {
  if (!pool || !desc || !out) return IC_ENULL;
  const int rc = check_batch(pool->cfg, desc, true);
  if (rc != IC_OK) return rc;
  PlanSizes ps;
  plan_sizes(pool, desc, ps);
  *out = ps.info;
  return IC_OK;
}

int ic_plan_image(const ic_pool* pool, const ic_batch_desc* desc, void* host_image, size_t host_bytes,
                  ic_plan_layout* out) {
  if (!pool || !desc || !out) return IC_ENULL;
  return guarded([&]() -> int {
  const int rc = check_batch(pool->cfg, desc, false);
  if (rc != IC_OK) return rc;
  PlanSizes ps;
  plan_sizes(pool, desc, ps);
  std::memset(out, 0, sizeof *out);
  out->image_bytes = (int64_t)ps.image_bytes;
  out->off_counters = (int64_t)ps.off_ctr;
  out->off_bt_off = (int64_t)ps.off_bt_off;
  out->off_bt_flat = (int64_t)ps.off_bt_flat;
  out->off_row_items = (int64_t)ps.off_row;
  out->off_tile_items = (int64_t)ps.off_tile;
  out->off_merge_items = (int64_t)ps.off_merge;
  out->off_row_dst = (int64_t)ps.off_row_dst;
  out->row_part_tokens = ps.row_part;
  out->span_part_tokens = ps.span_part;
  out->tile_query_rows = ps.tile_rows;
  out->tile_head_shift = ps.tile_g_shift;
  out->n_row_items = ps.info.row_items;
  out->n_tile_items = ps.info.tile_items;
  out->n_merge_items = ps.info.merge_rows;
  out->n_vector_row_items = ps.vec_items;
  if (host_image) {
    if (host_bytes < ps.image_bytes) return IC_ESIZE;
    std::memset(host_image, 0, ps.image_bytes);
    plan_fill(desc, ps, (char*)host_image);
  }
  return IC_OK;
  });
}

size_t paged_attn_mixed_workspace_bytes(const ic_pool* pool, const ic_batch_desc* desc) {
  if (!pool || !desc) return 0;
  if (check_batch(pool->cfg, desc, true) != IC_OK) return 0;
  PlanSizes ps;
  plan_sizes(pool, desc, ps);
  return ps.total_bytes;
}

// Upload of the descriptor image of a planned batch into the workspace (through the pinned ring).
static int upload_plan(ic_pool* pool, const ic_batch_desc* desc, const PlanSizes& ps, char* ws, hipStream_t st) {
  StagingSlot* slot = nullptr;
  const int rc = acquire_slot(pool, ps.image_bytes, &slot);
  if (rc != IC_OK) return rc;
  plan_fill(desc, ps, (char*)slot->host);
  {
    ProfScope ps_(pool, IC_K_UPLOAD, st);
    if (launch_upload(ws, slot->host, ps.image_bytes, st) != hipSuccess) return IC_EHIP;
  }
  if (hipEventRecord(slot->ev, st) != hipSuccess) return IC_EHIP;
  slot->pending = true;
  return IC_OK;
}

// The kernels of one attention call, for a descriptor image that is already in the workspace.
static int launch_attention(ic_pool* pool, const PlanSizes& ps, float scale, const void* dev_q, void* dev_out,
                            char* ws, hipStream_t st) {
  const int D = pool->cfg.head_dim;
  if (pool->num_cus == 0) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 8)
      return IC_EHIP;
    pool->num_cus = cus;
  }
  AttnParams p;
  p.pool = (const uint16_t*)pool->base;
  p.q = (const uint16_t*)dev_q;
  p.out = (uint16_t*)dev_out;
  p.bt_off = (const int32_t*)(ws + ps.off_bt_off);
  p.bt_flat = (const int32_t*)(ws + ps.off_bt_flat);
  p.row_items = (const RowItem*)(ws + ps.off_row);
  p.tile_items = (const TileItem*)(ws + ps.off_tile);
  p.merge_items = (const MergeItem*)(ws + ps.off_merge);
  p.part_o = (float*)(ws + ps.off_part_o);
  p.part_ml = (float*)(ws + ps.off_part_ml);
  p.num_heads = pool->cfg.num_heads;
  p.num_kv_heads = pool->cfg.num_kv_heads;
  p.group = pool->cfg.num_heads / pool->cfg.num_kv_heads;
  p.tile_g_shift = ps.tile_g_shift;
  p.n_row_items = ps.info.row_items;
  p.n_vec_items = ps.vec_items;
  p.n_tile_items = ps.info.tile_items;
  p.n_merge_items = ps.info.merge_rows;
  p.scale_log2e = scale * 1.4426950408889634f;
  p.row_variant = pool->tune.row_variant;
  p.tile_first = 0;
  p.counters = (int32_t*)(ws + ps.off_ctr);

  // Decode rows are memory-bound and span tiles are MFMA-bound (the complementarity Section 4.2
  // builds on): a batch that has both runs them as two persistent kernels side by side, one
  // workgroup of each per CU, the tile kernel on the pool's second stream (forked from and joined
  // back into the caller's stream by events).  The kernel beside the tile kernel is the slim row
  // kernel (multi-head pools) or the slim group kernel (grouped pools: head_dim 128, groups of up
  // to 16 heads).  serial_spans = 1 and the other grouped shapes run one kernel after the other instead.
  const int n_group_items = p.n_row_items - p.n_vec_items;
  const bool pair_ok = p.n_tile_items > 0 && !pool->tune.serial_spans;
  const bool beside_rows = pair_ok && p.n_vec_items > 0 && !ps.decode_as_group;
  const bool beside_group = pair_ok && n_group_items > 0 && D == 128 && p.group <= 16;
  const int row_slots = pool->tune.row_slots > 0 ? pool->tune.row_slots : pool->num_cus;
  if (beside_rows || beside_group) {
    if (!pool->side) {  // the stream is assigned last: a half-made set is retried by the next call
      if (!pool->ev_fork && hipEventCreateWithFlags(&pool->ev_fork, hipEventDisableTiming) != hipSuccess) return IC_EHIP;
      if (!pool->ev_join && hipEventCreateWithFlags(&pool->ev_join, hipEventDisableTiming) != hipSuccess) return IC_EHIP;
      if (!(pool->side = shared_side_stream())) return IC_EHIP;
    }
    if (hipEventRecord(pool->ev_fork, st) != hipSuccess) return IC_EHIP;
    if (hipStreamWaitEvent(pool->side, pool->ev_fork, 0) != hipSuccess) return IC_EHIP;
    // From here on the side stream may hold work that writes dev_out and the workspace: whatever fails
    // below, the caller's stream is still made to wait for it (or, failing that, the host does).
    // The kernel expected to end last runs on the caller's stream, where nothing but the upload is in front of it;
    // the other one pays the two cross-stream waits (some 10 us each).  A tile kernel that leads also asks for
    // issue priority: what it loses to its neighbour's waves is lost to the call (measured on the 70B-shaped
    // batch: tile kernel 0.455 instead of 0.492 ms, group kernel 0.24 instead of 0.21 ms, call 0.50 instead of 0.53).
    const bool tile_main = ps.tile_leads;
    hipStream_t s_tile = tile_main ? st : pool->side, s_rows = tile_main ? pool->side : st;
    p.tile_first = tile_main;
    bool ok = true;
    auto run_tile = [&] {
      ProfScope ps_(pool, IC_K_TILE, s_tile);
      ok = launch_tile_persist(p, D, pool->num_cus, true, s_tile) == hipSuccess;
    };
    auto run_rows = [&] {
      if (ok && beside_group) {
        ProfScope ps_(pool, IC_K_GROUP, s_rows);
        ok = launch_group_slim(p, D, row_slots, s_rows) == hipSuccess;
      }
      if (ok && p.n_vec_items > 0) {  // in a grouped pool: the rows with too few keys for the matrix cores
        ProfScope ps_(pool, IC_K_ROW, s_rows);
        ok = launch_row_persist_slim(p, D, row_slots, s_rows) == hipSuccess;
      }
    };
    // the tile workgroups are placed first either way: one per CU, the row workgroups fill in beside them
    bool joined;
    if (tile_main) {
      run_tile();
      run_rows();
      joined = hipEventRecord(pool->ev_join, pool->side) == hipSuccess;
    } else {
      run_tile();
      joined = hipEventRecord(pool->ev_join, pool->side) == hipSuccess;
      run_rows();
    }
    if (!joined || hipStreamWaitEvent(st, pool->ev_join, 0) != hipSuccess) {
      (void)hipStreamSynchronize(pool->side);
      return IC_EHIP;
    }
    if (!ok) return IC_EHIP;
  } else {
    if (p.n_tile_items > 0) {
      ProfScope ps_(pool, IC_K_TILE, st);
      // head_dim <= 128: the persistent launch also when no other kernel runs beside it.  Its per-XCD queues keep the
      // query tiles of one (sequence, head) on one L2: on 2048-row chunks the spans then fetch 2.6 x instead of 6.9 x
      // their keys from HBM and finish 7 % sooner (9.66 against 10.41 ms); shorter chunks and grouped pools: no change.
      // head_dim 256: one workgroup per work item; the persistent build is held to 208 registers for the sake of
      // its neighbour and is 19 % slower alone (0.197 against 0.166 ms on the GPT-J-shaped chunks).
      const hipError_t e = D <= 128 ? launch_tile_persist(p, D, pool->num_cus, false, st) : launch_tile_kernel(p, D, st);
      if (e != hipSuccess) return IC_EHIP;
    }
    if (n_group_items > 0) {
      ProfScope ps_(pool, IC_K_GROUP, st);
      const bool slim = pool->tune.row_launch == 3 && D == 128 && p.group <= 16;  // the side-by-side build, alone
      if ((slim ? launch_group_slim(p, D, row_slots, st) : launch_group_kernel(p, D, st)) != hipSuccess) return IC_EHIP;
    }
    if (p.n_vec_items > 0) {
      ProfScope ps_(pool, IC_K_ROW, st);
      const hipError_t e = pool->tune.row_launch == 3 ? launch_row_persist_slim(p, D, row_slots, st)
                           : pool->tune.row_launch != 1       ? launch_row_persist(p, D, row_slots, st)
                                                              : launch_row_kernel(p, D, st);
      if (e != hipSuccess) return IC_EHIP;
    }
  }
  if (p.n_merge_items > 0) {
    ProfScope ps_(pool, IC_K_MERGE, st);
    if (launch_merge_kernel(p, D, st) != hipSuccess) return IC_EHIP;
  }
  return IC_OK;
}


int paged_attn_mixed(ic_pool* pool, const ic_batch_desc* desc, const void* dev_q, void* dev_out,
                     void* dev_workspace, size_t workspace_bytes, void* hip_stream) {
  if (!pool || !desc || !dev_q || !dev_out || !dev_workspace) return IC_ENULL;
  return guarded([&]() -> int {
    int rc = check_batch(pool->cfg, desc, (desc->flags & IC_FLAG_TRUSTED) != 0);
    if (rc != IC_OK) return rc;
    if (misaligned(dev_q) || misaligned(dev_out) || ((uintptr_t)dev_workspace & 255u)) return IC_EALIGN;
    PlanSizes ps;
    plan_sizes(pool, desc, ps);
    if (workspace_bytes < ps.total_bytes) return IC_ESIZE;
    hipStream_t st = (hipStream_t)hip_stream;
    char* ws = (char*)dev_workspace;
    if ((rc = upload_plan(pool, desc, ps, ws, st)) != IC_OK) return rc;
    return launch_attention(pool, ps, desc->scale, dev_q, dev_out, ws, st);
  });
}

int paged_attn_plan_create(ic_pool* pool, const ic_batch_desc* desc, void* dev_workspace, size_t workspace_bytes,
                           void* hip_stream, ic_plan** out) {
  if (!pool || !desc || !dev_workspace || !out) return IC_ENULL;
  return guarded([&]() -> int {
  int rc = check_batch(pool->cfg, desc, (desc->flags & IC_FLAG_TRUSTED) != 0);
  if (rc != IC_OK) return rc;
  if ((uintptr_t)dev_workspace & 255u) return IC_EALIGN;
  std::unique_ptr<ic_plan> pl(new ic_plan());
  plan_sizes(pool, desc, pl->ps);
  if (workspace_bytes < pl->ps.total_bytes) return IC_ESIZE;
  pl->cfg = pool->cfg;
  pl->tune = pool->tune;
  pl->scale = desc->scale;
  pl->ws = (char*)dev_workspace;
  pl->total_q_rows = desc->total_q_rows;
  pl->append_checked = true;
  if (!(desc->flags & IC_FLAG_TRUSTED)) {
    std::vector<int32_t> dst((size_t)desc->total_q_rows, -1);
    append_destinations(desc, dst.data());
    pl->append_checked = destinations_distinct(pool->cfg, dst.data(), dst.size());
  }
  if ((rc = upload_plan(pool, desc, pl->ps, pl->ws, (hipStream_t)hip_stream)) != IC_OK) return rc;
  *out = pl.release();
  return IC_OK;
  });
}

int paged_attn_planned(ic_pool* pool, const ic_plan* plan, const void* dev_q, void* dev_out, void* hip_stream) {
  if (!pool || !plan || !dev_q || !dev_out) return IC_ENULL;
  const ic_pool_cfg &a = pool->cfg, &b = plan->cfg;
  if (a.num_blocks != b.num_blocks || a.block_size != b.block_size || a.num_heads != b.num_heads ||
      a.num_kv_heads != b.num_kv_heads || a.head_dim != b.head_dim || a.dtype != b.dtype || a.layout != b.layout)
    return IC_EINVAL;  // the plan was made for another shape
  if (std::memcmp(&pool->tune, &plan->tune, sizeof(ic_tuning)) != 0) return IC_EINVAL;  // or another launch plan
  if (misaligned(dev_q) || misaligned(dev_out)) return IC_EALIGN;
  return launch_attention(pool, plan->ps, plan->scale, dev_q, dev_out, plan->ws, (hipStream_t)hip_stream);
}

int kv_write_span_planned(ic_pool* pool, const ic_plan* plan, const void* dev_k_new, const void* dev_v_new,
                          void* hip_stream) {
  if (!pool || !plan || !dev_k_new || !dev_v_new) return IC_ENULL;
  const ic_pool_cfg &a = pool->cfg, &b = plan->cfg;
  if (a.num_blocks != b.num_blocks || a.block_size != b.block_size || a.num_heads != b.num_heads ||
      a.num_kv_heads != b.num_kv_heads || a.head_dim != b.head_dim || a.dtype != b.dtype || a.layout != b.layout)
    return IC_EINVAL;
  if (!plan->append_checked) return IC_EDUP;
  if (misaligned(dev_k_new) || misaligned(dev_v_new)) return IC_EALIGN;
  hipStream_t st = (hipStream_t)hip_stream;
  ProfScope ps_(pool, IC_K_APPEND, st);
  const hipError_t e = launch_append(pool->base, dev_k_new, dev_v_new, (const int32_t*)(plan->ws + plan->ps.off_row_dst),
                                     plan->total_q_rows, a.num_kv_heads, a.head_dim, st);
  return e == hipSuccess ? IC_OK : IC_EHIP;
}

int paged_attn_plan_destroy(ic_plan* plan) {
  if (!plan) return IC_ENULL;
  delete plan;
  return IC_OK;
}

// The pool's device-side int32 list (block ids of a swap, row destinations of an append).
static int ensure_dev_list(ic_pool* pool, int which, size_t bytes) {
  ic_pool::DevList& dl = pool->lists[which];
  if (dl.cap >= bytes) return IC_OK;
  const size_t cap = std::max(align_up(bytes, 4096), dev_list_bytes(pool, which));
  int32_t* fresh = nullptr;
  if (hipMalloc((void**)&fresh, cap) != hipSuccess) return IC_EHIP;
  if (dl.dev) pool->retired_dev.push_back(dl.dev);  // earlier launches may still read it
  dl.dev = fresh;
  dl.cap = cap;
  dl.held.clear();
  return IC_OK;
}

// Bring `n` ints into the pool's device list `which` on `st`, unless it holds exactly these already.
static int upload_list(ic_pool* pool, int which, const int32_t* host, size_t n, bool checked, hipStream_t st) {
  ic_pool::DevList& dl = pool->lists[which];
  const size_t bytes = align_up(sizeof(int32_t) * n, 16);
  int rc = ensure_dev_list(pool, which, bytes);
  if (rc != IC_OK) return rc;
  if (dl.held.size() == n && std::memcmp(dl.held.data(), host, sizeof(int32_t) * n) == 0) {
    dl.checked = dl.checked || checked;
    return IC_OK;
  }
  dl.held.clear();  // whatever fails below, the device copy is no longer known
  dl.checked = checked;
  StagingSlot* slot = nullptr;
  if ((rc = acquire_slot(pool, bytes, &slot)) != IC_OK) return rc;
  std::memcpy(slot->host, host, sizeof(int32_t) * n);
  std::memset((char*)slot->host + sizeof(int32_t) * n, 0xff, bytes - sizeof(int32_t) * n);
  {
    ProfScope ps_(pool, IC_K_UPLOAD, st);
    if (launch_upload(dl.dev, slot->host, bytes, st) != hipSuccess) return IC_EHIP;
  }
  if (hipEventRecord(slot->ev, st) != hipSuccess) return IC_EHIP;
  slot->pending = true;
  dl.held.assign(host, host + n);
  return IC_OK;
}

// The device list holds exactly these ints and they have passed the host checks.
static bool list_is_held(const ic_pool* pool, int which, const int32_t* host, size_t n) {
  const ic_pool::DevList& dl = pool->lists[which];
  return dl.checked && dl.held.size() == n && std::memcmp(dl.held.data(), host, sizeof(int32_t) * n) == 0;
}

static int swap_common(ic_pool* pool, const int32_t* host_ids, int32_t n, const void* dev_staging,
                       size_t staging_bytes, void* hip_stream, bool pack) {
  if (!pool) return IC_ENULL;
  if (n < 0) return IC_EINVAL;
  if (n == 0) return IC_OK;
  if (!host_ids || !dev_staging) return IC_ENULL;
  return guarded([&]() -> int {
  const int which = pack ? kListPack : kListUnpack;
  // a list the device copy already holds has passed these checks
  int rc = list_is_held(pool, which, host_ids, (size_t)n) ? IC_OK : check_ids(pool->cfg, host_ids, n, !pack);
  if (rc != IC_OK) return rc;
  if (misaligned(dev_staging)) return IC_EALIGN;
  if (staging_bytes / pool->block_bytes < (size_t)n) return IC_ESIZE;
  {  // staging must not overlap the pool
    const char* s0 = (const char*)dev_staging;
    const char* s1 = s0 + (size_t)n * pool->block_bytes;
    if (s0 < pool->base + pool->bytes && pool->base < s1) return IC_EINVAL;
  }
  hipStream_t st = (hipStream_t)hip_stream;
  if ((rc = upload_list(pool, which, host_ids, (size_t)n, true, st)) != IC_OK) return rc;
  const int32_t* dev_ids = pool->lists[which].dev;
  hipError_t e;
  {
    ProfScope ps_(pool, pack ? IC_K_PACK : IC_K_UNPACK, st);
    e = pack ? launch_pack(pool->base, (void*)dev_staging, dev_ids, n, pool->block_bytes, st)
             : launch_unpack(pool->base, dev_staging, dev_ids, n, pool->block_bytes, st);
  }
  return e == hipSuccess ? IC_OK : IC_EHIP;
  });
}

int kv_pack_blocks(ic_pool* pool, const int32_t* host_ids, int32_t n, void* dev_staging,
                   size_t staging_bytes, void* hip_stream) {
  return swap_common(pool, host_ids, n, dev_staging, staging_bytes, hip_stream, true);
}

int kv_unpack_blocks(ic_pool* pool, const int32_t* host_ids, int32_t n, const void* dev_staging,
                     size_t staging_bytes, void* hip_stream) {
  return swap_common(pool, host_ids, n, dev_staging, staging_bytes, hip_stream, false);
}

int kv_write_span(ic_pool* pool, const ic_batch_desc* desc, const void* dev_k_new, const void* dev_v_new,
                  void* hip_stream) {
  if (!pool || !desc || !dev_k_new || !dev_v_new) return IC_ENULL;
  return guarded([&]() -> int {
  const bool trusted = (desc->flags & IC_FLAG_TRUSTED) != 0;
  int rc = check_batch(pool->cfg, desc, trusted);
  if (rc != IC_OK) return rc;
  if (misaligned(dev_k_new) || misaligned(dev_v_new)) return IC_EALIGN;
  const size_t rows = (size_t)desc->total_q_rows;
  std::vector<int32_t> dst(rows, -1);
  append_destinations(desc, dst.data());
  if (!trusted && !list_is_held(pool, kListAppend, dst.data(), rows) && !destinations_distinct(pool->cfg, dst.data(), rows))
    return IC_EDUP;
  hipStream_t st = (hipStream_t)hip_stream;
  if ((rc = upload_list(pool, kListAppend, dst.data(), rows, !trusted, st)) != IC_OK) return rc;
  hipError_t e;
  {
    ProfScope ps_(pool, IC_K_APPEND, st);
    e = launch_append(pool->base, dev_k_new, dev_v_new, pool->lists[kListAppend].dev, desc->total_q_rows,
                      pool->cfg.num_kv_heads, pool->cfg.head_dim, st);
  }
  return e == hipSuccess ? IC_OK : IC_EHIP;
  });
}

int ic_prof_begin(ic_pool* pool, int32_t max_launches) {
  if (!pool) return IC_ENULL;
  if (max_launches < 1 || max_launches > (1 << 20)) return IC_EINVAL;
  return guarded([&]() -> int {
    ProfState& pr = pool->prof;
    pr.ev.reserve((size_t)max_launches * 2);
    while (pr.ev.size() < (size_t)max_launches * 2) {
      hipEvent_t e;
      if (hipEventCreate(&e) != hipSuccess) return IC_EHIP;
      pr.ev.push_back(e);
    }
    pr.kind.assign(pr.ev.size() / 2, 0);
    pr.used = 0;
    pr.on = true;
    return IC_OK;
  });
}

int ic_prof_end(ic_pool* pool, ic_prof_stats* out) {
  if (!pool || !out) return IC_ENULL;
  ProfState& pr = pool->prof;
  std::memset(out, 0, sizeof *out);
  pr.on = false;
  for (int i = 0; i < pr.used; ++i) {
    if (hipEventSynchronize(pr.ev[2 * i + 1]) != hipSuccess) return IC_EHIP;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, pr.ev[2 * i], pr.ev[2 * i + 1]) != hipSuccess) return IC_EHIP;
    const int k = pr.kind[i];
    if (out->launches[k] == 0 || ms < out->min_ms[k]) out->min_ms[k] = ms;
    if (out->launches[k] == 0 || ms > out->max_ms[k]) out->max_ms[k] = ms;
    out->launches[k] += 1;
    out->total_ms[k] += ms;
  }
  pr.used = 0;
  return IC_OK;
}

}  // extern "C"

// Layer-pipelined, chunked swap between the layers' paged pools and pinned host memory
// (Section 4.1: swap pipelining and swap chunking).  Host-side orchestration only: the bytes are
// moved by the block gather / scatter kernels of kv_swap.hip and by the copy engines.
//
// Two streams of default priority, one per direction, each running its layers in order:
//   out:  gather(pool_l -> stage), copy stage -> host, [record free(stage), done_l], next layer
//   in:   copy host -> stage, scatter(stage -> pool_l), [record free(stage), done_l], next layer
// Nothing is ordered against the caller's stream except at the start of a call, so the whole
// swap runs behind the forward pass, and the two directions (the link is full duplex, with a DMA
// engine each way) run beside each other.  Within one direction the gather kernel of layer l+1
// does not overlap the transfer of layer l: it takes under 2 % of the transfer's time, and a
// stream of its own would be the process's fifth (caller's, the attention call's side stream,
// these two).  With the default of four hardware queues a fifth stream shares a queue with
// another, and the attention call's tile kernel was measured waiting behind 3 ms transfers (call
// time doubled, swap rate halved).
// The staging buffers are handed out round-robin over both directions; free(stage) orders a
// buffer's next user, whichever stream that is, after its last one.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>

#include "ic_internal.h"

using namespace ic;

namespace {

constexpr int kIdSlots = 4;  // id lists in flight before a call has to wait for an old one

struct IdSlot {
  int32_t* host = nullptr;  // pinned mirror, max_blocks entries
  hipEvent_t ev = nullptr;  // recorded after the last kernel that reads the device copy
  bool pending = false;
};

struct Stage {
  hipEvent_t free_ = nullptr;  // the buffer's last user is through with it
  hipStream_t last = nullptr;  // the stream that recorded free_ (no wait needed from the same one)
  bool used = false;
};

bool misaligned16(const void* p) { return ((uintptr_t)p & 15u) != 0; }

bool same_shape(const ic_pool_cfg& a, const ic_pool_cfg& b) {
  return a.num_blocks == b.num_blocks && a.block_size == b.block_size && a.num_heads == b.num_heads &&
         a.num_kv_heads == b.num_kv_heads && a.head_dim == b.head_dim && a.dtype == b.dtype &&
         a.layout == b.layout;
}

// Pageable memory would turn every copy into a blocking, staged one.
int check_pinned(const void* p) {
  hipPointerAttribute_t a;
  std::memset(&a, 0, sizeof a);
  if (hipPointerGetAttributes(&a, p) != hipSuccess) {
    (void)hipGetLastError();  // the failed query must not surface in a later call
    return IC_EUNSUPPORTED;
  }
  return a.type == hipMemoryTypeHost ? IC_OK : IC_EUNSUPPORTED;
}

}  // namespace

struct ic_swapper {
  ic_swapper_cfg cfg;
  std::vector<ic_pool*> pools;
  std::vector<PoolView> views;
  size_t block_bytes = 0;
  char* staging = nullptr;
  size_t stage_bytes = 0;  // one staging buffer
  // runtime state, created by the first swap
  bool live = false;
  hipStream_t s_out = nullptr, s_in = nullptr;
  hipEvent_t ev_start = nullptr;
  std::vector<Stage> stages;
  int next_stage = 0;
  IdSlot ids[kIdSlots];
  int32_t* dev_ids = nullptr;  // kIdSlots lists of max_blocks
  int next_ids = 0;
  std::vector<hipEvent_t> done[2];
  std::vector<uint8_t> done_set[2];
};

namespace {

// Every object is created only if it is still missing, so a call that failed half-way is completed,
// not repeated, by the next one.
int init_runtime(ic_swapper* sw) {
  if (sw->live) return IC_OK;
  if (!sw->s_out && hipStreamCreateWithFlags(&sw->s_out, hipStreamNonBlocking) != hipSuccess) return IC_EHIP;
  if (!sw->s_in && hipStreamCreateWithFlags(&sw->s_in, hipStreamNonBlocking) != hipSuccess) return IC_EHIP;
  if (!sw->ev_start && hipEventCreateWithFlags(&sw->ev_start, hipEventDisableTiming) != hipSuccess) return IC_EHIP;
  for (Stage& s : sw->stages) {
    if (!s.free_ && hipEventCreateWithFlags(&s.free_, hipEventDisableTiming) != hipSuccess) return IC_EHIP;
  }
  for (int d = 0; d < 2; ++d)
    for (hipEvent_t& e : sw->done[d])
      if (!e && hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return IC_EHIP;
  const size_t list_bytes = (sizeof(int32_t) * (size_t)sw->cfg.max_blocks + 15) / 16 * 16;
  if (!sw->dev_ids && hipMalloc((void**)&sw->dev_ids, list_bytes * kIdSlots) != hipSuccess) return IC_EHIP;
  for (IdSlot& s : sw->ids) {
    if (!s.host && hipHostMalloc((void**)&s.host, list_bytes, hipHostMallocDefault) != hipSuccess) return IC_EHIP;
    if (!s.ev && hipEventCreateWithFlags(&s.ev, hipEventDisableTiming) != hipSuccess) return IC_EHIP;
  }
  sw->live = true;
  return IC_OK;
}

// Everything that can be checked without touching the GPU.
int check_call(const ic_swapper* sw, const int32_t* host_ids, int32_t n, const void* host,
               size_t layer_stride, bool distinct) {
  if (!sw) return IC_ENULL;
  if (n < 0 || n > sw->cfg.max_blocks) return IC_EINVAL;
  if (n == 0) return IC_OK;
  if (!host_ids || !host) return IC_ENULL;
  const int rc = ic_check_ids(&sw->views[0].cfg, host_ids, n, distinct ? 1 : 0);
  if (rc != IC_OK) return rc;
  if (layer_stride / sw->block_bytes < (size_t)n) return IC_ESIZE;
  if (misaligned16(host) || (layer_stride & 15u)) return IC_EALIGN;
  return IC_OK;
}

// One layer's blocks across the host link.  Issued as a pitched copy of n rows of one block each:
// the runtime hands pitched copies that touch host memory to the DMA engines, whereas it may run a
// flat hipMemcpyAsync as a copy kernel of one 8-wave workgroup per CU that stays resident for the
// whole transfer and takes registers the attention kernels count on (measured: attention calls
// running beside such copies took 1.8x as long).
hipError_t link_copy(void* dst, const void* src, size_t block_bytes, int32_t n, hipMemcpyKind kind,
                     hipStream_t st) {
  return hipMemcpy2DAsync(dst, block_bytes, src, block_bytes, block_bytes, (size_t)n, kind, st);
}

// Copy the id list to the device on st; *dev receives the device copy, *slot the ring entry whose
// event the caller records after its last kernel.
int upload_ids(ic_swapper* sw, hipStream_t st, const int32_t* host_ids, int32_t n, int32_t** dev, IdSlot** slot) {
  const int k = sw->next_ids;
  sw->next_ids = (k + 1) % kIdSlots;
  IdSlot& s = sw->ids[k];
  if (s.pending) {
    if (hipEventSynchronize(s.ev) != hipSuccess) return IC_EHIP;
    s.pending = false;
  }
  std::memcpy(s.host, host_ids, sizeof(int32_t) * (size_t)n);
  int32_t* d = sw->dev_ids + (size_t)k * ((sw->cfg.max_blocks + 3) / 4 * 4);
  const size_t padded = (sizeof(int32_t) * (size_t)n + 15) / 16 * 16;
  if (launch_upload(d, s.host, padded, st) != hipSuccess) return IC_EHIP;
  *dev = d;
  *slot = &s;
  return IC_OK;
}

}  // namespace

extern "C" {

size_t ic_swapper_staging_bytes(const ic_swapper_cfg* cfg, const ic_pool* pool0) {
  if (!cfg || !pool0) return 0;
  if (cfg->num_layers < 1 || cfg->max_blocks < 1 || cfg->num_stages < 2 || cfg->num_stages > 8 || cfg->reserved)
    return 0;
  return (size_t)cfg->num_stages * (size_t)cfg->max_blocks * kv_block_bytes(pool0);
}

int ic_swapper_create(const ic_swapper_cfg* cfg, ic_pool* const* layer_pools, void* dev_staging,
                      size_t staging_bytes, ic_swapper** out) {
  if (!cfg || !layer_pools || !dev_staging || !out) return IC_ENULL;
  if (cfg->num_layers < 1 || cfg->num_layers > 4096 || cfg->max_blocks < 1 || cfg->num_stages < 2 ||
      cfg->num_stages > 8 || cfg->reserved)
    return IC_EINVAL;
  for (int l = 0; l < cfg->num_layers; ++l)
    if (!layer_pools[l]) return IC_ENULL;
  const PoolView v0 = pool_view(layer_pools[0]);
  if (cfg->max_blocks > v0.cfg.num_blocks) return IC_EINVAL;
  if (misaligned16(dev_staging)) return IC_EALIGN;
  const size_t stage_bytes = (size_t)cfg->max_blocks * v0.block_bytes;
  if (staging_bytes / stage_bytes < (size_t)cfg->num_stages) return IC_ESIZE;
  ic_swapper* sw = new (std::nothrow) ic_swapper();
  if (!sw) return IC_ENOMEM;
  sw->cfg = *cfg;
  const char* s0 = (const char*)dev_staging;
  const char* s1 = s0 + stage_bytes * cfg->num_stages;
  for (int l = 0; l < cfg->num_layers; ++l) {
    const PoolView v = pool_view(layer_pools[l]);
    if (!same_shape(v.cfg, v0.cfg) || (s0 < v.base + v.bytes && v.base < s1)) {
      delete sw;
      return IC_EINVAL;
    }
    sw->pools.push_back(layer_pools[l]);
    sw->views.push_back(v);
  }
  sw->block_bytes = v0.block_bytes;
  sw->staging = (char*)dev_staging;
  sw->stage_bytes = stage_bytes;
  sw->stages.resize((size_t)cfg->num_stages);
  for (int d = 0; d < 2; ++d) {
    sw->done[d].assign((size_t)cfg->num_layers, nullptr);
    sw->done_set[d].assign((size_t)cfg->num_layers, 0);
  }
  *out = sw;
  return IC_OK;
}

int ic_swapper_sync(ic_swapper* sw) {
  if (!sw) return IC_ENULL;
  if (!sw->live) return IC_OK;
  if (hipStreamSynchronize(sw->s_out) != hipSuccess) return IC_EHIP;
  if (hipStreamSynchronize(sw->s_in) != hipSuccess) return IC_EHIP;
  return IC_OK;
}

int ic_swapper_destroy(ic_swapper* sw) {
  if (!sw) return IC_ENULL;
  const int rc = ic_swapper_sync(sw);
  if (sw->s_out) (void)hipStreamDestroy(sw->s_out);
  if (sw->s_in) (void)hipStreamDestroy(sw->s_in);
  if (sw->ev_start) (void)hipEventDestroy(sw->ev_start);
  for (Stage& s : sw->stages) {
    if (s.free_) (void)hipEventDestroy(s.free_);
  }
  for (int d = 0; d < 2; ++d)
    for (hipEvent_t e : sw->done[d])
      if (e) (void)hipEventDestroy(e);
  for (IdSlot& s : sw->ids) {
    if (s.ev) (void)hipEventDestroy(s.ev);
    if (s.host) (void)hipHostFree(s.host);
  }
  if (sw->dev_ids) (void)hipFree(sw->dev_ids);
  delete sw;
  return rc;
}

int kv_swap_out_layers(ic_swapper* sw, const int32_t* host_ids, int32_t n, void* pinned_host_dst,
                       size_t layer_stride_bytes, void* after_stream) {
  int rc = check_call(sw, host_ids, n, pinned_host_dst, layer_stride_bytes, false);
  if (rc != IC_OK || n == 0) return rc;
  if ((rc = check_pinned(pinned_host_dst)) != IC_OK) return rc;
  if ((rc = init_runtime(sw)) != IC_OK) return rc;
  // the blocks' last writer has to be through before the first gather
  hipStream_t st = sw->s_out;
  if (hipEventRecord(sw->ev_start, (hipStream_t)after_stream) != hipSuccess) return IC_EHIP;
  if (hipStreamWaitEvent(st, sw->ev_start, 0) != hipSuccess) return IC_EHIP;
  int32_t* dev_ids = nullptr;
  IdSlot* slot = nullptr;
  if ((rc = upload_ids(sw, st, host_ids, n, &dev_ids, &slot)) != IC_OK) return rc;
  for (int l = 0; l < sw->cfg.num_layers; ++l) {
    const int si = sw->next_stage;
    sw->next_stage = (si + 1) % sw->cfg.num_stages;
    Stage& sg = sw->stages[si];
    char* buf = sw->staging + (size_t)si * sw->stage_bytes;
    if (sg.used && sg.last != st && hipStreamWaitEvent(st, sg.free_, 0) != hipSuccess) return IC_EHIP;
    if (launch_pack(sw->views[l].base, buf, dev_ids, n, sw->block_bytes, st) != hipSuccess) return IC_EHIP;
    if (link_copy((char*)pinned_host_dst + (size_t)l * layer_stride_bytes, buf, sw->block_bytes, n,
                  hipMemcpyDeviceToHost, st) != hipSuccess)
      return IC_EHIP;
    if (hipEventRecord(sg.free_, st) != hipSuccess) return IC_EHIP;
    sg.used = true;
    sg.last = st;
    if (hipEventRecord(sw->done[IC_SWAP_OUT][l], st) != hipSuccess) return IC_EHIP;
    sw->done_set[IC_SWAP_OUT][l] = 1;
  }
  if (hipEventRecord(slot->ev, st) != hipSuccess) return IC_EHIP;
  slot->pending = true;
  return IC_OK;
}

int kv_swap_in_layers(ic_swapper* sw, const int32_t* host_ids, int32_t n, const void* pinned_host_src,
                      size_t layer_stride_bytes, void* after_stream) {
  int rc = check_call(sw, host_ids, n, pinned_host_src, layer_stride_bytes, true);
  if (rc != IC_OK || n == 0) return rc;
  if ((rc = check_pinned(pinned_host_src)) != IC_OK) return rc;
  if ((rc = init_runtime(sw)) != IC_OK) return rc;
  // whoever last used the destination blocks has to be through before the first scatter
  hipStream_t st = sw->s_in;
  if (hipEventRecord(sw->ev_start, (hipStream_t)after_stream) != hipSuccess) return IC_EHIP;
  if (hipStreamWaitEvent(st, sw->ev_start, 0) != hipSuccess) return IC_EHIP;
  int32_t* dev_ids = nullptr;
  IdSlot* slot = nullptr;
  if ((rc = upload_ids(sw, st, host_ids, n, &dev_ids, &slot)) != IC_OK) return rc;
  for (int l = 0; l < sw->cfg.num_layers; ++l) {
    const int si = sw->next_stage;
    sw->next_stage = (si + 1) % sw->cfg.num_stages;
    Stage& sg = sw->stages[si];
    char* buf = sw->staging + (size_t)si * sw->stage_bytes;
    if (sg.used && sg.last != st && hipStreamWaitEvent(st, sg.free_, 0) != hipSuccess) return IC_EHIP;
    if (link_copy(buf, (const char*)pinned_host_src + (size_t)l * layer_stride_bytes, sw->block_bytes, n,
                  hipMemcpyHostToDevice, st) != hipSuccess)
      return IC_EHIP;
    if (launch_unpack(sw->views[l].base, buf, dev_ids, n, sw->block_bytes, st) != hipSuccess) return IC_EHIP;
    if (hipEventRecord(sg.free_, st) != hipSuccess) return IC_EHIP;
    sg.used = true;
    sg.last = st;
    if (hipEventRecord(sw->done[IC_SWAP_IN][l], st) != hipSuccess) return IC_EHIP;
    sw->done_set[IC_SWAP_IN][l] = 1;
  }
  if (hipEventRecord(slot->ev, st) != hipSuccess) return IC_EHIP;
  slot->pending = true;
  return IC_OK;
}

int ic_swapper_wait_layer(ic_swapper* sw, int32_t direction, int32_t layer, void* hip_stream) {
  if (!sw) return IC_ENULL;
  if ((direction != IC_SWAP_OUT && direction != IC_SWAP_IN) || layer < 0 || layer >= sw->cfg.num_layers)
    return IC_EINVAL;
  if (!sw->live || !sw->done_set[direction][layer]) return IC_OK;  // nothing was ever queued
  return hipStreamWaitEvent((hipStream_t)hip_stream, sw->done[direction][layer], 0) == hipSuccess ? IC_OK : IC_EHIP;
}

int ic_swapper_sync_layer(ic_swapper* sw, int32_t direction, int32_t layer) {
  if (!sw) return IC_ENULL;
  if ((direction != IC_SWAP_OUT && direction != IC_SWAP_IN) || layer < 0 || layer >= sw->cfg.num_layers)
    return IC_EINVAL;
  if (!sw->live || !sw->done_set[direction][layer]) return IC_OK;
  return hipEventSynchronize(sw->done[direction][layer]) == hipSuccess ? IC_OK : IC_EHIP;
}

void* ic_host_alloc(size_t bytes) {
  void* p = nullptr;
  if (bytes == 0 || hipHostMalloc(&p, bytes, hipHostMallocDefault) != hipSuccess) {
    (void)hipGetLastError();
    return nullptr;
  }
  return p;
}

int ic_host_free(void* p) {
  if (!p) return IC_OK;
  return hipHostFree(p) == hipSuccess ? IC_OK : IC_EHIP;
}

int64_t ic_swap_limit_tokens(double t_fwd_s, double link_bytes_per_s, double token_bytes) {
  if (!(t_fwd_s >= 0.0) || !(link_bytes_per_s > 0.0) || !(token_bytes > 0.0)) return -1;
  const double tokens = std::floor(t_fwd_s * link_bytes_per_s / token_bytes);
  return tokens > 9.0e18 ? INT64_MAX : (int64_t)tokens;
}

int64_t ic_swap_schedule(int64_t total_blocks, int32_t block_size, const int64_t* limits, int64_t n_iters,
                         int64_t* out_blocks) {
  if (total_blocks < 0 || block_size < 1 || n_iters < 0 || (n_iters > 0 && (!limits || !out_blocks))) return -1;
  for (int64_t i = 0; i < n_iters; ++i)
    if (limits[i] < 0) return -1;
  int64_t remaining = total_blocks, last = 0;
  for (int64_t i = 0; i < n_iters; ++i) {
    const int64_t take = std::min<int64_t>(remaining, limits[i] / block_size);
    out_blocks[i] = take;
    remaining -= take;
    if (take > 0) last = i + 1;
  }
  return remaining > 0 ? n_iters + 1 : last;
}

}  // extern "C"

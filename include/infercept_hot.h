/*
 * infercept_hot.h - C ABI of the MI355X (gfx950) hot path of InferCept's intercept handling.
 *
 * Three operations, all on ONE layer's paged KV cache on ONE GPU:
 *   paged_attn_mixed   attention for one iteration's mixed batch: decode sequences (one query
 *                      row) and recomputation chunks (many query rows) read K/V through block tables
 *   kv_pack_blocks     gather scattered cache blocks into a contiguous staging buffer  (swap-out)
 *   kv_unpack_blocks   scatter a contiguous staging buffer back into cache blocks      (swap-in)
 *
 * General rules
 *   - Every function returns IC_OK (0) or a negative IC_E* code.  Nothing aborts, throws or prints.
 *     Arguments are validated before any kernel is launched: on error no device memory was written.
 *   - "dev" pointers are device (HBM) addresses owned by the caller (for example a PyTorch tensor's
 *     data_ptr) and must be 16-byte aligned.  "host" pointers are ordinary host memory; the library
 *     copies what it needs before returning, so host arrays may be reused at once.
 *   - Calls are asynchronous on `hip_stream` (a hipStream_t passed as void*, NULL = default stream);
 *     the caller synchronises.  All calls that use one ic_pool must be issued on one stream, or be
 *     ordered by the caller: the pool owns small descriptor buffers that successive calls reuse.
 *   - One process, one device: the device current at the first GPU call of a pool is the pool's.
 */
#ifndef INFERCEPT_HOT_H
#define INFERCEPT_HOT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  IC_OK = 0,
  IC_ENULL = -1,        /* a required pointer is NULL                                   */
  IC_EINVAL = -2,       /* a size, length or count is out of its legal range            */
  IC_ERANGE = -3,       /* a block id lies outside [0, num_blocks)                      */
  IC_ESIZE = -4,        /* a caller buffer (pool, staging, workspace, table) is too small */
  IC_EALIGN = -5,       /* a device pointer is not 16-byte aligned                      */
  IC_EDUP = -6,         /* duplicate destination id in kv_unpack_blocks                 */
  IC_EUNSUPPORTED = -7, /* dtype, layout, head_dim, block size ... not built            */
  IC_EOVERLAP = -8,     /* query-row ranges of two sequences overlap or leave [0,total) */
  IC_EHIP = -9,         /* the HIP runtime reported an error                            */
  IC_ENOMEM = -10,      /* host allocation failed                                       */
  IC_ELIMIT = -11       /* more than the fixed capacity of an allocation-free entry point */
};

/* Human-readable text for a return code (static storage, never NULL). */
const char* ic_strerror(int code);

/* ------------------------------------------------------------------------------------------
 * The block pool (paper Section 3.1: the KV cache is virtual memory whose pages are physical
 * blocks anywhere in GPU memory; Section 3.2 calls the per-token footprint M).
 *
 * layout 0:  pool[block][kv][kv_head][slot][dim], kv = 0 for K and 1 for V, bf16.
 *   One block = block_size tokens of ONE layer = block_size * M bytes, contiguous, so a swap
 *   moves whole blocks; inside it each (kv, head) tile of block_size x head_dim is contiguous,
 *   so attention reads it with full-width coalesced loads.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
  int32_t num_blocks;   /* >= 1                                                          */
  int32_t block_size;   /* tokens per block; 16 is the only size built                   */
  int32_t num_heads;    /* query heads                                                   */
  int32_t num_kv_heads; /* K/V heads in the pool; divides num_heads.  Equal: multi-head attention;
                           fewer: grouped-query attention, query head h reads K/V head
                           h / (num_heads / num_kv_heads)                                */
  int32_t head_dim;     /* 64, 128 or 256                                                */
  int32_t dtype;        /* 0 = bf16                                                      */
  int32_t layout;       /* 0 = the layout above                                          */
} ic_pool_cfg;

typedef struct ic_pool ic_pool; /* opaque; created by kv_pool_init, freed by kv_pool_destroy */

/*
 * Describe caller-owned pool memory to the library.  dev_pool_base: device, >= num_blocks *
 * block bytes (IC_ESIZE otherwise), 16-byte aligned.  Allocates no KV memory and touches no GPU
 * state.  The pool's own buffers are created by the first GPU call that needs them, sized from the
 * pool's shape so that later calls allocate nothing: four pinned host buffers for descriptors
 * (256 KiB + 8 bytes per block each) and three device int lists (block ids of a pack and of an
 * unpack: one int per block each; row destinations of an append: one int per cache slot).  Each
 * list remembers what it holds: a call whose list equals the previous one of its kind (the same
 * blocks moved for every layer of a model) uploads nothing.  A call that needs more (block tables that share blocks many times over, a pack list with
 * many duplicates, more query rows than cache slots) allocates a larger buffer and keeps the old one
 * until kv_pool_destroy; no call waits for the device.
 */
int kv_pool_init(const ic_pool_cfg* cfg, void* dev_pool_base, size_t pool_bytes, ic_pool** out);
int kv_pool_destroy(ic_pool* pool); /* frees library-owned buffers; never the KV memory */

/* block_size * 2 * num_kv_heads * head_dim * 2 bytes (K and V of one layer's block); 0 if pool is NULL. */
size_t kv_block_bytes(const ic_pool* pool);

/* ------------------------------------------------------------------------------------------
 * Mixed-batch paged attention (Section 4.2: decoding and recomputation have complementary
 * needs, so one iteration batches running requests' single decode tokens with one chunk of
 * each resumed request's discarded context; Section 4.3: a partially recomputed request keeps
 * its remaining tokens for later iterations).
 *
 * For sequence s and row i of its query span (0 <= i < q_len[s]) the row sits at absolute
 * position p = ctx_len[s] - q_len[s] + i and
 *      out[q_start[s] + i][h][:] = softmax_t( scale * q[q_start[s] + i][h] . K_t[h] ) V_t[h],  t = 0..p
 * where token t lives in block block_tables[s][t / block_size], slot t % block_size.  The span's
 * own K/V are already in the cache.  fp32 accumulation, bf16 result (round to nearest even).
 * Slots at t >= ctx_len[s], table entries past ceil(ctx_len/block_size) and unreferenced blocks
 * are never allowed to influence the result (they may hold NaN).
 * ------------------------------------------------------------------------------------------ */
enum {
  IC_FLAG_TRUSTED = 1 /* skip the O(total blocks) host checks of ids and row ranges (timing loops) */
};

typedef struct {
  int32_t num_seqs;           /* >= 1                                                          */
  const int32_t* ctx_len;     /* host [num_seqs]  KV tokens visible, INCLUDING the span's own  */
  const int32_t* q_len;       /* host [num_seqs]  1 = decode, >1 = recomputation chunk; 1..ctx_len */
  const int32_t* q_start;     /* host [num_seqs]  first row of the sequence in packed q / out  */
  const int32_t* block_tables;/* host [num_seqs][max_blocks_per_seq] row-major                 */
  int32_t max_blocks_per_seq; /* row stride of block_tables                                    */
  int32_t total_q_rows;       /* rows of q / out; every [q_start, q_start+q_len) inside, disjoint */
  float scale;                /* softmax scale, 1/sqrt(head_dim) in the usual case; finite and > 0
                                 (IC_EINVAL otherwise: the kernels fold it into the exponent after the
                                 row maximum is taken, which needs a positive factor)          */
  uint32_t flags;             /* IC_FLAG_*                                                     */
} ic_batch_desc;

/* Bytes of device workspace paged_attn_mixed needs for this batch (descriptor copy + split-KV
 * partial results); 0 if an argument is NULL or the descriptor is invalid. */
size_t paged_attn_mixed_workspace_bytes(const ic_pool* pool, const ic_batch_desc* desc);

/*
 * dev_q, dev_out: device bf16 [total_q_rows][num_heads][head_dim].  dev_workspace: device, 256-byte
 * aligned (IC_EALIGN otherwise; device allocators return such addresses), at least
 * paged_attn_mixed_workspace_bytes() (IC_ESIZE otherwise); its contents are scratch.
 * Deterministic: the same inputs give the same bits on every call.
 */
int paged_attn_mixed(ic_pool* pool, const ic_batch_desc* desc, const void* dev_q, void* dev_out,
                     void* dev_workspace, size_t workspace_bytes, void* hip_stream);

/*
 * KV append (Section 4.2: a recomputation chunk joins the batch; Section 4.3: a partly recomputed
 * request continues in later iterations, so what one chunk computes must be in the cache for the
 * next).  Writes the keys and values computed for this iteration's query positions into the paged
 * cache: for every sequence s and row i < q_len[s], position t = ctx_len[s] - q_len[s] + i,
 *      pool[block_tables[s][t / block_size]][K|V][h][t % block_size][:] = k_new|v_new[q_start[s] + i][h][:]
 * for decode sequences (q_len = 1: the new token) and chunks alike.  It is the step before
 * paged_attn_mixed on the same descriptor, on the same stream.  dev_k_new, dev_v_new: device bf16
 * [total_q_rows][num_kv_heads][head_dim]; rows no sequence owns are ignored.  Byte-exact; every
 * other slot of the cache keeps its bytes.  Two rows that address one slot (sequences sharing a
 * block they both write) give IC_EDUP; IC_FLAG_TRUSTED skips that check and the id checks.
 */
int kv_write_span(ic_pool* pool, const ic_batch_desc* desc, const void* dev_k_new, const void* dev_v_new,
                  void* hip_stream);

/*
 * Plan once, run for every layer.  One iteration's batch (Section 4.3) is the same for all layers of
 * the model; only the cache (one pool per layer), q and out change.  paged_attn_plan_create validates
 * and plans the batch for `pool`'s shape and tuning and uploads the descriptor image into
 * dev_workspace on hip_stream; paged_attn_planned then runs the attention of any pool of that shape
 * and tuning (IC_EINVAL otherwise) with nothing but kernel launches.  The workspace belongs to the
 * plan until paged_attn_plan_destroy; its partial-result area is reused by every run, so runs of one
 * plan must be ordered on one stream (after the stream the plan was created on has passed the
 * upload).  dev_workspace as for paged_attn_mixed (256-byte aligned, at least its workspace bytes).
 * Results are those of paged_attn_mixed, bit for bit.
 */
typedef struct ic_plan ic_plan;
int paged_attn_plan_create(ic_pool* pool, const ic_batch_desc* desc, void* dev_workspace, size_t workspace_bytes,
                           void* hip_stream, ic_plan** out);
int paged_attn_planned(ic_pool* pool, const ic_plan* plan, const void* dev_q, void* dev_out, void* hip_stream);
/* kv_write_span from the same plan (the rows' destinations are part of the image).  IC_EDUP if the
 * plan's descriptor was not trusted and two of its rows address one cache slot. */
int kv_write_span_planned(ic_pool* pool, const ic_plan* plan, const void* dev_k_new, const void* dev_v_new,
                          void* hip_stream);
int paged_attn_plan_destroy(ic_plan* plan);

/* Host-only validation of a descriptor against a pool shape (what paged_attn_mixed checks when
 * IC_FLAG_TRUSTED is clear).  Touches no GPU state. */
int ic_check_batch(const ic_pool_cfg* cfg, const ic_batch_desc* desc);

/* Launch plan knobs.  Partition sizes are in tokens and are rounded up to a multiple of 64;
 * 0 keeps the built-in choice.  Smaller values force the split-KV path on short contexts. */
typedef struct {
  int32_t decode_part_tokens; /* keys per work item of a decode row (built-in: 4096)         */
  int32_t span_part_tokens;   /* keys per work item of a span's query tile (built-in: 8192, or no split at all
                                 when the unsplit tiles already give every CU four workgroups) */
  int32_t span_kernel;        /* 0 = built-in choice (spans: MFMA tiles; decode rows: vector kernel, or the MFMA
                                 group kernel in a grouped-query pool), 1 = everything row by row on the vector
                                 kernel, 2 = MFMA tiles, in a grouped-query pool also for decode rows */
  int32_t row_variant;        /* vector-kernel build: bit 0 = prefetch two tiles ahead, bit 1 = cached (not non-temporal) KV loads */
  int32_t serial_spans;       /* 1 = run the span kernel, then the row kernel, on the caller's stream instead of
                                 two persistent kernels side by side (the tile kernel on the pool's own stream) */
  int32_t row_launch;         /* single-role row kernel: 0 = built-in choice (persistent, one workgroup per CU),
                                 1 = one workgroup per work item, 2 = persistent, 3 = persistent, the slim
                                 builds that otherwise run beside the tile kernel (in a grouped-query pool of
                                 head_dim 128 with groups of up to 16: the slim group kernel)  */
  int32_t row_slots;          /* resident workgroups of the persistent row kernel (and of the slim group kernel);
                                 0 = one per CU */
  int32_t mfma_min_keys;      /* query rows that see fewer keys than this run on the vector kernel, which keeps the
                                 softmax weights in fp32 (the matrix-core kernels round them to bf16, and with a
                                 handful of keys one weight's rounding shows in the output); 0 = built-in 64,
                                 1 = no such routing, at most 64                              */
  int32_t reserved[1];        /* must be 0                                                   */
} ic_tuning;
int ic_pool_set_tuning(ic_pool* pool, const ic_tuning* tuning);

/* What the planner would launch for this batch (host only; for tests and reports). */
typedef struct {
  int32_t decode_rows, span_rows;      /* query rows handled by each path                     */
  int32_t row_items;                   /* work items of the vector (row) kernel, per head     */
  int32_t tile_items;                  /* work items of the MFMA tile kernel, per head        */
  int32_t partial_slots;               /* split-KV partial results, per head                  */
  int32_t merge_rows;                  /* rows that need the merge pass                       */
  int64_t table_entries;               /* block-table entries copied to the device            */
} ic_plan_info;
int ic_plan_query(const ic_pool* pool, const ic_batch_desc* desc, ic_plan_info* out);

/* Host-only inspection of the launch plan, so that the planner can be tested without a GPU: writes
 * into host_image the descriptor image paged_attn_mixed would upload for this batch under the
 * pool's current tuning, and describes its layout.  All sections are int32 arrays at the given byte
 * offsets: counters[16] (zero) | bt_off[num_seqs] | bt_flat[table_entries] (the sequences' block
 * ids, back to back) | row items | tile items | merge items | row_dst[total_q_rows].
 *   row item   (8 x int32): seq, qrow, k_begin, k_end, slot (-1: whole row, direct output), 0, 0, 0
 *              one query row against keys [k_begin, k_end) of its sequence, all heads
 *   tile item  (8 x int32): seq, qrow0, n_rows, pos0, k_begin, k_end, slot0 (-1: direct), nparts
 *              n_rows consecutive query rows from qrow0, the first at position pos0, against keys
 *              [k_begin, k_end) cut at each row's own position; partial slot of row r: slot0 + r * nparts
 *   merge item (4 x int32): qrow, slot0, nparts, 0   (the row's partial slots are slot0 .. slot0 + nparts - 1)
 *   row_dst    cache slot (block * block_size + slot in block) kv_write_span writes each query row's
 *              K/V to, -1 for rows no sequence owns
 * host_image may be NULL (layout only); otherwise host_bytes >= the image size (IC_ESIZE).  The
 * descriptor is validated in full.  Touches no GPU state.
 */
typedef struct {
  int64_t image_bytes;
  int64_t off_counters, off_bt_off, off_bt_flat, off_row_items, off_tile_items, off_merge_items, off_row_dst;
  int32_t row_part_tokens;   /* keys per row item                                             */
  int32_t span_part_tokens;  /* keys per tile item (2^30: spans are not split)                */
  int32_t tile_query_rows;   /* query rows per tile item                                      */
  int32_t tile_head_shift;   /* log2 of the query heads one tile workgroup serves             */
  int32_t n_row_items, n_tile_items, n_merge_items;
  int32_t n_vector_row_items; /* row items [0, n) run on the vector kernel, the rest on the group kernel */
} ic_plan_layout;
int ic_plan_image(const ic_pool* pool, const ic_batch_desc* desc, void* host_image, size_t host_bytes,
                  ic_plan_layout* out);

/* ------------------------------------------------------------------------------------------
 * Swap of scattered blocks (Section 3.2, swap-based approach: a paged context is scattered over
 * many discontinuous regions, and moving it with one launch per region is launch-bound;
 * Section 4.1 moves it layer by layer, a bounded number of tokens per iteration).  One call moves
 * one layer's K+V of the listed blocks in ONE launch; a chunk of the swap is a shorter id list.
 *
 *   kv_pack_blocks:    staging[i] <- pool[host_ids[i]]   i < n   (list order; duplicates allowed)
 *   kv_unpack_blocks:  pool[host_ids[i]] <- staging[i]   i < n   (ids must be distinct: IC_EDUP)
 * dev_staging: device, n * kv_block_bytes() bytes (IC_ESIZE if staging_bytes is smaller), must not
 * overlap the pool.  n = 0 succeeds and does nothing.  Byte-exact.
 * ------------------------------------------------------------------------------------------ */
int kv_pack_blocks(ic_pool* pool, const int32_t* host_ids, int32_t n, void* dev_staging,
                   size_t staging_bytes, void* hip_stream);
int kv_unpack_blocks(ic_pool* pool, const int32_t* host_ids, int32_t n, const void* dev_staging,
                     size_t staging_bytes, void* hip_stream);

/*
 * kv_pack_blocks for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same result, same checks (byte-exact; the staging
 * buffer is still the caller's).  What differs is where the device-side copy of the id list lives:
 * kv_pack_blocks keeps it in a buffer the library allocates and uploads it through pinned host
 * memory it allocates; this call keeps it in a fixed array inside the library's device image
 * (IC_STATIC_PACK_MAX_BLOCKS ints = 256 KiB on every GPU the library runs on, held until the process
 * ends) and sends the ids as kernel arguments, 960 per launch, ahead of the one gather launch.  It
 * calls no allocating routine of the HIP runtime or of any library, and touches no pool-owned buffer.
 * n > IC_STATIC_PACK_MAX_BLOCKS gives IC_ELIMIT (split the list, or use kv_pack_blocks).
 * Every call on one GPU uses that GPU's one array: calls ordered on one stream are safe (the array
 * is rewritten for each call, nothing of the previous list survives), calls that overlap on
 * different streams of one GPU race.
 */
#define IC_STATIC_PACK_MAX_BLOCKS 65536
int kv_pack_blocks_static(ic_pool* pool, const int32_t* host_ids, int32_t n, void* dev_staging,
                          size_t staging_bytes, void* hip_stream);

/* Host-only validation of an id list: range, and distinctness when require_distinct != 0. */
int ic_check_ids(const ic_pool_cfg* cfg, const int32_t* host_ids, int32_t n, int require_distinct);

/* ------------------------------------------------------------------------------------------
 * Layer-pipelined, chunked swap between the paged pools of a model's layers and pinned host memory
 * (Section 4.1).  Swap pipelining: one layer's swapping is one pipeline stage; the stages run on the
 * swapper's own streams, behind the caller's forward pass, which waits only for the layer it needs.
 * Swap chunking: one call moves only as many blocks as the iteration's swap limit allows
 * (ic_swap_limit_tokens), the rest of the sequence follows in later iterations (ic_swap_schedule).
 *
 * A swapper serves L pools of ONE shape (the L layers of a model; a multi-layer cache is L pools).
 * It owns two streams of default priority, one per direction (swap-out and swap-in run beside each
 * other), and cycles `num_stages` staging buffers, each max_blocks * kv_block_bytes() bytes, carved from the
 * caller's dev_staging.  Per layer l and list position i, with blk = kv_block_bytes():
 *   kv_swap_out_layers:  host[l * layer_stride + i * blk ..+blk) <- pool_l[host_ids[i]]
 *   kv_swap_in_layers:   pool_l[host_ids[i]] <- host[l * layer_stride + i * blk ..+blk)   (ids distinct)
 * `host` is pinned host memory (ic_host_alloc, or any hipHostMalloc'ed block; pageable memory is
 * refused with IC_EUNSUPPORTED: copies from it would not be asynchronous) and must stay valid and
 * unmodified until the layers are through.  Both calls return at once.  Work already queued on
 * `after_stream` (NULL = default stream) when the call is made finishes before the first byte moves:
 * pass the stream that wrote (swap-out) or last read (swap-in) the listed blocks.
 * Order later work with ic_swapper_wait_layer (a stream waits until layer l of the latest call in
 * that direction is through: for swap-in the layer's blocks are then readable, for swap-out they
 * may be reused), ic_swapper_sync_layer or ic_swapper_sync (the host waits).
 * One host thread drives a swapper.  Byte-exact.  n = 0 succeeds and does nothing.
 * ------------------------------------------------------------------------------------------ */
typedef struct ic_swapper ic_swapper;

typedef struct {
  int32_t num_layers; /* L >= 1                                                        */
  int32_t max_blocks; /* most blocks one call may move per layer, >= 1                 */
  int32_t num_stages; /* staging buffers cycled layer by layer, 2..8                   */
  int32_t reserved;   /* must be 0                                                     */
} ic_swapper_cfg;

enum { IC_SWAP_OUT = 0, IC_SWAP_IN = 1 };

/* num_stages * max_blocks * kv_block_bytes(pool0); 0 on a NULL or invalid argument. */
size_t ic_swapper_staging_bytes(const ic_swapper_cfg* cfg, const ic_pool* pool0);

/* layer_pools: host array of L pools with identical ic_pool_cfg (IC_EINVAL otherwise); they must
 * outlive the swapper.  dev_staging: device, 16-byte aligned, >= ic_swapper_staging_bytes(), not
 * overlapping any pool.  Touches no GPU state: streams and events are created by the first swap. */
int ic_swapper_create(const ic_swapper_cfg* cfg, ic_pool* const* layer_pools, void* dev_staging,
                      size_t staging_bytes, ic_swapper** out);
int ic_swapper_destroy(ic_swapper* sw); /* waits for queued swaps, frees library-owned buffers */

int kv_swap_out_layers(ic_swapper* sw, const int32_t* host_ids, int32_t n, void* pinned_host_dst,
                       size_t layer_stride_bytes, void* after_stream);
int kv_swap_in_layers(ic_swapper* sw, const int32_t* host_ids, int32_t n, const void* pinned_host_src,
                      size_t layer_stride_bytes, void* after_stream);

int ic_swapper_wait_layer(ic_swapper* sw, int32_t direction, int32_t layer, void* hip_stream);
int ic_swapper_sync_layer(ic_swapper* sw, int32_t direction, int32_t layer);
int ic_swapper_sync(ic_swapper* sw);

/* Pinned host memory for swap targets (hipHostMalloc / hipHostFree).  NULL on failure. */
void* ic_host_alloc(size_t bytes);
int ic_host_free(void* p);

/*
 * Swap limit N_i of Section 4.1: with T_swap(N) = N * token_bytes / link_bytes_per_s, the number of
 * tokens whose swap takes as long as the iteration's forward pass, T_swap(N_i) = t_fwd_s, rounded
 * down to whole tokens (computed as floor(t_fwd_s * link_bytes_per_s / token_bytes) in fp64).
 * token_bytes is M summed over the layers that move.  Returns -1 on arguments outside the model.
 */
int64_t ic_swap_limit_tokens(double t_fwd_s, double link_bytes_per_s, double token_bytes);

/*
 * Split the swap of total_blocks blocks over iterations whose limits (tokens) are limits[0..n):
 * iteration i moves min(blocks left, limits[i] / block_size) whole blocks into out_blocks[i].
 * Returns the iterations used, n_iters + 1 if the limits do not cover the whole swap, -1 on bad
 * arguments.  Host only.
 */
int64_t ic_swap_schedule(int64_t total_blocks, int32_t block_size, const int64_t* limits,
                         int64_t n_iters, int64_t* out_blocks);

/* ------------------------------------------------------------------------------------------
 * The scheduler's arithmetic (host only, fp64): the GPU-memory-waste model, chunk sizing, the
 * saturation point and the interception schedule.  Waste is in byte-seconds when token_bytes is M in
 * bytes and times are in seconds.
 *
 * T_fwd (Section 3.2) gives an iteration's execution time as a function of the tokens scheduled in its
 * batch; here it comes from profiling: n points (tokens[k], seconds[k]), tokens positive and strictly
 * increasing.  Between points it is evaluated on straight lines, below the first
 * point on the line from the origin, beyond the last on the last segment's line.  Functions that
 * take a table return NaN if it is malformed.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
  int32_t n;
  const double* tokens;
  const double* seconds;
} ic_tfwd_table;

double ic_tfwd_eval(const ic_tfwd_table* table, double tokens);

/* Eq. 1 (Section 3.2): T_fwd(C) * C * M + T_fwd(C) * C_other * M. */
double ic_waste_discard(const ic_tfwd_table* table, double ctx_tokens, double other_tokens, double token_bytes);
/* Eq. 2: T_INT * C * M. */
double ic_waste_preserve(double t_int_s, double ctx_tokens, double token_bytes);
/* Eq. 3: 2 * T_swap(C) * C_batch * M (a swap that stalls the batch, out and back in). */
double ic_waste_swap(double t_swap_s, double batch_tokens, double token_bytes);
/* Eq. 4 (Section 4.2): T_fwd(C) * C * M / 2 + n * T_fwd(C / n) * C_other * M; NaN if n_chunks < 1. */
double ic_waste_chunked_discard(const ic_tfwd_table* table, double ctx_tokens, double other_tokens,
                                double token_bytes, int32_t n_chunks);

/* Section 4.2: chunk size = saturation point S - running group size, never below 0; and the
 * iterations a context then needs, ceil(C / chunk) (-1 if chunk < 1 or C < 0). */
int64_t ic_chunk_tokens(int64_t saturation_point, int64_t running_tokens);
int64_t ic_chunk_count(int64_t ctx_tokens, int64_t chunk_tokens);

/*
 * Saturation point S (Section 4.2) from a profile of iteration time against query tokens (increasing):
 * the smallest profiled token count whose throughput tokens / seconds reaches `frac` (0 < frac <= 1,
 * e.g. 0.95) of the best throughput in the profile.  -1 on bad input.
 */
int64_t ic_saturation_point(const double* query_tokens, const double* seconds, int32_t n, double frac);

/*
 * Scheduling intercepted requests (Section 4.3).  Waste_i = min(waste_preserve[i],
 * waste_chunked_discard[i]) (Eq. 5); requests are swapped out in descending order of that waste (ties:
 * lower index first) until swap_out_budget_tokens is spent, the last one possibly in part.
 * swap_tokens[i] receives the tokens of request i to swap out, action[i] what to do with the rest
 * of its context: IC_ACT_NONE (nothing left), IC_ACT_PRESERVE or IC_ACT_DISCARD, whichever of its
 * two wastes is smaller (preserve on a tie).  Wastes must be >= 0 and not NaN (IC_EINVAL).
 */
enum { IC_ACT_NONE = 0, IC_ACT_PRESERVE = 1, IC_ACT_DISCARD = 2 };
int ic_schedule_intercepted(int32_t n, const double* waste_preserve, const double* waste_chunked_discard,
                            const int64_t* ctx_tokens, int64_t swap_out_budget_tokens, int64_t* swap_tokens,
                            int32_t* action);

#ifdef __cplusplus
}
#endif
#endif /* INFERCEPT_HOT_H */

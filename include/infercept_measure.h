/*
 * infercept_measure.h - measurement aids of libinfercept_hot.so.  None of this is part of the method
 * (include/infercept_hot.h is the method's contract): per-kernel event timing for roofline reports
 * and three probes that say what this GPU reaches on the access patterns the kernels use.
 * Same conventions as infercept_hot.h: plain pointers and sizes, IC_OK or a negative IC_E* code,
 * nothing aborts, throws or prints, validation before any launch.
 */
#ifndef INFERCEPT_MEASURE_H
#define INFERCEPT_MEASURE_H

#include "infercept_hot.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ------------------------------------------------------------------------------------------
 * Per-kernel timing with HIP events on the launch stream (for roofline reports).  Between
 * ic_prof_begin and ic_prof_end every kernel the pool launches is bracketed by an event pair.
 * ic_prof_end synchronises the recorded events and returns totals per kernel kind.
 * ------------------------------------------------------------------------------------------ */
enum { IC_K_ROW = 0, IC_K_TILE = 1, IC_K_MERGE = 2, IC_K_PACK = 3, IC_K_UNPACK = 4, IC_K_UPLOAD = 5, IC_K_APPEND = 6,
       IC_K_GROUP = 7, IC_K_COUNT = 8 };
/* IC_K_UPLOAD: the kernel that copies a call's descriptor from pinned host memory to the device. */
typedef struct {
  int32_t launches[IC_K_COUNT];
  float total_ms[IC_K_COUNT];
  float min_ms[IC_K_COUNT];
  float max_ms[IC_K_COUNT];
} ic_prof_stats;
int ic_prof_begin(ic_pool* pool, int32_t max_launches);
int ic_prof_end(ic_pool* pool, ic_prof_stats* out);

/* ------------------------------------------------------------------------------------------
 * Measurement aid for roofline reports (not part of the method): the rate an MFMA-only loop reaches
 * on this GPU with the caller's operand data.  256 workgroups of 8 waves each issue iters x 4
 * back-to-back independent v_mfma_f32_32x32x16_bf16 on register operands taken from dev_operands
 * (bf16 bit patterns; zeros, ones or random values, the caller chooses), with no memory traffic in
 * the loop.  With random operands the chip's power limit lowers the shader clock, so the result is
 * below the vendor peak; *shader_ghz is the average shader clock inside the loop (shader-clock
 * ticks over 100 MHz real-time ticks of workgroup 0).
 *   dev_operands  DEVICE, 16-byte aligned, >= IC_CEILING_OPERAND_BYTES, only read
 *   dev_sink      DEVICE, 16-byte aligned, >= IC_CEILING_SINK_BYTES, overwritten (results the
 *                 compiler must not drop, and the clock readings)
 *   iters         1 .. 2^24
 * Synchronous: launches on hip_stream and waits for it.  Errors: IC_ENULL, IC_EINVAL, IC_ESIZE,
 * IC_EALIGN, IC_EHIP; nothing is launched on a validation error.
 */
#define IC_CEILING_OPERAND_BYTES ((size_t)1 << 20)
#define IC_CEILING_SINK_BYTES ((size_t)256 * 512 * 4 + (size_t)256 * 16)
int ic_mfma_ceiling(const void* dev_operands, size_t operand_bytes, void* dev_sink, size_t sink_bytes,
                    int32_t iters, void* hip_stream, double* tflops, double* shader_ghz);

/* Measurement aid: what a plain streaming kernel reaches on this GPU, for scale next to the 8 TB/s
 * vendor figure.  mode 0 reads `bytes` of dev_src once per repetition (dev_dst: >= 16 bytes, may
 * receive one 16-byte word); mode 1 copies dev_src to dev_dst (`bytes` each).  One-wave workgroups
 * (1 KiB each for the copy, 8 KiB for the read), non-temporal loads and stores.  *gbps = bytes moved
 * (read, or read + written) per second over `reps` back-to-back launches, by HIP events on
 * hip_stream.  Synchronous.
 *   bytes: a multiple of 8192, at most 2^31 KiB; reps 1 .. 10000; the two ranges must not overlap.
 * Errors: IC_ENULL, IC_EINVAL, IC_EALIGN, IC_EHIP; nothing is launched on a validation error.
 */
int ic_hbm_ceiling(const void* dev_src, void* dev_dst, size_t bytes, int32_t mode, int32_t reps,
                   void* hip_stream, double* gbps);

/* Measurement aid: the streaming-read rate of the decode kernels' ACCESS PATTERN with the arithmetic
 * taken out.  One one-wave workgroup per (listed block, K/V head) loads that head's K tile and V tile
 * of the block (block_size x head_dim bf16 each, non-temporal 16-byte loads) and folds them into a
 * word.  *gbps = n * kv_block_bytes * reps bytes over the time of `reps` back-to-back launches.
 * host_ids: n block ids in [0, num_blocks), duplicates allowed; dev_sink: device, 16 bytes, may be
 * written.  Allocates and frees its own device copy of the id list.  Synchronous.
 * Errors: IC_ENULL, IC_EINVAL, IC_ERANGE, IC_EALIGN, IC_EHIP. */
int ic_paged_read_ceiling(const ic_pool* pool, const int32_t* host_ids, int32_t n, void* dev_sink,
                          int32_t reps, void* hip_stream, double* gbps);

#ifdef __cplusplus
}
#endif
#endif /* INFERCEPT_MEASURE_H */

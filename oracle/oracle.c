/*
 * CPU oracle for the intercept hot path: TEST INFRASTRUCTURE ONLY.
 *
 * Only the test-suite, the smoke check and the benchmark's cpu_baseline leg may
 * call this file.  It shares no code with the HIP library and is deliberately
 * plain: fp64 arithmetic, the textbook definition written out, two passes over
 * the keys (max, then sum) instead of an online softmax, no blocking and no
 * intrinsics.  The only parallelism is one OpenMP loop over (query row, head).
 *
 * What it defines
 *  - Paged attention (paper Section 3.1: the KV cache is virtual memory mapped
 *    to non-contiguous physical blocks): logical token t of a sequence lives in
 *    physical block block_table[t / B], slot t % B.
 *  - Mixed batches (Section 4.2): a decode sequence contributes one query row,
 *    a recomputation chunk contributes q_len rows.  Row i of a chunk sits at
 *    absolute position p = ctx_len - q_len + i and attends to keys 0..p
 *    inclusive, so that recomputing a context chunk by chunk over several
 *    iterations (Section 4.3, partially recomputed requests stay queued)
 *    reproduces what a one-shot causal prefill would have produced.
 *  - Swap of scattered blocks (Section 3.2, swap-based approach): gather the
 *    listed blocks into a contiguous staging buffer, and scatter them back.
 *  - KV append (Sections 4.2, 4.3): the keys and values of a chunk's own
 *    positions are written into the paged cache before the chunk attends.
 *  - Swap pipelining and chunking (Section 4.1): what a layer-by-layer swap of
 *    the listed blocks leaves in host memory / in the pools (the pipeline only
 *    changes WHEN bytes move, so the result is the per-layer gather / scatter),
 *    the swap limit N_i that solves T_swap(N_i) = T_fwd(B_i), and the split of
 *    one sequence's swap over iterations under those limits.
 *
 *  - The GPU-memory-waste model (Eq. 1-5), the saturation point and the
 *    interception schedule (Sections 3.2, 4.2, 4.3).
 *
 * The attention formula itself is not printed in the paper (it inherits the
 * serving stack's kernels, Section 4.5); it is the standard scaled dot-product
 * causal attention  out = softmax(scale * q K^T) V.
 *
 * Pool layout (layout 0): [block][K=0 / V=1][head][slot][dim], bf16 bit patterns.
 * Every pinned property of this file is listed in tests/test_oracle_pins.py.
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double bf16_bits_to_double(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* address of element (block, kv, head, slot, 0) */
static const uint16_t *kv_row(const uint16_t *pool, int64_t block, int kv, int head, int slot,
                              int H, int B, int D)
{
    int64_t idx = ((((block * 2 + kv) * H + head) * (int64_t)B + slot) * (int64_t)D);
    return pool + idx;
}

/*
 * One (query row, head): returns 0, or -1 if scratch allocation fails.
 *   p        absolute position of the row (keys 0..p are visible)
 *   table    block table of the row's sequence
 *   qrow     D bf16 values of the query for this head
 *   out      D doubles
 */
static int attend_one(const uint16_t *pool, int H, int B, int D, const int32_t *table, int head,
                      int64_t p, const uint16_t *qrow, double scale, double *out)
{
    int64_t nkeys = p + 1;
    double *score = (double *)malloc(sizeof(double) * (size_t)nkeys);
    if (!score) return -1;

    /* pass 1: scores and their maximum */
    double smax = -INFINITY;
    for (int64_t t = 0; t < nkeys; ++t) {
        const uint16_t *k = kv_row(pool, table[t / B], 0, head, (int)(t % B), H, B, D);
        double dot = 0.0;
        for (int d = 0; d < D; ++d) dot += bf16_bits_to_double(qrow[d]) * bf16_bits_to_double(k[d]);
        score[t] = scale * dot;
        if (score[t] > smax) smax = score[t];
    }
    /* pass 2: normaliser */
    double denom = 0.0;
    for (int64_t t = 0; t < nkeys; ++t) {
        score[t] = exp(score[t] - smax);
        denom += score[t];
    }
    /* weighted sum of values */
    for (int d = 0; d < D; ++d) out[d] = 0.0;
    for (int64_t t = 0; t < nkeys; ++t) {
        const uint16_t *v = kv_row(pool, table[t / B], 1, head, (int)(t % B), H, B, D);
        double w = score[t] / denom;
        for (int d = 0; d < D; ++d) out[d] += w * bf16_bits_to_double(v[d]);
    }
    free(score);
    return 0;
}

/*
 * Attention for a list of (sequence, row-in-span) items; out is [n_items][H][D] fp64.
 * H query heads over Hkv key/value heads (the pool holds Hkv heads): Hkv = H is multi-head
 * attention; with grouped-query attention (the paper's largest model, Section 5) query head h
 * reads K/V head h / (H / Hkv), i.e. consecutive query heads share a K/V head (reading: the paper
 * does not print the mapping; this is the grouping of the model family it evaluates).
 * Returns 0 on success, -1 on allocation failure, -2 on an invalid descriptor.
 */
int oracle_paged_attn_items(const uint16_t *pool, int64_t num_blocks, int B, int H, int Hkv, int D,
                            int num_seqs, const int32_t *ctx_len, const int32_t *q_len,
                            const int32_t *q_start, const int32_t *block_tables,
                            int max_blocks_per_seq, const uint16_t *q, double scale,
                            int64_t n_items, const int32_t *item_seq, const int32_t *item_row,
                            double *out)
{
    if (Hkv < 1 || H < Hkv || H % Hkv != 0) return -2;
    const int group = H / Hkv;   /* query heads that share one K/V head */
    for (int64_t it = 0; it < n_items; ++it) {
        int s = item_seq[it];
        if (s < 0 || s >= num_seqs) return -2;
        if (ctx_len[s] < 1 || q_len[s] < 1 || q_len[s] > ctx_len[s]) return -2;
        if (item_row[it] < 0 || item_row[it] >= q_len[s]) return -2;
        int nb = (ctx_len[s] + B - 1) / B;
        if (nb > max_blocks_per_seq) return -2;
        for (int j = 0; j < nb; ++j) {
            int32_t id = block_tables[(int64_t)s * max_blocks_per_seq + j];
            if (id < 0 || id >= num_blocks) return -2;
        }
    }
    int failed = 0;
    int64_t work = n_items * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t w = 0; w < work; ++w) {
        int64_t it = w / H;
        int head = (int)(w % H);
        int s = item_seq[it];
        int i = item_row[it];
        int64_t p = (int64_t)ctx_len[s] - q_len[s] + i;
        const int32_t *table = block_tables + (int64_t)s * max_blocks_per_seq;
        const uint16_t *qrow = q + (((int64_t)q_start[s] + i) * H + head) * (int64_t)D;
        double *o = out + (it * H + head) * (int64_t)D;
        if (attend_one(pool, Hkv, B, D, table, head / group, p, qrow, scale, o) != 0) {
#pragma omp atomic write
            failed = 1;
        }
    }
    return failed ? -1 : 0;
}

/* Every row of every sequence; out is [total_q_rows][H][D] fp64, indexed by q_start[s] + i. */
int oracle_paged_attn(const uint16_t *pool, int64_t num_blocks, int B, int H, int Hkv, int D, int num_seqs,
                      const int32_t *ctx_len, const int32_t *q_len, const int32_t *q_start,
                      const int32_t *block_tables, int max_blocks_per_seq, const uint16_t *q,
                      double scale, double *out)
{
    int64_t n_items = 0;
    for (int s = 0; s < num_seqs; ++s) {
        if (q_len[s] < 1) return -2;
        n_items += q_len[s];
    }
    int32_t *iseq = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_items ? n_items : 1));
    int32_t *irow = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_items ? n_items : 1));
    int64_t *dst = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n_items ? n_items : 1));
    double *tmp = (double *)malloc(sizeof(double) * (size_t)(n_items ? n_items : 1) * H * D);
    if (!iseq || !irow || !dst || !tmp) { free(iseq); free(irow); free(dst); free(tmp); return -1; }
    int64_t n = 0;
    for (int s = 0; s < num_seqs; ++s)
        for (int i = 0; i < q_len[s]; ++i) {
            iseq[n] = s; irow[n] = i; dst[n] = (int64_t)q_start[s] + i; ++n;
        }
    int rc = oracle_paged_attn_items(pool, num_blocks, B, H, Hkv, D, num_seqs, ctx_len, q_len, q_start,
                                     block_tables, max_blocks_per_seq, q, scale, n_items, iseq, irow, tmp);
    if (rc == 0)
        for (int64_t k = 0; k < n_items; ++k)
            memcpy(out + dst[k] * H * D, tmp + k * H * D, sizeof(double) * (size_t)H * D);
    free(iseq); free(irow); free(dst); free(tmp);
    return rc;
}

/* staging[i] <- pool[ids[i]], i < n; list order; duplicate sources allowed. */
int oracle_pack_blocks(const uint8_t *pool, int64_t num_blocks, int64_t block_bytes,
                       const int32_t *ids, int64_t n, uint8_t *staging)
{
    for (int64_t i = 0; i < n; ++i)
        if (ids[i] < 0 || ids[i] >= num_blocks) return -2;
    for (int64_t i = 0; i < n; ++i)
        memcpy(staging + i * block_bytes, pool + (int64_t)ids[i] * block_bytes, (size_t)block_bytes);
    return 0;
}

/* pool[ids[i]] <- staging[i], i < n; destinations must be distinct (-3 otherwise). */
int oracle_unpack_blocks(uint8_t *pool, int64_t num_blocks, int64_t block_bytes,
                         const int32_t *ids, int64_t n, const uint8_t *staging)
{
    for (int64_t i = 0; i < n; ++i)
        if (ids[i] < 0 || ids[i] >= num_blocks) return -2;
    uint8_t *seen = (uint8_t *)calloc((size_t)(num_blocks ? num_blocks : 1), 1);
    if (!seen) return -1;
    for (int64_t i = 0; i < n; ++i) {
        if (seen[ids[i]]) { free(seen); return -3; }
        seen[ids[i]] = 1;
    }
    free(seen);
    for (int64_t i = 0; i < n; ++i)
        memcpy(pool + (int64_t)ids[i] * block_bytes, staging + i * block_bytes, (size_t)block_bytes);
    return 0;
}

/*
 * KV append (Sections 4.2 and 4.3): before a recomputation chunk (or a decode token) attends, the
 * keys and values just computed for its q_len[s] query positions enter the cache at logical
 * positions ctx_len[s] - q_len[s] .. ctx_len[s] - 1 of sequence s, i.e. in block
 * block_table[t / B], slot t % B, so that the attention of this iteration and the chunks of later
 * iterations find them there.  k_new / v_new: bf16 bit patterns [total rows][H][D], row
 * q_start[s] + i belongs to position ctx_len[s] - q_len[s] + i.  Every other slot keeps its bytes.
 * Returns -2 on an invalid descriptor or block id, -3 if two rows address the same slot.
 */
int oracle_kv_append(uint16_t *pool, int64_t num_blocks, int B, int H, int D, int num_seqs,
                     const int32_t *ctx_len, const int32_t *q_len, const int32_t *q_start,
                     const int32_t *block_tables, int max_blocks_per_seq, const uint16_t *k_new,
                     const uint16_t *v_new)
{
    if (num_seqs < 0 || B < 1 || H < 1 || D < 1) return -2;
    uint8_t *seen = (uint8_t *)calloc((size_t)(num_blocks * B > 0 ? num_blocks * B : 1), 1);
    if (!seen) return -1;
    for (int s = 0; s < num_seqs; ++s) {                      /* validate everything before writing */
        if (ctx_len[s] < 1 || q_len[s] < 1 || q_len[s] > ctx_len[s] || q_start[s] < 0 ||
            (ctx_len[s] + B - 1) / B > max_blocks_per_seq) { free(seen); return -2; }
        for (int i = 0; i < q_len[s]; ++i) {
            int t = ctx_len[s] - q_len[s] + i;
            int32_t blk = block_tables[(int64_t)s * max_blocks_per_seq + t / B];
            if (blk < 0 || blk >= num_blocks) { free(seen); return -2; }
            int64_t slot = (int64_t)blk * B + t % B;
            if (seen[slot]) { free(seen); return -3; }
            seen[slot] = 1;
        }
    }
    free(seen);
    for (int s = 0; s < num_seqs; ++s)
        for (int i = 0; i < q_len[s]; ++i) {
            int t = ctx_len[s] - q_len[s] + i;
            int64_t blk = block_tables[(int64_t)s * max_blocks_per_seq + t / B];
            int64_t row = (int64_t)q_start[s] + i;
            for (int h = 0; h < H; ++h) {
                uint16_t *kd = pool + ((((blk * 2 + 0) * H + h) * B) + t % B) * D;
                uint16_t *vd = pool + ((((blk * 2 + 1) * H + h) * B) + t % B) * D;
                memcpy(kd, k_new + (row * H + h) * D, sizeof(uint16_t) * (size_t)D);
                memcpy(vd, v_new + (row * H + h) * D, sizeof(uint16_t) * (size_t)D);
            }
        }
    return 0;
}

/*
 * Section 4.1, swap pipelining: each layer's swapping is one stage.  Whatever the overlap, once
 * all stages are through, layer l's listed blocks sit in list order at host + l * layer_stride.
 */
int oracle_swap_out_layers(const uint8_t *const *pools, int64_t num_layers, int64_t num_blocks,
                           int64_t block_bytes, const int32_t *ids, int64_t n, uint8_t *host,
                           int64_t layer_stride)
{
    if (layer_stride < n * block_bytes) return -2;
    for (int64_t l = 0; l < num_layers; ++l) {
        int rc = oracle_pack_blocks(pools[l], num_blocks, block_bytes, ids, n, host + l * layer_stride);
        if (rc) return rc;
    }
    return 0;
}

/* The way back: layer l's pool receives host + l * layer_stride at the listed (distinct) blocks. */
int oracle_swap_in_layers(uint8_t *const *pools, int64_t num_layers, int64_t num_blocks,
                          int64_t block_bytes, const int32_t *ids, int64_t n, const uint8_t *host,
                          int64_t layer_stride)
{
    if (layer_stride < n * block_bytes) return -2;
    for (int64_t l = 0; l < num_layers; ++l) {
        int rc = oracle_unpack_blocks(pools[l], num_blocks, block_bytes, ids, n, host + l * layer_stride);
        if (rc) return rc;
    }
    return 0;
}

/*
 * Section 4.1, swap chunking.  T_swap(N) = N * M / bandwidth (the paper computes T_swap from the
 * swapping bandwidth and the per-token memory M); the swap limit of an iteration whose forward
 * pass takes t_fwd is the N with T_swap(N) = t_fwd, i.e. the number of tokens whose movement
 * hides behind the forward pass.  Tokens are whole, so the limit is rounded down.
 * Returns -1 for arguments outside the model (negative time, non-positive bandwidth or M).
 */
int64_t oracle_swap_limit_tokens(double t_fwd, double bandwidth, double token_bytes)
{
    if (!(t_fwd >= 0.0) || !(bandwidth > 0.0) || !(token_bytes > 0.0)) return -1;
    double n = floor(t_fwd * bandwidth / token_bytes);
    if (n > 9.0e18) return INT64_MAX;
    return (int64_t)n;
}

/*
 * Section 4.1: the swap of one sequence is split over iterations so that iteration i moves at
 * most its swap limit limits[i] (tokens).  The cache moves in whole blocks of block_size tokens,
 * so an iteration moves floor(limit / block_size) blocks at most (reading: a partial block cannot
 * be moved, and rounding up would exceed what the forward pass hides).  out_blocks[i] receives
 * the blocks moved in iteration i; returns the number of iterations used (n_iters + 1 if the
 * limits given do not suffice), or -1 for bad arguments.
 */
int64_t oracle_swap_schedule(int64_t total_blocks, int64_t block_size, const int64_t *limits,
                             int64_t n_iters, int64_t *out_blocks)
{
    if (total_blocks < 0 || block_size < 1 || n_iters < 0) return -1;
    for (int64_t i = 0; i < n_iters; ++i)
        if (limits[i] < 0) return -1;
    int64_t left = total_blocks, used = 0;
    for (int64_t i = 0; i < n_iters; ++i) {
        int64_t can = limits[i] / block_size;
        int64_t mv = left < can ? left : can;
        out_blocks[i] = mv;
        left -= mv;
        if (mv > 0) used = i + 1;
        if (left == 0) { for (int64_t j = i + 1; j < n_iters; ++j) out_blocks[j] = 0; break; }
    }
    return left > 0 ? n_iters + 1 : used;
}

/* =====================================================================================
 * GPU-memory-waste model (Section 3.2: Eq. 1 discard, Eq. 2 preserve, Eq. 3 swap; Section 4.2:
 * Eq. 4 chunked discard; Section 4.3: Eq. 5 and the interception schedule) and the saturation
 * point S of Section 4.2.  All in fp64, each function the printed formula.
 *
 * T_fwd ("a mapping from the number of scheduled tokens in a batch to the execution time of
 * that iteration", obtained by offline profiling) is given as n measured points
 * (tokens[k], seconds[k]), tokens strictly increasing and positive.  Reading (the paper does not
 * say how the mapping is evaluated between profiled points): straight lines between
 * neighbouring points, the line through the origin and the first point below it, the last
 * segment's line beyond the last point (the first point's ray if n = 1).  NaN on a bad table.
 * ===================================================================================== */
double oracle_tfwd(const double *tokens, const double *seconds, int n, double x)
{
    if (n < 1 || !(x >= 0.0)) return NAN;
    for (int k = 0; k < n; ++k)
        if (!(tokens[k] > 0.0) || !(seconds[k] >= 0.0) || (k > 0 && !(tokens[k] > tokens[k - 1]))) return NAN;
    if (x <= tokens[0] || n == 1) return seconds[0] * (x / tokens[0]);
    int k = 1;
    while (k < n - 1 && x > tokens[k]) ++k;          /* segment [k-1, k]; the last one also serves beyond */
    double w = (x - tokens[k - 1]) / (tokens[k] - tokens[k - 1]);
    return seconds[k - 1] + w * (seconds[k] - seconds[k - 1]);
}

/* Eq. 1: recomputing C tokens in one iteration wastes their own memory and everybody else's
 * (C_other tokens) for T_fwd(C). */
double oracle_waste_discard(const double *tokens, const double *seconds, int n, double C, double C_other, double M)
{
    double t = oracle_tfwd(tokens, seconds, n, C);
    return t * C * M + t * C_other * M;
}

/* Eq. 2: a preserved context of C tokens is idle for the interception's duration. */
double oracle_waste_preserve(double T_int, double C, double M) { return T_int * C * M; }

/* Eq. 3: a synchronous swap stalls the whole batch (C_batch tokens) for T_swap, out and in. */
double oracle_waste_swap(double T_swap, double C_batch, double M) { return 2.0 * T_swap * C_batch * M; }

/* Eq. 4: recomputation in n chunks, one per iteration: half of Eq. 1's first term, and n times the
 * per-chunk added time T_fwd(C / n) charged to the other requests. */
double oracle_waste_chunked_discard(const double *tokens, const double *seconds, int n_pts, double C,
                                    double C_other, double M, int n_chunks)
{
    if (n_chunks < 1) return NAN;
    double whole = oracle_tfwd(tokens, seconds, n_pts, C);
    double per_chunk = oracle_tfwd(tokens, seconds, n_pts, C / n_chunks);
    return whole * C * M / 2.0 + n_chunks * per_chunk * C_other * M;
}

/* Section 4.2: chunk size = saturation point S minus the running group's size (never negative);
 * a context of C tokens then takes ceil(C / chunk) iterations. */
int64_t oracle_chunk_tokens(int64_t S, int64_t running) { return S > running ? S - running : 0; }
int64_t oracle_chunk_count(int64_t C, int64_t chunk)
{
    if (C < 0 || chunk < 1) return -1;
    return (C + chunk - 1) / chunk;
}

/* Section 4.2: S is the query-token count past which more tokens lengthen the iteration without
 * raising throughput.  From a profile of (query tokens q[k], iteration seconds t[k]), q increasing:
 * the smallest profiled q whose throughput q / t reaches frac (say 0.95) of the best throughput in
 * the profile (reading: the paper gives no numerical criterion for the knee).  -1 on bad input. */
int64_t oracle_saturation_point(const double *q, const double *t, int n, double frac)
{
    if (n < 1 || !(frac > 0.0) || frac > 1.0) return -1;
    double best = 0.0;
    for (int k = 0; k < n; ++k) {
        if (!(q[k] > 0.0) || !(t[k] > 0.0) || (k > 0 && !(q[k] > q[k - 1]))) return -1;
        if (q[k] / t[k] > best) best = q[k] / t[k];
    }
    for (int k = 0; k < n; ++k)
        if (q[k] / t[k] >= frac * best) return (int64_t)q[k];
    return -1;
}

/*
 * Section 4.3, scheduling intercepted requests.  Waste_i = min(WastePreserve_i, WasteChunkD_i)
 * (Eq. 5).  Requests are taken in descending order of that waste (equal wastes: lower index
 * first) and swapped out until the swap-out budget (tokens) is spent; a request the budget covers
 * only partly is swapped as far as it goes.  What is left of each request is preserved or
 * discarded, whichever of its two wastes is smaller (preserve on a tie).
 * Outputs: swap_tokens[i] tokens of request i to swap out; action[i] for the rest of its context:
 * 0 = nothing left, 1 = preserve, 2 = discard.  Returns 0, or -1 on bad arguments.
 */
int oracle_schedule_intercepted(int n, const double *waste_preserve, const double *waste_chunkd,
                                const int64_t *ctx_tokens, int64_t budget, int64_t *swap_tokens,
                                int32_t *action)
{
    if (n < 0 || budget < 0) return -1;
    int *order = (int *)malloc(sizeof(int) * (size_t)(n ? n : 1));
    if (!order) return -1;
    for (int i = 0; i < n; ++i) {
        if (ctx_tokens[i] < 0 || !(waste_preserve[i] >= 0.0) || !(waste_chunkd[i] >= 0.0)) { free(order); return -1; }
        order[i] = i;
    }
    for (int a = 1; a < n; ++a) {                     /* insertion sort: stable, descending waste */
        int v = order[a];
        double wv = fmin(waste_preserve[v], waste_chunkd[v]);
        int b = a - 1;
        while (b >= 0 && fmin(waste_preserve[order[b]], waste_chunkd[order[b]]) < wv) { order[b + 1] = order[b]; --b; }
        order[b + 1] = v;
    }
    int64_t left = budget;
    for (int r = 0; r < n; ++r) {
        int i = order[r];
        int64_t take = ctx_tokens[i] < left ? ctx_tokens[i] : left;
        swap_tokens[i] = take;
        left -= take;
        if (ctx_tokens[i] - take == 0) action[i] = 0;
        else action[i] = waste_preserve[i] <= waste_chunkd[i] ? 1 : 2;
    }
    free(order);
    return 0;
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}

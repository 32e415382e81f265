// Tile path of the attention kernels: the query rows of a recomputation chunk (Section 4.2) against a range of their
// sequence's paged keys.  Here QK^T and PV are dense contractions (hundreds of rows share every
// key), so they run on the matrix cores: v_mfma_f32_32x32x16_bf16, fp32 accumulation.  (The kernels use this body for
// head_dim 64 and 128; head_dim 256 runs tile16_body.h, where a wave takes 16 rows.)
//
// One workgroup = one TileItem x one head group (one head with multi-head attention; with grouped
// queries the G heads that share a K/V head): up to tile_rows(D) rows = query rows x heads of the
// group, one wave per 32 rows.
//   - K and V tiles of 64 keys (4 cache blocks, looked up in the block table) are fetched with
//     16-byte coalesced loads into registers two tiles ahead, then staged in one of two LDS
//     buffers and shared by all waves; one barrier per tile.
//   - S^T = K Q^T: A operand = 32 keys x 16 dims from LDS, B operand = this wave's Q^T kept in
//     registers for the whole item.  In the 32x32 accumulator layout every lane then owns ONE
//     query column (lane % 32) and 16 of a subtile's 32 keys, so the online softmax needs a
//     single cross-lane exchange per tile (with lane ^ 32).
//   - O^T += V^T P^T: the accumulator registers of S^T, rounded to bf16, already ARE the B
//     operand (8 keys per lane per MFMA, slot j of lane half hl <-> key 8*(j/4) + 4*hl + j%4).
//     V stays [key][dim] in LDS; the A operand (one dim, 8 keys per lane, in that key order) comes
//     from two ds_read_b64_tr_b16 transpose loads, so no register transposition is needed.
//   - Causality: query row r of the item sits at position pos0 + r and sees keys <= that position.
//     Only tiles that straddle a wave's diagonal are masked; tiles beyond it are skipped.
// Dead slots (keys >= k_end, possibly NaN) get score -inf by select and V = 0 in LDS.
#pragma once

#include "ic_internal.h"

namespace ic {
namespace tilep {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

constexpr float kNegBig = -1.0e30f;
constexpr float kLazyLog2 = 8.0f;  // slack of the online softmax's reference maximum, in log2 units
constexpr int kTileK = 64;    // keys per staged tile
// Waves (of 32 query rows each) per workgroup: tile_rows(D) / 32.  More rows per workgroup means
// fewer workgroups re-reading the same keys from L2 / HBM.
template <int D>
struct TW {
  static constexpr int kWaves = tile_rows(D) / 32;
  static constexpr int kThreads = 64 * kWaves;
};

template <int D>
struct TG {
  static constexpr int kKStride = D + 8;        // bf16 per LDS row of K (16-byte pad)
  static constexpr int kVStride = D + 32;       // bf16 per LDS row of V: rows shift by 16 banks
  static constexpr int kChunks = D / 8;         // 16-byte chunks per token row
  static constexpr int kThreads = TW<D>::kThreads;
  static constexpr int kKLoads = kTileK * kChunks / kThreads;      // K chunks per thread
  static_assert(kTileK * kChunks % kThreads == 0, "K tile must split evenly over the threads");
  static constexpr int kQSteps = D / 16;        // MFMA k-steps of Q K^T
  static constexpr int kDTiles = D / 32;        // 32-row tiles of O^T
};

template <int D>
struct Staging {
  u32x4 k[TG<D>::kKLoads];
  u32x4 v[TG<D>::kKLoads];
};

// Global -> registers for chunk pair j of one 64-key tile (K chunk and V chunk at the same offset).
// ids = the 4 block ids of the tile (wave-uniform).  Thread u takes 16-byte chunk u of the K tile
// and of the V tile: consecutive lanes read consecutive addresses of a (block, head) tile, so every
// load instruction is fully coalesced.
template <int D>
__device__ __forceinline__ void fetch_chunk(Staging<D>& st, int j, const char* pool, const int (&ids)[4],
                                            int head, int H, int tid) {
  using G = TG<D>;
  constexpr int kTileBytes = kBlockSize * D * 2;
  const int64_t blk_stride = (int64_t)2 * H * kTileBytes;
  const int u = tid + G::kThreads * j;    // 16-byte chunk of the tile
  const int tok = u / G::kChunks;         // 0..63
  const int c = u % G::kChunks;
  // the chunks one wave loads in one instruction never straddle a block: tok / 16 is wave-uniform
  const int bsel = __builtin_amdgcn_readfirstlane(tok / kBlockSize);
  const char* a = pool + (int64_t)head * kTileBytes + (int64_t)ids[bsel] * blk_stride +
                  (tok % kBlockSize) * (D * 2) + c * 16;
  st.k[j] = *(const u32x4*)a;
  st.v[j] = *(const u32x4*)(a + (int64_t)H * kTileBytes);
}

template <int D>
__device__ __forceinline__ void fetch_tile(Staging<D>& st, const char* pool, const int (&ids)[4],
                                           int head, int H, int tid) {
#pragma unroll
  for (int j = 0; j < TG<D>::kKLoads; ++j) fetch_chunk<D>(st, j, pool, ids, head, H, tid);
}

// Registers -> LDS, K (which = 0) or V (which = 1) of a staged tile, as [key][dim] rows (padded).
// V of keys >= n_valid is zeroed (dead slots may hold NaN, and 0 * NaN would poison the PV product).
template <int D>
__device__ __forceinline__ void stage_half(const Staging<D>& st, int which, uint16_t* ks, uint16_t* vs,
                                           int tid, int n_valid) {
  using G = TG<D>;
#pragma unroll
  for (int j = 0; j < G::kKLoads; ++j) {
    const int u = tid + G::kThreads * j;
    const int tok = u / G::kChunks, c = u % G::kChunks;
    if (which == 0) {
      *(u32x4*)(ks + tok * G::kKStride + c * 8) = st.k[j];
    } else {
      u32x4 v = st.v[j];
      if (tok >= n_valid) v = (u32x4){0u, 0u, 0u, 0u};
      *(u32x4*)(vs + tok * G::kVStride + c * 8) = v;
    }
  }
}

// A operand of O^T += V^T P^T for MFMA rows d = d0 .. d0+31 (this lane: d0 + lane % 32) and the 8 keys
// of k-step ksp that belong to this lane half, read with the LDS transpose load.  In each group of
// 16 lanes, lane i supplies the address of an 8-byte row and receives column i % 4 of the rows
// supplied by lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12 (layout measured on gfx950).  So lane j points at
// V[key j/4][dims 4 (j % 4) ..+3] of its group's 16 dims, and lane i gets V[4 keys][dim i]: two loads
// give the 8 keys in accumulator order (slots 0-3: keys 4 hl ..+3, slots 4-7: keys 8 + 4 hl ..+3).
template <int D>
__device__ __forceinline__ bf16x8 read_vt_operand(const uint16_t* vs, int d0, int ksp, int lane) {
  using G = TG<D>;
  typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
  const int hl = lane >> 5;
  const int j = lane & 15;
  const uint16_t* a = vs + (16 * ksp + 4 * hl + (j >> 2)) * G::kVStride + d0 + 16 * ((lane & 31) >> 4) + 4 * (j & 3);
  const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)a);
  const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(a + 8 * G::kVStride));
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// One 64-key tile for one wave: S^T = K Q^T, online softmax, O^T += V^T P^T.  mask is set only for
// tiles that straddle the wave's causal diagonal.
template <int D>
__device__ __forceinline__ void wave_step(const uint16_t* ks, const uint16_t* vs,
                                          const bf16x8 (&qreg)[TG<D>::kQSteps],
                                          f32x16 (&acc_o)[TG<D>::kDTiles], float& m, float& l, int kt,
                                          int pos, int col, int hl, float sc, bool mask) {
  using G = TG<D>;
  f32x16 s_acc[2];
#pragma unroll
  for (int tt = 0; tt < 2; ++tt)
#pragma unroll
    for (int i = 0; i < 16; ++i) s_acc[tt][i] = 0.f;
  // Both 32-key subtiles advance together (two independent accumulators alternate in the MFMA
  // pipe) and the A operands of the next k-step are read from LDS before this step's MFMAs issue.
  {
    const uint16_t* kp0 = ks + col * G::kKStride + 8 * hl;
    const uint16_t* kp1 = kp0 + 32 * G::kKStride;
    bf16x8 a0 = *(const bf16x8*)kp0, a1 = *(const bf16x8*)kp1;
#pragma unroll
    for (int s = 0; s < G::kQSteps; ++s) {
      bf16x8 n0 = a0, n1 = a1;
      if (s + 1 < G::kQSteps) {
        n0 = *(const bf16x8*)(kp0 + 16 * (s + 1));
        n1 = *(const bf16x8*)(kp1 + 16 * (s + 1));
      }
      s_acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, qreg[s], s_acc[0], 0, 0, 0);
      s_acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, qreg[s], s_acc[1], 0, 0, 0);
      a0 = n0;
      a1 = n1;
    }
  }
  // Scores stay unscaled in the accumulators; the scale (> 0, in log2 units) is folded into the
  // exponent: p = 2^(s*sc - m).
  if (mask) {  // wave-uniform; the empty asm keeps this a branch instead of 32 always-on selects
    asm volatile("" ::: "memory");
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = kt + 32 * tt + 8 * (i / 4) + 4 * hl + (i % 4);
        s_acc[tt][i] = key > pos ? -__builtin_inff() : s_acc[tt][i];
      }
  }
  float tmax = -__builtin_inff();
#pragma unroll
  for (int tt = 0; tt < 2; ++tt)
#pragma unroll
    for (int i = 0; i < 16; ++i) tmax = __builtin_fmaxf(tmax, s_acc[tt][i]);
  tmax = __builtin_fmaxf(tmax, __shfl_xor(tmax, 32));
  // Lazy reference: the running maximum m only has to bound the scores loosely.  It is moved (and the
  // accumulators rescaled, 16 multiplies per 32 output rows) only when a score exceeds it by more than
  // kLazyLog2; until then weights may reach 2^kLazyLog2, which fp32 sums and bf16 weights hold easily.
  const float m_cand = __builtin_fmaxf(m, tmax * sc);
  const bool grew = m_cand > m + kLazyLog2;
  const float m_new = grew ? m_cand : m;
  const float alpha = grew ? __builtin_amdgcn_exp2f(m - m_cand) : 1.0f;
  m = m_new;
  // Weights: rounded to bf16 in pairs (one v_cvt_pk_bf16_f32), and summed AS ROUNDED by a bf16 dot
  // product with (1, 1): the normaliser then counts exactly what the matrix core will multiply, so
  // the output stays an exact convex combination of the values and a row dominated by one key
  // (short contexts) does not inherit the 2^-9 relative rounding error of its weight.
  float psum = 0.f;
  bf16x8 pb[4];
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
  for (int tt = 0; tt < 2; ++tt)
#pragma unroll
    for (int i = 0; i < 16; i += 2) {
      const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[tt][i], sc, -m_new));
      const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[tt][i + 1], sc, -m_new));
      const bf16x2 pr = {(__bf16)p0, (__bf16)p1};
      psum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, psum, false);
      pb[2 * tt + i / 8][i % 8] = pr[0];
      pb[2 * tt + i / 8][i % 8 + 1] = pr[1];
    }
  l = l * alpha + psum;
  if (__builtin_amdgcn_ballot_w64(grew) != 0) {  // rescale only when some row's maximum moved
#pragma unroll
    for (int dt = 0; dt < G::kDTiles; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc_o[dt][i] *= alpha;
  }
  // O^T += V^T P^T, k-step outer so that the kDTiles independent accumulators alternate
  {
    const int lane = col + 32 * hl;
    bf16x8 a[G::kDTiles];
#pragma unroll
    for (int dt = 0; dt < G::kDTiles; ++dt) a[dt] = read_vt_operand<D>(vs, 32 * dt, 0, lane);
#pragma unroll
    for (int ksp = 0; ksp < 4; ++ksp) {
      bf16x8 n[G::kDTiles];
#pragma unroll
      for (int dt = 0; dt < G::kDTiles; ++dt)
        n[dt] = ksp + 1 < 4 ? read_vt_operand<D>(vs, 32 * dt, ksp + 1, lane) : a[dt];
#pragma unroll
      for (int dt = 0; dt < G::kDTiles; ++dt)
        acc_o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[dt], pb[ksp], acc_o[dt], 0, 0, 0);
#pragma unroll
      for (int dt = 0; dt < G::kDTiles; ++dt) a[dt] = n[dt];
    }
  }
}

// One staged tile: K rows then V rows.
template <int D>
constexpr int tile_buf_elems() {
  return kTileK * TG<D>::kKStride + kTileK * TG<D>::kVStride;
}

template <int D>
constexpr int tile_lds_bytes() {
  return 2 * tile_buf_elems<D>() * 2;  // two buffers of bf16
}

// One TileItem x one group of (1 << p.tile_g_shift) query heads that share a K/V head, executed by a
// workgroup of tile_rows(D) / 32 waves.  th = index of the head group: its heads are
// th << shift .. ((th + 1) << shift) - 1.  Row r of the tile is query row r >> shift of the item for
// head (th << shift) + (r & mask): with multi-head attention (shift 0) a tile is 256 rows of one head,
// with grouped-query attention the heads of a group ride on one staging of their common keys.
// lds: at least tile_lds_bytes<D>() bytes of workgroup LDS, 16-byte aligned.
template <int D>
__device__ __forceinline__ void tile_body(const AttnParams& p, const TileItem& it, int th, uint16_t* lds) {
  using G = TG<D>;

  const int H = p.num_heads;
  const int Hk = p.num_kv_heads;
  const int gs = p.tile_g_shift;
  const int head0 = th << gs;
  const int kvh = head0 / p.group;
  const int n_rows_t = it.n_rows << gs;               // rows of the tile: query rows x heads of the group
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31;  // query column of this lane inside the wave's 32 rows
  const int hl = lane >> 5;

  // ---- this wave's Q^T operand (registers for the whole item) and causal limits
  const int r = 32 * w + col;                       // row inside the tile
  const int r_eff = min(r, n_rows_t - 1);           // dead rows mirror the last live one
  const int pos = it.pos0 + (r_eff >> gs);          // last visible key of this lane's row
  const int wave_pos_lo = it.pos0 + min((32 * w) >> gs, it.n_rows - 1);        // smallest limit in the wave
  const int wave_pos_hi = it.pos0 + min((32 * w + 31) >> gs, it.n_rows - 1);   // largest limit in the wave
  bf16x8 qreg[G::kQSteps];
  {
    const int qr = r_eff >> gs;                     // query row inside the item
    const int head = head0 + (r_eff & ((1 << gs) - 1));
    const uint16_t* qp = p.q + ((int64_t)(it.qrow0 + qr) * H + head) * D + 8 * hl;
#pragma unroll
    for (int s = 0; s < G::kQSteps; ++s) qreg[s] = *(const bf16x8*)(qp + 16 * s);
  }

  f32x16 acc_o[G::kDTiles];
#pragma unroll
  for (int dt = 0; dt < G::kDTiles; ++dt)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc_o[dt][i] = 0.f;
  float m = kNegBig, l = 0.f;

  const char* pool = (const char*)p.pool;
  // The block table is read through the constant address space: its entries are wave-uniform and nothing
  // writes them while the kernel runs, so they can come as scalar loads.  As vector loads they would be
  // the youngest loads in flight whenever the next tile's addresses are needed, and waiting for them
  // (loads return in order) would also wait for every K/V tile load issued before them, which cuts
  // the prefetch distance from two tiles to one.
  typedef __attribute__((address_space(4))) const int32_t const_i32;
  const_i32* bt = (const_i32*)(p.bt_flat + p.bt_off[it.seq]);
  const int last_blk = (it.k_end - 1) / kBlockSize;  // last table entry this item may touch
  const int n_tiles = (it.k_end - it.k_begin + kTileK - 1) / kTileK;
  const float sc = p.scale_log2e;

  auto tile_ids = [&](int t, int (&ids)[4]) {
    const int b0 = (it.k_begin + t * kTileK) / kBlockSize;
#pragma unroll
    for (int i = 0; i < 4; ++i) ids[i] = bt[min(b0 + i, last_blk)];
  };

  // Pipeline.  LDS holds two tile buffers; registers hold PFD staged tiles (PFD = 2, or 1 for
  // head_dim 256, which has no registers for a second set).  In step t every wave
  //   - computes on LDS buffer t % 2,
  //   - copies tile t+1 from its register set into the other LDS buffer,
  //   - reloads that register set with tile t+1+PFD,
  // and ONE barrier ends the step: it publishes tile t+1 and guarantees nobody still reads the
  // buffer that step t+1 will overwrite.  (Slipping the copies and loads between the MFMAs instead
  // of issuing them after the tile's arithmetic costs about 45 more registers and was slower.)
  // ids always holds the block ids of the tile the next fetch will read, loaded a step ahead.
  // Every fetch is issued unconditionally; tiles past the item's end re-read its last block (tile_ids
  // clamps to it) and are never staged.  Loads return in order and a wait names how many younger loads
  // may stay in flight, so the compiler can let the newer register set's loads fly while the older
  // set is copied to LDS only if that number is the same on every path through the loop.  With
  // fetches skipped at the tail it is not, every copy waits for all loads, and the prefetch distance
  // drops from two tiles to one.  For the same reason the two-set loop always runs whole pairs of
  // steps; the odd one out does no arithmetic and no copy.
  constexpr int PFD = D <= 128 ? 2 : 1;
  constexpr int kBuf = tile_buf_elems<D>();
  Staging<D> st[PFD];
  int ids[4];
  tile_ids(0, ids);
  fetch_tile<D>(st[0], pool, ids, kvh, Hk, tid);
  if (PFD == 2) {
    tile_ids(1, ids);
    fetch_tile<D>(st[PFD - 1], pool, ids, kvh, Hk, tid);
  }
  stage_half<D>(st[0], 0, lds, lds + kTileK * G::kKStride, tid, it.k_end - it.k_begin);
  stage_half<D>(st[0], 1, lds, lds + kTileK * G::kKStride, tid, it.k_end - it.k_begin);
  tile_ids(PFD, ids);
  fetch_tile<D>(st[0], pool, ids, kvh, Hk, tid);
  tile_ids(PFD + 1, ids);
  __syncthreads();

  // Waves w and w + 4 share a SIMD.  The first does its arithmetic, then its copy to LDS; the second
  // the other way round, so that between two barriers one wave of a SIMD is in the matrix and vector
  // pipes while the other waits on memory and LDS writes, instead of both doing the same thing at
  // the same time.  The loads that refill the register set come last for both: with no load between
  // the two possible places of the copy, the number of younger loads in flight is the same at both.
  const bool copy_first = TW<D>::kWaves == 8 && (w & 4) != 0;  // wave-uniform
  // step t with its register set fixed at compile time (RS = (t + 1) % PFD holds tile t + 1)
  auto step = [&](int t, Staging<D>& sreg) {
    const int kt = it.k_begin + t * kTileK;
    const uint16_t* ks = lds + (t & 1) * kBuf;
    const uint16_t* vs = ks + kTileK * G::kKStride;
    uint16_t* nks = lds + ((t + 1) & 1) * kBuf;
    uint16_t* nvs = nks + kTileK * G::kKStride;
    auto copy = [&]() {
      if (t + 1 < n_tiles) {
        const int n_valid_next = it.k_end - (kt + kTileK);
        stage_half<D>(sreg, 0, nks, nvs, tid, n_valid_next);
        stage_half<D>(sreg, 1, nks, nvs, tid, n_valid_next);
      }
    };
    if (copy_first) copy();
    if (t < n_tiles && kt <= wave_pos_hi)  // otherwise every key of the tile is in this wave's future
      wave_step<D>(ks, vs, qreg, acc_o, m, l, kt, pos, col, hl, sc, kt + kTileK - 1 > wave_pos_lo);
    if (!copy_first) copy();
    fetch_tile<D>(sreg, pool, ids, kvh, Hk, tid);
    tile_ids(t + 2 + PFD, ids);
    __syncthreads();
  };
  if constexpr (PFD == 2) {
    for (int t = 0; t < n_tiles; t += 2) {
      step(t, st[1]);
      step(t + 1, st[0]);
    }
  } else {
    for (int t = 0; t < n_tiles; ++t) step(t, st[0]);
  }

  // ---- epilogue: lane holds O^T[d][col] for d = 32 dt + 8 (i/4) + 4 hl + i%4
  l += __shfl_xor(l, 32);
  // (row coordinates are worked out again here rather than kept in registers across the key loop)
  if (r < n_rows_t) {
    const int qr = r >> gs;
    const int head = head0 + (r & ((1 << gs) - 1));
    if (it.slot0 < 0) {
      const float inv = 1.0f / l;
      uint16_t* op = p.out + ((int64_t)(it.qrow0 + qr) * H + head) * D;
#pragma unroll
      for (int dt = 0; dt < G::kDTiles; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int d = 32 * dt + 8 * g + 4 * hl;
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (__bf16)(acc_o[dt][4 * g + e] * inv);  // round to nearest even
          *(bf16x4*)(op + d) = o;
        }
    } else {
      const int64_t ps = (int64_t)(it.slot0 + qr * it.nparts) * H + head;
      float* op = p.part_o + ps * D;
#pragma unroll
      for (int dt = 0; dt < G::kDTiles; ++dt)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int d = 32 * dt + 8 * g + 4 * hl;
          *(f32x4*)(op + d) = (f32x4){acc_o[dt][4 * g], acc_o[dt][4 * g + 1], acc_o[dt][4 * g + 2],
                                      acc_o[dt][4 * g + 3]};
        }
      if (hl == 0) {
        p.part_ml[ps * 2] = m;
        p.part_ml[ps * 2 + 1] = l;
      }
    }
  }
}

}  // namespace tilep
}  // namespace ic

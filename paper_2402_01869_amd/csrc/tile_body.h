// Tile path of the attention kernels: the query rows of a recomputation chunk (Section 4.2) against a range of their
// sequence's paged keys.  Here QK^T and PV are dense contractions (hundreds of rows share every
// key), so they run on the matrix cores: v_mfma_f32_32x32x16_bf16, fp32 accumulation.
//
// One workgroup = one TileItem x one head: up to tile_rows(D) query rows, one wave per 32 rows.
//   - K and V tiles of 64 keys (4 cache blocks, looked up in the block table) are fetched with
//     16-byte coalesced loads into registers one tile ahead, then staged in LDS and shared by
//     the 4 waves.
//   - S^T = K Q^T: A operand = 32 keys x 16 dims from LDS, B operand = this wave's Q^T kept in
//     registers for the whole item.  In the 32x32 accumulator layout every lane then owns ONE
//     query column (lane % 32) and 16 of a subtile's 32 keys, so the online softmax needs a
//     single cross-lane exchange per tile (with lane ^ 32).
//   - O^T += V^T P^T: the accumulator registers of S^T, rounded to bf16, already ARE the B
//     operand (8 keys per lane per MFMA); V is transposed once per workgroup on its way into
//     LDS, with the keys of each group of 16 stored in the order the accumulator layout yields
//     them (slot 8*hl + j  <->  key 8*(j/4) + 4*hl + j%4, hl = lane / 32), so the A operand is
//     one 16-byte LDS read.
//   - Causality: row r of the item sits at position pos0 + r and sees keys <= that position.
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

constexpr float kNegBig = -1.0e30f;
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
  static constexpr int kVStride = kTileK + 8;   // bf16 per LDS row of V^T
  static constexpr int kChunks = D / 8;         // 16-byte chunks per token row
  static constexpr int kThreads = TW<D>::kThreads;
  static constexpr int kKLoads = kTileK * kChunks / kThreads;      // K chunks per thread
  static constexpr int kVUnits = 16 * kChunks;                     // (key quad, dim chunk) pairs
  static constexpr int kVPasses = (kVUnits + kThreads - 1) / kThreads;
  static_assert(kTileK * kChunks % kThreads == 0, "K tile must split evenly over the threads");
  static constexpr int kQSteps = D / 16;        // MFMA k-steps of Q K^T
  static constexpr int kDTiles = D / 32;        // 32-row tiles of O^T
};

template <int D>
struct Staging {
  u32x4 k[TG<D>::kKLoads];
  u32x4 v[TG<D>::kVPasses][4];
};

// Work split of the V tile among threads: unit u = (dim chunk c, key quad tq), tq fastest, so the
// 64 lanes of a wave cover all 16 key quads of 4 dim chunks.  The transposed 8-byte LDS stores of a
// wave then fall on distinct banks (measured: the chunk-fastest split is 4-way conflicted).
template <int D>
struct VUnit {
  int tq, c;
  __device__ __forceinline__ VUnit(int u) : tq(u % 16), c(u / 16) {}
};

// Global -> registers for one 64-key tile.  ids = the 4 block ids of the tile (wave-uniform).
template <int D>
__device__ __forceinline__ void fetch_tile(Staging<D>& st, const char* pool, const int (&ids)[4],
                                           int head, int H, int tid) {
  using G = TG<D>;
  constexpr int kTileBytes = kBlockSize * D * 2;
  const int64_t blk_stride = (int64_t)2 * H * kTileBytes;
  const char* kbase = pool + (int64_t)head * kTileBytes;
  const char* vbase = kbase + (int64_t)H * kTileBytes;
#pragma unroll
  for (int j = 0; j < G::kKLoads; ++j) {
    const int u = tid + G::kThreads * j;    // 16-byte chunk of the K tile
    const int tok = u / G::kChunks;         // 0..63
    const int c = u % G::kChunks;
    // 256 consecutive chunks never straddle more than one wave-uniform block boundary: tok / 16 is
    // the same for all lanes of a wave for every supported D
    const int bsel = __builtin_amdgcn_readfirstlane(tok / kBlockSize);
    const int64_t blk = ids[bsel];
    st.k[j] = *(const u32x4*)(kbase + blk * blk_stride + (tok % kBlockSize) * (D * 2) + c * 16);
  }
#pragma unroll
  for (int ps = 0; ps < G::kVPasses; ++ps) {
    const int u = tid + G::kThreads * ps;
    if (u < G::kVUnits) {
      const VUnit<D> vu(u);
      const int64_t blk = ids[vu.tq / 4];
      const char* a = vbase + blk * blk_stride + ((vu.tq % 4) * 4) * (D * 2) + vu.c * 16;
#pragma unroll
      for (int i = 0; i < 4; ++i) st.v[ps][i] = *(const u32x4*)(a + i * (D * 2));
    }
  }
}

// Registers -> LDS.  K as is; V transposed (dims become rows); with ZERO, keys >= n_valid are zeroed.
template <int D, bool ZERO>
__device__ __forceinline__ void stage_tile(const Staging<D>& st, uint16_t* ks, uint16_t* vs, int tid,
                                           int n_valid) {
  using G = TG<D>;
#pragma unroll
  for (int j = 0; j < G::kKLoads; ++j) {
    const int u = tid + G::kThreads * j;
    const int tok = u / G::kChunks, c = u % G::kChunks;
    *(u32x4*)(ks + tok * G::kKStride + c * 8) = st.k[j];
  }
#pragma unroll
  for (int ps = 0; ps < G::kVPasses; ++ps) {
    const int u = tid + G::kThreads * ps;
    if (u < G::kVUnits) {
      const VUnit<D> vu(u);
      const int tq = vu.tq, c = vu.c;
      u32x4 r[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        r[i] = st.v[ps][i];
        if (ZERO && 4 * tq + i >= n_valid) r[i] = (u32x4){0u, 0u, 0u, 0u};
      }
      // key quad tq = (group of 16: tq / 4, quad in group: qd): slots 8*(qd % 2) + 4*(qd / 2) ..+3
      const int qd = tq % 4;
      const int col = 16 * (tq / 4) + 8 * (qd % 2) + 4 * (qd / 2);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        // dims 2kk (low halves) and 2kk+1 (high halves) of the 4 keys
        u32x2 lo, hi;
        lo[0] = __builtin_amdgcn_perm(r[1][kk], r[0][kk], 0x05040100u);
        lo[1] = __builtin_amdgcn_perm(r[3][kk], r[2][kk], 0x05040100u);
        hi[0] = __builtin_amdgcn_perm(r[1][kk], r[0][kk], 0x07060302u);
        hi[1] = __builtin_amdgcn_perm(r[3][kk], r[2][kk], 0x07060302u);
        *(u32x2*)(vs + (c * 8 + 2 * kk) * G::kVStride + col) = lo;
        *(u32x2*)(vs + (c * 8 + 2 * kk + 1) * G::kVStride + col) = hi;
      }
    }
  }
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
  for (int tt = 0; tt < 2; ++tt) {
#pragma unroll
    for (int i = 0; i < 16; ++i) s_acc[tt][i] = 0.f;
    const uint16_t* kp = ks + (32 * tt + col) * G::kKStride + 8 * hl;
#pragma unroll
    for (int s = 0; s < G::kQSteps; ++s) {
      const bf16x8 a = *(const bf16x8*)(kp + 16 * s);
      s_acc[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[s], s_acc[tt], 0, 0, 0);
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
  const float m_new = __builtin_fmaxf(m, tmax * sc);
  const bool grew = m_new > m;
  const float alpha = __builtin_amdgcn_exp2f(m - m_new);
  m = m_new;
  float psum = 0.f;
  bf16x8 pb[4];
#pragma unroll
  for (int tt = 0; tt < 2; ++tt)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[tt][i], sc, -m_new));
      psum += pv;
      pb[2 * tt + i / 8][i % 8] = (__bf16)pv;
    }
  l = l * alpha + psum;
  if (__builtin_amdgcn_ballot_w64(grew) != 0) {  // rescale only when some row's maximum moved
#pragma unroll
    for (int dt = 0; dt < G::kDTiles; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc_o[dt][i] *= alpha;
  }
#pragma unroll
  for (int dt = 0; dt < G::kDTiles; ++dt) {
    const uint16_t* vp = vs + (32 * dt + col) * G::kVStride + 8 * hl;
#pragma unroll
    for (int ksp = 0; ksp < 4; ++ksp) {
      const bf16x8 a = *(const bf16x8*)(vp + 16 * ksp);
      acc_o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[ksp], acc_o[dt], 0, 0, 0);
    }
  }
}

template <int D>
constexpr int tile_lds_bytes() {
  return (kTileK * TG<D>::kKStride + D * TG<D>::kVStride) * 2;
}

// One TileItem x one head, executed by a workgroup of tile_rows(D) / 32 waves.
// lds: at least tile_lds_bytes<D>() bytes of workgroup LDS, 16-byte aligned.
template <int D>
__device__ __forceinline__ void tile_body(const AttnParams& p, const TileItem& it, int head, uint16_t* lds) {
  using G = TG<D>;
  uint16_t* ks = lds;
  uint16_t* vs = lds + kTileK * G::kKStride;

  const int H = p.num_heads;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31;  // query column of this lane inside the wave's 32 rows
  const int hl = lane >> 5;

  // ---- this wave's Q^T operand (registers for the whole item) and causal limits
  const int r = 32 * w + col;                       // row inside the item
  const bool row_ok = r < it.n_rows;
  const int r_eff = row_ok ? r : it.n_rows - 1;     // dead rows mirror the last live one
  const int pos = it.pos0 + r_eff;                  // last visible key of this lane's row
  const int wave_pos_lo = it.pos0 + min(32 * w, it.n_rows - 1);        // smallest limit in the wave
  const int wave_pos_hi = it.pos0 + min(32 * w + 31, it.n_rows - 1);   // largest limit in the wave
  bf16x8 qreg[G::kQSteps];
  {
    const uint16_t* qp = p.q + ((int64_t)(it.qrow0 + r_eff) * H + head) * D + 8 * hl;
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
  const int32_t* bt = p.bt_flat + p.bt_off[it.seq];
  const int last_blk = (it.k_end - 1) / kBlockSize;  // last table entry this item may touch
  const int n_tiles = (it.k_end - it.k_begin + kTileK - 1) / kTileK;
  const float sc = p.scale_log2e;

  auto tile_ids = [&](int t, int (&ids)[4]) {
    const int b0 = (it.k_begin + t * kTileK) / kBlockSize;
#pragma unroll
    for (int i = 0; i < 4; ++i) ids[i] = bt[min(b0 + i, last_blk)];
  };

  Staging<D> st;
  int ids_cur[4], ids_nxt[4];
  tile_ids(0, ids_cur);
  fetch_tile<D>(st, pool, ids_cur, head, H, tid);
  if (n_tiles > 1) tile_ids(1, ids_nxt);

  for (int t = 0; t < n_tiles; ++t) {
    const int kt = it.k_begin + t * kTileK;
    if (it.k_end - kt >= kTileK)
      stage_tile<D, false>(st, ks, vs, tid, kTileK);
    else
      stage_tile<D, true>(st, ks, vs, tid, it.k_end - kt);
    __syncthreads();
    if (t + 1 < n_tiles) {
      fetch_tile<D>(st, pool, ids_nxt, head, H, tid);
      if (t + 2 < n_tiles) tile_ids(t + 2, ids_nxt);
    }
    if (kt <= wave_pos_hi) {  // otherwise every key of the tile is in this wave's future
      wave_step<D>(ks, vs, qreg, acc_o, m, l, kt, pos, col, hl, sc, kt + kTileK - 1 > wave_pos_lo);
    }
    __syncthreads();
  }

  // ---- epilogue: lane holds O^T[d][col] for d = 32 dt + 8 (i/4) + 4 hl + i%4
  l += __shfl_xor(l, 32);
  if (row_ok) {
    if (it.slot0 < 0) {
      const float inv = 1.0f / l;
      uint16_t* op = p.out + ((int64_t)(it.qrow0 + r) * H + head) * D;
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
      const int64_t ps = (int64_t)(it.slot0 + r * it.nparts) * H + head;
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

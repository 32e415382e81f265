// Tile path for head_dim 256: the work item, staging, online softmax and epilogue of tile_body.h (recomputation
// chunks, Section 4.2, on the matrix cores), with 16 query rows per wave instead of 32.
//
// Why: 32 rows x 256 dims of fp32 accumulators (128 registers) plus the wave's Q^T (64) leave no room for a second
// wave on a SIMD, and a lone wave has nothing to hide its LDS and memory waits behind.  With 16 rows per wave
// (v_mfma_f32_16x16x32_bf16) a wave holds 64 accumulator and 32 Q^T registers, a workgroup is 8 waves of 16 rows
// (the same 128-row tile), and two waves share every SIMD.  The price is LDS traffic: every K and V operand read now
// feeds half as many multiply-adds.
//   - S^T = K Q^T per 16-key subtile: A = K[16 keys][32 dims] from LDS (lane: key = lane % 16, dims 8 (lane / 16) ..+7),
//     B = Q^T from registers; result: lane holds query column lane % 16, keys 4 (lane / 16) ..+3 of the subtile.
//   - O^T += V^T P^T per 32 keys (two subtiles) and 16 dims: the two subtiles' weights of a lane, rounded to bf16, ARE
//     the B operand (slot j < 4 of lane group g <-> key 4 g + j of the first subtile, slot 4 + j <-> the same key of the
//     second); the A operand comes from two LDS transpose loads in that key order.
#pragma once

#include "tile_body.h"

namespace ic {
namespace tile16 {

using namespace tilep;

template <int D>
struct G16 {
  static constexpr int kRows = 16;                        // query rows (x heads of a group) per wave
  static constexpr int kWaves = tile_rows(D) / kRows;     // 8 for head_dim 256
  static constexpr int kThreads = 64 * kWaves;
  // bf16 per LDS row of K and of V: rows shift by 8 of the 64 banks (32 bytes).  An operand read of K takes 16 bytes of
  // 16 keys per quarter wave, a transpose read of V 32 bytes of 8 keys per half wave: both then cover all banks once
  // (measured: with the 16-byte shift of tile_body.h the K reads of this layout are 5 % slower, with its 64-byte
  // shift the V reads conflict two ways).
  static constexpr int kKStride = D + 16;
  static constexpr int kVStride = D + 16;
  static constexpr int kChunks = D / 8;                   // 16-byte chunks per token row
  static constexpr int kLoads = kTileK * kChunks / kThreads;  // K (and V) chunks per thread and tile
  static constexpr int kQSteps = D / 32;                  // MFMA k-steps of Q K^T
  static constexpr int kDTiles = D / 16;                  // 16-row tiles of O^T
  static_assert(kTileK * kChunks % kThreads == 0, "a tile must split evenly over the threads");
  static_assert(kThreads <= 1024, "workgroup size");
};

template <int D>
struct Staging16 {
  u32x4 k[G16<D>::kLoads];
  u32x4 v[G16<D>::kLoads];
};

// Global -> registers for one 64-key tile: thread u takes 16-byte chunk u + kThreads j of the K tile and of the V
// tile; a wave's 64 chunks of one load lie in one (block, head) tile and are consecutive: fully coalesced.
template <int D>
__device__ __forceinline__ void fetch_tile16(Staging16<D>& st, const char* pool, const int (&ids)[4], int head, int H,
                                             int tid) {
  using G = G16<D>;
  constexpr int kTileBytes = kBlockSize * D * 2;
  const int64_t blk_stride = (int64_t)2 * H * kTileBytes;
#pragma unroll
  for (int j = 0; j < G::kLoads; ++j) {
    const int u = tid + G::kThreads * j;
    const int tok = u / G::kChunks;  // 0..63
    const int c = u % G::kChunks;
    const int bsel = __builtin_amdgcn_readfirstlane(tok / kBlockSize);  // wave-uniform
    const char* a = pool + (int64_t)head * kTileBytes + (int64_t)ids[bsel] * blk_stride + (tok % kBlockSize) * (D * 2) + c * 16;
    st.k[j] = *(const u32x4*)a;
    st.v[j] = *(const u32x4*)(a + (int64_t)H * kTileBytes);
  }
}

// Registers -> LDS as [key][dim] rows (padded).  V of keys >= n_valid is zeroed (dead slots may hold NaN).
template <int D>
__device__ __forceinline__ void stage_tile16(const Staging16<D>& st, uint16_t* ks, uint16_t* vs, int tid, int n_valid) {
  using G = G16<D>;
#pragma unroll
  for (int j = 0; j < G::kLoads; ++j) {
    const int u = tid + G::kThreads * j;
    const int tok = u / G::kChunks, c = u % G::kChunks;
    *(u32x4*)(ks + tok * G::kKStride + c * 8) = st.k[j];
    u32x4 v = st.v[j];
    if (tok >= n_valid) v = (u32x4){0u, 0u, 0u, 0u};
    *(u32x4*)(vs + tok * G::kVStride + c * 8) = v;
  }
}

// A operand of O^T += V^T P^T for dims d0 .. d0 + 15 and the 32 keys of half h of the tile, in the key order of the
// weights (see the head of this file).  The LDS transpose load (layout measured on gfx950): in a group of 16 lanes,
// lane j points at 8 bytes and lane i receives element i % 4 of the pieces of lanes i / 4, i / 4 + 4, i / 4 + 8,
// i / 4 + 12.  Lane j of group g points at V[key 4 g + j / 4][dims d0 + 4 (j % 4) ..+3]; lane i then holds dim d0 + i
// of keys 4 g ..+3.
template <int D>
__device__ __forceinline__ bf16x8 read_vt16(const uint16_t* vs, int d0, int h, int lane) {
  using G = G16<D>;
  typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
  const int g = lane >> 4, j = lane & 15;
  const uint16_t* a = vs + (32 * h + 4 * g + (j >> 2)) * G::kVStride + d0 + 4 * (j & 3);
  const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)a);
  const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(a + 16 * G::kVStride));
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// One 64-key tile for one wave.  mask is set only for tiles that straddle the wave's causal diagonal.
// kPin: pin the order of operand reads and MFMAs written here (costs about ten registers; the build that shares its
// SIMDs with another kernel cannot afford them).
template <int D, bool kPin>
__device__ __forceinline__ void wave_step16(const uint16_t* ks, const uint16_t* vs, const bf16x8 (&qreg)[G16<D>::kQSteps],
                                            f32x4 (&acc_o)[G16<D>::kDTiles], float& m, float& l, int kt, int pos, int lane,
                                            float sc, bool mask) {
  using G = G16<D>;
  const int col = lane & 15, g = lane >> 4;
  f32x4 s[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) s[u] = (f32x4){0.f, 0.f, 0.f, 0.f};
  {
    // The four 16-key subtiles advance together (four independent accumulators alternate in the matrix pipe), and the
    // A operands of the next k-step are read from LDS before this step's MFMAs issue: the kernel is bound by LDS
    // operand reads, and left to itself the compiler keeps only one or two of them in flight per wave.
    const uint16_t* kp = ks + col * G::kKStride + 8 * g;
    bf16x8 a[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) a[u] = *(const bf16x8*)(kp + 16 * u * G::kKStride);
#pragma unroll
    for (int t = 0; t < G::kQSteps; ++t) {
      bf16x8 n[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) n[u] = t + 1 < G::kQSteps ? *(const bf16x8*)(kp + 16 * u * G::kKStride + 32 * (t + 1)) : a[u];
#pragma unroll
      for (int u = 0; u < 4; ++u) s[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u], qreg[t], s[u], 0, 0, 0);
#pragma unroll
      for (int u = 0; u < 4; ++u) a[u] = n[u];
    }
    // pin that order (0x100: LDS reads, 0x008: MFMAs): the scheduler otherwise moves every read next to its use
    if constexpr (kPin) {
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
      for (int t = 0; t + 1 < G::kQSteps; ++t) {
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
    }
  }
  // this lane: query column col, keys kt + 16 u + 4 g + i
  if (mask) {  // wave-uniform; the empty asm keeps this a branch instead of 16 always-on selects
    asm volatile("" ::: "memory");
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i) s[u][i] = kt + 16 * u + 4 * g + i > pos ? -__builtin_inff() : s[u][i];
  }
  float tmax = -__builtin_inff();
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int i = 0; i < 4; ++i) tmax = __builtin_fmaxf(tmax, s[u][i]);
  tmax *= sc;
  // Lazy reference maximum: a lane looks at its own 16 scores; the wave reduces across the four lanes of a column
  // (and rescales) only when some score exceeds its column's reference by more than 2^kLazyLog2.
  if (__builtin_amdgcn_ballot_w64(tmax > m + kLazyLog2) != 0) {
    tmax = __builtin_fmaxf(tmax, __shfl_xor(tmax, 16));
    tmax = __builtin_fmaxf(tmax, __shfl_xor(tmax, 32));
    const float m_cand = __builtin_fmaxf(m, tmax);
    const bool grew = m_cand > m + kLazyLog2;  // the same in the four lanes of a column
    const float alpha = grew ? __builtin_amdgcn_exp2f(m - m_cand) : 1.0f;
    m = grew ? m_cand : m;
    l *= alpha;
#pragma unroll
    for (int dt = 0; dt < G::kDTiles; ++dt)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc_o[dt][i] *= alpha;
  }
  // weights rounded to bf16 in pairs and summed as rounded: the normaliser counts what the matrix core multiplies
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
  bf16x8 pb[2];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int i = 0; i < 4; i += 2) {
      const bf16x2 pr = {(__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(s[u][i], sc, -m)),
                         (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(s[u][i + 1], sc, -m))};
      l = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, l, false);
      pb[u >> 1][4 * (u & 1) + i] = pr[0];
      pb[u >> 1][4 * (u & 1) + i + 1] = pr[1];
    }
  // O^T += V^T P^T: the 32-key half outer, so that the kDTiles independent accumulators alternate; operands are
  // read four MFMAs ahead.
  {
    constexpr int kAhead = 4, kOps = 2 * G::kDTiles;
    bf16x8 a[kAhead];
#pragma unroll
    for (int i = 0; i < kAhead; ++i) a[i] = read_vt16<D>(vs, 16 * (i % G::kDTiles), i / G::kDTiles, lane);
#pragma unroll
    for (int i = 0; i < kOps; ++i) {
      const bf16x8 cur = a[i % kAhead];
      if (i + kAhead < kOps) a[i % kAhead] = read_vt16<D>(vs, 16 * ((i + kAhead) % G::kDTiles), (i + kAhead) / G::kDTiles, lane);
      acc_o[i % G::kDTiles] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(cur, pb[i / G::kDTiles], acc_o[i % G::kDTiles], 0, 0, 0);
    }
    if constexpr (kPin) {  // two transpose loads per operand
      __builtin_amdgcn_sched_group_barrier(0x100, 2 * kAhead, 0);
#pragma unroll
      for (int i = 0; i < kOps; ++i) {
        if (i + kAhead < kOps) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      }
    }
  }
}

template <int D>
constexpr int tile16_buf_elems() {
  return kTileK * G16<D>::kKStride + kTileK * G16<D>::kVStride;
}
template <int D>
constexpr int tile16_lds_bytes() {
  return 2 * tile16_buf_elems<D>() * 2;  // two buffers of bf16
}

// One TileItem x one group of (1 << p.tile_g_shift) query heads that share a K/V head, executed by a workgroup of
// tile_rows(D) / 16 waves (see tile_body in tile_body.h for the row mapping).  lds: tile16_lds_bytes<D>() bytes.
template <int D, bool kPin>
__device__ __forceinline__ void tile16_body(const AttnParams& p, const TileItem& it, int th, uint16_t* lds) {
  using G = G16<D>;
  const int H = p.num_heads, Hk = p.num_kv_heads, gs = p.tile_g_shift;
  const int head0 = th << gs;
  const int kvh = head0 / p.group;
  const int n_rows_t = it.n_rows << gs;  // rows of the tile: query rows x heads of the group
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 15, g = lane >> 4;

  const int r = G::kRows * w + col;                  // row inside the tile
  const int r_eff = min(r, n_rows_t - 1);            // dead rows mirror the last live one
  const int pos = it.pos0 + (r_eff >> gs);           // last visible key of this lane's row
  const int wave_pos_lo = it.pos0 + min((G::kRows * w) >> gs, it.n_rows - 1);
  const int wave_pos_hi = it.pos0 + min((G::kRows * w + G::kRows - 1) >> gs, it.n_rows - 1);
  bf16x8 qreg[G::kQSteps];
  {
    const int head = head0 + (r_eff & ((1 << gs) - 1));
    const uint16_t* qp = p.q + ((int64_t)(it.qrow0 + (r_eff >> gs)) * H + head) * D + 8 * g;
#pragma unroll
    for (int t = 0; t < G::kQSteps; ++t) qreg[t] = *(const bf16x8*)(qp + 32 * t);
  }
  f32x4 acc_o[G::kDTiles];
#pragma unroll
  for (int dt = 0; dt < G::kDTiles; ++dt) acc_o[dt] = (f32x4){0.f, 0.f, 0.f, 0.f};
  float m = kNegBig, l = 0.f;

  const char* pool = (const char*)p.pool;
  typedef __attribute__((address_space(4))) const int32_t const_i32;
  const_i32* bt = (const_i32*)(p.bt_flat + p.bt_off[it.seq]);  // wave-uniform, read-only: scalar loads
  const int last_blk = (it.k_end - 1) / kBlockSize;
  const int n_tiles = (it.k_end - it.k_begin + kTileK - 1) / kTileK;
  const float sc = p.scale_log2e;
  auto tile_ids = [&](int t, int (&ids)[4]) {
    const int b0 = (it.k_begin + t * kTileK) / kBlockSize;
#pragma unroll
    for (int i = 0; i < 4; ++i) ids[i] = bt[min(b0 + i, last_blk)];
  };

  // Pipeline as in tile_body.h with one register set: in step t every wave computes on LDS buffer t % 2, copies
  // tile t + 1 from its registers into the other buffer, reloads the registers with tile t + 2; one barrier ends
  // the step.  Fetches are unconditional: tiles past the item's end re-read its last block and are never staged.
  constexpr int kBuf = tile16_buf_elems<D>();
  Staging16<D> st;
  int ids[4];
  tile_ids(0, ids);
  fetch_tile16<D>(st, pool, ids, kvh, Hk, tid);
  stage_tile16<D>(st, lds, lds + kTileK * G::kKStride, tid, it.k_end - it.k_begin);
  tile_ids(1, ids);
  fetch_tile16<D>(st, pool, ids, kvh, Hk, tid);
  tile_ids(2, ids);
  __syncthreads();
  // Waves w and w + 4 share a SIMD: one does its arithmetic first and its copy after, the other the reverse.
  const bool copy_first = (w & 4) != 0;
  for (int t = 0; t < n_tiles; ++t) {
    const int kt = it.k_begin + t * kTileK;
    const uint16_t* ks = lds + (t & 1) * kBuf;
    const uint16_t* vs = ks + kTileK * G::kKStride;
    uint16_t* nks = lds + ((t + 1) & 1) * kBuf;
    auto copy = [&]() {
      if (t + 1 < n_tiles) stage_tile16<D>(st, nks, nks + kTileK * G::kKStride, tid, it.k_end - (kt + kTileK));
    };
    if (copy_first) copy();
    if (kt <= wave_pos_hi)  // otherwise every key of the tile is in this wave's future
      wave_step16<D, kPin>(ks, vs, qreg, acc_o, m, l, kt, pos, lane, sc, kt + kTileK - 1 > wave_pos_lo);
    if (!copy_first) copy();
    fetch_tile16<D>(st, pool, ids, kvh, Hk, tid);
    tile_ids(t + 3, ids);
    __syncthreads();
  }

  // ---- epilogue: lane holds O^T[d][col] for d = 16 dt + 4 g + i
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  if (r < n_rows_t) {
    const int qr = r >> gs;
    const int head = head0 + (r & ((1 << gs) - 1));
    if (it.slot0 < 0) {
      const float inv = 1.0f / l;
      uint16_t* op = p.out + ((int64_t)(it.qrow0 + qr) * H + head) * D;
#pragma unroll
      for (int dt = 0; dt < G::kDTiles; ++dt) {
        bf16x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (__bf16)(acc_o[dt][e] * inv);  // round to nearest even
        *(bf16x4*)(op + 16 * dt + 4 * g) = o;
      }
    } else {
      const int64_t ps = (int64_t)(it.slot0 + qr * it.nparts) * H + head;
      float* op = p.part_o + ps * D;
#pragma unroll
      for (int dt = 0; dt < G::kDTiles; ++dt) *(f32x4*)(op + 16 * dt + 4 * g) = acc_o[dt];
      if (g == 0) {
        p.part_ml[ps * 2] = m;
        p.part_ml[ps * 2 + 1] = l;
      }
    }
  }
}

}  // namespace tile16
}  // namespace ic

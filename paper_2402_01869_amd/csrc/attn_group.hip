// Group kernel: decode rows of a grouped-query pool (Section 5's largest model has 64 query heads over
// 8 K/V heads).  The G query heads of a group read the same keys, so one workgroup takes a RowItem
// for a whole group: the G heads are the columns of an MFMA tile (padded to 32), every key is read
// from HBM once per group instead of once per head, and the arithmetic per key byte (G times that
// of multi-head decode) runs on the matrix cores while the kernel stays HBM-bound.
//
// One workgroup = one RowItem x one K/V head, 4 waves.  The waves work independently, without
// barriers: wave w takes the item's 32-key tiles w, w+4, ...; for each it
//   - loads the tile (2 cache blocks of K and of V, 16-byte coalesced loads) into registers, one tile
//     ahead of the arithmetic,
//   - copies it to its OWN slice of LDS ([key][dim] rows, padded; V of dead slots zeroed),
//   - S^T = K Q^T (keys x heads), online softmax per head, O^T += V^T P^T, as in the tile kernel
//     (same operand layouts, V through the LDS transpose loads).
// At the end the four waves' (m, l, O) are combined through LDS and written as bf16 rows, or as
// split-KV partial results for the merge kernel.
#include "tile_body.h"

namespace ic {

namespace {

using namespace tilep;

constexpr int kGroupWaves = 4;
constexpr int kGT = 32;  // keys per wave tile: two cache blocks

template <int D>
constexpr int wave_lds_elems() {
  return kGT * (TG<D>::kKStride + TG<D>::kVStride);  // bf16 elements of one wave's K and V tile
}
template <int D>
constexpr int group_lds_bytes() {
  return kGroupWaves * wave_lds_elems<D>() * 2;
}

template <int D>
struct GStage {
  static constexpr int kLoads = kGT * (D / 8) / 64;  // 16-byte chunks per lane for K (and for V)
  u32x4 k[kLoads];
  u32x4 v[kLoads];
};

// Chunk c of a 32-key tile (c = lane + 64 j): block c / (16 D/8), then linear inside the block's
// (K or V, head) tile, which is contiguous in the pool.
template <int D>
__device__ __forceinline__ void group_fetch(GStage<D>& st, const char* pool, int id0, int id1, int kvh, int Hk,
                                            int lane) {
  constexpr int kTileBytes = kBlockSize * D * 2;
  constexpr int kChunksPerBlock = kBlockSize * D / 8;
  const int64_t blk_stride = (int64_t)2 * Hk * kTileBytes;
  const char* base = pool + (int64_t)kvh * kTileBytes;
#pragma unroll
  for (int j = 0; j < GStage<D>::kLoads; ++j) {
    const int c = lane + 64 * j;
    const int id = (c / kChunksPerBlock) ? id1 : id0;  // uniform per j: 64 divides kChunksPerBlock
    const char* a = base + (int64_t)id * blk_stride + (c % kChunksPerBlock) * 16;
    st.k[j] = __builtin_nontemporal_load((const u32x4*)a);
    st.v[j] = __builtin_nontemporal_load((const u32x4*)(a + (int64_t)Hk * kTileBytes));
  }
}

template <int D>
__device__ __forceinline__ void group_stage(const GStage<D>& st, uint16_t* ks, uint16_t* vs, int lane, int n_valid) {
  using G = TG<D>;
#pragma unroll
  for (int j = 0; j < GStage<D>::kLoads; ++j) {
    const int c = lane + 64 * j;
    const int tok = c / (D / 8), dc = c % (D / 8);
    *(u32x4*)(ks + tok * G::kKStride + dc * 8) = st.k[j];
    u32x4 v = st.v[j];
    if (tok >= n_valid) v = (u32x4){0u, 0u, 0u, 0u};  // dead slots may hold NaN
    *(u32x4*)(vs + tok * G::kVStride + dc * 8) = v;
  }
}

// One 32-key tile for one wave.  n_valid < 32 only for the last tile of the item.
template <int D>
__device__ __forceinline__ void group_step(const uint16_t* ks, const uint16_t* vs, const bf16x8 (&qreg)[TG<D>::kQSteps],
                                           f32x16 (&acc_o)[TG<D>::kDTiles], float& m, float& l, int n_valid, int col,
                                           int hl, float sc) {
  using G = TG<D>;
  f32x16 s_acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) s_acc[i] = 0.f;
  {
    const uint16_t* kp = ks + col * G::kKStride + 8 * hl;
    bf16x8 a = *(const bf16x8*)kp;
#pragma unroll
    for (int s = 0; s < G::kQSteps; ++s) {
      bf16x8 n = a;
      if (s + 1 < G::kQSteps) n = *(const bf16x8*)(kp + 16 * (s + 1));
      s_acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[s], s_acc, 0, 0, 0);
      a = n;
    }
  }
  if (n_valid < kGT) {  // wave-uniform
    asm volatile("" ::: "memory");
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int key = 8 * (i / 4) + 4 * hl + (i % 4);
      s_acc[i] = key >= n_valid ? -__builtin_inff() : s_acc[i];
    }
  }
  float tmax = -__builtin_inff();
#pragma unroll
  for (int i = 0; i < 16; ++i) tmax = __builtin_fmaxf(tmax, s_acc[i]);
  tmax = __builtin_fmaxf(tmax, __shfl_xor(tmax, 32));
  // Lazy reference: the running maximum m only has to bound the scores loosely.  It is moved (and the
  // accumulators rescaled, 16 multiplies per 32 output rows) only when a score exceeds it by more than
  // kLazyLog2; until then weights may reach 2^kLazyLog2, which fp32 sums and bf16 weights hold easily.
  const float m_cand = __builtin_fmaxf(m, tmax * sc);
  const bool grew = m_cand > m + kLazyLog2;
  const float m_new = grew ? m_cand : m;
  const float alpha = grew ? __builtin_amdgcn_exp2f(m - m_cand) : 1.0f;
  m = m_new;
  // weights rounded to bf16 in pairs and summed as rounded (bf16 dot product with (1, 1)): the
  // normaliser counts exactly what the matrix core multiplies
  float psum = 0.f;
  bf16x8 pb[2];
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
  for (int i = 0; i < 16; i += 2) {
    const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[i], sc, -m_new));
    const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_acc[i + 1], sc, -m_new));
    const bf16x2 pr = {(__bf16)p0, (__bf16)p1};
    psum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, psum, false);
    pb[i / 8][i % 8] = pr[0];
    pb[i / 8][i % 8 + 1] = pr[1];
  }
  l = l * alpha + psum;
  if (__builtin_amdgcn_ballot_w64(grew) != 0) {
#pragma unroll
    for (int dt = 0; dt < G::kDTiles; ++dt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc_o[dt][i] *= alpha;
  }
  const int lane = col + 32 * hl;
#pragma unroll
  for (int ksp = 0; ksp < 2; ++ksp) {
    bf16x8 a[G::kDTiles];
#pragma unroll
    for (int dt = 0; dt < G::kDTiles; ++dt) a[dt] = read_vt_operand<D>(vs, 32 * dt, ksp, lane);
#pragma unroll
    for (int dt = 0; dt < G::kDTiles; ++dt)
      acc_o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[dt], pb[ksp], acc_o[dt], 0, 0, 0);
  }
}

template <int D>
__device__ __forceinline__ void group_body(const AttnParams& p, const RowItem& it, int kvh, uint16_t* lds) {
  using G = TG<D>;
  const int H = p.num_heads, Hk = p.num_kv_heads, Gq = p.group;  // Gq <= 32 query heads per K/V head
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31, hl = lane >> 5;
  const int head = kvh * Gq + min(col, Gq - 1);  // columns past the group mirror its last head

  bf16x8 qreg[G::kQSteps];
  {
    const uint16_t* qp = p.q + ((int64_t)it.qrow * H + head) * D + 8 * hl;
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
  const int last_blk = (it.k_end - 1) / kBlockSize;
  const int n_tiles = (it.k_end - it.k_begin + kGT - 1) / kGT;
  const float sc = p.scale_log2e;
  uint16_t* ks = lds + w * wave_lds_elems<D>();
  uint16_t* vs = ks + kGT * G::kKStride;

  auto fetch = [&](GStage<D>& st, int t) {
    const int b0 = (it.k_begin + t * kGT) / kBlockSize;
    group_fetch<D>(st, pool, bt[b0], bt[min(b0 + 1, last_blk)], kvh, Hk, lane);
  };
  GStage<D> st;
  if (w < n_tiles) fetch(st, w);
  for (int t = w; t < n_tiles; t += kGroupWaves) {
    const int n_valid = it.k_end - (it.k_begin + t * kGT);
    group_stage<D>(st, ks, vs, lane, n_valid);
    if (t + kGroupWaves < n_tiles) fetch(st, t + kGroupWaves);
    // the slice is private to this wave, whose LDS operations execute in order: a fence is enough
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
    group_step<D>(ks, vs, qreg, acc_o, m, l, n_valid, col, hl, sc);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");
  }

  // ---- combine the waves: each parks O^T (live columns), m and l in its own slice
  l += __shfl_xor(l, 32);
  float* my_o = (float*)(lds + w * wave_lds_elems<D>());  // [col][d]
  float* my_ml = my_o + 32 * D;                            // [col][2]
  static_assert((32 * D + 64) * 4 <= wave_lds_elems<D>() * 2, "wave slice too small for the combine");
  if (col < Gq) {
#pragma unroll
    for (int dt = 0; dt < G::kDTiles; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int d = 32 * dt + 8 * g + 4 * hl;
        *(f32x4*)(my_o + col * D + d) =
            (f32x4){acc_o[dt][4 * g], acc_o[dt][4 * g + 1], acc_o[dt][4 * g + 2], acc_o[dt][4 * g + 3]};
      }
    if (hl == 0) {
      my_ml[2 * col] = m;
      my_ml[2 * col + 1] = l;
    }
  }
  __syncthreads();
  const float* base = (const float*)lds;
  constexpr int kSliceF = wave_lds_elems<D>() / 2;  // floats per wave slice
  for (int idx = tid; idx < Gq * D; idx += 64 * kGroupWaves) {
    const int c = idx / D, d = idx - c * D;
    float M = kNegBig;
#pragma unroll
    for (int ww = 0; ww < kGroupWaves; ++ww) M = __builtin_fmaxf(M, base[ww * kSliceF + 32 * D + 2 * c]);
    float L = 0.f, O = 0.f;
#pragma unroll
    for (int ww = 0; ww < kGroupWaves; ++ww) {
      const float* sl = base + ww * kSliceF;
      const float wgt = __builtin_amdgcn_exp2f(sl[32 * D + 2 * c] - M);
      L = __builtin_fmaf(sl[32 * D + 2 * c + 1], wgt, L);
      O = __builtin_fmaf(sl[c * D + d], wgt, O);
    }
    const int hq = kvh * Gq + c;
    if (it.slot < 0) {
      const __bf16 o = (__bf16)(O / L);  // round to nearest even
      p.out[((int64_t)it.qrow * H + hq) * D + d] = __builtin_bit_cast(uint16_t, o);
    } else {
      const int64_t ps = (int64_t)it.slot * H + hq;
      p.part_o[ps * D + d] = O;
      if (d == 0) {
        p.part_ml[ps * 2] = M;
        p.part_ml[ps * 2 + 1] = L;
      }
    }
  }
}

template <int D>
__global__ __launch_bounds__(64 * kGroupWaves, (D <= 128 ? 2 : 1)) void group_attn_kernel(AttnParams p) {
  __shared__ __attribute__((aligned(16))) uint16_t lds[group_lds_bytes<D>() / 2];
  const int Hk = p.num_kv_heads;
  const uint32_t wg = blockIdx.x;
  const int item_idx = wg / Hk;
  const int kvh = wg - item_idx * Hk;
  const RowItem it = p.row_items[p.n_vec_items + item_idx];  // the group kernel's items follow the vector kernel's
  group_body<D>(p, it, kvh, lds);
}

}  // namespace

hipError_t launch_group_kernel(const AttnParams& p, int head_dim, hipStream_t st) {
  const int n_items = p.n_row_items - p.n_vec_items;
  if (n_items <= 0) return hipSuccess;
  if (p.group < 2 || p.group > 32) return hipErrorInvalidValue;
  const uint64_t grid = (uint64_t)n_items * (uint64_t)p.num_kv_heads;
  if (grid > 0x7fffffffull) return hipErrorInvalidValue;
  const dim3 g((uint32_t)grid), b(64 * kGroupWaves);
  switch (head_dim) {
    case 64: hipLaunchKernelGGL(group_attn_kernel<64>, g, b, 0, st, p); break;
    case 128: hipLaunchKernelGGL(group_attn_kernel<128>, g, b, 0, st, p); break;
    case 256: hipLaunchKernelGGL(group_attn_kernel<256>, g, b, 0, st, p); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace ic

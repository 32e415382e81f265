// Row path of the attention kernels: one query row (a decode token, Section 4.2) against a range
// of its sequence's paged keys.  One flop per KV byte, so this path is HBM-bound and runs on the
// vector ALU: the job is to keep many 16-byte loads in flight, not to feed MFMA.
//
// Mapping (one workgroup of 4 waves = one RowItem x one head):
//   - a (block, K or V, head) tile is 16 tokens x D bf16, contiguous; a wave reads it as D/32
//     loads of 1 KiB, lane l taking bytes [16 l, 16 l + 16): fully coalesced, block-table driven
//   - a token row is D/8 adjacent lanes, each holding 8 dims; q . k is 4 v_dot2_f32_bf16 per lane
//     and a D/8-lane all-reduce (DPP inside a 16-lane row)
//   - every D/8-lane group keeps its own online-softmax state (m, l, acc[8]); groups and waves
//     are combined once, through LDS, at the end of the item
//   - wave w owns blocks w, w+4, ... of the item; tiles are register multi-buffered so the
//     next tiles' loads are in flight while the current one is consumed
// Scores are kept in log2 units (multiplied by scale * log2 e) so exp is one v_exp_f32.
#pragma once

#include "ic_internal.h"

namespace ic {
namespace rowp {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr float kNegBig = -1.0e30f;  // finite "no key seen yet" maximum (keeps exp2(m - m) = 1)

__device__ __forceinline__ float bf16lo(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float bf16hi(uint32_t u) {
  return __builtin_bit_cast(float, u & 0xffff0000u);
}

// fp32 -> bf16 bits, round to nearest even; NaN stays NaN.
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, false));
}

// Sum over groups of LANES adjacent lanes (LANES = 8, 16 or 32); every lane gets the total.
template <int LANES>
__device__ __forceinline__ float group_sum(float x) {
  x += dpp_f32<0xB1>(x);   // quad_perm [1,0,3,2]
  x += dpp_f32<0x4E>(x);   // quad_perm [2,3,0,1]
  x += dpp_f32<0x141>(x);  // row_half_mirror: the other quad of each 8
  if (LANES >= 16) x += dpp_f32<0x140>(x);  // row_mirror: the other half of each 16
  if (LANES >= 32) x += __shfl_xor(x, 16);
  return x;
}

template <int D>
struct Geo {
  static constexpr int kLanesPerTok = D / 8;             // 8, 16, 32
  static constexpr int kTokPerLoad = 64 / kLanesPerTok;  // 8, 4, 2
  static constexpr int kLoads = 16 / kTokPerLoad;        // 2, 4, 8 loads of 1 KiB per tile
  static constexpr int kGroups = kRowWaves * kTokPerLoad;
};

// NL loads of 1 KiB of K and of V: a whole (block, head) tile (NL = kLoads), or half of one.
template <int D, int NL = Geo<D>::kLoads>
struct Tile {
  u32x4 k[NL];
  u32x4 v[NL];
};

// j0: first 1 KiB piece of the (block, head) tile to load (0 for a whole tile).
template <int D, bool NT, int NL = Geo<D>::kLoads>
__device__ __forceinline__ void load_tile(Tile<D, NL>& t, const char* pool, int64_t blk, int head,
                                          int H, int lane, int j0 = 0) {
  constexpr int kTileBytes = kBlockSize * D * 2;
  const char* kb = pool + ((blk * 2) * H + head) * (int64_t)kTileBytes + lane * 16 + j0 * 1024;
  const char* vb = kb + (int64_t)H * kTileBytes;
#pragma unroll
  for (int j = 0; j < NL; ++j)
    t.k[j] = NT ? __builtin_nontemporal_load((const u32x4*)(kb + j * 1024))
                : *(const u32x4*)(kb + j * 1024);
#pragma unroll
  for (int j = 0; j < NL; ++j)
    t.v[j] = NT ? __builtin_nontemporal_load((const u32x4*)(vb + j * 1024))
                : *(const u32x4*)(vb + j * 1024);
}

// Consume one 16-token tile.  n_valid < 16 only for the last, partial block of a sequence: its
// dead slots may hold anything (NaN included), so their score is forced to -inf and their V to 0.
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c,
                                         false);
}

// n_valid counts from the first token this Tile holds.
template <int D, bool MASK, int NL = Geo<D>::kLoads>
__device__ __forceinline__ void consume_tile(const Tile<D, NL>& t, const u32x4& q2, float sc, float& m,
                                             float& l, float (&acc)[8], int n_valid, int lane) {
  float s[NL];
#pragma unroll
  for (int j = 0; j < NL; ++j) {
    // q . k over this lane's 8 dims: four bf16-pair dot products with fp32 accumulation
    const u32x4 kk = t.k[j];
    float d = dot2(q2[0], kk[0], 0.f);
    d = dot2(q2[1], kk[1], d);
    d = dot2(q2[2], kk[2], d);
    d = dot2(q2[3], kk[3], d);
    s[j] = group_sum<Geo<D>::kLanesPerTok>(d) * sc;
  }
  bool ok[NL];
  float m_new = m;
#pragma unroll
  for (int j = 0; j < NL; ++j) {
    ok[j] = true;
    if (MASK) {
      const int tok = j * Geo<D>::kTokPerLoad + lane / Geo<D>::kLanesPerTok;
      ok[j] = tok < n_valid;
      s[j] = ok[j] ? s[j] : -__builtin_inff();
    }
    m_new = __builtin_fmaxf(m_new, s[j]);
  }
  const float alpha = __builtin_amdgcn_exp2f(m - m_new);
  m = m_new;
  l *= alpha;
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] *= alpha;
#pragma unroll
  for (int j = 0; j < NL; ++j) {
    const float p = __builtin_amdgcn_exp2f(s[j] - m_new);
    l += p;
    u32x4 vv = t.v[j];
    if (MASK && !ok[j]) vv = (u32x4){0u, 0u, 0u, 0u};
    acc[0] = __builtin_fmaf(p, bf16lo(vv[0]), acc[0]);
    acc[1] = __builtin_fmaf(p, bf16hi(vv[0]), acc[1]);
    acc[2] = __builtin_fmaf(p, bf16lo(vv[1]), acc[2]);
    acc[3] = __builtin_fmaf(p, bf16hi(vv[1]), acc[3]);
    acc[4] = __builtin_fmaf(p, bf16lo(vv[2]), acc[4]);
    acc[5] = __builtin_fmaf(p, bf16hi(vv[2]), acc[5]);
    acc[6] = __builtin_fmaf(p, bf16lo(vv[3]), acc[6]);
    acc[7] = __builtin_fmaf(p, bf16hi(vv[3]), acc[7]);
  }
}

template <int D>
constexpr int row_lds_bytes() {
  return (Geo<D>::kGroups * D + 2 * Geo<D>::kGroups) * (int)sizeof(float);
}

// One RowItem x one head, executed by a workgroup of 4 waves.  PF = tiles prefetched ahead,
// NT = non-temporal KV loads.  lds: at least row_lds_bytes<D>() bytes of workgroup LDS.
// HALF (with PF = 0 only): a block is loaded and consumed in two halves of 8 tokens, which halves the registers a
// tile takes: the slim build for head_dim 256.
template <int D, int PF, bool NT, bool HALF = false>
__device__ __forceinline__ void row_body(const AttnParams& p, const RowItem& it, int head, float* lds) {
  using G = Geo<D>;
  constexpr int STAGES = PF + 1;  // register buffers
  static_assert(!HALF || (PF == 0 && G::kLoads % 2 == 0), "half-block steps have no prefetch");

  const int H = p.num_heads;
  const int Hk = p.num_kv_heads;
  const int kvh = head / p.group;   // the K/V head this query head reads
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

  const int k_begin = it.k_begin, k_end = it.k_end;
  const int nblk = (k_end - k_begin + kBlockSize - 1) / kBlockSize;
  const int32_t* bt = p.bt_flat + p.bt_off[it.seq] + k_begin / kBlockSize;
  // wave w owns blocks w, w+4, ...: lane i keeps the id of the wave's i-th block
  const int nb_w = (nblk - w + kRowWaves - 1) / kRowWaves;
  int my_id = 0;
  if (lane < nb_w) my_id = bt[w + kRowWaves * lane];

  // this lane's 8 query dims as bf16 pairs; scores are scaled into log2 units after the dot product
  const u32x4 q2 = *(const u32x4*)(p.q + ((int64_t)it.qrow * H + head) * D + (lane % G::kLanesPerTok) * 8);
  const float sc = p.scale_log2e;

  float m = kNegBig, l = 0.f;
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;

  const char* pool = (const char*)p.pool;
  if constexpr (HALF) {
    constexpr int NH = G::kLoads / 2;            // 1 KiB pieces per half
    constexpr int kHalfTok = kBlockSize / 2;
    for (int i = 0; i < nb_w; ++i) {
      const int id = __builtin_amdgcn_readlane(my_id, i);
      const int tok0 = k_begin + (w + kRowWaves * i) * kBlockSize;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int n_valid = k_end - tok0 - h * kHalfTok;
        if (n_valid <= 0) break;  // wave-uniform
        Tile<D, NH> t;
        load_tile<D, NT, NH>(t, pool, id, kvh, Hk, lane, h * NH);
        if (n_valid >= kHalfTok)
          consume_tile<D, false, NH>(t, q2, sc, m, l, acc, kHalfTok, lane);
        else
          consume_tile<D, true, NH>(t, q2, sc, m, l, acc, n_valid, lane);
      }
    }
  } else {
  Tile<D> buf[STAGES];
#pragma unroll
  for (int s = 0; s < PF; ++s)
    if (s < nb_w) load_tile<D, NT>(buf[s], pool, __builtin_amdgcn_readlane(my_id, s), kvh, Hk, lane);

  for (int it0 = 0; it0 < nb_w; it0 += STAGES) {
#pragma unroll
    for (int s = 0; s < STAGES; ++s) {
      const int i = it0 + s;
      if (i < nb_w) {
        if (i + PF < nb_w)
          load_tile<D, NT>(buf[(s + PF) % STAGES], pool, __builtin_amdgcn_readlane(my_id, i + PF), kvh,
                       Hk, lane);
        const int tok0 = k_begin + (w + kRowWaves * i) * kBlockSize;
        const int n_valid = k_end - tok0;
        if (n_valid >= kBlockSize)
          consume_tile<D, false>(buf[s], q2, sc, m, l, acc, kBlockSize, lane);
        else
          consume_tile<D, true>(buf[s], q2, sc, m, l, acc, n_valid, lane);
      }
    }
  }
  }

  // combine the lane groups of all waves through LDS
  float (*s_acc)[D] = (float (*)[D])lds;
  float* s_m = lds + G::kGroups * D;
  float* s_l = s_m + G::kGroups;
  {
    const int g = w * G::kTokPerLoad + lane / G::kLanesPerTok;
    const int d0 = (lane % G::kLanesPerTok) * 8;
    *(f32x4*)&s_acc[g][d0] = (f32x4){acc[0], acc[1], acc[2], acc[3]};
    *(f32x4*)&s_acc[g][d0 + 4] = (f32x4){acc[4], acc[5], acc[6], acc[7]};
    if (lane % G::kLanesPerTok == 0) {
      s_m[g] = m;
      s_l[g] = l;
    }
  }
  __syncthreads();
  const int d = threadIdx.x;
  if (d < D) {
    float M = kNegBig;
#pragma unroll
    for (int g = 0; g < G::kGroups; ++g) M = __builtin_fmaxf(M, s_m[g]);
    float L = 0.f, O = 0.f;
#pragma unroll
    for (int g = 0; g < G::kGroups; ++g) {
      const float wgt = __builtin_amdgcn_exp2f(s_m[g] - M);
      L = __builtin_fmaf(s_l[g], wgt, L);
      O = __builtin_fmaf(s_acc[g][d], wgt, O);
    }
    if (it.slot < 0) {
      p.out[((int64_t)it.qrow * H + head) * D + d] = (uint16_t)f32_to_bf16(O / L);
    } else {
      const int64_t ps = (int64_t)it.slot * H + head;
      p.part_o[ps * D + d] = O;
      if (d == 0) {
        p.part_ml[ps * 2] = M;
        p.part_ml[ps * 2 + 1] = L;
      }
    }
  }
}

}  // namespace rowp
}  // namespace ic

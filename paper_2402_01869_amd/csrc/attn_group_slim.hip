// Slim group kernel: the decode rows of a grouped-query pool (Section 5's largest model: 64 query heads over
// 8 K/V heads) for running BESIDE the tile kernel, as the slim row kernel does for multi-head pools.  Decode is
// memory-bound and recomputation is compute-bound (the complementarity Section 4.2 builds on), so one workgroup
// of each kind shares a CU.  Next to the two tile waves of a SIMD (208 registers each) 96 registers are left
// for one wave of this kernel; that budget shapes everything here:
//   - K and V travel from the paged pool STRAIGHT into LDS (global_load_lds_dwordx4): no staging registers, and
//     the loads in flight are bounded by LDS, not by the register file.  Every wave owns a ring of two stages
//     (one cache block of K and of V each, 16 keys); waves never wait for each other inside an item.
//   - The G <= 16 query heads of the group are the 16 columns of 16 x 16 MFMA tiles (the group kernel pads to
//     32): S^T = K Q^T with v_mfma_f32_16x16x32_bf16 (4 per block), O^T += V^T P^T with v_mfma_f32_16x16x16_bf16
//     (8 per block), whose B operand is exactly the layout S^T comes out in (lane: head = lane % 16, keys
//     4 (lane / 16) ..+3).  Accumulators: 32 registers, Q^T: 16.
//   - LDS rows are unpadded; bank conflicts are avoided by an XOR swizzle of the 16-byte chunk index applied on
//     the global side of the copy (every lane of a copy instruction owns the LDS slot of its lane number and
//     chooses which chunk of its key's row it fetches into it).
//   - Online softmax with a lazy reference maximum: a lane looks at its own four scores only, and the wave
//     reduces across lanes (and rescales) only when some score exceeds the reference by more than 2^8.
// Work items are the group kernel's (RowItem x K/V head), pulled from a queue by persistent workgroups of 4 waves;
// wave w takes the item's blocks w, w+4, ...; the four (m, l, O) are combined through LDS at the end.
#include <mutex>

#include "tile_body.h"

namespace ic {

namespace {

using namespace tilep;

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void glb_void;
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;

constexpr int kSlimWaves = 4;
constexpr int kSD = 128;                                  // head_dim (the only one built)
constexpr int kRowBytes = kSD * 2;                        // one key's K (or V) row
constexpr int kStageBytes = kBlockSize * kRowBytes;       // one block's K (or V) for one head: 4 KiB
constexpr int kWaveBytes = 4 * kStageBytes;               // K ring of two, V ring of two
// The request is padded past half of a CU's 160 KiB on purpose: two of these workgroups then never share a CU
// (which would leave no room for the tile workgroup, 74 KiB, that is meant to sit beside one of them).
constexpr int kSlimLdsBytes = 82 * 1024;
static_assert(kSlimWaves * kWaveBytes <= kSlimLdsBytes, "rings must fit the request");
static_assert(2 * kSlimLdsBytes > 160 * 1024, "two workgroups must not fit one CU");

// Swizzle terms: the value XORed into the chunk index (0..15) of key k's row.
//   K: 16 lanes read the same chunk of 16 keys -> 16 different slots of a 256-byte bank row.
//   V: the transpose read of 16 lanes covers 4 keys x 32 bytes, of 32 lanes 8 keys x 32 bytes -> 8 different
//      32-byte slots.
__device__ __forceinline__ int kswz(int key) { return key & 15; }
__device__ __forceinline__ int vswz(int key) { return ((key & 3) << 2) | (((key >> 2) & 1) << 1); }

// Wait until at most N vector-memory operations of this wave are outstanding and all of its LDS and scalar
// loads have completed (s_waitcnt, gfx9 encoding: vmcnt in bits 3:0 and 15:14, lgkmcnt in 11:8, expcnt 6:4
// left at "no wait").  The direct-to-LDS copies are invisible to the compiler's wait insertion, so the waits
// for them are written out, fenced against reordering by the compiler.
template <int N>
__device__ __forceinline__ void wait_vm() {
  static_assert(N >= 0 && N < 64, "vmcnt is six bits");
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (0 << 8));
  asm volatile("" ::: "memory");
}

// Direct copy of one block's K and V rows for one K/V head into a stage.  ks, vs: the stage's K and V buffers
// (wave-uniform); blk: the block's K rows for the head (wave-uniform), its V rows v_off bytes further; ko, vo: this
// lane's byte offsets for instruction 0 (see slim_body).  Instruction i covers keys 4 i .. 4 i + 3, lane =
// 16 (key % 4) + slot.  Buffer loads, because their address is a scalar base plus ONE register per lane (a global
// load wants a 64-bit address per lane and copy, 16 registers this kernel does not have); the descriptor covers
// exactly the bytes from the head's K rows to the end of its V rows in this block.  8 vector-memory operations.
template <int I>
__device__ __forceinline__ void copy_keys(__amdgpu_buffer_rsrc_t rsrc, char* ks, char* vs, uint32_t v_off, uint32_t ko,
                                          uint32_t vo) {
  // key 4 I + g: its row lies 1024 I further; the swizzle term of K changes by 4 I (chunk bits 3:2), of V by bit 1.
  // The instruction's immediate offset moves BOTH ends of the copy: the source address and the LDS address.
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void*)ks, 16, (int)(ko ^ (uint32_t)(I << 6)), 0, 1024 * I, 0);
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void*)vs, 16, (int)(vo ^ (uint32_t)((I & 1) << 5)), (int)v_off, 1024 * I, 0);
}
__device__ __forceinline__ void copy_block(char* ks, char* vs, const char* blk, uint32_t v_off, uint32_t ko, uint32_t vo) {
  const __amdgpu_buffer_rsrc_t rsrc =
      __builtin_amdgcn_make_buffer_rsrc((void*)blk, 0, (int)(v_off + kStageBytes), 0x00020000);
  copy_keys<0>(rsrc, ks, vs, v_off, ko, vo);
  copy_keys<1>(rsrc, ks, vs, v_off, ko, vo);
  copy_keys<2>(rsrc, ks, vs, v_off, ko, vo);
  copy_keys<3>(rsrc, ks, vs, v_off, ko, vo);
}

// LDS reads of copied data are written as assembly: the compiler orders every LDS read it knows of behind ALL
// direct-to-LDS copies in flight (it cannot tell the stages apart), which would end the prefetch.  The reads'
// completion is therefore waited for by hand (lds_wait); LDS operations of one wave execute in order.
__device__ __forceinline__ bf16x8 lds_read_b128(uint32_t addr) {
  bf16x8 v;
  asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr) : "memory");
  return v;
}
__device__ __forceinline__ bf16x4 lds_read_tr(uint32_t addr) {
  bf16x4 v;
  asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(v) : "v"(addr) : "memory");
  return v;
}
// All LDS reads of this wave have returned; the named registers are only valid after it.
__device__ __forceinline__ void lds_wait(bf16x8& a, bf16x8& b, bf16x8& c, bf16x8& d) {
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d)::"memory");
}
__device__ __forceinline__ void lds_wait(bf16x4 (&a)[8]) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7])::"memory");
}

// One block of 16 keys for one wave.  ks, vs: LDS byte addresses of the stage.  n_valid < 16 only for the last
// block of the item.
__device__ __forceinline__ void slim_step(uint32_t ks, uint32_t vs, const bf16x8 (&qreg)[4], f32x4 (&acc_o)[8],
                                          float& m, float& l, int n_valid, int lane, float sc) {
  const int col = lane & 15, g = lane >> 4;
  f32x4 s = {0.f, 0.f, 0.f, 0.f};
  {
    // A operand of k-step t: key col, dims 32 t + 8 g ..+7 = chunk 4 t + g, at slot (4 t + g) ^ kswz(col)
    const uint32_t a0 = ks + (uint32_t)(col * kRowBytes) + (uint32_t)((g ^ kswz(col)) << 4);
    bf16x8 a[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) a[t] = lds_read_b128(a0 ^ (uint32_t)(t << 6));
    lds_wait(a[0], a[1], a[2], a[3]);
#pragma unroll
    for (int t = 0; t < 4; ++t) s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[t], qreg[t], s, 0, 0, 0);
  }
  // A operands of O^T += V^T P^T for dims 16 dt ..+15: the LDS transpose load (layout measured on gfx950: in a
  // group of 16 lanes, lane j points at 8 bytes and lane i receives element i % 4 of the pieces of lanes i / 4,
  // i / 4 + 4, i / 4 + 8, i / 4 + 12).  Lane j points at V[key 4 g + j / 4][dims 16 dt + 4 (j % 4) ..+3]; lane i
  // then holds dim 16 dt + i of keys 4 g ..+3.  Issued here so that they return under the softmax arithmetic.
  bf16x4 va[8];
  {
    const int j = lane & 15, key = 4 * g + (j >> 2);
    const uint32_t va0 = vs + (uint32_t)(key * kRowBytes) + (uint32_t)((((j & 3) >> 1) ^ vswz(key)) << 4) + (uint32_t)((j & 1) << 3);
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) va[dt] = lds_read_tr(va0 ^ (uint32_t)(dt << 5));
  }
  // this lane: head col, keys 4 g + i
  if (n_valid < kBlockSize) {  // wave-uniform
#pragma unroll
    for (int i = 0; i < 4; ++i) s[i] = 4 * g + i >= n_valid ? -__builtin_inff() : s[i];
  }
  float tmax = __builtin_fmaxf(__builtin_fmaxf(s[0], s[1]), __builtin_fmaxf(s[2], s[3])) * sc;
  if (__builtin_amdgcn_ballot_w64(tmax > m + kLazyLog2) != 0) {
    // some score is far above its head's reference: move the references to the heads' maxima over the block
    tmax = __builtin_fmaxf(tmax, __shfl_xor(tmax, 16));
    tmax = __builtin_fmaxf(tmax, __shfl_xor(tmax, 32));
    const float m_cand = __builtin_fmaxf(m, tmax);
    const bool grew = m_cand > m + kLazyLog2;  // the same in the four lanes of a head
    const float alpha = grew ? __builtin_amdgcn_exp2f(m - m_cand) : 1.0f;
    m = grew ? m_cand : m;
    l *= alpha;
#pragma unroll
    for (int dt = 0; dt < 8; ++dt)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc_o[dt][i] *= alpha;
  }
  // weights rounded to bf16 in pairs and summed as rounded: the normaliser counts what the matrix core multiplies
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
  const bf16x2 p01 = {(__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(s[0], sc, -m)),
                      (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(s[1], sc, -m))};
  const bf16x2 p23 = {(__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(s[2], sc, -m)),
                      (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(s[3], sc, -m))};
  l = __builtin_amdgcn_fdot2_f32_bf16(p01, ones, l, false);
  l = __builtin_amdgcn_fdot2_f32_bf16(p23, ones, l, false);
  const bf16x4 pb4 = {p01[0], p01[1], p23[0], p23[1]};
  const s16x4 pb = __builtin_bit_cast(s16x4, pb4);
  lds_wait(va);
#pragma unroll
  for (int dt = 0; dt < 8; ++dt)
    acc_o[dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, va[dt]), pb, acc_o[dt], 0, 0, 0);
}

__device__ __forceinline__ void slim_body(const AttnParams& p, const RowItem& it, int kvh, char* lds) {
  constexpr int D = kSD;
  const int H = p.num_heads, Hk = p.num_kv_heads, Gq = p.group;  // 2 <= Gq <= 16
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 15, g = lane >> 4;
  const int head = kvh * Gq + min(col, Gq - 1);  // columns past the group mirror its last head

  bf16x8 qreg[4];
  {
    const uint16_t* qp = p.q + ((int64_t)it.qrow * H + head) * D + 8 * g;
#pragma unroll
    for (int t = 0; t < 4; ++t) qreg[t] = *(const bf16x8*)(qp + 32 * t);
  }
  f32x4 acc_o[8];
#pragma unroll
  for (int dt = 0; dt < 8; ++dt) acc_o[dt] = (f32x4){0.f, 0.f, 0.f, 0.f};
  float m = kNegBig, l = 0.f;

  typedef __attribute__((address_space(4))) const int32_t const_i32;
  const_i32* bt = (const_i32*)(p.bt_flat + p.bt_off[it.seq]) + it.k_begin / kBlockSize;
  const int n_blocks = (it.k_end - it.k_begin + kBlockSize - 1) / kBlockSize;
  const int n_mine = n_blocks > w ? (n_blocks - w + kSlimWaves - 1) / kSlimWaves : 0;  // blocks w, w + 4, ...
  const float sc = p.scale_log2e;
  constexpr int kBlkTileBytes = kBlockSize * D * 2;
  const int64_t blk_stride = (int64_t)2 * Hk * kBlkTileBytes;
  const uint32_t v_off = (uint32_t)Hk * kBlkTileBytes;  // from a block's K rows of a head to its V rows
  const char* pool = (const char*)p.pool + (int64_t)kvh * kBlkTileBytes;
  char* ring = lds + w * kWaveBytes;  // K stage s at ring + s * 4 KiB, V stage s at ring + (2 + s) * 4 KiB
  const uint32_t ring_a = (uint32_t)(uintptr_t)(lds_void*)ring;  // its LDS byte address
  // this lane's source offsets inside a block for copy instruction 0: key g, chunk slot ^ swizzle(g)
  const uint32_t ko = (uint32_t)(g * kRowBytes) + (uint32_t)(((lane & 15) ^ kswz(g)) << 4);
  const uint32_t vo = (uint32_t)(g * kRowBytes) + (uint32_t)(((lane & 15) ^ vswz(g)) << 4);

  auto block_id = [&](int jj) { return bt[w + kSlimWaves * min(jj, n_mine - 1)]; };
  auto issue = [&](int jj, int id) {
    char* ks = ring + (jj & 1) * kStageBytes;
    copy_block(ks, ks + 2 * kStageBytes, pool + (int64_t)id * blk_stride, v_off, ko, vo);
  };
  // Every store of the previous item and the Q loads above are out of the way before the copies are counted.
  wait_vm<0>();
  if (n_mine > 0) issue(0, block_id(0));
  if (n_mine > 1) issue(1, block_id(1));
  for (int jj = 0; jj < n_mine; ++jj) {
    const int id_next = block_id(jj + 2);  // a scalar load, back long before the copy below needs it
    // copies complete in order: all but the 8 of the younger stage have landed
    if (jj + 1 < n_mine) wait_vm<8>(); else wait_vm<0>();
    const int n_valid = it.k_end - it.k_begin - kBlockSize * (w + kSlimWaves * jj);
    if (n_valid < kBlockSize) {
      // dead slots may hold NaN, and 0 * NaN would poison the PV product: zero their V rows (a row is 256 bytes)
      char* vs = ring + ((jj & 1) + 2) * kStageBytes;
      for (int r = n_valid; r < kBlockSize; ++r) *(uint32_t*)(vs + r * kRowBytes + 4 * lane) = 0u;
    }
    const uint32_t ks_a = ring_a + (uint32_t)((jj & 1) * kStageBytes);
    slim_step(ks_a, ks_a + 2 * kStageBytes, qreg, acc_o, m, l, n_valid, lane, sc);
    if (jj + 2 < n_mine) {
      wait_vm<8>();  // no wait for copies (8 are in flight): this wave's reads of the stage have returned
      issue(jj + 2, id_next);
    }
  }

  // ---- combine the waves: each parks O^T (live columns), m and l in its own slice
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  wait_vm<0>();
  float* my_o = (float*)ring;        // [col][d]
  float* my_ml = my_o + 16 * D;      // [col][2]
  static_assert((16 * D + 32) * 4 <= kWaveBytes, "wave slice too small for the combine");
  if (col < Gq) {
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) *(f32x4*)(my_o + col * D + 16 * dt + 4 * g) = acc_o[dt];
    if (g == 0) {
      my_ml[2 * col] = m;
      my_ml[2 * col + 1] = l;
    }
  }
  __syncthreads();
  constexpr int kSliceF = kWaveBytes / 4;  // floats per wave slice
  const float* base = (const float*)lds;
  for (int idx = tid; idx < Gq * D; idx += 64 * kSlimWaves) {
    const int c = idx / D, d = idx - c * D;
    float M = kNegBig;
#pragma unroll
    for (int ww = 0; ww < kSlimWaves; ++ww) M = __builtin_fmaxf(M, base[ww * kSliceF + 16 * D + 2 * c]);
    float L = 0.f, O = 0.f;
#pragma unroll
    for (int ww = 0; ww < kSlimWaves; ++ww) {
      const float* sl = base + ww * kSliceF;
      const float wgt = __builtin_amdgcn_exp2f(sl[16 * D + 2 * c] - M);
      L = __builtin_fmaf(sl[16 * D + 2 * c + 1], wgt, L);
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

}  // namespace

// Persistent launch: `slots` workgroups pull (row item, K/V head) pairs from one queue (counters[kCtrGroupQueue],
// zero when the kernel starts; the last workgroup out puts it back to zero).  Register budget: 96 per lane (five
// waves per SIMD asked for), checked by the test-suite from the compiler's resource report.
__global__ __launch_bounds__(64 * kSlimWaves, 5) void group_slim_kernel(AttnParams p) {
  // Launch-time LDS: with the size in the kernel the compiler sees that one workgroup fits a CU, takes that as
  // leave to use the whole register file, and the workgroup no longer fits beside a tile workgroup.
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  __shared__ int s_next;
  const uint32_t Hk = (uint32_t)p.num_kv_heads;
  const uint32_t n = (uint32_t)(p.n_row_items - p.n_vec_items) * Hk;
  for (;;) {
    if (threadIdx.x == 0) s_next = atomicAdd(&p.counters[kCtrGroupQueue], 1);
    __syncthreads();
    const uint32_t idx = (uint32_t)s_next;
    __syncthreads();  // s_next is rewritten at the top of the next round
    if (idx >= n) break;
    const uint32_t item = idx / Hk;
    const RowItem it = p.row_items[(uint32_t)p.n_vec_items + item];  // the group kernels' items follow the vector kernel's
    slim_body(p, it, (int)(idx - item * Hk), lds);
    __syncthreads();  // the combine reads every wave's slice
  }
  queue_leave(p.counters, kCtrGroupQueue, 1, -1, kCtrGroupLeft);
}

hipError_t launch_group_slim(const AttnParams& p, int head_dim, int slots, hipStream_t st) {
  const int n_items = p.n_row_items - p.n_vec_items;
  if (n_items <= 0) return hipSuccess;
  if (head_dim != kSD || p.group < 2 || p.group > 16 || !p.counters || slots < 1) return hipErrorInvalidValue;
  if ((uint64_t)n_items * (uint64_t)p.num_kv_heads > 0x7fffffffull) return hipErrorInvalidValue;
  {  // more than 64 KiB of launch-time LDS has to be asked for, once per device
    static std::mutex mu;
    static bool asked[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!asked[dev]) {
      const hipError_t e =
          hipFuncSetAttribute((const void*)group_slim_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kSlimLdsBytes);
      if (e != hipSuccess) return e;
      asked[dev] = true;
    }
  }
  hipLaunchKernelGGL(group_slim_kernel, dim3((uint32_t)slots), dim3(64 * kSlimWaves), kSlimLdsBytes, st, p);
  return hipGetLastError();
}

}  // namespace ic

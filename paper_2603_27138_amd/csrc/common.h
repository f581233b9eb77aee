// Shared device helpers for the gfx950 kernels (wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "scout.h"

namespace scout {

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Internal launch parameters derived once on the host from scout_problem.
struct Dims {
  int B, Hq, Hkv, G, d, S, max_blocks, k;
  float sm_scale;
  int n_sink, n_tail;  // always-kept blocks at the start and at the end of a sequence
  int group_max;       // block importance: 0 = sum over the group's heads, 1 = their maximum
  int digest_kind;     // 0 = channel-wise min and max in the element type, 1 = binary32 sums of the keys (mean pooling)
  int share;           // consecutive pairs that share one digest / block-table row: 1, or with a selection
                       // per query head the real group size (then Hkv = Hq and G = 1 here)
  uint32_t share_magic;  // ceil(2^32 / share) for share > 1: pair / share without a division
  int s_shift;         // log2(S): integer divisions are slow enough here to show in the launch heads
  int tile_stride;     // elements from one slot's tile to the next, in k_pool and in v_pool alike: S * d for
                       // two dense pools, 2 * S * d where a slot's K tile and V tile lie next to each other
  const int32_t* ctx_len;
};

// Per-split partial results in the workspace, per pair and split:
//   o [pairs][nsplit][G][d]  unnormalised weighted value sums
//   m [pairs][nsplit][G]     maximum logit in base-2 units
//   l [pairs][nsplit][G]     sum of 2^(logit - m)
struct Partials {
  float* o;
  float* m;
  float* l;
  int nsplit;
  uint32_t waves_magic;  // MFMA family: ceil(2^32 / (nsplit * waves per workgroup)), 0 if that is 1
};

// What happens to a finished (sequence, query head) result.
//   mode 0: the workgroup's partial goes to the workspace (several splits per pair)
//   mode 1: export the GPU partial (o, m, l), m in natural-log units
//   mode 2: merge with the host's partial (Alg. 1 Merge) and write the final output
struct Epilogue {
  int mode;
  float* o;
  float* m;
  float* l;
  const float* host_o;
  const float* host_m;
  const float* host_l;
  void* out;
  float* lse;
  int dtype_out;
};

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t hi16) {
  return __uint_as_float(hi16 << 16);
}
// low / high half of a dword that packs two bf16 values
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// binary32 -> bf16 bits, round to nearest even (finite inputs; NaN stays NaN)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

// Index of the digest / block-table row a pair reads: pair / share.  Exact for pair < 2^16 and
// share <= 16 (the multiplication's error stays below 1 / share).
__device__ __forceinline__ int kv_row(const Dims& D, int pair) {
  return D.share == 1 ? pair : (int)__umulhi((uint32_t)pair, D.share_magic);
}

// Kernels that work pair by pair are launched with the KV head in grid dimension y and the sequence
// in z, so that neither has to be divided out of a pair index.
__device__ __forceinline__ int grid_pair() { return blockIdx.z * gridDim.y + blockIdx.y; }

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

__device__ __forceinline__ int num_blocks_of(const Dims& D, int b) {
  int ctx = D.ctx_len[b];
  if (ctx < 0) ctx = 0;
  int nb = (ctx + D.S - 1) >> D.s_shift;
  return nb < D.max_blocks ? nb : D.max_blocks;
}

// number of lanes below this one whose bit is set in a 64-bit wave mask
__device__ __forceinline__ int mbcnt64(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// Exchanges between the four 16-lane rows of a wave on the vector ALU (no trip through the LDS
// crossbar): v_permlane16_swap trades the odd rows of its first operand with the even rows of its
// second, v_permlane32_swap the upper half of the first with the lower half of the second.  Fed the
// same value twice, the two results hold, lane for lane, the value of the lane and of its partner
// (lane ^ 16, lane ^ 32), in an order that does not matter to a commutative operation.
__device__ __forceinline__ float max_xor16(float x) {
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float max_xor32(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_xor16(float x) {
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float sum_xor32(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// The value that the partner lane holds, for the butterfly partner of level LEVEL: lane ^ 32 and
// lane ^ 16 through the row swaps (own ^ both results leaves the partner's bits), lane ^ 15, ^ 7, ^ 3,
// ^ 1 through the DPP mirrors inside a 16-lane row.  The XOR masks 32, 16, 15, 7, 3, 1 are
// independent, so a reduction that walks the levels downwards covers the same lane groups as the
// usual 32, 16, 8, 4, 2, 1 butterfly, and bit LEVEL of the lane index still tells the two partners
// apart.  All on the vector ALU: no trip through the LDS crossbar.
template <int LEVEL>
__device__ __forceinline__ uint32_t partner_u32(uint32_t x) {
  if constexpr (LEVEL == 5) {
    const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    return r[0] ^ r[1] ^ x;
  } else if constexpr (LEVEL == 4) {
    const auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
    return r[0] ^ r[1] ^ x;
  } else {
    constexpr int ctrl = LEVEL == 3 ? 0x140 /* row_mirror */ : LEVEL == 2 ? 0x141 /* row_half_mirror */
                       : LEVEL == 1 ? 0x1B /* quad_perm 3,2,1,0 */ : 0xB1 /* quad_perm 1,0,3,2 */;
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, ctrl, 0xf, 0xf, false);
  }
}
template <int LEVEL>
__device__ __forceinline__ double partner_f64(double x) {
  const uint64_t u = __double_as_longlong(x);
  const uint32_t lo = partner_u32<LEVEL>((uint32_t)u), hi = partner_u32<LEVEL>((uint32_t)(u >> 32));
  return __longlong_as_double(((uint64_t)hi << 32) | lo);
}

// Load 8 consecutive elements of storage type as binary32.
template <int DT>
__device__ __forceinline__ void load8(const void* base, size_t elem_off, float (&x)[8]);

template <>
__device__ __forceinline__ void load8<SCOUT_BF16>(const void* base, size_t elem_off, float (&x)[8]) {
  const uint4 w = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(base) + elem_off);
  x[0] = bf16_lo(w.x); x[1] = bf16_hi(w.x);
  x[2] = bf16_lo(w.y); x[3] = bf16_hi(w.y);
  x[4] = bf16_lo(w.z); x[5] = bf16_hi(w.z);
  x[6] = bf16_lo(w.w); x[7] = bf16_hi(w.w);
}
template <>
__device__ __forceinline__ void load8<SCOUT_F32>(const void* base, size_t elem_off, float (&x)[8]) {
  const float4* p = reinterpret_cast<const float4*>(static_cast<const float*>(base) + elem_off);
  const float4 a = p[0], b = p[1];
  x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
  x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}

template <int DT>
__device__ __forceinline__ float load1(const void* base, size_t elem_off) {
  if (DT == SCOUT_BF16) return bf16_bits_to_f32(static_cast<const uint16_t*>(base)[elem_off]);
  return static_cast<const float*>(base)[elem_off];
}

}  // namespace scout

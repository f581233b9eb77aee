// Digest construction and block-importance scoring.
//
// Digest: channel-wise min/max pooling over the keys of a block (Sec. 2.2).
// Score: query against the digest (Sec. 2.2, Sec. 3.2, Alg. 1 TopK argument);
// for a min/max digest each channel contributes max(q*min, q*max), summed over
// channels and over the G query heads of the KV head.  Because the sum over
// heads commutes with the sum over channels, the group folds into two
// coefficient vectors  P_c = sum_h max(q_hc, 0),  N_c = sum_h min(q_hc, 0)  and
// score(j) = sum_c (P_c * max_j[c] + N_c * min_j[c]):  two FMAs per channel
// whatever G is.  The pass is a pure stream over the digest cache (HBM-bound);
// accumulation is binary64 so the binary32 result is the correctly rounded
// score except for ties of the last binary64 bit.
#include "common.h"

namespace scout {

// ------------------------------------------------------------------ digest

template <int DT>
__global__ __launch_bounds__(256) void digest_kernel(Dims D, const void* __restrict__ k_blocks,
                                                     void* __restrict__ digest) {
  const int pair = blockIdx.y;
  const int b = pair / D.Hkv;
  const int cpt = D.d / 8;  // 8-channel chunks per token row
  const int j = blockIdx.x * (blockDim.x / cpt) + threadIdx.x / cpt;
  const int c0 = (threadIdx.x % cpt) * 8;
  const int nb = num_blocks_of(D, b);
  if (j >= nb) return;
  int ctx = D.ctx_len[b];
  int valid = ctx - j * D.S;
  if (valid > D.S) valid = D.S;
  const size_t row0 = ((size_t)pair * D.max_blocks + j) * D.S;
  float mn[8], mx[8], x[8];
  load8<DT>(k_blocks, row0 * D.d + c0, mn);
#pragma unroll
  for (int i = 0; i < 8; ++i) mx[i] = mn[i];
  for (int t = 1; t < valid; ++t) {
    load8<DT>(k_blocks, (row0 + t) * D.d + c0, x);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      mn[i] = x[i] < mn[i] ? x[i] : mn[i];
      mx[i] = x[i] > mx[i] ? x[i] : mx[i];
    }
  }
  const size_t o_min = (((size_t)pair * D.max_blocks + j) * 2 + 0) * D.d + c0;
  const size_t o_max = o_min + D.d;
  if (DT == SCOUT_BF16) {
    // the values came out of bf16 storage, so the upper halves are exact
    uint16_t* dg = static_cast<uint16_t*>(digest);
    uint4 a, c;
    a.x = (__float_as_uint(mn[0]) >> 16) | (__float_as_uint(mn[1]) & 0xffff0000u);
    a.y = (__float_as_uint(mn[2]) >> 16) | (__float_as_uint(mn[3]) & 0xffff0000u);
    a.z = (__float_as_uint(mn[4]) >> 16) | (__float_as_uint(mn[5]) & 0xffff0000u);
    a.w = (__float_as_uint(mn[6]) >> 16) | (__float_as_uint(mn[7]) & 0xffff0000u);
    c.x = (__float_as_uint(mx[0]) >> 16) | (__float_as_uint(mx[1]) & 0xffff0000u);
    c.y = (__float_as_uint(mx[2]) >> 16) | (__float_as_uint(mx[3]) & 0xffff0000u);
    c.z = (__float_as_uint(mx[4]) >> 16) | (__float_as_uint(mx[5]) & 0xffff0000u);
    c.w = (__float_as_uint(mx[6]) >> 16) | (__float_as_uint(mx[7]) & 0xffff0000u);
    *reinterpret_cast<uint4*>(dg + o_min) = a;
    *reinterpret_cast<uint4*>(dg + o_max) = c;
  } else {
    float* dg = static_cast<float*>(digest);
    float4* pmin = reinterpret_cast<float4*>(dg + o_min);
    float4* pmax = reinterpret_cast<float4*>(dg + o_max);
    pmin[0] = make_float4(mn[0], mn[1], mn[2], mn[3]);
    pmin[1] = make_float4(mn[4], mn[5], mn[6], mn[7]);
    pmax[0] = make_float4(mx[0], mx[1], mx[2], mx[3]);
    pmax[1] = make_float4(mx[4], mx[5], mx[6], mx[7]);
  }
}

// ------------------------------------------------------------------- score

constexpr int kScoreBlocksPerWave = 16;
constexpr int kScoreWaves = 4;
constexpr int kScoreBlocksPerWg = kScoreBlocksPerWave * kScoreWaves;

// One digest entry (min row + max row = 2*DH elements) is spread over LPB
// consecutive lanes, 16 bytes per lane, so that each wave-wide load reads one
// contiguous kilobyte of the digest cache.
template <int DT, int DH>
__global__ __launch_bounds__(kScoreWaves * kWave) void score_kernel(
    Dims D, const void* __restrict__ q, const void* __restrict__ digest, float* __restrict__ scores) {
  constexpr int EPL = (DT == SCOUT_BF16) ? 8 : 4;  // elements per 16-byte load
  constexpr int LPB = 2 * DH / EPL;                // lanes per block
  constexpr int BPW = kWave / LPB;                 // blocks per wave-wide load
  constexpr int ITERS = kScoreBlocksPerWave / BPW;
  static_assert(LPB <= kWave && ITERS >= 1, "layout");

  const int pair = blockIdx.y;
  const int b = pair / D.Hkv, g = pair % D.Hkv;
  const int lane = lane_id(), wave = threadIdx.x / kWave;
  const int nb = num_blocks_of(D, b);
  const int j_wave = blockIdx.x * kScoreBlocksPerWg + wave * kScoreBlocksPerWave;
  if (j_wave >= D.max_blocks) return;

  const int sub = lane % LPB;          // position inside the digest entry
  const int e0 = sub * EPL;            // first element: [0, DH) min row, [DH, 2DH) max row
  const bool is_max = e0 >= DH;
  const int c0 = e0 % DH;

  // issue the digest loads first, fold the query group while they are in flight
  uint4 raw[ITERS];
  const char* dbase = static_cast<const char*>(digest);
  constexpr size_t ESZ = (DT == SCOUT_BF16) ? 2 : 4;
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int j = j_wave + it * BPW + lane / LPB;
    raw[it] = make_uint4(0, 0, 0, 0);
    if (j < nb) {
      const size_t off = (((size_t)pair * D.max_blocks + j) * 2 * DH + e0) * ESZ;
      raw[it] = *reinterpret_cast<const uint4*>(dbase + off);
    }
  }

  double coef[EPL];
#pragma unroll
  for (int i = 0; i < EPL; ++i) coef[i] = 0.0;
  for (int h = 0; h < D.G; ++h) {
    const size_t qoff = (((size_t)b * D.Hq + g * D.G + h) * DH + c0) * ESZ;
    const uint4 w = *reinterpret_cast<const uint4*>(static_cast<const char*>(q) + qoff);
    float qv[8];
    if (DT == SCOUT_BF16) {
      qv[0] = bf16_lo(w.x); qv[1] = bf16_hi(w.x); qv[2] = bf16_lo(w.y); qv[3] = bf16_hi(w.y);
      qv[4] = bf16_lo(w.z); qv[5] = bf16_hi(w.z); qv[6] = bf16_lo(w.w); qv[7] = bf16_hi(w.w);
    } else {
      qv[0] = __uint_as_float(w.x); qv[1] = __uint_as_float(w.y);
      qv[2] = __uint_as_float(w.z); qv[3] = __uint_as_float(w.w);
      qv[4] = qv[5] = qv[6] = qv[7] = 0.0f;
    }
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
      const float part = is_max ? fmaxf(qv[i], 0.0f) : fminf(qv[i], 0.0f);
      coef[i] += (double)part;
    }
  }

#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int j = j_wave + it * BPW + lane / LPB;
    double acc = 0.0;
    if (DT == SCOUT_BF16) {
      acc = fma(coef[0], (double)bf16_lo(raw[it].x), acc);
      acc = fma(coef[1], (double)bf16_hi(raw[it].x), acc);
      acc = fma(coef[2 % EPL], (double)bf16_lo(raw[it].y), acc);
      acc = fma(coef[3 % EPL], (double)bf16_hi(raw[it].y), acc);
      acc = fma(coef[4 % EPL], (double)bf16_lo(raw[it].z), acc);
      acc = fma(coef[5 % EPL], (double)bf16_hi(raw[it].z), acc);
      acc = fma(coef[6 % EPL], (double)bf16_lo(raw[it].w), acc);
      acc = fma(coef[7 % EPL], (double)bf16_hi(raw[it].w), acc);
    } else {
      acc = fma(coef[0], (double)__uint_as_float(raw[it].x), acc);
      acc = fma(coef[1], (double)__uint_as_float(raw[it].y), acc);
      acc = fma(coef[2], (double)__uint_as_float(raw[it].z), acc);
      acc = fma(coef[3], (double)__uint_as_float(raw[it].w), acc);
    }
#pragma unroll
    for (int off = 1; off < LPB; off <<= 1) acc += __shfl_xor(acc, off);
    if (sub == 0 && j < D.max_blocks)
      scores[(size_t)pair * D.max_blocks + j] = j < nb ? (float)acc : -INFINITY;
  }
}

// ------------------------------------------------------------ host launchers

int launch_digest(const Dims& D, int dtype, const void* k_blocks, void* digest, hipStream_t st) {
  const int cpt = D.d / 8;
  const int blocks_per_wg = 256 / cpt;
  dim3 grid((D.max_blocks + blocks_per_wg - 1) / blocks_per_wg, D.B * D.Hkv);
  if (grid.x == 0 || grid.y == 0) return SCOUT_OK;
  if (dtype == SCOUT_BF16)
    hipLaunchKernelGGL(digest_kernel<SCOUT_BF16>, grid, dim3(256), 0, st, D, k_blocks, digest);
  else
    hipLaunchKernelGGL(digest_kernel<SCOUT_F32>, grid, dim3(256), 0, st, D, k_blocks, digest);
  return hipGetLastError() == hipSuccess ? SCOUT_OK : SCOUT_EHIP;
}

int launch_score(const Dims& D, int dtype, const void* q, const void* digest, float* scores,
                 hipStream_t st) {
  dim3 grid((D.max_blocks + kScoreBlocksPerWg - 1) / kScoreBlocksPerWg, D.B * D.Hkv);
  dim3 block(kScoreWaves * kWave);
  if (grid.x == 0 || grid.y == 0) return SCOUT_OK;
  if (dtype == SCOUT_BF16 && D.d == 128)
    hipLaunchKernelGGL((score_kernel<SCOUT_BF16, 128>), grid, block, 0, st, D, q, digest, scores);
  else if (dtype == SCOUT_BF16 && D.d == 64)
    hipLaunchKernelGGL((score_kernel<SCOUT_BF16, 64>), grid, block, 0, st, D, q, digest, scores);
  else if (dtype == SCOUT_F32 && D.d == 128)
    hipLaunchKernelGGL((score_kernel<SCOUT_F32, 128>), grid, block, 0, st, D, q, digest, scores);
  else if (dtype == SCOUT_F32 && D.d == 64)
    hipLaunchKernelGGL((score_kernel<SCOUT_F32, 64>), grid, block, 0, st, D, q, digest, scores);
  else
    return SCOUT_EUNSUPPORTED;
  return hipGetLastError() == hipSuccess ? SCOUT_OK : SCOUT_EHIP;
}

}  // namespace scout

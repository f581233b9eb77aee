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

constexpr int kScoreWaves = 4;      // waves per workgroup
constexpr int kScoreBatch = 8;      // wave-wide loads per batch
constexpr int kScoreBatches = 4;    // batches per wave

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// One digest entry (min row + max row = 2*DH elements) is spread over LPB
// consecutive lanes, 16 bytes per lane, so that each wave-wide load reads one
// contiguous kilobyte of the digest cache.  A wave walks over kScoreBatches
// batches of kScoreBatch such loads and keeps two batches in flight.  The loads
// go through a buffer descriptor that ends at the pair's last valid block:
// blocks beyond it read as zero without touching memory, so the issue path has
// no branches.  Per batch every lane ends up with kScoreBatch partial sums (one
// per load) that still have to be added across the LPB lanes of an entry; the
// first three reduction steps exchange half of the remaining sums each, so the
// batch needs 4+2+1 exchanges plus log2(LPB)-3 plain ones instead of
// kScoreBatch*log2(LPB).
template <int DT, int DH>
__global__ __launch_bounds__(kScoreWaves* kWave) void score_kernel(
    Dims D, const void* __restrict__ q, const void* __restrict__ digest, float* __restrict__ scores) {
  constexpr int EPL = (DT == SCOUT_BF16) ? 8 : 4;  // elements per 16-byte load
  constexpr int ESZ = (DT == SCOUT_BF16) ? 2 : 4;
  constexpr int LPB = 2 * DH / EPL;                // lanes per block
  constexpr int BPW = kWave / LPB;                 // blocks per wave-wide load
  constexpr int BLK_PER_WAVE = BPW * kScoreBatch * kScoreBatches;
  static_assert(LPB >= 16 && LPB <= kWave, "layout");

  const int pair = blockIdx.y;
  const int b = pair / D.Hkv, g = pair % D.Hkv;
  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int nb = num_blocks_of(D, b);
  const int j_wave = (blockIdx.x * kScoreWaves + wave) * BLK_PER_WAVE;
  if (j_wave >= D.max_blocks) return;

  const int sub = lane % LPB;  // position inside the digest entry
  const int grp = lane / LPB;  // which of the BPW blocks of a load
  const int e0 = sub * EPL;    // first element: [0, DH) min row, [DH, 2DH) max row
  const bool is_max = e0 >= DH;
  const int c0 = e0 % DH;

  // the group's queries first, so that they arrive before the digest stream
  u32x4 qraw[16];
  const char* qbase = static_cast<const char*>(q) + (((size_t)b * D.Hq + g * D.G) * DH + c0) * ESZ;
#pragma unroll
  for (int h = 0; h < 16; ++h) {  // rows beyond the group re-read its last row and are ignored below
    const int hs = h < D.G ? h : D.G - 1;
    qraw[h] = *reinterpret_cast<const u32x4*>(qbase + (size_t)hs * DH * ESZ);
  }

  const char* dpair = static_cast<const char*>(digest) + (size_t)pair * D.max_blocks * 2 * DH * ESZ;
  const __amdgpu_buffer_rsrc_t rs =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(dpair), 0, nb * 2 * DH * ESZ, 0x00020000);
  const int voff0 = ((j_wave + grp) * 2 * DH + e0) * ESZ;
  constexpr int LOAD_STRIDE = BPW * 2 * DH * ESZ;  // bytes between consecutive loads of a wave (1 KiB)

  u32x4 raw[2][kScoreBatch];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int it = 0; it < kScoreBatch; ++it)
      raw[t][it] = __builtin_bit_cast(
          u32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, voff0 + (t * kScoreBatch + it) * LOAD_STRIDE, 0, 0));

  // fold the query group: P_c = sum of positive parts (pairs with the max row),
  // N_c = sum of negative parts (pairs with the min row)
  double coef[EPL];
#pragma unroll
  for (int i = 0; i < EPL; ++i) coef[i] = 0.0;
#pragma unroll
  for (int h = 0; h < 16; ++h) {
    float qv[8];
    if (DT == SCOUT_BF16) {
      qv[0] = bf16_lo(qraw[h][0]); qv[1] = bf16_hi(qraw[h][0]); qv[2] = bf16_lo(qraw[h][1]); qv[3] = bf16_hi(qraw[h][1]);
      qv[4] = bf16_lo(qraw[h][2]); qv[5] = bf16_hi(qraw[h][2]); qv[6] = bf16_lo(qraw[h][3]); qv[7] = bf16_hi(qraw[h][3]);
    } else {
      qv[0] = __uint_as_float(qraw[h][0]); qv[1] = __uint_as_float(qraw[h][1]);
      qv[2] = __uint_as_float(qraw[h][2]); qv[3] = __uint_as_float(qraw[h][3]);
      qv[4] = qv[5] = qv[6] = qv[7] = 0.0f;
    }
    if (h < D.G) {
#pragma unroll
      for (int i = 0; i < EPL; ++i) coef[i] += (double)(is_max ? fmaxf(qv[i], 0.0f) : fminf(qv[i], 0.0f));
    }
  }

  constexpr int LV = LPB == 64 ? 5 : LPB == 32 ? 4 : LPB == 16 ? 3 : 2;  // top butterfly level inside an entry
  const bool hiA = (lane >> LV) & 1, hiB = (lane >> (LV - 1)) & 1, hiC = (lane >> (LV - 2)) & 1;
  const int my_it = (hiA ? 4 : 0) + (hiB ? 2 : 0) + (hiC ? 1 : 0);
  const bool writer = (sub & (LPB / 8 - 1)) == 0;

#pragma unroll
  for (int t = 0; t < kScoreBatches; ++t) {
    u32x4(&cur)[kScoreBatch] = raw[t & 1];
    double a[kScoreBatch];
#pragma unroll
    for (int it = 0; it < kScoreBatch; ++it) {
      double acc = 0.0;
      if (DT == SCOUT_BF16) {
        acc = fma(coef[0], (double)bf16_lo(cur[it][0]), acc);
        acc = fma(coef[1], (double)bf16_hi(cur[it][0]), acc);
        acc = fma(coef[2 % EPL], (double)bf16_lo(cur[it][1]), acc);
        acc = fma(coef[3 % EPL], (double)bf16_hi(cur[it][1]), acc);
        acc = fma(coef[4 % EPL], (double)bf16_lo(cur[it][2]), acc);
        acc = fma(coef[5 % EPL], (double)bf16_hi(cur[it][2]), acc);
        acc = fma(coef[6 % EPL], (double)bf16_lo(cur[it][3]), acc);
        acc = fma(coef[7 % EPL], (double)bf16_hi(cur[it][3]), acc);
      } else {
        acc = fma(coef[0], (double)__uint_as_float(cur[it][0]), acc);
        acc = fma(coef[1], (double)__uint_as_float(cur[it][1]), acc);
        acc = fma(coef[2], (double)__uint_as_float(cur[it][2]), acc);
        acc = fma(coef[3], (double)__uint_as_float(cur[it][3]), acc);
      }
      a[it] = acc;
    }
    // the batch after next takes over this buffer
    if (t + 2 < kScoreBatches) {
#pragma unroll
      for (int it = 0; it < kScoreBatch; ++it)
        cur[it] = __builtin_bit_cast(
            u32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, voff0 + ((t + 2) * kScoreBatch + it) * LOAD_STRIDE, 0, 0));
    }
    // exchange-and-halve reduction across the LPB lanes of an entry: at each of the first three
    // levels a lane keeps half of its sums and hands the other half to its partner
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const double keep = hiA ? a[i + 4] : a[i], send = hiA ? a[i] : a[i + 4];
      a[i] = keep + partner_f64<LV>(send);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const double keep = hiB ? a[i + 2] : a[i], send = hiB ? a[i] : a[i + 2];
      a[i] = keep + partner_f64<LV - 1>(send);
    }
    {
      const double keep = hiC ? a[1] : a[0], send = hiC ? a[0] : a[1];
      a[0] = keep + partner_f64<LV - 2>(send);
    }
    if constexpr (LV - 3 >= 0) a[0] += partner_f64<(LV - 3 >= 0 ? LV - 3 : 0)>(a[0]);
    if constexpr (LV - 4 >= 0) a[0] += partner_f64<(LV - 4 >= 0 ? LV - 4 : 0)>(a[0]);
    if constexpr (LV - 5 >= 0) a[0] += partner_f64<(LV - 5 >= 0 ? LV - 5 : 0)>(a[0]);
    // a[0]: score of the block that load my_it of this batch brought to this lane group
    const int j = j_wave + (t * kScoreBatch + my_it) * BPW + grp;
    if (writer && j < D.max_blocks) scores[(size_t)pair * D.max_blocks + j] = j < nb ? (float)a[0] : -INFINITY;
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
  const int epl = dtype == SCOUT_BF16 ? 8 : 4;
  const int blocks_per_wg = (kWave / (2 * D.d / epl)) * kScoreBatch * kScoreBatches * kScoreWaves;
  dim3 grid((D.max_blocks + blocks_per_wg - 1) / blocks_per_wg, D.B * D.Hkv);
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

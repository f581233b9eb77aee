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
  const int pair = grid_pair();  // grid (x, Hkv, B)
  const int b = blockIdx.z;
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

// Mean pooling (Sec. 2.2 names it next to min/max pooling): the digest of a block is the sum of its
// valid keys in binary32, added in token order, one rounding per token, so that the append of a token
// is one addition and gives the bits a rebuild would give; the mean is sum / count where it is used.
template <int DT>
__global__ __launch_bounds__(256) void digest_sum_kernel(Dims D, const void* __restrict__ k_blocks,
                                                         float* __restrict__ digest) {
  const int pair = grid_pair();  // grid (x, Hkv, B)
  const int b = blockIdx.z;
  const int cpt = D.d / 8;
  const int j = blockIdx.x * (blockDim.x / cpt) + threadIdx.x / cpt;
  const int c0 = (threadIdx.x % cpt) * 8;
  const int nb = num_blocks_of(D, b);
  if (j >= nb) return;
  int valid = D.ctx_len[b] - j * D.S;
  if (valid > D.S) valid = D.S;
  const size_t row0 = ((size_t)pair * D.max_blocks + j) * D.S;
  float sum[8], x[8];
  load8<DT>(k_blocks, row0 * D.d + c0, sum);
  for (int t = 1; t < valid; ++t) {
    load8<DT>(k_blocks, (row0 + t) * D.d + c0, x);
#pragma unroll
    for (int i = 0; i < 8; ++i) sum[i] = sum[i] + x[i];
  }
  float4* out = reinterpret_cast<float4*>(digest + ((size_t)pair * D.max_blocks + j) * D.d + c0);
  out[0] = make_float4(sum[0], sum[1], sum[2], sum[3]);
  out[1] = make_float4(sum[4], sum[5], sum[6], sum[7]);
}

// ------------------------------------------------------------------- score

constexpr int kScoreWaves = 4;      // waves per workgroup
constexpr int kScoreBatch = 8;      // wave-wide loads per batch
constexpr int kScoreBatches = 1;    // batches per wave (with more than one, two are kept in flight)

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// The score of a block is sum_c P_c*max_j[c] + N_c*min_j[c], with P_c (N_c) the sum over the group's
// query heads of the positive (negative) parts of q[c]: the group is folded before the stream.
//
// Stream layout: a wave-wide load takes one 128-byte line from each of 8 consecutive digest entries
// (8 lanes x 16 bytes per entry), and NL such loads cover the entries whole.  A lane therefore adds
// the products of NL loads into one partial sum, and only the 8 lanes of an entry remain to be added
// across lanes: three DPP steps.  Where a batch of kScoreBatch loads holds several 8-entry groups,
// the first steps exchange half of the remaining sums each instead of adding all of them everywhere.
// A wave takes one batch, all of it requested at once: many small waves (8192 at 128 pairs x 1024
// blocks, 8 KiB each) measured faster than fewer waves that walk over several batches (13.5 vs 14.5 us
// for 64 MiB).  The loads go through a buffer
// descriptor that ends at the pair's last valid block: blocks beyond it read as zero without touching
// memory, so the issue path has no branches.
//
// The fold of the query group is done once per workgroup (one channel and one sign per thread) and
// handed to the lanes through LDS, while the first digest loads are in flight.  The pointers are
// deliberately not marked restrict: loads that the compiler knows to be invariant float freely, and
// here the order of issue matters (queries first, then batch by batch), because a wait for one load
// is a wait for every load issued before it.
//
// MEAN: the digest entry is one row of binary32 sums of the block's keys (mean pooling) whatever the
// element type of the queries; the score is (sum over heads of q) . sums / count, so there is one
// coefficient vector instead of two and a division by the block's token count at the end.
template <int DT, int DH, bool MEAN>
__global__ __launch_bounds__(kScoreWaves* kWave) void score_kernel(
    Dims D, const void* q, const void* digest, float* scores) {
  constexpr bool DIG16 = DT == SCOUT_BF16 && !MEAN;  // digest elements are bf16
  constexpr int EPL = DIG16 ? 8 : 4;               // digest elements per 16-byte load
  constexpr int ESZ = (DT == SCOUT_BF16) ? 2 : 4;  // bytes per query element
  constexpr int DSZ = DIG16 ? 2 : 4;               // bytes per digest element
  constexpr int EB = (MEAN ? 1 : 2) * DH * DSZ;    // bytes per digest entry
  constexpr int NL = EB / 128;                     // 128-byte lines per entry
  constexpr int NG = kScoreBatch / NL;             // 8-entry groups per batch
  constexpr int BLK_PER_WAVE = NG * 8 * kScoreBatches;
  constexpr int NT = kScoreWaves * kWave;
  static_assert(NL >= 2 && NL <= kScoreBatch && 2 * DH <= NT, "layout");

  __shared__ __align__(16) double coef_lds[2][DH];  // [0]: N_c (goes with the min row), [1]: P_c

  const int pair = grid_pair();  // grid (x, Hkv, B)
  const int b = blockIdx.z, g = blockIdx.y;
  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int nb = num_blocks_of(D, b);
  const int j_wave = (blockIdx.x * kScoreWaves + wave) * BLK_PER_WAVE;
  const bool active = j_wave < D.max_blocks;  // a wave past the row still helps with the fold

  // the group's queries first: thread t takes channel t % DH, negative (t < DH) or positive parts
  const int fc = threadIdx.x % DH;
  const bool fpos = threadIdx.x >= DH;
  const char* qbase = static_cast<const char*>(q) + (((size_t)b * D.Hq + g * D.G) * DH + fc) * ESZ;
  float qv[16];
#pragma unroll
  for (int h = 0; h < 16; ++h) {  // rows beyond the group re-read its last row and are ignored below
    const int hs = h < D.G ? h : D.G - 1;
    if (DT == SCOUT_BF16)
      qv[h] = __uint_as_float((uint32_t) * reinterpret_cast<const uint16_t*>(qbase + (size_t)hs * DH * ESZ) << 16);
    else
      qv[h] = *reinterpret_cast<const float*>(qbase + (size_t)hs * DH * ESZ);
  }

  // (the query loads above do not wait for the sequence's length; this is the first thing that does)
  if ((int)blockIdx.x * kScoreWaves * BLK_PER_WAVE >= nb) {
    // the whole workgroup lies beyond the sequence's last block (a ragged batch has many of these):
    // nothing to read, only the row's tail to mark
    const int j = (int)blockIdx.x * kScoreWaves * BLK_PER_WAVE + threadIdx.x;
    if (threadIdx.x < kScoreWaves * BLK_PER_WAVE && j < D.max_blocks) scores[(size_t)pair * D.max_blocks + j] = -INFINITY;
    return;
  }
  const char* dpair = static_cast<const char*>(digest) + (size_t)kv_row(D, pair) * D.max_blocks * EB;
  const __amdgpu_buffer_rsrc_t rs =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(dpair), 0, active ? nb * EB : 0, 0x00020000);
  const int voff0 = (j_wave + (lane >> 3)) * EB + (lane & 7) * 16;
  // byte offset of load `it` of batch `t`: group it / NL of the batch, line it % NL of its entries
  auto load_off = [&](int t, int it) { return voff0 + (t * NG + it / NL) * 8 * EB + (it % NL) * 128; };

  u32x4 raw[kScoreBatches < 2 ? 1 : 2][kScoreBatch];
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int t = 0; t < (kScoreBatches < 2 ? kScoreBatches : 2); ++t) {
#pragma unroll
    for (int it = 0; it < kScoreBatch; ++it)
      raw[t][it] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, load_off(t, it), 0, 0));
    __builtin_amdgcn_sched_barrier(0);
  }

  {
    double f = 0.0;
#pragma unroll
    for (int h = 0; h < 16; ++h)
      if (h < D.G) f += MEAN ? (double)qv[h] : (double)(fpos ? fmaxf(qv[h], 0.0f) : fminf(qv[h], 0.0f));
    if (threadIdx.x < 2 * DH) coef_lds[fpos ? 1 : 0][fc] = f;  // MEAN: both rows hold the plain sum
  }
  __syncthreads();
  // line u of an entry: min row for u < NL/2, max row after (MEAN: the one row of sums);
  // channels (u % lines per row) * 128/DSZ + 8 lanes x EPL
  constexpr int LPR = MEAN ? NL : NL / 2;  // lines per digest row
  double coef[NL][EPL];
#pragma unroll
  for (int u = 0; u < NL; ++u)
#pragma unroll
    for (int i = 0; i < EPL; ++i)
      coef[u][i] = coef_lds[u >= LPR ? 1 : 0][(u % LPR) * (128 / DSZ) + (lane & 7) * EPL + i];

  const bool hi2 = (lane >> 2) & 1, hi1 = (lane >> 1) & 1;
  const int my_g = NG == 4 ? (hi2 ? 2 : 0) + (hi1 ? 1 : 0) : NG == 2 ? (hi2 ? 1 : 0) : 0;
  const bool writer = NG == 4 ? (lane & 1) == 0 : NG == 2 ? (lane & 3) == 0 : (lane & 7) == 0;

#pragma unroll
  for (int t = 0; t < kScoreBatches; ++t) {
    u32x4(&cur)[kScoreBatch] = raw[t & 1];
    double a[NG];
#pragma unroll
    for (int gq = 0; gq < NG; ++gq) {
      double acc = 0.0;
#pragma unroll
      for (int u = 0; u < NL; ++u) {
        const u32x4 w = cur[gq * NL + u];
        if (DIG16) {
          acc = fma(coef[u][0], (double)bf16_lo(w[0]), acc);
          acc = fma(coef[u][1], (double)bf16_hi(w[0]), acc);
          acc = fma(coef[u][2 % EPL], (double)bf16_lo(w[1]), acc);
          acc = fma(coef[u][3 % EPL], (double)bf16_hi(w[1]), acc);
          acc = fma(coef[u][4 % EPL], (double)bf16_lo(w[2]), acc);
          acc = fma(coef[u][5 % EPL], (double)bf16_hi(w[2]), acc);
          acc = fma(coef[u][6 % EPL], (double)bf16_lo(w[3]), acc);
          acc = fma(coef[u][7 % EPL], (double)bf16_hi(w[3]), acc);
        } else {
          acc = fma(coef[u][0], (double)__uint_as_float(w[0]), acc);
          acc = fma(coef[u][1], (double)__uint_as_float(w[1]), acc);
          acc = fma(coef[u][2], (double)__uint_as_float(w[2]), acc);
          acc = fma(coef[u][3], (double)__uint_as_float(w[3]), acc);
        }
      }
      a[gq] = acc;
    }
    // the batch after next takes over this buffer
    if (t + 2 < kScoreBatches) {
#pragma unroll
      for (int it = 0; it < kScoreBatch; ++it)
        cur[it] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, load_off(t + 2, it), 0, 0));
    }
    // add across the 8 lanes of an entry; with several groups the first steps exchange and halve
    if constexpr (NG == 4) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const double keep = hi2 ? a[i + 2] : a[i], send = hi2 ? a[i] : a[i + 2];
        a[i] = keep + partner_f64<2>(send);
      }
      const double keep = hi1 ? a[1] : a[0], send = hi1 ? a[0] : a[1];
      a[0] = keep + partner_f64<1>(send);
    } else if constexpr (NG == 2) {
      const double keep = hi2 ? a[1] : a[0], send = hi2 ? a[0] : a[1];
      a[0] = keep + partner_f64<2>(send);
      a[0] += partner_f64<1>(a[0]);
    } else {
      a[0] += partner_f64<2>(a[0]);
      a[0] += partner_f64<1>(a[0]);
    }
    a[0] += partner_f64<0>(a[0]);
    // a[0]: score of entry lane/8 of group my_g of this batch
    const int j = j_wave + (t * NG + my_g) * 8 + (lane >> 3);
    if (writer && j < D.max_blocks) {
      const bool kept = j < D.n_sink || j >= nb - D.n_tail;  // always-kept blocks rank above every score
      double sc = a[0];
      if (MEAN) {  // sums -> means: the block's token count (the last block may be partly filled)
        int cnt = D.ctx_len[b] - j * D.S;
        cnt = cnt > D.S ? D.S : (cnt < 1 ? 1 : cnt);
        sc = sc / (double)cnt;
      }
      scores[(size_t)pair * D.max_blocks + j] = j < nb ? (kept ? INFINITY : (float)sc) : -INFINITY;
    }
  }
}

// The same stream with the group's heads combined by their maximum instead of their sum.  The fold of
// the group is not possible then: every head keeps its own estimate, sum over channels of the larger
// of q*min and q*max, which is P_h . max + N_h . min with the positive and negative parts of that head's
// queries.  G times the multiply-adds of the folded kernel on the same loads, so the arithmetic, not the
// stream, sets the pace, and everything around the multiply-adds is kept small:
//  * the per-head coefficients are made once per workgroup, as binary64 in LDS, and a wave takes
//    16 loads per lane (2 to 8 entries per lane) so that each coefficient it reads serves that many entries;
//  * heads are taken four at a time, or eight where the group has more than four (one pass, an element
//    converted to binary64 once, for the common group of eight);
//  * the sums of (entries per lane) x 4 heads are added across the 8 lanes of an entry by a butterfly
//    that exchanges half of the remaining sums at each of its three steps, instead of three steps for
//    every sum: 7/8 of a step per sum.
// Heads beyond G in the last pass repeat head G - 1, which leaves the maximum as it is.
template <int N, int LEVEL>
__device__ __forceinline__ void halve_across(double* a, bool hi) {
#pragma unroll
  for (int i = 0; i < N / 2; ++i) {
    const double keep = hi ? a[i + N / 2] : a[i], send = hi ? a[i] : a[i + N / 2];
    a[i] = keep + partner_f64<LEVEL>(send);
  }
}

constexpr int score_max_entries(int lines) { return 16 / lines < 4 ? 16 / lines : 4; }  // per lane

// ROWS: every head's estimate goes to a row of its own, scores[B][Hq][max_blocks] (a selection per query head:
// one pass over the KV head's digests serves its G query heads), instead of their maximum into the KV head's row.
template <int DT, int DH, int HC, bool ROWS>
__global__ __launch_bounds__(kScoreWaves* kWave) void score_max_kernel(Dims D, const void* q, const void* digest,
                                                                      float* scores) {
  constexpr int EPL = (DT == SCOUT_BF16) ? 8 : 4;   // elements per 16-byte load
  constexpr int ESZ = (DT == SCOUT_BF16) ? 2 : 4;
  constexpr int EB = 2 * DH * ESZ;                  // bytes per digest entry
  constexpr int NL = EB / 128;                      // 128-byte lines per entry
  constexpr int E = score_max_entries(NL);          // entries per lane
  constexpr int V = E * HC;                         // sums per lane and pass (HC heads per pass: 4 or 8)
  constexpr int W = HC == 8 ? 2 : 4;                // elements per step of the inner loop
  constexpr int BLK_PER_WAVE = 8 * E;
  constexpr int NT = kScoreWaves * kWave;
  static_assert(NL >= 2 && NL <= 8 && V >= 8 && (HC / (V / 8) == 2 || HC / (V / 8) == 4), "layout");

  // [head][0: N_h, goes with the min row; 1: P_h][channel], the channels of a row in the order in which the
  // lanes read them: a lane's EPL channels of a line are EPL / 2 reads of 16 bytes, and the 8 lanes of an
  // entry read 128 consecutive bytes each time (channel by channel they would be 64 bytes apart and
  // collide on the banks)
  __shared__ __align__(16) double coef_lds[16][2][DH];
  constexpr int CPL = 128 / ESZ;  // channels per line
  auto coef_at = [](int c) {      // where channel c of a row sits
    const int lr = c / CPL, l8 = (c % CPL) / EPL, i = c % EPL;
    return ((lr * (EPL / 2) + i / 2) * 8 + l8) * 2 + (i & 1);
  };

  const int pair = grid_pair();  // grid (x, Hkv, B)
  const int b = blockIdx.z, g = blockIdx.y;
  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int nb = num_blocks_of(D, b);
  const int j_wave = (blockIdx.x * kScoreWaves + wave) * BLK_PER_WAVE;
  const bool active = j_wave < D.max_blocks;
  const int n_rows = ROWS ? D.G : 1;  // rows of `scores` per pair
  if ((int)blockIdx.x * kScoreWaves * BLK_PER_WAVE >= nb) {  // as in score_kernel: only the rows' tails to mark
    for (int t = threadIdx.x; t < kScoreWaves * BLK_PER_WAVE; t += NT) {
      const int j = (int)blockIdx.x * kScoreWaves * BLK_PER_WAVE + t;
      if (j < D.max_blocks)
        for (int r = 0; r < n_rows; ++r) scores[((size_t)pair * n_rows + r) * D.max_blocks + j] = -INFINITY;
    }
    return;
  }

  // queries first (see score_kernel for why the order of issue matters)
  constexpr int QPT = 16 * DH / NT;  // elements per thread
  static_assert(16 * DH % NT == 0, "layout");
  const int heads4 = (D.G + HC - 1) & ~(HC - 1);  // heads that are read, the repeated ones included
  float qreg[QPT];
#pragma unroll
  for (int i = 0; i < QPT; ++i) {
    const int e = threadIdx.x + i * NT, h = e / DH, c = e % DH;
    const int hs = h < D.G ? h : D.G - 1;
    qreg[i] = load1<DT>(q, ((size_t)b * D.Hq + g * D.G + hs) * DH + c);
  }
  const char* dpair = static_cast<const char*>(digest) + (size_t)kv_row(D, pair) * D.max_blocks * EB;
  const __amdgpu_buffer_rsrc_t rs =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(dpair), 0, active ? nb * EB : 0, 0x00020000);
  const int voff0 = (j_wave + (lane >> 3)) * EB + (lane & 7) * 16;
  u32x4 raw[E * NL];  // load gq * NL + u: line u of the lane's entry in group gq of 8 entries
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int u = 0; u < NL; ++u)  // requested in the order of use: line by line, the E entries of a line together
#pragma unroll
    for (int gq = 0; gq < E; ++gq)
      raw[gq * NL + u] = __builtin_bit_cast(
          u32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, voff0 + gq * 8 * EB + u * 128, 0, 0));
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < QPT; ++i) {
    const int e = threadIdx.x + i * NT, h = e / DH, c = e % DH;
    if (h < heads4) {
      coef_lds[h][0][coef_at(c)] = (double)fminf(qreg[i], 0.0f);
      coef_lds[h][1][coef_at(c)] = (double)fmaxf(qreg[i], 0.0f);
    }
  }
  __syncthreads();

  const bool b2 = (lane >> 2) & 1, b1 = (lane >> 1) & 1, b0 = lane & 1;
  // what the butterfly below leaves in this lane: sums (lane & 7) * V / 8 + r of the V, that is heads
  // hh_mine + r of the pass for the entry of group gq_mine
  constexpr int R = V / 8;
  const int gq_mine = (lane & 7) * R / HC, hh_mine = (lane & 7) * R % HC;
  const int j = j_wave + gq_mine * 8 + (lane >> 3);
  const bool kept = j < D.n_sink || j >= nb - D.n_tail;  // always-kept blocks rank above every score
  double best = -INFINITY;
  for (int h0 = 0; h0 < D.G; h0 += HC) {
    double acc[V];  // sum of entry group gq, head h0 + hh at gq * HC + hh
#pragma unroll
    for (int i = 0; i < V; ++i) acc[i] = 0.0;
    // (the loaded words are declared changed here: otherwise their binary64 forms, which do not depend on
    // the pass, are all made ahead of the loop and take four times the registers of the words themselves)
#pragma unroll
    for (int it = 0; it < E * NL; ++it)
      asm volatile("" : "+v"(raw[it][0]), "+v"(raw[it][1]), "+v"(raw[it][2]), "+v"(raw[it][3]));
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      // line u of an entry: min row for u < NL/2, max row after; channels c0 .. c0 + EPL of that row
      const int row = u / (NL / 2), c0 = (u % (NL / 2)) * CPL + (lane & 7) * EPL;
#pragma unroll
      for (int i0 = 0; i0 < EPL; i0 += W) {  // W elements at a time: HC x W coefficients in registers
        double cf[HC][W];
#pragma unroll
        for (int hh = 0; hh < HC; ++hh)
#pragma unroll
          for (int i = 0; i < W; ++i) cf[hh][i] = coef_lds[h0 + hh][row][coef_at(c0 + i0 + i)];
#pragma unroll
        for (int gq = 0; gq < E; ++gq) {
          const u32x4 w = raw[gq * NL + u];
          double x[W];
#pragma unroll
          for (int i = 0; i < W; ++i) {
            if (DT == SCOUT_BF16)
              x[i] = (double)(((i0 + i) & 1) ? bf16_hi(w[(i0 + i) >> 1]) : bf16_lo(w[(i0 + i) >> 1]));
            else
              x[i] = (double)__uint_as_float(w[i0 + i]);
          }
#pragma unroll
          for (int hh = 0; hh < HC; ++hh)
#pragma unroll
            for (int i = 0; i < W; ++i) acc[gq * HC + hh] = fma(cf[hh][i], x[i], acc[gq * HC + hh]);
        }
      }
    }
    // across the 8 lanes of an entry: each step keeps the half of the sums that the lane's bit names and
    // adds the partner's; V / 8 finished sums remain, index (4 b2 + 2 b1 + b0) * V / 8 + r of the V
    halve_across<V, 2>(acc, b2);
    halve_across<V / 2, 1>(acc, b1);
    halve_across<V / 4, 0>(acc, b0);
    if constexpr (ROWS) {
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const int h = h0 + hh_mine + r;
        if (h < D.G && j < D.max_blocks)
          scores[((size_t)pair * D.G + h) * D.max_blocks + j] = j < nb ? (kept ? INFINITY : (float)acc[r]) : -INFINITY;
      }
    } else {
#pragma unroll
      for (int r = 0; r < R; ++r) best = acc[r] > best ? acc[r] : best;  // heads of one entry (R divides HC)
    }
  }
  if constexpr (!ROWS) {
    // lanes whose finished sums were heads of the same entry: HC / R of them, neighbours
    if constexpr (HC / R >= 4) {
      const double o = partner_f64<1>(best);
      best = o > best ? o : best;
    }
    if constexpr (HC / R >= 2) {
      const double o = partner_f64<0>(best);
      best = o > best ? o : best;
    }
    if (hh_mine == 0 && j < D.max_blocks)
      scores[(size_t)pair * D.max_blocks + j] = j < nb ? (kept ? INFINITY : (float)best) : -INFINITY;
  }
}

// ------------------------------------------------------------ host launchers

int launch_digest(const Dims& D, int dtype, const void* k_blocks, void* digest, hipStream_t st) {
  const int cpt = D.d / 8;
  const int blocks_per_wg = 256 / cpt;
  dim3 grid((D.max_blocks + blocks_per_wg - 1) / blocks_per_wg, D.Hkv, D.B);
  if (grid.x == 0 || grid.y == 0 || grid.z == 0) return SCOUT_OK;
  if (D.digest_kind == 1) {
    float* sums = static_cast<float*>(digest);
    if (dtype == SCOUT_BF16)
      hipLaunchKernelGGL(digest_sum_kernel<SCOUT_BF16>, grid, dim3(256), 0, st, D, k_blocks, sums);
    else
      hipLaunchKernelGGL(digest_sum_kernel<SCOUT_F32>, grid, dim3(256), 0, st, D, k_blocks, sums);
    return hipGetLastError() == hipSuccess ? SCOUT_OK : SCOUT_EHIP;
  }
  if (dtype == SCOUT_BF16)
    hipLaunchKernelGGL(digest_kernel<SCOUT_BF16>, grid, dim3(256), 0, st, D, k_blocks, digest);
  else
    hipLaunchKernelGGL(digest_kernel<SCOUT_F32>, grid, dim3(256), 0, st, D, k_blocks, digest);
  return hipGetLastError() == hipSuccess ? SCOUT_OK : SCOUT_EHIP;
}

template <int HC, bool ROWS>
static int launch_score_max_hc(const Dims& D, int dtype, const void* q, const void* digest, float* scores,
                               hipStream_t st) {
  const int lines = 2 * D.d * (dtype == SCOUT_BF16 ? 2 : 4) / 128;
  const int blocks_per_wg = score_max_entries(lines) * 8 * kScoreWaves;  // 8 entries per wave-wide load
  dim3 grid((D.max_blocks + blocks_per_wg - 1) / blocks_per_wg, D.Hkv, D.B);
  dim3 block(kScoreWaves * kWave);
  if (grid.x == 0 || grid.y == 0 || grid.z == 0) return SCOUT_OK;
  if (dtype == SCOUT_BF16 && D.d == 128)
    hipLaunchKernelGGL((score_max_kernel<SCOUT_BF16, 128, HC, ROWS>), grid, block, 0, st, D, q, digest, scores);
  else if (dtype == SCOUT_BF16 && D.d == 64)
    hipLaunchKernelGGL((score_max_kernel<SCOUT_BF16, 64, HC, ROWS>), grid, block, 0, st, D, q, digest, scores);
  else if (dtype == SCOUT_F32 && D.d == 128)
    hipLaunchKernelGGL((score_max_kernel<SCOUT_F32, 128, HC, ROWS>), grid, block, 0, st, D, q, digest, scores);
  else if (dtype == SCOUT_F32 && D.d == 64)
    hipLaunchKernelGGL((score_max_kernel<SCOUT_F32, 64, HC, ROWS>), grid, block, 0, st, D, q, digest, scores);
  else
    return SCOUT_EUNSUPPORTED;
  return hipGetLastError() == hipSuccess ? SCOUT_OK : SCOUT_EHIP;
}

int launch_score_max(const Dims& D, int dtype, const void* q, const void* digest, float* scores, hipStream_t st) {
  // groups of 5 to 8 heads in one pass of eight, every other size in passes of four
  if (D.G > 4 && D.G <= 8) return launch_score_max_hc<8, false>(D, dtype, q, digest, scores, st);
  return launch_score_max_hc<4, false>(D, dtype, q, digest, scores, st);
}

// A selection per query head (D describes every query head as a pair of its own that shares its KV head's
// rows): the same kernel over the KV heads, every head's estimate to its own row.
static int launch_score_rows(const Dims& D, int dtype, const void* q, const void* digest, float* scores,
                             hipStream_t st) {
  Dims K = D;
  K.G = D.share;
  K.Hkv = D.Hkv / D.share;
  K.share = 1;
  K.share_magic = 0;
  if (K.G > 4 && K.G <= 8) return launch_score_max_hc<8, true>(K, dtype, q, digest, scores, st);
  return launch_score_max_hc<4, true>(K, dtype, q, digest, scores, st);
}

template <bool MEAN>
static int launch_score_sum(const Dims& D, int dtype, const void* q, const void* digest, float* scores,
                            hipStream_t st) {
  const int entry_bytes = MEAN ? D.d * 4 : 2 * D.d * (dtype == SCOUT_BF16 ? 2 : 4);
  const int lines = entry_bytes / 128;  // 128-byte lines per digest entry
  const int blocks_per_wg = kScoreBatch / lines * 8 * kScoreBatches * kScoreWaves;
  dim3 grid((D.max_blocks + blocks_per_wg - 1) / blocks_per_wg, D.Hkv, D.B);
  dim3 block(kScoreWaves * kWave);
  if (grid.x == 0 || grid.y == 0 || grid.z == 0) return SCOUT_OK;
  if (dtype == SCOUT_BF16 && D.d == 128)
    hipLaunchKernelGGL((score_kernel<SCOUT_BF16, 128, MEAN>), grid, block, 0, st, D, q, digest, scores);
  else if (dtype == SCOUT_BF16 && D.d == 64)
    hipLaunchKernelGGL((score_kernel<SCOUT_BF16, 64, MEAN>), grid, block, 0, st, D, q, digest, scores);
  else if (dtype == SCOUT_F32 && D.d == 128)
    hipLaunchKernelGGL((score_kernel<SCOUT_F32, 128, MEAN>), grid, block, 0, st, D, q, digest, scores);
  else if (dtype == SCOUT_F32 && D.d == 64)
    hipLaunchKernelGGL((score_kernel<SCOUT_F32, 64, MEAN>), grid, block, 0, st, D, q, digest, scores);
  else
    return SCOUT_EUNSUPPORTED;
  return hipGetLastError() == hipSuccess ? SCOUT_OK : SCOUT_EHIP;
}

int launch_score(const Dims& D, int dtype, const void* q, const void* digest, float* scores,
                 hipStream_t st) {
  if (D.digest_kind == 1) return D.group_max ? SCOUT_EUNSUPPORTED : launch_score_sum<true>(D, dtype, q, digest, scores, st);
  if (D.group_max) return launch_score_max(D, dtype, q, digest, scores, st);
  if (D.share > 1) return launch_score_rows(D, dtype, q, digest, scores, st);
  return launch_score_sum<false>(D, dtype, q, digest, scores, st);
}

}  // namespace scout

// Top-k block selection, residency split and the recall plan.
//
// Selection (Alg. 1, TopK): the k best blocks of a pair under the total order
// (score descending, block index ascending).  Integer work only: scores are
// mapped to order-preserving 32-bit keys, the k-th largest key is found by a
// bit-by-bit threshold search whose counts are wave ballots and scalar
// population counts (no sort, no shared-memory traffic for one wave), and the
// winners are written in ascending index order by a ballot prefix count.
// Residency split (Alg. 1: predicted blocks minus resident blocks) and the
// recall plan (Sec. 3.4) reuse the same machinery.
//
// Element i of a pair lives in wave i / (64*KPL), register (i / 64) % KPL,
// lane i % 64: loads are coalesced and index order is (wave, register, lane).
#include "common.h"

namespace scout {

// binary32 -> key with  a < b  <=>  key(a) < key(b);  -0 and +0 share a key;
// NaN -> 1 (below -inf); 0 is reserved for "not a candidate".
__device__ __forceinline__ uint32_t score_key(float s) {
  uint32_t u = __float_as_uint(s);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 1u;
  if ((u << 1) == 0u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Sum a wave-uniform value over the waves of the workgroup; also the sum over
// the waves before this one.  lds holds 2*WAVES ints, used alternately so one
// barrier per call is enough.
template <int WAVES>
__device__ __forceinline__ void wg_exchange(int v, int* lds, int& phase, int wave, int& total,
                                            int& before) {
  if (WAVES == 1) {
    total = v;
    before = 0;
    return;
  }
  int* buf = lds + (phase & 1) * WAVES;
  if (lane_id() == 0) buf[wave] = v;
  __syncthreads();
  total = 0;
  before = 0;
#pragma unroll
  for (int w = 0; w < WAVES; ++w) {
    const int x = buf[w];
    total += x;
    before += (w < wave) ? x : 0;
  }
  ++phase;
}

template <int WAVES, int KPL>
struct Selector {
  int* lds;
  int phase;
  int wave;

  // number of keys >= cand over the whole workgroup
  __device__ __forceinline__ int count_ge(const uint32_t (&key)[KPL], uint32_t cand) {
    int c = 0;
#pragma unroll
    for (int r = 0; r < KPL; ++r) c += __popcll(__ballot(key[r] >= cand));
    int total, before;
    wg_exchange<WAVES>(c, lds, phase, wave, total, before);
    return total;
  }

  // total number of set bits of a per-lane register mask, and (per element) the
  // number of set elements that precede it in index order
  __device__ __forceinline__ int positions(uint32_t bits, int (&pos)[KPL]) {
    int c = 0;
#pragma unroll
    for (int r = 0; r < KPL; ++r) c += __popcll(__ballot((bits >> r) & 1u));
    int total, off;
    wg_exchange<WAVES>(c, lds, phase, wave, total, off);
#pragma unroll
    for (int r = 0; r < KPL; ++r) {
      const uint64_t m = __ballot((bits >> r) & 1u);
      pos[r] = off + mbcnt64(m);
      off += __popcll(m);
    }
    return total;
  }

  __device__ __forceinline__ int count(uint32_t bits) {
    int c = 0;
#pragma unroll
    for (int r = 0; r < KPL; ++r) c += __popcll(__ballot((bits >> r) & 1u));
    int total, before;
    wg_exchange<WAVES>(c, lds, phase, wave, total, before);
    return total;
  }

  // Bits of the kk best candidates (key > 0) under (key descending, then index
  // ascending, or descending when high_index_first).  Needs 1 <= kk <= number
  // of candidates.
  __device__ __forceinline__ uint32_t best(const uint32_t (&key)[KPL], int kk, bool high_index_first) {
    // the largest T with  count(key >= T) >= kk  is the kk-th largest key
    uint32_t T = 0;
    for (int bit = 31; bit >= 0; --bit) {
      const uint32_t cand = T | (1u << bit);
      const int c = count_ge(key, cand);
      if (c >= kk) T = cand;
      if (c == kk) break;  // {key >= cand} is exactly the answer; lower bits cannot matter
    }
    uint32_t gt = 0, eq = 0;
#pragma unroll
    for (int r = 0; r < KPL; ++r) {
      gt |= (key[r] > T ? 1u : 0u) << r;
      eq |= (key[r] == T ? 1u : 0u) << r;
    }
    // after an early break T may lie between two keys: then everything >= T is taken
    int rank[KPL];
    const int n_eq = positions(eq, rank);
    const int n_gt = count(gt);
    int need = kk - n_gt;
    // keys above T but counted as ">= cand" at the break: those are all in gt already
    uint32_t out = gt;
#pragma unroll
    for (int r = 0; r < KPL; ++r) {
      const int rk = high_index_first ? (n_eq - 1 - rank[r]) : rank[r];
      if (((eq >> r) & 1u) && rk < need) out |= 1u << r;
    }
    return out;
  }
};

// Keys and table entries of a pair.  Every load is issued unconditionally (the index is clamped
// into the row, the value masked afterwards) so that all of them are in flight together.
template <int WAVES, int KPL>
__device__ __forceinline__ void load_keys(const Dims& D, const float* __restrict__ scores,
                                          const int32_t* __restrict__ table, int pair, int nb, int wave,
                                          int lane, uint32_t (&key)[KPL], int (&slot)[KPL]) {
  const size_t row = (size_t)pair * D.max_blocks;
  float sc[KPL];
#pragma unroll
  for (int r = 0; r < KPL; ++r) {
    const int i = (wave * KPL + r) * kWave + lane;
    const int ic = i < D.max_blocks ? i : D.max_blocks - 1;
    sc[r] = scores[row + ic];
    slot[r] = table[row + ic];
  }
#pragma unroll
  for (int r = 0; r < KPL; ++r) {
    const int i = (wave * KPL + r) * kWave + lane;
    key[r] = i < nb ? score_key(sc[r]) : 0u;
    slot[r] = i < nb ? slot[r] : -1;
  }
}

template <int WAVES, int KPL>
__global__ __launch_bounds__(WAVES* kWave) void topk_kernel(
    Dims D, const float* __restrict__ scores, const int32_t* __restrict__ table,
    int32_t* __restrict__ sel_all, int32_t* __restrict__ sel_gpu, int32_t* __restrict__ slot_gpu,
    int32_t* __restrict__ n_gpu, int32_t* __restrict__ sel_host, int32_t* __restrict__ n_host) {
  __shared__ int lds[2 * WAVES];
  const int pair = blockIdx.x, b = pair / D.Hkv;
  const int lane = lane_id(), wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int nb = num_blocks_of(D, b);
  const int k_eff = D.k < nb ? D.k : nb;

  uint32_t key[KPL];
  int slot[KPL];
  load_keys<WAVES, KPL>(D, scores, table, pair, nb, wave, lane, key, slot);
  Selector<WAVES, KPL> S{lds, 0, wave};

  uint32_t sel = 0;
  if (k_eff > 0) sel = S.best(key, k_eff, false);

  uint32_t gpu = 0;
#pragma unroll
  for (int r = 0; r < KPL; ++r)
    if (((sel >> r) & 1u) && slot[r] >= 0) gpu |= 1u << r;
  int pos_all[KPL], pos_gpu[KPL];
  S.positions(sel, pos_all);
  const int ng = S.positions(gpu, pos_gpu);
  const int nh = k_eff - ng;
  const size_t out0 = (size_t)pair * D.k;
#pragma unroll
  for (int r = 0; r < KPL; ++r) {
    if ((sel >> r) & 1u) {
      const int i = (wave * KPL + r) * kWave + lane;
      sel_all[out0 + pos_all[r]] = i;
      if ((gpu >> r) & 1u) {
        sel_gpu[out0 + pos_gpu[r]] = i;
        slot_gpu[out0 + pos_gpu[r]] = slot[r];
      } else {
        sel_host[out0 + pos_all[r] - pos_gpu[r]] = i;
      }
    }
  }
  for (int t = threadIdx.x; t < D.k; t += WAVES * kWave) {
    if (t >= k_eff) sel_all[out0 + t] = -1;
    if (t >= ng) {
      sel_gpu[out0 + t] = -1;
      slot_gpu[out0 + t] = -1;
    }
    if (t >= nh) sel_host[out0 + t] = -1;
  }
  if (threadIdx.x == 0) {
    n_gpu[pair] = ng;
    n_host[pair] = nh;
  }
}

constexpr int kMaxK = 1024;

template <int WAVES, int KPL>
__global__ __launch_bounds__(WAVES* kWave) void recall_kernel(
    Dims D, const float* __restrict__ scores, int32_t* __restrict__ table,
    int32_t* __restrict__ recall_blk, int32_t* __restrict__ recall_slot,
    int32_t* __restrict__ evict_blk, int32_t* __restrict__ n_recall) {
  __shared__ int lds[2 * WAVES];
  __shared__ int freed[kMaxK];  // slots of the evicted blocks, in ascending block order
  const int pair = blockIdx.x, b = pair / D.Hkv;
  const int lane = lane_id(), wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int nb = num_blocks_of(D, b);
  const int k_eff = D.k < nb ? D.k : nb;

  uint32_t key[KPL];
  int slot[KPL];
  load_keys<WAVES, KPL>(D, scores, table, pair, nb, wave, lane, key, slot);
  Selector<WAVES, KPL> S{lds, 0, wave};

  uint32_t top = 0;
  if (k_eff > 0) top = S.best(key, k_eff, false);

  uint32_t res = 0;
#pragma unroll
  for (int r = 0; r < KPL; ++r)
    if (slot[r] >= 0) res |= 1u << r;
  const uint32_t missing = top & ~res;  // important now, but in host memory
  const uint32_t spare = res & ~top;    // resident, not in the current top-k
  const int n_missing = S.count(missing);
  const int n_spare = S.count(spare);
  const int n = n_missing < n_spare ? n_missing : n_spare;

  uint32_t rec = 0, evi = 0;
  if (n > 0) {
    uint32_t kk[KPL];
    if (n == n_missing) {
      rec = missing;
    } else {  // the cache has room for only n of them: best-ranked first
#pragma unroll
      for (int r = 0; r < KPL; ++r) kk[r] = ((missing >> r) & 1u) ? key[r] : 0u;
      rec = S.best(kk, n, false);
    }
    // worst-ranked spare blocks go: lowest score first, equal scores by higher index
#pragma unroll
    for (int r = 0; r < KPL; ++r) kk[r] = ((spare >> r) & 1u) ? ~key[r] : 0u;
    evi = S.best(kk, n, true);
  }
  int pos_r[KPL], pos_e[KPL];
  S.positions(rec, pos_r);
  S.positions(evi, pos_e);
  const size_t out0 = (size_t)pair * D.k;
#pragma unroll
  for (int r = 0; r < KPL; ++r) {
    if ((evi >> r) & 1u) {
      const int i = (wave * KPL + r) * kWave + lane;
      freed[pos_e[r]] = slot[r];
      recall_slot[out0 + pos_e[r]] = slot[r];
      evict_blk[out0 + pos_e[r]] = i;
      table[(size_t)pair * D.max_blocks + i] = -1;
    }
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < KPL; ++r) {
    if ((rec >> r) & 1u) {
      const int i = (wave * KPL + r) * kWave + lane;
      recall_blk[out0 + pos_r[r]] = i;
      table[(size_t)pair * D.max_blocks + i] = freed[pos_r[r]];
    }
  }
  for (int t = threadIdx.x; t < D.k; t += WAVES * kWave) {
    if (t >= n) {
      recall_blk[out0 + t] = -1;
      recall_slot[out0 + t] = -1;
      evict_blk[out0 + t] = -1;
    }
  }
  if (threadIdx.x == 0) n_recall[pair] = n;
}

// ------------------------------------------------------------ host launchers

#define SCOUT_TOPK_DISPATCH(KERNEL, ...)                                                     \
  do {                                                                                       \
    dim3 grid(D.B* D.Hkv);                                                                   \
    if (grid.x == 0) return SCOUT_OK;                                                        \
    if (D.max_blocks <= 256)                                                                 \
      hipLaunchKernelGGL((KERNEL<1, 4>), grid, dim3(kWave), 0, st, __VA_ARGS__);             \
    else if (D.max_blocks <= 1024)                                                           \
      hipLaunchKernelGGL((KERNEL<1, 16>), grid, dim3(kWave), 0, st, __VA_ARGS__);            \
    else if (D.max_blocks <= 4096)                                                           \
      hipLaunchKernelGGL((KERNEL<4, 16>), grid, dim3(4 * kWave), 0, st, __VA_ARGS__);        \
    else if (D.max_blocks <= 16384)                                                          \
      hipLaunchKernelGGL((KERNEL<16, 16>), grid, dim3(16 * kWave), 0, st, __VA_ARGS__);      \
    else                                                                                     \
      return SCOUT_EUNSUPPORTED;                                                             \
  } while (0)

int launch_topk(const Dims& D, const float* scores, const int32_t* table, int32_t* sel_all,
                int32_t* sel_gpu, int32_t* slot_gpu, int32_t* n_gpu, int32_t* sel_host,
                int32_t* n_host, hipStream_t st) {
  SCOUT_TOPK_DISPATCH(topk_kernel, D, scores, table, sel_all, sel_gpu, slot_gpu, n_gpu, sel_host,
                      n_host);
  return hipGetLastError() == hipSuccess ? SCOUT_OK : SCOUT_EHIP;
}

int launch_recall(const Dims& D, const float* scores, int32_t* table, int32_t* recall_blk,
                  int32_t* recall_slot, int32_t* evict_blk, int32_t* n_recall, hipStream_t st) {
  if (D.k > kMaxK) return SCOUT_EUNSUPPORTED;
  SCOUT_TOPK_DISPATCH(recall_kernel, D, scores, table, recall_blk, recall_slot, evict_blk, n_recall);
  return hipGetLastError() == hipSuccess ? SCOUT_OK : SCOUT_EHIP;
}

}  // namespace scout

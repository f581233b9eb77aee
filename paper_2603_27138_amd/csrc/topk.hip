// Top-k block selection with residency split (Alg. 1: TopK, then predicted
// blocks minus resident blocks) and the recall plan (Sec. 3.4), one workgroup
// per (sequence, KV head) pair.
#include "select.h"

namespace scout {

template <int WAVES, int KPL>
__global__ __launch_bounds__(WAVES* kWave) void topk_kernel(
    Dims D, const float* __restrict__ scores, const int32_t* __restrict__ table,
    int32_t* __restrict__ sel_all, int32_t* __restrict__ sel_gpu, int32_t* __restrict__ slot_gpu,
    int32_t* __restrict__ n_gpu, int32_t* __restrict__ sel_host, int32_t* __restrict__ n_host) {
  __shared__ __attribute__((aligned(16))) int lds[selector_lds_ints<WAVES>()];
  const int b = blockIdx.z, pair = grid_pair();  // grid (1, Hkv, B)
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
  const int ng = S.positions2(sel, pos_all, gpu, pos_gpu);
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
  __shared__ __attribute__((aligned(16))) int lds[selector_lds_ints<WAVES>()];
  __shared__ int freed[kMaxK];  // slots of the evicted blocks, in ascending block order
  const int b = blockIdx.z, pair = grid_pair();  // grid (1, Hkv, B)
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
  S.positions2(rec, pos_r, evi, pos_e);
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

// Waves per pair and keys per lane by row length.  Few keys per lane and many waves win although the
// waves then exchange through LDS: a wave with 16 keys per lane issues its ballots one after the
// other (1024 blocks: 4.6 us with 8 waves x 2 keys against 8.9 us with one wave x 16; 4096 blocks:
// 6.0 us with 16 waves x 4 against 9.3 us with 4 waves x 16).

#define SCOUT_TOPK_DISPATCH(KERNEL, ...)                                                     \
  do {                                                                                       \
    dim3 grid(1, D.Hkv, D.B);                                                                   \
    if (grid.x == 0) return SCOUT_OK;                                                        \
    if (D.max_blocks <= 256)                                                                 \
      hipLaunchKernelGGL((KERNEL<1, 4>), grid, dim3(kWave), 0, st, __VA_ARGS__);             \
    else if (D.max_blocks <= 1024)                                                           \
      hipLaunchKernelGGL((KERNEL<8, 2>), grid, dim3(8 * kWave), 0, st, __VA_ARGS__);         \
    else if (D.max_blocks <= 4096)                                                           \
      hipLaunchKernelGGL((KERNEL<16, 4>), grid, dim3(16 * kWave), 0, st, __VA_ARGS__);       \
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

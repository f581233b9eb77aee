// Data movement of a periodic recall (Sec. 3.4): the blocks that the recall plan names come back from
// host memory into the pool slots that the plan freed, after the layer's attention and off its
// critical path.
//
// The source is host memory that the GPU can address (pinned), read by the kernel itself: one launch
// gathers every tile of every pair, with the plan read where it was written (device memory), instead
// of one small copy per 16 KiB tile issued from the host.  A workgroup moves one block (its K tile and
// its V tile); every thread has all its 16-byte reads in flight before the first write, because over
// the host link it is the number of outstanding reads that makes the rate.
#include "common.h"

namespace scout {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
constexpr int kFetchThreads = 256;
constexpr int kFetchMaxPieces = 8;  // 16-byte pieces per thread and tile: tiles up to 32 KiB

__global__ __launch_bounds__(kFetchThreads) void recall_fetch_kernel(
    Dims D, int tile_bytes, const char* __restrict__ src_k, const char* __restrict__ src_v,
    const int32_t* __restrict__ recall_blk, const int32_t* __restrict__ recall_slot,
    const int32_t* __restrict__ n_recall, char* __restrict__ k_pool, char* __restrict__ v_pool,
    long long n_slots) {
  const int pair = blockIdx.y, i = blockIdx.x;
  int n = n_recall[pair];
  n = n < D.k ? n : D.k;
  if (i >= n) return;
  const int blk = recall_blk[(size_t)pair * D.k + i], slot = recall_slot[(size_t)pair * D.k + i];
  if (blk < 0 || blk >= D.max_blocks || slot < 0 || slot >= n_slots) return;
  const size_t src = ((size_t)pair * D.max_blocks + blk) * tile_bytes, dst = (size_t)slot * tile_bytes;
  const int pieces = tile_bytes / 16;
  u32x4 rk[kFetchMaxPieces], rv[kFetchMaxPieces];
#pragma unroll
  for (int u = 0; u < kFetchMaxPieces; ++u) {
    const int pc = threadIdx.x + u * kFetchThreads;
    if (pc < pieces) {
      rk[u] = *reinterpret_cast<const u32x4*>(src_k + src + (size_t)pc * 16);
      rv[u] = *reinterpret_cast<const u32x4*>(src_v + src + (size_t)pc * 16);
    }
  }
#pragma unroll
  for (int u = 0; u < kFetchMaxPieces; ++u) {
    const int pc = threadIdx.x + u * kFetchThreads;
    if (pc < pieces) {
      *reinterpret_cast<u32x4*>(k_pool + dst + (size_t)pc * 16) = rk[u];
      *reinterpret_cast<u32x4*>(v_pool + dst + (size_t)pc * 16) = rv[u];
    }
  }
}

int launch_recall_fetch(const Dims& D, int dtype, const void* src_k, const void* src_v, const int32_t* recall_blk,
                        const int32_t* recall_slot, const int32_t* n_recall, void* k_pool, void* v_pool,
                        long long n_slots, hipStream_t st) {
  const int tile_bytes = D.S * D.d * (dtype == SCOUT_BF16 ? 2 : 4);
  if (tile_bytes % 16 != 0 || tile_bytes / 16 > kFetchMaxPieces * kFetchThreads) return SCOUT_EUNSUPPORTED;
  dim3 grid(D.k, D.B * D.Hkv);
  if (grid.x == 0 || grid.y == 0) return SCOUT_OK;
  hipLaunchKernelGGL(recall_fetch_kernel, grid, dim3(kFetchThreads), 0, st, D, tile_bytes,
                     static_cast<const char*>(src_k), static_cast<const char*>(src_v), recall_blk, recall_slot,
                     n_recall, static_cast<char*>(k_pool), static_cast<char*>(v_pool), n_slots);
  return hipGetLastError() == hipSuccess ? SCOUT_OK : SCOUT_EHIP;
}

}  // namespace scout

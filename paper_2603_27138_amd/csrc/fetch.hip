// Data movement of a periodic recall (Sec. 3.4): the blocks that the recall plan names come back from
// host memory into the pool slots that the plan freed, after the layer's attention and off its
// critical path.
//
// The source is host memory that the GPU can address (pinned), read by the kernel itself: one launch
// gathers every tile of every pair, with the plan read where it was written (device memory), instead
// of one small copy per 16 KiB tile issued from the host.  A workgroup moves one block at a time (its
// K tile and its V tile); every thread has all its 16-byte reads in flight before the first write,
// because over the host link it is the number of outstanding reads that makes the rate.
//
// The launch is small (a few dozen workgroups keep far more bytes in flight than the host link's
// latency needs).
//
// Reads that wave loads send over the host link hold up the memory system for everything else on the
// GPU: kernels that run beside this one (layer steps, a GEMM, a plain copy) were measured 1.7 to 1.9
// times slower while it ran, however few workgroups it used, whereas a copy by the DMA engine left
// them within a few per cent.  So when the transfer is to overlap with compute, the staged route is
// the one to use: the host packs the planned tiles (scout_host_stage_recall), one contiguous copy by
// the DMA engine brings them over, and recall_scatter_kernel, device to device, puts them into their
// slots.  The direct kernel remains for callers that recall with nothing else running.
#include "common.h"

namespace scout {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
constexpr int kFetchThreads = 256;
constexpr int kFetchMaxPieces = 8;  // 16-byte pieces per thread and tile: tiles up to 32 KiB
constexpr int kFetchWgs = 64;

// One tile pair by one workgroup: all reads of a thread in flight before its first write.
__device__ __forceinline__ void move_tiles(const char* __restrict__ from_k, const char* __restrict__ from_v,
                                           char* __restrict__ to_k, char* __restrict__ to_v, int pieces) {
  u32x4 rk[kFetchMaxPieces], rv[kFetchMaxPieces];
#pragma unroll
  for (int u = 0; u < kFetchMaxPieces; ++u) {
    const int pc = threadIdx.x + u * kFetchThreads;
    if (pc < pieces) {
      rk[u] = *reinterpret_cast<const u32x4*>(from_k + (size_t)pc * 16);
      rv[u] = *reinterpret_cast<const u32x4*>(from_v + (size_t)pc * 16);
    }
  }
#pragma unroll
  for (int u = 0; u < kFetchMaxPieces; ++u) {
    const int pc = threadIdx.x + u * kFetchThreads;
    if (pc < pieces) {
      *reinterpret_cast<u32x4*>(to_k + (size_t)pc * 16) = rk[u];
      *reinterpret_cast<u32x4*>(to_v + (size_t)pc * 16) = rv[u];
    }
  }
}

// Workgroup w of W: if there are fewer pairs than workgroups, W / pairs workgroups share a pair and
// deal its entries round robin; otherwise workgroups take whole pairs, W apart.
__global__ __launch_bounds__(kFetchThreads) void recall_fetch_kernel(
    Dims D, int tile_bytes, int stride_bytes, int wgs_per_pair, const char* __restrict__ src_k, const char* __restrict__ src_v,
    const int32_t* __restrict__ recall_blk, const int32_t* __restrict__ recall_slot,
    const int32_t* __restrict__ n_recall, char* __restrict__ k_pool, char* __restrict__ v_pool,
    long long n_slots) {
  const int pairs = D.B * D.Hkv;
  const int first_pair = blockIdx.x / wgs_per_pair, first_entry = blockIdx.x % wgs_per_pair;
  const int pair_step = (gridDim.x + wgs_per_pair - 1) / wgs_per_pair;
  for (int pair = first_pair; pair < pairs; pair += pair_step) {
    int n = n_recall[pair];
    n = n < D.k ? n : D.k;
    for (int i = first_entry; i < n; i += wgs_per_pair) {
      const int blk = recall_blk[(size_t)pair * D.k + i], slot = recall_slot[(size_t)pair * D.k + i];
      if (blk < 0 || blk >= D.max_blocks || slot < 0 || slot >= n_slots) continue;
      const size_t src = ((size_t)pair * D.max_blocks + blk) * tile_bytes, dst = (size_t)slot * stride_bytes;
      move_tiles(src_k + src, src_v + src, k_pool + dst, v_pool + dst, tile_bytes / 16);
    }
  }
}

// The staged route: the tiles already sit in device memory, packed by the host in plan order (tile
// tile_off[pair] + i of entry i: K rows, then V rows).  Device to device: gridDim.x workgroups per pair
// deal the pair's entries round robin (a recall moves a fraction of the budget, so a workgroup per
// possible entry would mostly launch workgroups that find nothing to do).
__global__ __launch_bounds__(kFetchThreads) void recall_scatter_kernel(
    Dims D, int tile_bytes, int stride_bytes, const char* __restrict__ staged, long long n_tiles,
    const int32_t* __restrict__ tile_off, const int32_t* __restrict__ recall_blk,
    const int32_t* __restrict__ recall_slot, const int32_t* __restrict__ n_recall, char* __restrict__ k_pool,
    char* __restrict__ v_pool, long long n_slots) {
  const int pair = blockIdx.y;
  int n = n_recall[pair];
  n = n < D.k ? n : D.k;
  if ((int)blockIdx.x >= n) return;
  const long long first = tile_off[pair];
  for (int i = blockIdx.x; i < n; i += gridDim.x) {
    const int blk = recall_blk[(size_t)pair * D.k + i], slot = recall_slot[(size_t)pair * D.k + i];
    if (blk < 0 || blk >= D.max_blocks || slot < 0 || slot >= n_slots) continue;
    if (first < 0 || first + i >= n_tiles) continue;  // an offset that points outside the buffer moves nothing
    const char* from = staged + (size_t)(first + i) * 2 * tile_bytes;
    const size_t dst = (size_t)slot * stride_bytes;
    move_tiles(from, from + tile_bytes, k_pool + dst, v_pool + dst, tile_bytes / 16);
  }
}

int launch_recall_fetch(const Dims& D, int dtype, const void* src_k, const void* src_v, const int32_t* recall_blk,
                        const int32_t* recall_slot, const int32_t* n_recall, void* k_pool, void* v_pool,
                        long long n_slots, hipStream_t st) {
  const int tile_bytes = D.S * D.d * (dtype == SCOUT_BF16 ? 2 : 4);
  if (tile_bytes % 16 != 0 || tile_bytes / 16 > kFetchMaxPieces * kFetchThreads) return SCOUT_EUNSUPPORTED;
  const long long pairs = (long long)D.B * D.Hkv;
  if (pairs == 0) return SCOUT_OK;
  int wgs_per_pair = pairs < kFetchWgs ? (int)(kFetchWgs / pairs) : 1;
  if (wgs_per_pair > D.k) wgs_per_pair = D.k;
  const long long want = pairs * wgs_per_pair;
  const unsigned grid = (unsigned)(want < kFetchWgs ? want : kFetchWgs);
  const int stride_bytes = D.tile_stride * (dtype == SCOUT_BF16 ? 2 : 4);
  hipLaunchKernelGGL(recall_fetch_kernel, dim3(grid), dim3(kFetchThreads), 0, st, D, tile_bytes, stride_bytes, wgs_per_pair,
                     static_cast<const char*>(src_k), static_cast<const char*>(src_v), recall_blk, recall_slot,
                     n_recall, static_cast<char*>(k_pool), static_cast<char*>(v_pool), n_slots);
  return hipGetLastError() == hipSuccess ? SCOUT_OK : SCOUT_EHIP;
}

int launch_recall_scatter(const Dims& D, int dtype, const void* staged, long long n_tiles, const int32_t* tile_off,
                          const int32_t* recall_blk, const int32_t* recall_slot, const int32_t* n_recall,
                          void* k_pool, void* v_pool, long long n_slots, hipStream_t st) {
  const int tile_bytes = D.S * D.d * (dtype == SCOUT_BF16 ? 2 : 4);
  if (tile_bytes % 16 != 0 || tile_bytes / 16 > kFetchMaxPieces * kFetchThreads) return SCOUT_EUNSUPPORTED;
  dim3 grid(D.k < 16 ? D.k : 16, D.B * D.Hkv);
  if (grid.x == 0 || grid.y == 0) return SCOUT_OK;
  const int stride_bytes = D.tile_stride * (dtype == SCOUT_BF16 ? 2 : 4);
  hipLaunchKernelGGL(recall_scatter_kernel, grid, dim3(kFetchThreads), 0, st, D, tile_bytes, stride_bytes,
                     static_cast<const char*>(staged), n_tiles, tile_off, recall_blk, recall_slot, n_recall,
                     static_cast<char*>(k_pool), static_cast<char*>(v_pool), n_slots);
  return hipGetLastError() == hipSuccess ? SCOUT_OK : SCOUT_EHIP;
}

}  // namespace scout

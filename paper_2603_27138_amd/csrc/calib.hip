// Measurement aids, a library of their own (libscout_calib.so): nothing of the method runs here.
// A plain copy of known size to scale HBM byte counters, and the two access patterns of the path with
// nothing computed (a read-only stream, a gather of K/V tiles by slot), so that a benchmark can state
// what this GPU sustains for them next to the kernels' own rates.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "scout_calib.h"

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Reference for HBM byte counters: a plain copy with the same 16-byte accesses the kernels use.
__global__ __launch_bounds__(256) void calib_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                         size_t n16) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

// Measured ceilings for the two access patterns of the path, nothing computed: a read-only stream
// (what the digest pass does) and a gather of whole K and V tiles by slot (what the attention does).
// Many small waves, everything requested at once: 8 loads of 16 bytes per lane.
__global__ __launch_bounds__(256) void calib_read_kernel(const uint4* __restrict__ src, size_t n16, uint32_t* sink) {
  const size_t base = ((size_t)blockIdx.x * 256 * 8) + threadIdx.x;
  uint4 v[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const size_t i = base + (size_t)u * 256;
    v[u] = i < n16 ? src[i] : make_uint4(0, 0, 0, 0);
  }
  uint32_t acc = 0;
#pragma unroll
  for (int u = 0; u < 8; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  if (acc == 0x9e3779b9u && sink != nullptr) sink[0] = acc;  // keeps the loads alive; practically never true
}

// grid (ceil(k/2), pairs), four waves per workgroup: waves 0 and 1 read the K and the V tile of entry
// blockIdx.x of the pair's list, waves 2 and 3 those of entry k-1-blockIdx.x, if the list is that long
// (a list is rarely full, so folding it keeps most workgroups from being launched for nothing).
__global__ __launch_bounds__(256) void calib_gather_kernel(const char* __restrict__ k_pool,
                                                           const char* __restrict__ v_pool, long long n_slots,
                                                           int tile_bytes, int stride_bytes,
                                                           const int32_t* __restrict__ slot_gpu,
                                                           const int32_t* __restrict__ n_gpu, int k, uint32_t* sink) {
  const int pair = blockIdx.y, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = wave < 2 ? (int)blockIdx.x : k - 1 - (int)blockIdx.x;
  if (wave >= 2 && i <= (int)blockIdx.x) return;  // the middle entry of an odd k belongs to waves 0 and 1
  const long long slot = slot_gpu[(size_t)pair * k + i];  // read with the count, not after it
  int n = n_gpu[pair];
  n = n < k ? n : k;
  if (i >= n || slot < 0 || slot >= n_slots) return;
  const char* tile = ((wave & 1) ? v_pool : k_pool) + (size_t)slot * stride_bytes;
  uint32_t acc = 0;
  for (int off = lane * 16; off < tile_bytes; off += 8 * 1024) {  // 8 KiB per trip: 8 loads in flight
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      v[u] = off + u * 1024 < tile_bytes ? *reinterpret_cast<const uint4*>(tile + off + u * 1024) : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  if (acc == 0x9e3779b9u && sink != nullptr) sink[0] = acc;
}

}  // namespace

extern "C" {

int scout_calib_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst || !aligned16(src) || !aligned16(dst) || bytes % 16 != 0) return SCOUT_EINVAL;
  if (bytes == 0) return SCOUT_OK;
  hipLaunchKernelGGL(calib_copy_kernel, dim3(4096), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint4*>(src), static_cast<uint4*>(dst), bytes / 16);
  return hipGetLastError() == hipSuccess ? SCOUT_OK : SCOUT_EHIP;
}

int scout_calib_read(const void* src, size_t bytes, void* sink, void* stream) {
  if (!src || !aligned16(src) || bytes % 16 != 0) return SCOUT_EINVAL;
  if (bytes == 0) return SCOUT_OK;
  const size_t n16 = bytes / 16, per_wg = 256 * 8;
  hipLaunchKernelGGL(calib_read_kernel, dim3((unsigned)((n16 + per_wg - 1) / per_wg)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<const uint4*>(src), n16,
                     static_cast<uint32_t*>(sink));
  return hipGetLastError() == hipSuccess ? SCOUT_OK : SCOUT_EHIP;
}

int scout_calib_gather(const scout_problem* p, const void* k_pool, const void* v_pool, int64_t n_slots,
                       const int32_t* slot_gpu, const int32_t* n_gpu, void* sink, void* stream) {
  if (p == nullptr || p->B < 0 || p->Hkv < 1 || p->k < 1 || p->S < 1 || p->d < 8 || p->d % 8 != 0 ||
      (p->dtype != SCOUT_F32 && p->dtype != SCOUT_BF16) || (long long)p->B * p->Hkv > 65535)
    return SCOUT_EINVAL;
  if (!k_pool || !v_pool || !slot_gpu || !n_gpu || !aligned16(k_pool) || !aligned16(v_pool) || n_slots < 0)
    return SCOUT_EINVAL;
  const int esize = p->dtype == SCOUT_BF16 ? 2 : 4;
  const int tile_bytes = p->S * p->d * esize;
  if (p->tile_stride != 0 && (p->tile_stride < p->S * p->d || p->tile_stride % 8 != 0)) return SCOUT_EINVAL;
  const int stride_bytes = p->tile_stride != 0 ? p->tile_stride * esize : tile_bytes;
  dim3 grid((p->k + 1) / 2, p->B * p->Hkv);
  if (grid.y == 0) return SCOUT_OK;
  hipLaunchKernelGGL(calib_gather_kernel, grid, dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const char*>(k_pool), static_cast<const char*>(v_pool), (long long)n_slots,
                     tile_bytes, stride_bytes, slot_gpu, n_gpu, p->k, static_cast<uint32_t*>(sink));
  return hipGetLastError() == hipSuccess ? SCOUT_OK : SCOUT_EHIP;
}

}  // extern "C"

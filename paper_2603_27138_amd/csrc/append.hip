// Decode append: the key and value of the token that decode just produced join the cache, and the
// digest of the block they fall into (Sec. 2.2: channel-wise min/max over the block's keys, or their
// sum for mean pooling) is kept up to date, so that the digests of all blocks stay on the GPU as Sec. 3.2 requires while the
// sequence grows.
//
// One workgroup per sequence, one thread per (KV head, channel) element: a few kilobytes per call,
// bound by latency, not by bandwidth.  Every thread reads the sequence's length before the barrier
// and one thread advances it after, so the length can be updated in place.
#include <type_traits>

#include "common.h"

namespace scout {

template <int DT>
__global__ __launch_bounds__(1024) void append_kernel(Dims D, int32_t* ctx_len, const void* __restrict__ k_new,
                                                     const void* __restrict__ v_new,
                                                     const int32_t* __restrict__ new_slot, void* digest,
                                                     int32_t* block_table, void* k_pool, void* v_pool,
                                                     long long n_slots, void* host_k, void* host_v) {
  using E = typename std::conditional<DT == SCOUT_BF16, uint16_t, float>::type;
  const int b = blockIdx.x;
  const int t = ctx_len[b];
  const bool room = t >= 0 && t < D.max_blocks * D.S;  // a full sequence is left as it is
  if (room) {
    const int j = t >> D.s_shift, r = t & (D.S - 1);  // S and d are powers of two
    const E* kn = static_cast<const E*>(k_new);
    const E* vn = static_cast<const E*>(v_new);
    E* dg = static_cast<E*>(digest);
    E* kp = static_cast<E*>(k_pool);
    E* vp = static_cast<E*>(v_pool);
    E* hk = static_cast<E*>(host_k);  // the host's copy of every block (pinned memory), or null
    E* hv = static_cast<E*>(host_v);
    const int d_shift = D.d == 64 ? 6 : 7;
    for (int e = threadIdx.x; e < D.Hkv * D.d; e += blockDim.x) {
      const int g = e >> d_shift, c = e & (D.d - 1);
      const size_t pair = (size_t)b * D.Hkv + g;
      int32_t* entry = block_table + pair * D.max_blocks + j;
      // a block's first token opens it with the slot the caller chose; later tokens follow the table
      const int slot = r == 0 ? new_slot[pair] : *entry;
      const E k = kn[pair * D.d + c], v = vn[pair * D.d + c];
      const size_t i_min = ((pair * D.max_blocks + j) * 2) * D.d + c, i_max = i_min + D.d;
      if (D.digest_kind == 1) {  // mean pooling: the block's running sum in binary32, one addition per token
        float* sums = static_cast<float*>(digest);
        const size_t i_sum = (pair * D.max_blocks + j) * D.d + c;
        const float kf = load1<DT>(kn, pair * D.d + c);
        sums[i_sum] = r == 0 ? kf : sums[i_sum] + kf;
      } else if (r == 0) {
        dg[i_min] = k;
        dg[i_max] = k;
      } else {
        // strict comparisons: of equal elements the older one stays, as in a first-occurrence min/max
        const float kf = load1<DT>(kn, pair * D.d + c);
        if (kf < load1<DT>(dg, i_min)) dg[i_min] = k;
        if (kf > load1<DT>(dg, i_max)) dg[i_max] = k;
      }
      if (slot >= 0 && slot < n_slots) {
        const size_t row = (size_t)slot * D.tile_stride + (size_t)r * D.d + c;
        kp[row] = k;
        vp[row] = v;
      }
      if (hk != nullptr) {  // whatever the residency: this is what a later recall reads, and why an
                            // eviction has nothing to move
        const size_t row = ((pair * D.max_blocks + j) * D.S + r) * D.d + c;
        hk[row] = k;
        hv[row] = v;
      }
      if (r == 0 && c == 0) *entry = slot;  // nobody reads the entry in this call when r == 0
    }
  }
  __syncthreads();
  if (room && threadIdx.x == 0) ctx_len[b] = t + 1;
}

int launch_append(const Dims& D, int dtype, int32_t* ctx_len, const void* k_new, const void* v_new,
                  const int32_t* new_slot, void* digest, int32_t* block_table, void* k_pool, void* v_pool,
                  long long n_slots, void* host_k, void* host_v, hipStream_t st) {
  if (D.B == 0) return SCOUT_OK;
  // one element per thread where the sequence's row fits a workgroup: the call is a chain of
  // dependent round trips (length, table entry, digest), so it should walk that chain once
  const int elems = D.Hkv * D.d;
  const dim3 block(elems >= 1024 ? 1024 : (elems + 63) / 64 * 64);
  if (dtype == SCOUT_BF16)
    hipLaunchKernelGGL(append_kernel<SCOUT_BF16>, dim3(D.B), block, 0, st, D, ctx_len, k_new, v_new, new_slot,
                       digest, block_table, k_pool, v_pool, n_slots, host_k, host_v);
  else
    hipLaunchKernelGGL(append_kernel<SCOUT_F32>, dim3(D.B), block, 0, st, D, ctx_len, k_new, v_new, new_slot,
                       digest, block_table, k_pool, v_pool, n_slots, host_k, host_v);
  return hipGetLastError() == hipSuccess ? SCOUT_OK : SCOUT_EHIP;
}

}  // namespace scout

// Selection machinery shared by the top-k kernels and the fused select-and-attend kernel.
//
// Selection (Alg. 1, TopK): the k best blocks of a pair under the total order
// (score descending, block index ascending).  Integer work only: scores are
// mapped to order-preserving 32-bit keys, the k-th largest key is found by a
// bit-by-bit threshold search that starts below the prefix all keys share and
// whose counts are wave ballots and scalar population counts (no sort), and the
// winners are put in ascending index order by a ballot prefix count.
//
// Element i of a pair lives in wave i / (64*KPL), register (i / 64) % KPL,
// lane i % 64: loads are coalesced and index order is (wave, register, lane).
#pragma once
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

// Inclusive prefix sum over the 64 lanes on the vector ALU (DPP row shifts, then the two
// row-to-row broadcasts), no LDS traffic.
__device__ __forceinline__ int wave_inclusive_scan(int x) {
  int v = x;
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);  // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);  // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);  // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);  // row_shr:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1 and 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2 and 3
  return v;
}

// OR over the 64 lanes, result in every lane: rotations inside the 16-lane rows (DPP), then the
// row exchanges, all on the vector ALU.
__device__ __forceinline__ uint32_t wave_or(uint32_t v) {
  v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x128, 0xf, 0xf, false);  // row_ror:8
  v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x124, 0xf, 0xf, false);  // row_ror:4
  v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x122, 0xf, 0xf, false);  // row_ror:2
  v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x121, 0xf, 0xf, false);  // row_ror:1
  auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
  v = r[0] | r[1];
  r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return r[0] | r[1];
}

template <int WAVES, int KPL>
struct Selector {
  int* lds;
  int phase;
  int wave;
  // Histogram rounds done so far by this Selector, over all its best() calls (several waves only).
  // Round r counts into bin array r % 3 and, after its barrier, clears array (r + 2) % 3 for round
  // r + 2.  The numbering runs on from one call to the next, which is what makes back-to-back calls
  // safe without a barrier between them: a call that ends with round r (its reads of array r % 3 are
  // followed by no barrier) leaves array (r + 1) % 3 clean (cleared in round r - 1, or by the first
  // call's opening clear) and array (r + 2) % 3 being cleared; the next call starts with round r + 1,
  // touches array r % 3 only after the barrier of that round (its clear for round r + 3), and a wave
  // still reading array r % 3 for the previous call has not yet arrived at the barriers (the common
  // prefix exchange, then round r + 1) that every wave must pass before that clear.  Wave-uniform.
  int hround = 0;

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

  // positions() of two masks with one exchange: the two per-wave counts travel in the halves of one
  // word (a workgroup holds at most 16384 elements, so neither half can carry into the other).
  // Returns the total of the second mask.
  __device__ __forceinline__ int positions2(uint32_t bits_a, int (&pos_a)[KPL], uint32_t bits_b, int (&pos_b)[KPL]) {
    int ca = 0, cb = 0;
#pragma unroll
    for (int r = 0; r < KPL; ++r) {
      ca += __popcll(__ballot((bits_a >> r) & 1u));
      cb += __popcll(__ballot((bits_b >> r) & 1u));
    }
    int total, off;
    wg_exchange<WAVES>(ca | (cb << 16), lds, phase, wave, total, off);
    int off_a = off & 0xffff, off_b = off >> 16;
#pragma unroll
    for (int r = 0; r < KPL; ++r) {
      const uint64_t ma = __ballot((bits_a >> r) & 1u), mb = __ballot((bits_b >> r) & 1u);
      pos_a[r] = off_a + mbcnt64(ma);
      pos_b[r] = off_b + mbcnt64(mb);
      off_a += __popcll(ma);
      off_b += __popcll(mb);
    }
    return total >> 16;
  }

  __device__ __forceinline__ int count(uint32_t bits) {
    int c = 0;
#pragma unroll
    for (int r = 0; r < KPL; ++r) c += __popcll(__ballot((bits >> r) & 1u));
    int total, before;
    wg_exchange<WAVES>(c, lds, phase, wave, total, before);
    return total;
  }

  // OR and AND of a per-lane word over the whole workgroup
  __device__ __forceinline__ void or_and(uint32_t vo, uint32_t va, uint32_t& all_or, uint32_t& all_and) {
    vo = wave_or(vo);
    va = ~wave_or(~va);
    if (WAVES > 1) {
      int* buf = lds + (phase & 1) * WAVES;  // same alternation as wg_exchange
      int* buf2 = lds + 2 * WAVES + (phase & 1) * WAVES;
      if (lane_id() == 0) {
        buf[wave] = (int)vo;
        buf2[wave] = (int)va;
      }
      __syncthreads();
      vo = 0;
      va = 0xffffffffu;
#pragma unroll
      for (int w = 0; w < WAVES; ++w) {
        vo |= (uint32_t)buf[w];
        va &= (uint32_t)buf2[w];
      }
      ++phase;
    }
    all_or = vo;
    all_and = va;
  }

  // Bits of the kk best candidates (key > 0) under (key descending, then index
  // ascending, or descending when high_index_first).  Needs 1 <= kk <= number
  // of candidates.
  __device__ __forceinline__ uint32_t best(const uint32_t (&key)[KPL], int kk, bool high_index_first) {
    // Bits on which all candidates agree need no search: start below the common prefix.
    uint32_t vo = 0, va = 0xffffffffu;
#pragma unroll
    for (int r = 0; r < KPL; ++r) {
      vo |= key[r];
      va &= key[r] ? key[r] : 0xffffffffu;
    }
    if constexpr (WAVES > 1) {
      // Before the first histogram round of this Selector, bin arrays 0 and 1 are cleared here, so that
      // the barrier inside or_and also publishes the zeros.  Later calls find their arrays clean (see
      // hround) and must not clear here: a slower wave may still be reading the last round's array.
      if (hround == 0) {
        int* hist = lds + 4 * WAVES;
        for (int i = wave * kWave + lane_id(); i < 2 * 256; i += WAVES * kWave) hist[i] = 0;
      }
    }
    uint32_t all_or, all_and;
    or_and(vo, va, all_or, all_and);
    const uint32_t diff = all_or ^ all_and;
    // the largest T with  count(key >= T) >= kk  is the kk-th largest key
    uint32_t T = diff ? (all_and & ~(0xffffffffu >> __builtin_clz(diff))) : all_and;
    int n_ge = -1;
    if constexpr (WAVES == 1) {
      for (int bit = diff ? 31 - __builtin_clz(diff) : -1; bit >= 0; --bit) {
        const uint32_t cand = T | (1u << bit);
        const int c = count_ge(key, cand);
        if (c >= kk) T = cand;
        if (c == kk) {  // {key >= cand} is exactly the answer; lower bits cannot matter
          n_ge = c;
          break;
        }
      }
    } else {
      // Several waves: every exchange through LDS costs a barrier's latency, so the threshold is
      // settled eight bits per round by a histogram.  Keys that agree with the bits found so far
      // add one to the bin of their next digit (LDS atomics), one barrier, then every wave reads the
      // 256 bins (four per lane), forms the suffix sums with a vector-ALU scan and picks the largest
      // digit whose suffix count, added to the keys already known to be above, still reaches kk.
      // Three bin arrays rotate: the one for the round after next is cleared while this round's is read.
      int* hist = lds + 4 * WAVES;
      const int tid = wave * kWave + lane_id();
      int n_above = 0;  // keys whose settled bits are larger than T's
      int bit = diff ? 31 - __builtin_clz(diff) : -1;
      while (bit >= 0) {
        const int nbits = bit >= 7 ? 8 : bit + 1;
        const int shift = bit - nbits + 1;
        const int hslot = hround % 3;
        int* h = hist + hslot * 256;
        int* hz = hist + (hslot == 0 ? 2 : hslot - 1) * 256;  // (hround + 2) % 3
        ++hround;  // counted whether or not this round ends the search
        const uint32_t hi_mask = bit == 31 ? 0u : ~((2u << bit) - 1u);  // bits above this round's digit
#pragma unroll
        for (int r = 0; r < KPL; ++r) {
          if (key[r] != 0u && (key[r] & hi_mask) == (T & hi_mask))
            atomicAdd(&h[(key[r] >> shift) & ((1u << nbits) - 1u)], 1);
        }
        __syncthreads();
        // every wave is past the previous round's reads now: clear the array of the round after next
        for (int i = tid; i < 256; i += WAVES * kWave) hz[i] = 0;
        // lane l owns digits 4l .. 4l+3
        const int4 b4 = *reinterpret_cast<const int4*>(h + 4 * lane_id());
        const int lane_sum = b4.x + b4.y + b4.z + b4.w;
        const int incl = wave_inclusive_scan(lane_sum);
        const int total = __builtin_amdgcn_readlane(incl, kWave - 1);
        // suffix counts (keys with digit >= d), plus the keys already above
        const int s3 = n_above + total - incl + b4.w;
        const int s2 = s3 + b4.z, s1 = s2 + b4.y, s0 = s1 + b4.x;
        const int n_ok = (s0 >= kk) + (s1 >= kk) + (s2 >= kk) + (s3 >= kk);  // a prefix of the four
        const uint64_t any = __ballot(n_ok > 0);
        // some digit qualifies: digit 0 counts every candidate that matches so far
        const int top_lane = 63 - __builtin_clzll(any);
        const int top_ok = __builtin_amdgcn_readlane(n_ok, top_lane);
        const int dstar = 4 * top_lane + top_ok - 1;
        const int s_at = __builtin_amdgcn_readlane(top_ok == 1 ? s0 : top_ok == 2 ? s1 : top_ok == 3 ? s2 : s3, top_lane);
        const int h_at = __builtin_amdgcn_readlane(top_ok == 1 ? b4.x : top_ok == 2 ? b4.y : top_ok == 3 ? b4.z : b4.w,
                                                   top_lane);
        T |= (uint32_t)dstar << shift;
        n_above = s_at - h_at;
        if (s_at == kk) {  // {key >= T} is exactly the answer; lower bits cannot matter
          n_ge = kk;
          break;
        }
        bit -= nbits;
      }
    }
    uint32_t ge = 0;
#pragma unroll
    for (int r = 0; r < KPL; ++r) ge |= (key[r] >= T ? 1u : 0u) << r;
    if (n_ge == kk) return ge;  // wave-uniform
    // ties at the threshold: take them in index order until kk are chosen
    uint32_t gt = 0, eq = 0;
#pragma unroll
    for (int r = 0; r < KPL; ++r) {
      gt |= (key[r] > T ? 1u : 0u) << r;
      eq |= (key[r] == T ? 1u : 0u) << r;
    }
    int rank[KPL];
    const int n_eq = positions(eq, rank);
    const int n_gt = count(gt);
    const int need = kk - n_gt;
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
  const size_t trow = (size_t)kv_row(D, pair) * D.max_blocks;  // the table belongs to the KV head
  float sc[KPL];
#pragma unroll
  for (int r = 0; r < KPL; ++r) {
    const int i = (wave * KPL + r) * kWave + lane;
    const int ic = i < D.max_blocks ? i : D.max_blocks - 1;
    sc[r] = scores[row + ic];
    slot[r] = table[trow + ic];
  }
#pragma unroll
  for (int r = 0; r < KPL; ++r) {
    const int i = (wave * KPL + r) * kWave + lane;
    key[r] = i < nb ? score_key(sc[r]) : 0u;
    slot[r] = i < nb ? slot[r] : -1;
  }
}

// LDS words a Selector needs for WAVES waves
template <int WAVES>
constexpr int selector_lds_ints() { return 4 * WAVES + 3 * 256; }

}  // namespace scout

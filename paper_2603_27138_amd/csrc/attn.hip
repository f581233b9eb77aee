// Block-sparse paged decode attention over the selected GPU-resident blocks
// (Sec. 3.2; Alg. 1 GPUAttn) and the merge of partial results (Alg. 1 Merge).
//
// A partial result of a token set is (o, m, l): m the largest logit, l the sum
// of exp(logit - m), o the weighted value sum.  Partials of disjoint sets
// combine exactly (FlashAttention rescaling), which is used three times: across
// the blocks a wave walks through, across the waves / workgroups that split a
// pair's block list, and finally with the host's partial.
//
// Inside the kernels logits are kept in base-2 units (x * log2(e)), so the
// exponentials are bare v_exp_f32; m is converted back to natural-log units
// where it leaves the library.
//
// Two kernel families write the same per-split partials into the workspace:
//   attn_mfma_kernel  bf16, d = 128: the G query heads of a KV head form one MFMA
//                     operand, K and V rows go from HBM straight into MFMA operand
//                     registers (no LDS), in units of 16 tokens.
//   attn_valu_kernel  any supported (dtype, d, S): plain vector ALU, used for
//                     fp32 and the other shapes.
// combine_kernel folds the splits (and optionally the host partial) together.
#include "select.h"

namespace scout {

// bare v_exp_f32: results below 2^-126 flush to zero, which is what a softmax weight wants
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float exp2_diff(float a, float b) {
  // 2^(a-b) with the convention 2^(-inf - anything) = 0
  return a == -INFINITY ? 0.0f : fast_exp2(a - b);
}

// ---------------------------------------------------------------- MFMA family

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// Pack the low (sel = 0) or high (sel = 1) bf16 of two dwords into one dword:
// result.lo = half(a), result.hi = half(b).  One v_perm_b32: its selector bytes
// 0-3 address the second source operand, 4-7 the first.
__device__ __forceinline__ uint32_t pack_halves(uint32_t a, uint32_t b, int sel) {
  return sel ? __builtin_amdgcn_perm(b, a, 0x07060302u) : __builtin_amdgcn_perm(b, a, 0x05040100u);
}

typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

// two binary32 -> one dword of two bf16 (round to nearest even), x in the low half
__device__ __forceinline__ uint32_t cvt_pk_bf16(float x, float y) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){x, y}, bf16x2));
}

constexpr int kMfmaD = 128;

// The host's partial for one output element (mode 2 only); loaded ahead of the point of use so
// that its latency hides behind the fold.
struct HostPart {
  float o, m, l;
};

__device__ __forceinline__ HostPart load_host(const Dims& D, const Epilogue& E, int bh, int c) {
  HostPart hp{0.0f, -INFINITY, 0.0f};
  if (E.mode == 2 && E.host_o != nullptr) {
    hp.m = E.host_m[bh];
    hp.l = E.host_l[bh];
    hp.o = E.host_o[(size_t)bh * D.d + c];
  }
  return hp;
}

// acc: unnormalised weighted value sum of channel c, l: weight sum, M2: base-2 maximum
__device__ __forceinline__ void finish(const Dims& D, const Epilogue& E, int bh, int c, float acc,
                                       float l, float M2, const HostPart& hp) {
  const float m_nat = M2 * kLn2;  // -inf stays -inf
  const float o_norm = l > 0.0f ? acc / l : 0.0f;
  if (E.mode == 1) {
    E.o[(size_t)bh * D.d + c] = o_norm;
    if (c == 0) {
      E.m[bh] = m_nat;
      E.l[bh] = l;
    }
    return;
  }
  const float mb = hp.m, lb = hp.l, ob = hp.o;
  float ms = -INFINITY;
  if (l > 0.0f) ms = fmaxf(ms, m_nat);
  if (lb > 0.0f) ms = fmaxf(ms, mb);
  const float wa = l > 0.0f ? l * expf(m_nat - ms) : 0.0f;
  const float wb = lb > 0.0f ? lb * expf(mb - ms) : 0.0f;
  const float ls = wa + wb;
  float r = 0.0f;
  if (wa > 0.0f) r += wa * o_norm;
  if (wb > 0.0f) r += wb * ob;
  r = ls > 0.0f ? r / ls : 0.0f;
  if (E.dtype_out == SCOUT_BF16)
    static_cast<uint16_t*>(E.out)[(size_t)bh * D.d + c] = (uint16_t)f32_to_bf16_bits(r);
  else
    static_cast<float*>(E.out)[(size_t)bh * D.d + c] = r;
  if (E.lse != nullptr && c == 0) E.lse[bh] = ls > 0.0f ? ms + logf(ls) : -INFINITY;
}

// The work of a pair is cut into units of 16 tokens (a block of S tokens is S/16 units; a unit's K
// rows and V rows are 4 KiB each, contiguous).  The pair's units are dealt to the waves that share
// the pair (all waves of all its workgroups) in contiguous ranges whose lengths differ by at most
// one, so no wave waits for a neighbour that got a whole block more.  For each unit:
//   logits^T[token][head] = K[token][:] . Q[head][:]            4 x mfma 16x16x32
//   online softmax per head (heads live in lane % 16)
//   out^T[dim][head]    += V^T[dim][token] . P^T[token][head]   8 x mfma 16x16x16
// Operand layout of the 16x16 MFMAs: lane L supplies, for A, row L%16 and for B, column L%16, the
// contraction elements of group L/16 (8 of them for x32, 4 for x16); the result has column L%16 and
// rows 4*(L/16)+i.  The contraction index may be labelled freely as long as A and B agree, which
// lets the logits leave the first product in exactly the registers the second one needs: lane L
// ends up with the logits of head L%16 for tokens 4*(L/16) + i (i = 0..3), so the value rows are
// loaded in that same token order.  Element r of a lane's 16-byte value chunk feeds product r, whose
// output row index then means channel 8*row + r.
//
// The waves of a workgroup fold their partials through LDS; with one split per pair the workgroup
// finishes the pair itself (Epilogue modes 1 and 2), so the whole attention is one launch and
// nothing goes through the workspace.

constexpr int kUnitTokens = 16;
constexpr int kUnitBytes = kUnitTokens * kMfmaD * 2;  // of K, and of V

typedef __attribute__((ext_vector_type(4))) short s16x4;

// K and V rows of one unit in MFMA operand registers (32 VGPRs).
struct UnitRegs {
  u32x4 k[4];  // contraction step s: row = token ln, 16-byte chunk 4*s + kg
  u32x4 v[4];  // row = token 4*kg + i, 16-byte chunk ln
};

// One unit, checked: where it starts in the pools (element offset) and how many of its tokens
// count (0 = nothing to read).
struct Entry {
  size_t elem_off;
  int valid;
};

// sel / slot_list point at the pair's list (global memory or LDS); u is wave-uniform.
__device__ __forceinline__ Entry read_entry(const int32_t* sel, const int32_t* slot_list, int u, int u_end,
                                            int ush, int S, int ctx, long long n_slots, int tile_stride) {
  Entry e{0, 0};
  if (u < u_end) {
    const int i = u >> ush, sub = u - (i << ush);  // ush = log2(units per block)
    const int j = __builtin_amdgcn_readfirstlane(sel[i]);
    const long long slot = __builtin_amdgcn_readfirstlane(slot_list[i]);
    int valid = ctx - j * S - sub * kUnitTokens;
    valid = valid > kUnitTokens ? kUnitTokens : valid;
    if (j >= 0 && valid > 0 && slot >= 0 && slot < n_slots) {
      e.elem_off = (size_t)slot * tile_stride + sub * kUnitTokens * kMfmaD;
      e.valid = valid;
    }
  }
  return e;
}

// Request a unit.  The loads go through a buffer descriptor that covers exactly the unit, or nothing
// when the entry is void: then every lane gets zeros without touching memory.  That keeps the issue
// path free of branches, so the compiler can count outstanding loads exactly and a wave can wait for
// one unit while the next ones are still in flight.
__device__ __forceinline__ void issue_unit(UnitRegs& T, const uint16_t* __restrict__ k_pool,
                                           const uint16_t* __restrict__ v_pool, const Entry& e, int ln,
                                           int kg) {
  const int bytes = e.valid > 0 ? kUnitBytes : 0;
  const __amdgpu_buffer_rsrc_t kr =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(k_pool + e.elem_off), 0, bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t vr =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(v_pool + e.elem_off), 0, bytes, 0x00020000);
  const int koff = ln * 256 + kg * 16;   // row ln, 16-byte chunk 4*s + kg
  const int voff = kg * 1024 + ln * 16;  // row 4*kg + i, chunk ln
#pragma unroll
  for (int s = 0; s < 4; ++s)
    T.k[s] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(kr, koff + s * 64, 0, 0));
#pragma unroll
  for (int i = 0; i < 4; ++i)
    T.v[i] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(vr, voff + i * 256, 0, 0));
}

// Online-softmax state of one wave: head ln, channels 8*(4*kg + i) + r in acc[r][i].
struct WaveState {
  f32x4 acc[8];
  float m, l;
};

// Fold one unit into the wave's state.  `valid` tokens of the unit count (0: the unit is void and
// leaves the state as it is), so this too runs without a data-dependent branch around loads.
__device__ __forceinline__ void consume_unit(WaveState& W, UnitRegs& T, const u32x4 (&qreg)[4], int valid,
                                             float scale2, int kg) {
  f32x4 st = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < 4; ++s)
    st = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(T.k[s]), as_bf16x8(qreg[s]), st, 0, 0, 0);
  // st[i] = logit of head ln, token 4*kg + i
  float x[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) x[i] = st[i] * scale2;
  if (valid < kUnitTokens) {  // wave-uniform and rare: a void unit, or the partly filled last block
                              // of a sequence; tokens beyond `valid` are dropped, their value rows zeroed
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (4 * kg + i >= valid) {
        x[i] = -INFINITY;
        T.v[i] = (u32x4){0, 0, 0, 0};
      }
    }
  }
  float bm = fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3]));
  bm = max_xor32(max_xor16(bm));  // over the four lanes that share the head
  const float m_new = fmaxf(W.m, bm);
  const float m_sub = m_new == -INFINITY ? 0.0f : m_new;  // nothing seen yet: weights are 2^-inf = 0
  float p[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) p[i] = fast_exp2(x[i] - m_sub);
  if (__ballot(m_new != W.m) != 0) {  // some head's maximum moved: rescale what has been gathered
    const float alpha = exp2_diff(W.m, m_new);
    W.l *= alpha;
#pragma unroll
    for (int r = 0; r < 8; ++r) W.acc[r] *= alpha;
    W.m = m_new;
  }
  // weights go into the second product as bf16; sum what is actually used
  const uint32_t p01 = cvt_pk_bf16(p[0], p[1]), p23 = cvt_pk_bf16(p[2], p[3]);
  W.l += (bf16_lo(p01) + bf16_hi(p01)) + (bf16_lo(p23) + bf16_hi(p23));
  const s16x4 preg = __builtin_bit_cast(s16x4, (uint2){p01, p23});
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const uint32_t a01 = pack_halves(T.v[0][r >> 1], T.v[1][r >> 1], r & 1);
    const uint32_t a23 = pack_halves(T.v[2][r >> 1], T.v[3][r >> 1], r & 1);
    W.acc[r] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, (uint2){a01, a23}), preg,
                                                         W.acc[r], 0, 0, 0);
  }
}

// B operand of the first product: Q^T, column = head ln, zero beyond G
__device__ __forceinline__ void load_q(u32x4 (&qreg)[4], const Dims& D, const uint16_t* __restrict__ q, int b,
                                       int g, int ln, int kg) {
  const int G = D.G;
  const int hsafe = ln < G ? ln : G - 1;
  const uint16_t* qrow = q + ((size_t)b * D.Hq + g * G + hsafe) * kMfmaD + kg * 8;
#pragma unroll
  for (int s = 0; s < 4; ++s) qreg[s] = *reinterpret_cast<const u32x4*>(qrow + s * 32);
  const uint32_t keep = ln < G ? 0xffffffffu : 0u;
#pragma unroll
  for (int s = 0; s < 4; ++s) qreg[s] &= keep;
}

// The attention of one workgroup: its share (split) of the pair's list, folded over the waves
// through LDS, then the epilogue.  sel / slot_list: the pair's list in global memory or LDS.
// PRIVATE: the wave holds its own list entries in registers instead (lane j: the entry of the wave's
// j-th unit, units dealt to the pair's waves in stride: v, v + waves, ...), fetched by the wave
// itself in the same trip as the count: no staging through LDS and no barrier before the first tile
// request.  At most 64 units per wave; sel / slot_list are not read.
template <int WAVES, int DEPTH, bool PRIVATE = false>
__device__ __forceinline__ void attend_pair(const Dims& D, int b, int g, int split, const u32x4 (&qreg)[4],
                                            const uint16_t* __restrict__ k_pool,
                                            const uint16_t* __restrict__ v_pool, long long n_slots,
                                            const int32_t* sel, const int32_t* slot_list, int n, int ctx,
                                            const Partials& P, const Epilogue& E, float* smem, int my_sel = -1,
                                            int my_slot = -1) {
  // per wave: [G][132] floats of o (padded rows), then m[16], l[16]
  constexpr int ROW = kMfmaD + 4;
  const int pair = b * D.Hkv + g;
  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int ln = lane & 15, kg = lane >> 4;
  const int G = D.G;
  const int wstride = G * ROW + 32;  // floats of LDS per wave

  n = n < 0 ? 0 : (n > D.k ? D.k : n);
  if (n_slots <= 0) n = 0;
  // ctx (the sequence's length) is handed in: read here, after the caller's barrier and its stores, it
  // would be a fresh trip to memory in front of the first tile request
  const float scale2 = D.sm_scale * kLog2e;
  const int S = D.S, ush = D.s_shift - 4;  // a block is 2^ush units of 16 tokens

  // this wave's contiguous share of the pair's units: the first (units mod waves) waves take one unit
  // more than the others.  The quotient comes from a multiplication with a reciprocal made on the host
  // (at most 4096 units over at most 1024 waves: exact); an integer division here delays the first
  // tile request by a noticeable fraction of a microsecond.
  const int n_units = n << ush, n_waves = P.nsplit * WAVES, v = split * WAVES + wave;
  const int per = P.waves_magic ? (int)__umulhi((uint32_t)n_units, P.waves_magic) : n_units;
  const int extra = n_units - per * n_waves;
  const int u0 = v * per + (v < extra ? v : extra);
  const int u1 = u0 + per + (v < extra ? 1 : 0);

  WaveState W;
#pragma unroll
  for (int r = 0; r < 8; ++r) W.acc[r] = (f32x4){0.f, 0.f, 0.f, 0.f};
  W.m = -INFINITY;
  W.l = 0.0f;

  // DEPTH units are kept in flight per wave: the loads of the next ones are issued before a unit is
  // consumed.  Measured at the benchmark shapes, one unit in flight per wave with eight waves per
  // workgroup (64 KiB requested per compute unit at any time) beats two, three and four (17.0, 17.4,
  // 17.7 and 19.0 us for 64.5 MiB of tiles).
  if constexpr (PRIVATE) {
    static_assert(DEPTH == 1, "one unit in flight");
    // unit v + j * n_waves of the pair is this wave's j-th; its list entry sits in lane j
    auto entry = [&](int j, int u) {
      Entry e{0, 0};
      if (u < n_units) {
        const int bj = __builtin_amdgcn_readlane(my_sel, j);
        const long long slot = __builtin_amdgcn_readlane(my_slot, j);
        const int sub = u & ((1 << ush) - 1);
        int valid = ctx - bj * S - sub * kUnitTokens;
        valid = valid > kUnitTokens ? kUnitTokens : valid;
        if (bj >= 0 && valid > 0 && slot >= 0 && slot < n_slots) {
          e.elem_off = (size_t)slot * D.tile_stride + sub * kUnitTokens * kMfmaD;
          e.valid = valid;
        }
      }
      return e;
    };
    UnitRegs b0;
    Entry e0 = entry(0, v);
    issue_unit(b0, k_pool, v_pool, e0, ln, kg);
    int j = 0;
    for (int u = v; u < n_units; u += n_waves) {
      ++j;
      const Entry nx = entry(j, u + n_waves);
      consume_unit(W, b0, qreg, e0.valid, scale2, kg);
      e0 = nx;
      issue_unit(b0, k_pool, v_pool, nx, ln, kg);
    }
  } else {
    UnitRegs buf[DEPTH];
    Entry ent[DEPTH];
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      ent[d] = read_entry(sel, slot_list, u0 + d, u1, ush, S, ctx, n_slots, D.tile_stride);
      issue_unit(buf[d], k_pool, v_pool, ent[d], ln, kg);
    }
    for (int u = u0; u < u1; u += DEPTH) {
#pragma unroll
      for (int d = 0; d < DEPTH; ++d) {
        const Entry nx = read_entry(sel, slot_list, u + d + DEPTH, u1, ush, S, ctx, n_slots, D.tile_stride);
        consume_unit(W, buf[d], qreg, ent[d].valid, scale2, kg);
        ent[d] = nx;
        issue_unit(buf[d], k_pool, v_pool, nx, ln, kg);
      }
    }
  }
  f32x4(&acc)[8] = W.acc;
  float m_run = W.m, l_run = W.l;

  // lanes kg = 0..3 of a head saw disjoint tokens under a common maximum
  l_run = sum_xor32(sum_xor16(l_run));

  // the host's partial for the outputs this thread will finish: requested now, used after the fold
  constexpr int kOutPerThread = 16 * kMfmaD / (WAVES * kWave);
  HostPart hp[kOutPerThread];
#pragma unroll
  for (int t = 0; t < kOutPerThread; ++t) {
    const int idx = threadIdx.x + t * WAVES * kWave;
    const int hh = idx < G * kMfmaD ? idx / kMfmaD : 0;
    hp[t] = load_host(D, E, b * D.Hq + g * G + hh, idx % kMfmaD);
  }

  // fold the waves of the workgroup through LDS
  float* wo = smem + (size_t)wave * wstride;
  float* wm = wo + G * ROW;
  float* wl = wm + 16;
  if (ln < G) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      // acc[r][i]: channel 8*(4*kg + i) + r
      float* dst = wo + ln * ROW + 8 * (4 * kg + i);
      *reinterpret_cast<float4*>(dst) = make_float4(acc[0][i], acc[1][i], acc[2][i], acc[3][i]);
      *reinterpret_cast<float4*>(dst + 4) = make_float4(acc[4][i], acc[5][i], acc[6][i], acc[7][i]);
    }
    if (kg == 0) {
      wm[ln] = m_run;
      wl[ln] = l_run;
    }
  }
  __syncthreads();
  const size_t pbase = (size_t)pair * P.nsplit + split;
  if (E.mode == 0) {
    // partial of this split: four channels per thread, 16-byte LDS reads and one 16-byte store
    for (int item = threadIdx.x; item < G * (kMfmaD / 4); item += WAVES * kWave) {
      const int h = item / (kMfmaD / 4), c = (item % (kMfmaD / 4)) * 4;
      float mw[WAVES];
      float M = -INFINITY;
#pragma unroll
      for (int w = 0; w < WAVES; ++w) {
        mw[w] = smem[(size_t)w * wstride + G * ROW + h];
        M = fmaxf(M, mw[w]);
      }
      float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
      float l = 0.0f;
#pragma unroll
      for (int w = 0; w < WAVES; ++w) {
        const float* base = smem + (size_t)w * wstride;
        const float f = exp2_diff(mw[w], M);
        const float4 x = *reinterpret_cast<const float4*>(base + h * ROW + c);
        o.x += f * x.x; o.y += f * x.y; o.z += f * x.z; o.w += f * x.w;
        l += f * base[G * ROW + 16 + h];
      }
      *reinterpret_cast<float4*>(P.o + (pbase * G + h) * kMfmaD + c) = o;
      if (c == 0) {
        P.m[pbase * G + h] = M;
        P.l[pbase * G + h] = l;
      }
    }
    return;
  }
#pragma unroll
  for (int t = 0; t < kOutPerThread; ++t) {
    const int idx = threadIdx.x + t * WAVES * kWave;
    if (idx >= G * kMfmaD) break;
    const int h = idx / kMfmaD, c = idx % kMfmaD;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) M = fmaxf(M, smem[(size_t)w * wstride + G * ROW + h]);
    float o = 0.0f, l = 0.0f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      const float* base = smem + (size_t)w * wstride;
      const float f = exp2_diff(base[G * ROW + h], M);
      o += f * base[h * ROW + c];
      l += f * base[G * ROW + 16 + h];
    }
    if (E.mode == 0) {
      P.o[(pbase * G + h) * kMfmaD + c] = o;
      if (c == 0) {
        P.m[pbase * G + h] = M;
        P.l[pbase * G + h] = l;
      }
    } else {
      finish(D, E, b * D.Hq + g * G + h, c, o, l, M, hp[t]);
    }
  }
}

// Which (sequence, KV head, pair, split) a workgroup of the attention kernels works on.  Normally the grid
// is (splits, KV heads, sequences).  With a selection per query head and one workgroup per head, the launcher
// asks for a grid of one dimension instead (REMAP, a kernel instance of its own so that the usual path keeps its
// short head): the heads of a KV head choose overlapping blocks,
// so they get workgroup ids 8 apart, which the dispatcher hands to the same XCD one after the other: what one
// head reads from memory the others find in that XCD's L2 (a layer-step with per-head selection at config 3's
// shape: 96 us instead of 111 us).
template <bool REMAP>
__device__ __forceinline__ void which_pair(const Dims& D, int& b, int& g, int& pair, int& split) {
  b = blockIdx.z;
  g = blockIdx.y;
  pair = grid_pair();
  split = blockIdx.x;
  if constexpr (REMAP) {
    const int L = blockIdx.x, t = L >> 3;
    const int row = ((t / D.share) << 3) | (L & 7);  // the KV head's row; its heads are t % share
    pair = row * D.share + t % D.share;
    b = pair / D.Hkv;
    g = pair - b * D.Hkv;
    split = 0;
  }
}

// True, and the grid to launch, if the pairs that share a row can be placed on one XCD (see which_pair).
static bool xcd_grid(const Dims& D, int nsplit, dim3& grid) {
  const int pairs = D.B * D.Hkv;
  if (D.share > 1 && nsplit == 1 && (pairs / D.share) % 8 == 0) {
    grid = dim3(pairs, 1, 1);
    return true;
  }
  return false;
}

template <int WAVES, int DEPTH>
__global__ __launch_bounds__(WAVES* kWave) void attn_mfma_kernel(
    Dims D, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k_pool,
    const uint16_t* __restrict__ v_pool, long long n_slots, const int32_t* __restrict__ sel_gpu,
    const int32_t* __restrict__ slot_gpu, const int32_t* __restrict__ n_gpu, Partials P, Epilogue E) {
  extern __shared__ float smem[];
  int b, g, pair, split;
  which_pair<false>(D, b, g, pair, split);
  const int lane = lane_id();
  // The pair's whole list is copied to LDS by all threads at once, in the same round trip that
  // brings the count and the queries: which entries a wave needs depends on the count, and a
  // second, dependent trip to memory would cost more than the few hundred bytes read in vain.
  int* l_sel = reinterpret_cast<int*>(smem + WAVES * (D.G * (kMfmaD + 4) + 32));
  int* l_slot = l_sel + D.k;
  const size_t list0 = (size_t)pair * D.k;
  const int n = n_gpu[pair];
  const int ctx = D.ctx_len[b];
  for (int t = threadIdx.x; t < D.k; t += WAVES * kWave) {
    l_sel[t] = sel_gpu[list0 + t];
    l_slot[t] = slot_gpu[list0 + t];
  }
  u32x4 qreg[4];
  load_q(qreg, D, q, b, g, lane & 15, lane >> 4);
  __syncthreads();
  attend_pair<WAVES, DEPTH>(D, b, g, split, qreg, k_pool, v_pool, n_slots, l_sel, l_slot, n, ctx, P, E, smem);
}

// The same attention with the list entries fetched by the waves themselves (see attend_pair, PRIVATE):
// used when no wave can have more than 64 units.  Without the staging of the list through LDS and its
// barrier the first tile request leaves one trip to memory after the wave started: 16.4 us against
// 17.0 us for config 3's 64.5 MiB of tiles (config 2: 10.4 against 10.9, config 5: 30.0 against 30.6).
template <int WAVES, bool REMAP>
__global__ __launch_bounds__(WAVES* kWave) void attn_mfma_private_kernel(
    Dims D, const uint16_t* __restrict__ q, const uint16_t* __restrict__ k_pool,
    const uint16_t* __restrict__ v_pool, long long n_slots, const int32_t* __restrict__ sel_gpu,
    const int32_t* __restrict__ slot_gpu, const int32_t* __restrict__ n_gpu, Partials P, Epilogue E) {
  extern __shared__ float smem[];
  int b, g, pair, split;
  which_pair<REMAP>(D, b, g, pair, split);
  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const size_t list0 = (size_t)pair * D.k;
  const int n_waves = P.nsplit * WAVES, v = split * WAVES + wave;
  const int e = (v + lane * n_waves) >> (D.s_shift - 4);  // the block of this wave's unit number `lane`
  int my_sel = -1, my_slot = -1;
  if (e < D.k) {
    my_sel = sel_gpu[list0 + e];
    my_slot = slot_gpu[list0 + e];
  }
  const int n = n_gpu[pair];
  const int ctx = D.ctx_len[b];
  u32x4 qreg[4];
  load_q(qreg, D, q, b, g, lane & 15, lane >> 4);
  attend_pair<WAVES, 1, true>(D, b, g, split, qreg, k_pool, v_pool, n_slots, nullptr, nullptr, n, ctx, P, E, smem,
                              my_sel, my_slot);
}

// A hint from the lists as the caller left them (in a decode loop: the previous step's lists of this
// layer; adjacent decode tokens attend to highly overlapping sets of blocks, Sec. 1).  While the waves of
// a workgroup select, they ask memory for nothing; the unit a wave would start with under the old lists
// is touched just before, one dword of every 64 bytes, so that its rows are on their way from HBM into
// the caches meanwhile (one unit per wave is what memory delivers in that time: touching two measured
// no gain).  A hint is only ever a slot number inside [0, n_slots): whatever the arrays hold, the touch
// stays inside the pools, and its value is never used.  Budgets above 128 blocks take no hint.  (Not in
// step_kernel: its workgroups are at different stages at any time, memory is never idle there, and the
// touch measured no gain: 65.5 against 65.2 us at 256 ragged pairs.)
struct Hint {
  int n_old, s_lo, s_hi;  // the old count; lane l: old slot entries l and 64 + l
};

// Requested in the same trip as whatever else the kernel asks for first.
__device__ __forceinline__ Hint load_hint(const Dims& D, int pair, int lane, const int32_t* slot_gpu,
                                          const int32_t* n_gpu) {
  Hint h{0, -1, -1};
  if (D.k <= 2 * kWave) {
    const size_t row = (size_t)pair * D.k;
    h.n_old = n_gpu[pair];
    h.s_lo = slot_gpu[row + (lane < D.k ? lane : D.k - 1)];
    h.s_hi = slot_gpu[row + (kWave + lane < D.k ? kWave + lane : D.k - 1)];
  }
  return h;
}

// Wave v of the pair's P.nsplit * WAVES waves touches the first unit of its share of the old list.  To be
// issued when the loads whose values are needed next have returned (a wave's loads return in the order
// they were issued, and a touch takes a loaded memory system's full latency).  The touch goes through a
// buffer descriptor that covers the unit, or nothing: no branch, so nothing ever waits for its value.
// The caller keeps tk and tv alive (an empty asm that names them) until its own later loads have returned.
template <int WAVES>
__device__ __forceinline__ void touch_hint(const Dims& D, const Hint& h, const Partials& P, int v, int lane,
                                           const uint16_t* k_pool, const uint16_t* v_pool, long long n_slots,
                                           uint32_t& tk, uint32_t& tv) {
  int n = __builtin_amdgcn_readfirstlane(h.n_old);
  n = n < 0 ? 0 : (n > D.k ? D.k : n);
  const int ush = D.s_shift - 4;
  const int n_units = D.k <= 2 * kWave ? n << ush : 0;
  const int per = P.waves_magic ? (int)__umulhi((uint32_t)n_units, P.waves_magic) : n_units;
  const int extra = n_units - per * (P.nsplit * WAVES);
  const int u0 = v * per + (v < extra ? v : extra);  // the first unit of this wave's share of the old list
  const int uc = u0 < n_units ? u0 : 0;
  const int e = uc >> ush, sub = uc & ((1 << ush) - 1);
  long long slot = e < kWave ? __builtin_amdgcn_readlane(h.s_lo, e & (kWave - 1))
                             : __builtin_amdgcn_readlane(h.s_hi, e & (kWave - 1));
  const bool ok = u0 < n_units && slot >= 0 && slot < n_slots;
  slot = ok ? slot : 0;
  const size_t off = (size_t)slot * D.tile_stride + sub * kUnitTokens * kMfmaD;
  const int bytes = ok ? kUnitBytes : 0;
  const __amdgpu_buffer_rsrc_t kr =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(k_pool + off), 0, bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t vr =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(v_pool + off), 0, bytes, 0x00020000);
  tk = __builtin_amdgcn_raw_buffer_load_b32(kr, lane * 64, 0, 0);  // one dword of every 64 bytes of the unit
  tv = __builtin_amdgcn_raw_buffer_load_b32(vr, lane * 64, 0, 0);
}

// Selection and attention of a pair in one launch (the non-pipelined description of Sec. 3.2:
// identify the top-k blocks, then attend to the resident ones).  Every workgroup of the pair
// repeats the cheap selection from the scores (integer work on a few KiB of keys), keeps the
// resident list in LDS and goes straight on to its share of the units; split 0 also writes the
// lists out, because the host needs to know which selected blocks are its own.
// SEL_WAVES = 8: all waves share the keys and exchange counts through LDS; SEL_WAVES = 1: one wave
// holds all keys and selects without a barrier while the others wait (kept for comparison).
template <int SEL_WAVES, int KPL, bool REMAP>
__global__ __launch_bounds__(8 * kWave) void select_attend_kernel(
    Dims D, const uint16_t* __restrict__ q, const float* __restrict__ scores,
    const int32_t* __restrict__ table, const uint16_t* __restrict__ k_pool,
    const uint16_t* __restrict__ v_pool, long long n_slots, int32_t* __restrict__ sel_all,
    int32_t* __restrict__ sel_gpu, int32_t* __restrict__ slot_gpu, int32_t* __restrict__ n_gpu,
    int32_t* __restrict__ sel_host, int32_t* __restrict__ n_host, Partials P, Epilogue E) {
  constexpr int WAVES = 8;
  extern __shared__ float smem[];
  int b, g, pair, split;
  which_pair<REMAP>(D, b, g, pair, split);
  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  // LDS after the fold area: resident list (block, slot), the selector's exchange words, the count
  const int kpad = (D.k + 3) & ~3;  // keeps what follows 16-byte aligned
  int* l_sel = reinterpret_cast<int*>(smem + WAVES * (D.G * (kMfmaD + 4) + 32));
  int* l_slot = l_sel + kpad;
  int* l_x = l_slot + kpad;
  int* l_n = l_x + selector_lds_ints<WAVES>();

  u32x4 qreg[4];
  load_q(qreg, D, q, b, g, lane & 15, lane >> 4);
  const int ctx = D.ctx_len[b];  // once, here: the attention below must not wait for it again

  const Hint hint = load_hint(D, pair, lane, slot_gpu, n_gpu);
  uint32_t touched_k = 0, touched_v = 0;

  if (SEL_WAVES == WAVES || wave == 0) {  // wave-uniform
    const int sw = SEL_WAVES == WAVES ? wave : 0;
    int nb = (ctx < 0 ? 0 : ctx + D.S - 1) >> D.s_shift;
    nb = nb < D.max_blocks ? nb : D.max_blocks;
    const int k_eff = D.k < nb ? D.k : nb;
    uint32_t key[KPL];
    int slot[KPL];
    load_keys<SEL_WAVES, KPL>(D, scores, table, pair, nb, sw, lane, key, slot);
    __builtin_amdgcn_sched_barrier(0);
    touch_hint<WAVES>(D, hint, P, split * WAVES + wave, lane, k_pool, v_pool, n_slots, touched_k, touched_v);
    __builtin_amdgcn_sched_barrier(0);
    Selector<SEL_WAVES, KPL> S{l_x, 0, sw};
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
    const bool writer = split == 0;
#pragma unroll
    for (int r = 0; r < KPL; ++r) {
      if ((sel >> r) & 1u) {
        const int i = (sw * KPL + r) * kWave + lane;
        if (writer) sel_all[out0 + pos_all[r]] = i;
        if ((gpu >> r) & 1u) {
          l_sel[pos_gpu[r]] = i;
          l_slot[pos_gpu[r]] = slot[r];
          if (writer) {
            sel_gpu[out0 + pos_gpu[r]] = i;
            slot_gpu[out0 + pos_gpu[r]] = slot[r];
          }
        } else if (writer) {
          sel_host[out0 + pos_all[r] - pos_gpu[r]] = i;
        }
      }
    }
    const int tid = sw * kWave + lane;
    if (writer) {
      for (int t = tid; t < D.k; t += SEL_WAVES * kWave) {
        if (t >= k_eff) sel_all[out0 + t] = -1;
        if (t >= ng) {
          sel_gpu[out0 + t] = -1;
          slot_gpu[out0 + t] = -1;
        }
        if (t >= nh) sel_host[out0 + t] = -1;
      }
      if (tid == 0) {
        n_gpu[pair] = ng;
        n_host[pair] = nh;
      }
    }
    if (tid == 0) l_n[0] = ng;
  }
  __syncthreads();
  attend_pair<WAVES, 1>(D, b, g, split, qreg, k_pool, v_pool, n_slots, l_sel, l_slot, l_n[0], ctx, P, E, smem);
  asm volatile("" ::"v"(touched_k), "v"(touched_v));  // the touches stay loads, their registers reserved until they have returned
}

// The whole layer-step of a pair in one launch (the non-pipelined sequence of Sec. 3.2: score every
// block against its digest, keep the top-k, attend to the resident ones, merge with the host's
// partial), for launches in which the pairs alone fill the chip (one workgroup per pair, nothing to
// combine afterwards).  The workgroup streams the pair's digest rows, keeps the scores as selection
// keys in LDS (they go to global memory only if the caller wants them), selects, and goes on to the
// attention without a second launch or a trip of the scores through HBM.  bf16, d = 128, min/max
// digests, the group's heads summed.
//
// Scoring repeats score_kernel's arithmetic operation for operation (the same stream layout, the same
// order of the binary64 FMAs, the same three exchange steps), so a score has the same bits whichever
// kernel made it.  A wave keeps one batch of 16 blocks (8 KiB) in flight, the next requested as soon
// as one is scored (two or four in flight measured the same: 62.8, 62.0 against 62.2 us at batch 32).
constexpr int kStepBatch = 8;         // wave-wide loads per batch: 16 blocks
constexpr int kStepEntryBytes = 512;  // one digest entry: min row and max row of 128 bf16

template <int KPL>
__global__ __launch_bounds__(8 * kWave) void step_kernel(
    Dims D, const uint16_t* q, const char* digest, const int32_t* __restrict__ table,
    const uint16_t* __restrict__ k_pool, const uint16_t* __restrict__ v_pool, long long n_slots,
    float* scores, int32_t* __restrict__ sel_all, int32_t* __restrict__ sel_gpu,
    int32_t* __restrict__ slot_gpu, int32_t* __restrict__ n_gpu, int32_t* __restrict__ sel_host,
    int32_t* __restrict__ n_host, Partials P, Epilogue E) {
  constexpr int WAVES = 8;
  extern __shared__ float smem[];
  const int b = blockIdx.z, g = blockIdx.y, pair = grid_pair();
  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int kpad = (D.k + 3) & ~3;
  int* l_sel = reinterpret_cast<int*>(smem + WAVES * (D.G * (kMfmaD + 4) + 32));
  int* l_slot = l_sel + kpad;
  int* l_x = l_slot + kpad;
  int* l_n = l_x + selector_lds_ints<WAVES>();
  uint32_t* l_key = reinterpret_cast<uint32_t*>(l_n + 4);                       // [WAVES * 64 * KPL]
  double* coef_lds = reinterpret_cast<double*>(l_key + WAVES * kWave * KPL);    // [2][128]: N_c, P_c

  // table entries of the elements this thread will hold in the selection: requested first, used last
  const size_t trow = (size_t)kv_row(D, pair) * D.max_blocks;
  int slot[KPL];
#pragma unroll
  for (int r = 0; r < KPL; ++r) {
    const int i = (wave * KPL + r) * kWave + lane;
    slot[r] = table[trow + (i < D.max_blocks ? i : D.max_blocks - 1)];
  }
  // the group's queries: thread t < 256 folds channel t % 128, negative (t < 128) or positive parts
  const int fc = threadIdx.x & (kMfmaD - 1);
  const bool fpos = threadIdx.x >= kMfmaD;
  const uint16_t* qbase = q + ((size_t)b * D.Hq + g * D.G) * kMfmaD + fc;
  float qv[16];
  if (threadIdx.x < 2 * kMfmaD) {
#pragma unroll
    for (int h = 0; h < 16; ++h) qv[h] = bf16_bits_to_f32(qbase[(size_t)(h < D.G ? h : D.G - 1) * kMfmaD]);
  }
  const int ctx = D.ctx_len[b];
  int nb = (ctx < 0 ? 0 : ctx + D.S - 1) >> D.s_shift;
  nb = nb < D.max_blocks ? nb : D.max_blocks;

  const char* dpair = digest + trow * kStepEntryBytes;
  const __amdgpu_buffer_rsrc_t rs =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(dpair), 0, nb * kStepEntryBytes, 0x00020000);
  const int n_batches = (nb + 15) >> 4;
  // byte offset of load `it` of the batch that starts at block j0: group it / 4, line it % 4 of its entries
  const int voff0 = (lane >> 3) * kStepEntryBytes + (lane & 7) * 16;
  auto load_batch = [&](u32x4(&dst)[kStepBatch], int batch) {
    const int base = batch < n_batches ? batch * 16 * kStepEntryBytes + voff0 : nb * kStepEntryBytes;  // beyond: reads zeros
#pragma unroll
    for (int it = 0; it < kStepBatch; ++it)
      dst[it] = __builtin_bit_cast(
          u32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, base + (it >> 2) * 8 * kStepEntryBytes + (it & 3) * 128, 0, 0));
  };
  u32x4 raw[kStepBatch];
  load_batch(raw, wave);

  if (threadIdx.x < 2 * kMfmaD) {
    double f = 0.0;
#pragma unroll
    for (int h = 0; h < 16; ++h)
      if (h < D.G) f += (double)(fpos ? fmaxf(qv[h], 0.0f) : fminf(qv[h], 0.0f));
    coef_lds[(fpos ? kMfmaD : 0) + fc] = f;
  }
  // rows of the key array that no batch will write
  for (int i = n_batches * 16 + threadIdx.x; i < WAVES * kWave * KPL; i += WAVES * kWave) l_key[i] = 0u;
  __syncthreads();
  double coef[4][8];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int i = 0; i < 8; ++i) coef[u][i] = coef_lds[(u >= 2 ? kMfmaD : 0) + (u & 1) * 64 + (lane & 7) * 8 + i];

  const bool hi2 = (lane >> 2) & 1;
  const size_t srow = (size_t)pair * D.max_blocks;
  // scores of the 16 blocks of one batch from its eight loads; a batch beyond the last one holds zeros
  // and only marks rows beyond the sequence
  auto score_batch = [&](const u32x4(&cur)[kStepBatch], int batch) {
    double a[2];
#pragma unroll
    for (int gq = 0; gq < 2; ++gq) {
      double acc = 0.0;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const u32x4 w = cur[gq * 4 + u];
        acc = fma(coef[u][0], (double)bf16_lo(w[0]), acc);
        acc = fma(coef[u][1], (double)bf16_hi(w[0]), acc);
        acc = fma(coef[u][2], (double)bf16_lo(w[1]), acc);
        acc = fma(coef[u][3], (double)bf16_hi(w[1]), acc);
        acc = fma(coef[u][4], (double)bf16_lo(w[2]), acc);
        acc = fma(coef[u][5], (double)bf16_hi(w[2]), acc);
        acc = fma(coef[u][6], (double)bf16_lo(w[3]), acc);
        acc = fma(coef[u][7], (double)bf16_hi(w[3]), acc);
      }
      a[gq] = acc;
    }
    const double keep = hi2 ? a[1] : a[0], send = hi2 ? a[0] : a[1];
    double sc = keep + partner_f64<2>(send);
    sc += partner_f64<1>(sc);
    sc += partner_f64<0>(sc);
    const int j = batch * 16 + (hi2 ? 8 : 0) + (lane >> 3);
    if ((lane & 3) == 0) {
      const bool kept = j < D.n_sink || j >= nb - D.n_tail;  // always-kept blocks rank above every score
      const float val = j < nb ? (kept ? INFINITY : (float)sc) : -INFINITY;
      if (j < WAVES * kWave * KPL) l_key[j] = j < nb ? score_key(val) : 0u;
      if (scores != nullptr && j < D.max_blocks) scores[srow + j] = val;
    }
  };
  for (int batch = wave; batch < n_batches; batch += WAVES) {
    score_batch(raw, batch);
    load_batch(raw, batch + WAVES);
  }
  if (scores != nullptr)  // the row's tail beyond the last batch
    for (int j = n_batches * 16 + threadIdx.x; j < D.max_blocks; j += WAVES * kWave) scores[srow + j] = -INFINITY;

  u32x4 qreg[4];
  load_q(qreg, D, q, b, g, lane & 15, lane >> 4);
  __syncthreads();

  const int k_eff = D.k < nb ? D.k : nb;
  uint32_t key[KPL];
#pragma unroll
  for (int r = 0; r < KPL; ++r) {
    const int i = (wave * KPL + r) * kWave + lane;
    key[r] = l_key[i];  // 0 beyond nb
    slot[r] = i < nb ? slot[r] : -1;
  }
  Selector<WAVES, KPL> S{l_x, 0, wave};
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
        l_sel[pos_gpu[r]] = i;
        l_slot[pos_gpu[r]] = slot[r];
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
    l_n[0] = ng;
  }
  __syncthreads();
  attend_pair<WAVES, 1>(D, b, g, 0, qreg, k_pool, v_pool, n_slots, l_sel, l_slot, l_n[0], ctx, P, E, smem);
}

// ---------------------------------------------------------------- VALU family

constexpr int kValuHeads = 4;  // query heads per wave

// One wave per (pair, split, chunk of kValuHeads heads).  A token row is spread
// over LPT = DH/8 lanes (8 channels each); the 64/LPT lane groups take different
// tokens of a block and each keeps an online-softmax stream of its own, so the
// block loop needs no cross-group traffic; the streams are folded at the end.
template <int DT, int DH>
__global__ __launch_bounds__(kWave) void attn_valu_kernel(
    Dims D, const void* __restrict__ q, const void* __restrict__ k_pool,
    const void* __restrict__ v_pool, long long n_slots, const int32_t* __restrict__ sel_gpu,
    const int32_t* __restrict__ slot_gpu, const int32_t* __restrict__ n_gpu, Partials P) {
  constexpr int LPT = DH / 8;      // lanes per token
  constexpr int TPW = kWave / LPT; // tokens per wave pass
  const int pair = blockIdx.y, split = blockIdx.x, h0 = blockIdx.z * kValuHeads;
  const int b = pair / D.Hkv, g = pair % D.Hkv;
  const int lane = lane_id();
  const int tl = lane / LPT, c0 = (lane % LPT) * 8;
  const int G = D.G;
  const int nh = (G - h0) < kValuHeads ? (G - h0) : kValuHeads;

  int n = n_gpu[pair];
  n = n < 0 ? 0 : (n > D.k ? D.k : n);
  const int ctx = D.ctx_len[b];
  const float scale2 = D.sm_scale * kLog2e;

  float qv[kValuHeads][8];
#pragma unroll
  for (int h = 0; h < kValuHeads; ++h) {
    if (h < nh) {
      load8<DT>(q, ((size_t)b * D.Hq + g * G + h0 + h) * DH + c0, qv[h]);
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) qv[h][i] = 0.0f;
    }
  }
  float m_run[kValuHeads], l_run[kValuHeads], o[kValuHeads][8];
#pragma unroll
  for (int h = 0; h < kValuHeads; ++h) {
    m_run[h] = -INFINITY;
    l_run[h] = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[h][i] = 0.0f;
  }

  for (int i = split; i < n; i += P.nsplit) {
    const int j = sel_gpu[(size_t)pair * D.k + i];
    const long long slot = slot_gpu[(size_t)pair * D.k + i];
    int valid = ctx - j * D.S;
    valid = valid > D.S ? D.S : valid;
    if (j < 0 || valid <= 0 || slot < 0 || slot >= n_slots) continue;
    const size_t tile = (size_t)slot * D.tile_stride;
    for (int t0 = 0; t0 < D.S; t0 += TPW) {
      const int t = t0 + tl;
      const bool live = t < valid;
      float kx[8], vx[8];
      if (live) {
        load8<DT>(k_pool, tile + (size_t)t * DH + c0, kx);
        load8<DT>(v_pool, tile + (size_t)t * DH + c0, vx);
      } else {
#pragma unroll
        for (int c = 0; c < 8; ++c) kx[c] = vx[c] = 0.0f;
      }
#pragma unroll
      for (int h = 0; h < kValuHeads; ++h) {
        float dot = 0.0f;
#pragma unroll
        for (int c = 0; c < 8; ++c) dot = fmaf(qv[h][c], kx[c], dot);
#pragma unroll
        for (int off = 1; off < LPT; off <<= 1) dot += __shfl_xor(dot, off);
        if (live) {
          const float x = dot * scale2;
          const float m_new = fmaxf(m_run[h], x);
          const float a = exp2_diff(m_run[h], m_new);
          const float pw = exp2f(x - m_new);
          l_run[h] = l_run[h] * a + pw;
#pragma unroll
          for (int c = 0; c < 8; ++c) o[h][c] = fmaf(pw, vx[c], o[h][c] * a);
          m_run[h] = m_new;
        }
      }
    }
  }

  // fold the TPW token streams of the wave
#pragma unroll
  for (int h = 0; h < kValuHeads; ++h) {
#pragma unroll
    for (int off = LPT; off < kWave; off <<= 1) {
      const float m2 = __shfl_xor(m_run[h], off), l2 = __shfl_xor(l_run[h], off);
      const float M = fmaxf(m_run[h], m2);
      const float fa = exp2_diff(m_run[h], M), fb = exp2_diff(m2, M);
      l_run[h] = l_run[h] * fa + l2 * fb;
#pragma unroll
      for (int c = 0; c < 8; ++c) o[h][c] = o[h][c] * fa + __shfl_xor(o[h][c], off) * fb;
      m_run[h] = M;
    }
  }
  if (tl == 0) {
    const size_t pbase = (size_t)pair * P.nsplit + split;
#pragma unroll
    for (int h = 0; h < kValuHeads; ++h) {
      if (h < nh) {
        float* dst = P.o + (pbase * G + h0 + h) * DH + c0;
        *reinterpret_cast<float4*>(dst) = make_float4(o[h][0], o[h][1], o[h][2], o[h][3]);
        *reinterpret_cast<float4*>(dst + 4) = make_float4(o[h][4], o[h][5], o[h][6], o[h][7]);
        if (c0 == 0) {
          P.m[pbase * G + h0 + h] = m_run[h];
          P.l[pbase * G + h0 + h] = l_run[h];
        }
      }
    }
  }
}

// ------------------------------------------------------- combine and merge

// Fold the nsplit partials of every (sequence, query head), then export the GPU
// partial or go straight on to the merge with the host's partial (Epilogue modes
// 1 and 2).  One workgroup of d threads per head.
template <int GROUP>
__global__ void combine_kernel(Dims D, Partials P, Epilogue E) {
  // grid (G, Hkv, B): head within the group, KV head, sequence
  const int h = blockIdx.x;
  const int pair = grid_pair(), bh = pair * D.G + h;
  const int c = threadIdx.x;
  const size_t p0 = (size_t)pair * P.nsplit;
  const HostPart hp = load_host(D, E, bh, c);
  // one pass with a running maximum, GROUP splits at a time: every load of a group is independent
  // of the others, so a group costs one trip to memory (GROUP covers the split count where it can)
  float M = -INFINITY, acc = 0.0f, l = 0.0f;
  for (int s0 = 0; s0 < P.nsplit; s0 += GROUP) {
    float ms[GROUP], ls[GROUP], os[GROUP];
#pragma unroll
    for (int j = 0; j < GROUP; ++j) {
      const int sp = s0 + j < P.nsplit ? s0 + j : P.nsplit - 1;
      const size_t r = (p0 + sp) * D.G + h;
      ms[j] = P.m[r];
      ls[j] = P.l[r];
      os[j] = P.o[r * D.d + c];
    }
    float Mn = M;
#pragma unroll
    for (int j = 0; j < GROUP; ++j)
      if (s0 + j < P.nsplit) Mn = fmaxf(Mn, ms[j]);
    const float f0 = exp2_diff(M, Mn);
    acc *= f0;
    l *= f0;
#pragma unroll
    for (int j = 0; j < GROUP; ++j) {
      if (s0 + j < P.nsplit) {
        const float f = exp2_diff(ms[j], Mn);
        acc += f * os[j];
        l += f * ls[j];
      }
    }
    M = Mn;
  }
  finish(D, E, bh, c, acc, l, M, hp);
}

// Stand-alone merge of two partials given in natural-log units (Alg. 1 Merge).
template <int DT_OUT>
__global__ void merge_kernel(Dims D, const float* __restrict__ o_a, const float* __restrict__ m_a,
                             const float* __restrict__ l_a, const float* __restrict__ o_b,
                             const float* __restrict__ m_b, const float* __restrict__ l_b,
                             void* __restrict__ out, float* __restrict__ lse) {
  const int bh = blockIdx.x, c = threadIdx.x;
  const float ma = m_a[bh], la = l_a[bh];
  float mb = -INFINITY, lb = 0.0f, ob = 0.0f;
  if (o_b != nullptr) {
    mb = m_b[bh];
    lb = l_b[bh];
    ob = o_b[(size_t)bh * D.d + c];
  }
  float ms = -INFINITY;
  if (la > 0.0f) ms = fmaxf(ms, ma);
  if (lb > 0.0f) ms = fmaxf(ms, mb);
  const float wa = la > 0.0f ? la * expf(ma - ms) : 0.0f;
  const float wb = lb > 0.0f ? lb * expf(mb - ms) : 0.0f;
  const float ls = wa + wb;
  float r = 0.0f;
  if (wa > 0.0f) r += wa * o_a[(size_t)bh * D.d + c];
  if (wb > 0.0f) r += wb * ob;
  r = ls > 0.0f ? r / ls : 0.0f;
  if (DT_OUT == SCOUT_BF16)
    static_cast<uint16_t*>(out)[(size_t)bh * D.d + c] = (uint16_t)f32_to_bf16_bits(r);
  else
    static_cast<float*>(out)[(size_t)bh * D.d + c] = r;
  if (lse != nullptr && c == 0) lse[bh] = ls > 0.0f ? ms + logf(ls) : -INFINITY;
}

// ------------------------------------------------------------ host launchers

bool mfma_supported(const Dims& D, int dtype) {
  return dtype == SCOUT_BF16 && D.d == kMfmaD && D.S % kUnitTokens == 0 && D.G <= 16;
}

size_t mfma_smem_bytes(const Dims& D, int waves) {
  return (size_t)waves * (D.G * (kMfmaD + 4) + 32) * sizeof(float);
}

// family 2: MFMA kernel with `waves` waves per workgroup (8 or 16); family 1: vector ALU.
// E.mode != 0 requires P.nsplit == 1 and family 2 (the workgroup finishes the pair itself).
int launch_attn(const Dims& D, int dtype, int family, int waves, const void* q, const void* k_pool,
                const void* v_pool, long long n_slots, const int32_t* sel_gpu,
                const int32_t* slot_gpu, const int32_t* n_gpu, Partials P, Epilogue E, hipStream_t st) {
  const int pairs = D.B * D.Hkv;
  if (pairs == 0) return SCOUT_OK;
  if (family == 2) {
    dim3 grid(P.nsplit, D.Hkv, D.B), block(waves * kWave);
    const size_t lds = mfma_smem_bytes(D, waves) + 2 * (size_t)D.k * sizeof(int);
    const uint16_t* q16 = static_cast<const uint16_t*>(q);
    const uint16_t* k16 = static_cast<const uint16_t*>(k_pool);
    const uint16_t* v16 = static_cast<const uint16_t*>(v_pool);
#define SCOUT_ATTN(W, DP)                                                                               \
  hipLaunchKernelGGL((attn_mfma_kernel<W, DP>), grid, block, lds, st, D, q16, k16, v16, n_slots, sel_gpu, \
                     slot_gpu, n_gpu, P, E)
    // units in flight per wave: few.  Requests that only queue in the memory system buy nothing (a
    // compute unit's loads return in the order they were issued), and fewer registers leave room for
    // the next workgroup to start its head while this one folds.
    const long long units_per_wave = (((long long)D.k * (D.S / kUnitTokens)) + P.nsplit * waves - 1) / (P.nsplit * waves);
    if (waves == 16)
      SCOUT_ATTN(16, 1);
    else if (waves == 8 && units_per_wave <= 64 && xcd_grid(D, P.nsplit, grid))
      hipLaunchKernelGGL((attn_mfma_private_kernel<8, true>), grid, block, mfma_smem_bytes(D, 8), st, D, q16, k16, v16,
                         n_slots, sel_gpu, slot_gpu, n_gpu, P, E);
    else if (waves == 8 && units_per_wave <= 64)
      hipLaunchKernelGGL((attn_mfma_private_kernel<8, false>), grid, block, mfma_smem_bytes(D, 8), st, D, q16, k16, v16,
                         n_slots, sel_gpu, slot_gpu, n_gpu, P, E);
    else if (waves == 8)
      SCOUT_ATTN(8, 1);
    else if (waves == 4)
      SCOUT_ATTN(4, 2);
    else
      return SCOUT_EINVAL;
#undef SCOUT_ATTN
  } else {
    if (E.mode != 0) return SCOUT_EINVAL;
    dim3 grid(P.nsplit, pairs, (D.G + kValuHeads - 1) / kValuHeads), block(kWave);
    if (dtype == SCOUT_BF16 && D.d == 128)
      hipLaunchKernelGGL((attn_valu_kernel<SCOUT_BF16, 128>), grid, block, 0, st, D, q, k_pool, v_pool,
                         n_slots, sel_gpu, slot_gpu, n_gpu, P);
    else if (dtype == SCOUT_BF16 && D.d == 64)
      hipLaunchKernelGGL((attn_valu_kernel<SCOUT_BF16, 64>), grid, block, 0, st, D, q, k_pool, v_pool,
                         n_slots, sel_gpu, slot_gpu, n_gpu, P);
    else if (dtype == SCOUT_F32 && D.d == 128)
      hipLaunchKernelGGL((attn_valu_kernel<SCOUT_F32, 128>), grid, block, 0, st, D, q, k_pool, v_pool,
                         n_slots, sel_gpu, slot_gpu, n_gpu, P);
    else if (dtype == SCOUT_F32 && D.d == 64)
      hipLaunchKernelGGL((attn_valu_kernel<SCOUT_F32, 64>), grid, block, 0, st, D, q, k_pool, v_pool,
                         n_slots, sel_gpu, slot_gpu, n_gpu, P);
    else
      return SCOUT_EUNSUPPORTED;
  }
  return hipGetLastError() == hipSuccess ? SCOUT_OK : SCOUT_EHIP;
}

bool select_attend_supported(const Dims& D, int dtype) {
  return mfma_supported(D, dtype) && D.max_blocks <= 8 * kWave * 16;
}

// Selection fused into the head of the MFMA attention kernel (8 waves per workgroup).
int launch_select_attend(const Dims& D, const void* q, const float* scores, const int32_t* table,
                         const void* k_pool, const void* v_pool, long long n_slots, int32_t* sel_all,
                         int32_t* sel_gpu, int32_t* slot_gpu, int32_t* n_gpu, int32_t* sel_host,
                         int32_t* n_host, Partials P, Epilogue E, hipStream_t st) {
  const int pairs = D.B * D.Hkv;
  if (pairs == 0) return SCOUT_OK;
  dim3 grid(P.nsplit, D.Hkv, D.B), block(8 * kWave);
  const bool remap = xcd_grid(D, P.nsplit, grid);
  const size_t lds = mfma_smem_bytes(D, 8) + (2 * (size_t)((D.k + 3) & ~3) + selector_lds_ints<8>() + 4) * sizeof(int);
  const uint16_t* q16 = static_cast<const uint16_t*>(q);
  const uint16_t* k16 = static_cast<const uint16_t*>(k_pool);
  const uint16_t* v16 = static_cast<const uint16_t*>(v_pool);
#define SCOUT_SA(SW, KPL)                                                                                      \
  do {                                                                                                         \
    if (remap)                                                                                                 \
      hipLaunchKernelGGL((select_attend_kernel<SW, KPL, true>), grid, block, lds, st, D, q16, scores, table, k16, \
                         v16, n_slots, sel_all, sel_gpu, slot_gpu, n_gpu, sel_host, n_host, P, E);             \
    else                                                                                                       \
      hipLaunchKernelGGL((select_attend_kernel<SW, KPL, false>), grid, block, lds, st, D, q16, scores, table, k16, \
                         v16, n_slots, sel_all, sel_gpu, slot_gpu, n_gpu, sel_host, n_host, P, E);             \
  } while (0)
  // All eight waves share the keys: measured faster than one wave selecting alone while seven wait
  // (46.9 vs 44.1 us per step at 1024 blocks per pair), a lone wave issues too slowly.
  const int per_lane = (D.max_blocks + 8 * kWave - 1) / (8 * kWave);
  if (per_lane <= 2)
    SCOUT_SA(8, 2);
  else if (per_lane <= 4)
    SCOUT_SA(8, 4);
  else if (per_lane <= 8)
    SCOUT_SA(8, 8);
  else if (per_lane <= 16)
    SCOUT_SA(8, 16);
  else
    return SCOUT_EUNSUPPORTED;
#undef SCOUT_SA
  return hipGetLastError() == hipSuccess ? SCOUT_OK : SCOUT_EHIP;
}

// One workgroup streams its pair's whole digest row: worth it while a row is short enough that one
// long sequence among short ones cannot hold the launch up for long (2048 blocks = 1 MiB of digest).
bool step_kernel_supported(const Dims& D, int dtype) {
  // (with a selection per query head the scoring pass of its own serves the G heads of a row in one reading)
  return select_attend_supported(D, dtype) && D.digest_kind == 0 && D.group_max == 0 && D.share == 1 &&
         D.max_blocks <= 2048;
}

// Scoring, selection, attention and merge of every pair in one launch, one workgroup per pair
// (P.nsplit must be 1, E.mode 2).  `scores` may be null.
int launch_step(const Dims& D, const void* q, const void* digest, const int32_t* table, const void* k_pool,
                const void* v_pool, long long n_slots, float* scores, int32_t* sel_all, int32_t* sel_gpu,
                int32_t* slot_gpu, int32_t* n_gpu, int32_t* sel_host, int32_t* n_host, Partials P, Epilogue E,
                hipStream_t st) {
  if (D.B * D.Hkv == 0) return SCOUT_OK;
  if (P.nsplit != 1 || E.mode != 2) return SCOUT_EINVAL;
  dim3 grid(1, D.Hkv, D.B), block(8 * kWave);
  const int per_lane = (D.max_blocks + 8 * kWave - 1) / (8 * kWave);
  const int kpl = per_lane <= 2 ? 2 : per_lane <= 4 ? 4 : per_lane <= 8 ? 8 : 16;
  const size_t lds = mfma_smem_bytes(D, 8) +
                     (2 * (size_t)((D.k + 3) & ~3) + selector_lds_ints<8>() + 4 + 8 * kWave * kpl) * sizeof(int) +
                     2 * kMfmaD * sizeof(double);
  const uint16_t* q16 = static_cast<const uint16_t*>(q);
  const char* dg = static_cast<const char*>(digest);
  const uint16_t* k16 = static_cast<const uint16_t*>(k_pool);
  const uint16_t* v16 = static_cast<const uint16_t*>(v_pool);
#define SCOUT_STEP(KPL)                                                                                      \
  hipLaunchKernelGGL((step_kernel<KPL>), grid, block, lds, st, D, q16, dg, table, k16, v16, n_slots, scores, \
                     sel_all, sel_gpu, slot_gpu, n_gpu, sel_host, n_host, P, E)
  if (kpl == 2)
    SCOUT_STEP(2);
  else if (kpl == 4)
    SCOUT_STEP(4);
  else  // rows beyond 2048 blocks: see step_kernel_supported
    return SCOUT_EUNSUPPORTED;
#undef SCOUT_STEP
  return hipGetLastError() == hipSuccess ? SCOUT_OK : SCOUT_EHIP;
}

int launch_combine(const Dims& D, Partials P, Epilogue E, hipStream_t st) {
  dim3 grid(D.G, D.Hkv, D.B), block(D.d);
  if (grid.z == 0) return SCOUT_OK;
  if (P.nsplit <= 2)
    hipLaunchKernelGGL(combine_kernel<2>, grid, block, 0, st, D, P, E);
  else if (P.nsplit <= 4)
    hipLaunchKernelGGL(combine_kernel<4>, grid, block, 0, st, D, P, E);
  else
    hipLaunchKernelGGL(combine_kernel<8>, grid, block, 0, st, D, P, E);
  return hipGetLastError() == hipSuccess ? SCOUT_OK : SCOUT_EHIP;
}

int launch_merge(const Dims& D, int dtype_out, const float* o_a, const float* m_a, const float* l_a,
                 const float* o_b, const float* m_b, const float* l_b, void* out, float* lse,
                 hipStream_t st) {
  dim3 grid(D.B * D.Hq), block(D.d);
  if (grid.x == 0) return SCOUT_OK;
  if (dtype_out == SCOUT_BF16)
    hipLaunchKernelGGL(merge_kernel<SCOUT_BF16>, grid, block, 0, st, D, o_a, m_a, l_a, o_b, m_b, l_b, out,
                       lse);
  else
    hipLaunchKernelGGL(merge_kernel<SCOUT_F32>, grid, block, 0, st, D, o_a, m_a, l_a, o_b, m_b, l_b, out,
                       lse);
  return hipGetLastError() == hipSuccess ? SCOUT_OK : SCOUT_EHIP;
}

}  // namespace scout

// C ABI: argument validation, workspace carving, kernel-family choice.
// Nothing here computes; every step of the path runs in the kernels.
#include <hip/hip_runtime.h>

#include <cmath>
#include <mutex>

#include "common.h"

namespace scout {

int launch_digest(const Dims&, int, const void*, void*, hipStream_t);
int launch_score(const Dims&, int, const void*, const void*, float*, hipStream_t);
int launch_recall_fetch(const Dims&, int, const void*, const void*, const int32_t*, const int32_t*, const int32_t*,
                        void*, void*, long long, hipStream_t);
int launch_recall_scatter(const Dims&, int, const void*, long long, const int32_t*, const int32_t*, const int32_t*,
                          const int32_t*, void*, void*, long long, hipStream_t);
int launch_append(const Dims&, int, int32_t*, const void*, const void*, const int32_t*, void*, int32_t*, void*, void*,
                  long long, void*, void*, hipStream_t);
int launch_topk(const Dims&, const float*, const int32_t*, int32_t*, int32_t*, int32_t*, int32_t*,
                int32_t*, int32_t*, hipStream_t);
int launch_recall(const Dims&, const float*, int32_t*, int32_t*, int32_t*, int32_t*, int32_t*,
                  hipStream_t);
bool mfma_supported(const Dims&, int);
int launch_attn(const Dims&, int, int, int, const void*, const void*, const void*, long long,
                const int32_t*, const int32_t*, const int32_t*, Partials, Epilogue, hipStream_t);
int launch_combine(const Dims&, Partials, Epilogue, hipStream_t);
bool select_attend_supported(const Dims&, int);
int launch_select_attend(const Dims&, const void*, const float*, const int32_t*, const void*, const void*,
                         long long, int32_t*, int32_t*, int32_t*, int32_t*, int32_t*, int32_t*, Partials,
                         Epilogue, hipStream_t);
bool step_kernel_supported(const Dims&, int);
int launch_step(const Dims&, const void*, const void*, const int32_t*, const void*, const void*, long long, float*,
                int32_t*, int32_t*, int32_t*, int32_t*, int32_t*, int32_t*, Partials, Epilogue, hipStream_t);
int launch_merge(const Dims&, int, const float*, const float*, const float*, const float*,
                 const float*, const float*, void*, float*, hipStream_t);

constexpr int kMaxSplit = 64;
constexpr int kValuHeadsPerWave = 4;

static thread_local int g_family = 0;  // 0 auto, 1 vector ALU, 2 MFMA
static thread_local int g_nsplit = 0;  // 0 auto
static thread_local int g_waves = 0;   // 0 auto; MFMA family only
static thread_local int g_fuse_select = 1;  // scout_layer_step: selection inside the attention launch
static thread_local int g_fuse_step = 1;    // scout_layer_step: scoring too, where one workgroup per pair fills the chip

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static int check_problem(const scout_problem* p, Dims* D) {
  if (p == nullptr) return SCOUT_EINVAL;
  if (p->B < 0 || p->Hq <= 0 || p->Hkv <= 0 || p->Hq % p->Hkv != 0) return SCOUT_EINVAL;
  if (p->max_blocks < 1 || p->k < 1) return SCOUT_EINVAL;
  if (p->dtype != SCOUT_F32 && p->dtype != SCOUT_BF16) return SCOUT_EINVAL;
  if (!(p->sm_scale >= 0.0f) || std::isinf(p->sm_scale)) return SCOUT_EINVAL;
  if (p->n_sink < 0 || p->n_tail < 0 || (p->group_max != 0 && p->group_max != 1)) return SCOUT_EINVAL;
  if (p->per_head != 0 && p->per_head != 1) return SCOUT_EINVAL;
  if (p->digest_kind != 0 && p->digest_kind != 1) return SCOUT_EINVAL;
  if (p->digest_kind == 1 && p->group_max) return SCOUT_EUNSUPPORTED;
  if (p->ctx_len == nullptr) return SCOUT_EINVAL;
  if (p->d != 64 && p->d != 128) return SCOUT_EUNSUPPORTED;
  if (p->S != 16 && p->S != 32 && p->S != 64) return SCOUT_EUNSUPPORTED;
  if (p->Hq / p->Hkv > 16) return SCOUT_EUNSUPPORTED;
  if (p->max_blocks > 16384 || p->k > 1024) return SCOUT_EUNSUPPORTED;
  if ((long long)p->B * p->Hq > (1ll << 30)) return SCOUT_EUNSUPPORTED;
  D->B = p->B;
  D->Hq = p->Hq;
  D->Hkv = p->Hkv;
  D->G = p->Hq / p->Hkv;
  D->d = p->d;
  D->S = p->S;
  D->max_blocks = p->max_blocks;
  D->k = p->k;
  D->sm_scale = p->sm_scale > 0.0f ? p->sm_scale : 1.0f / std::sqrt((float)p->d);
  D->n_sink = p->n_sink;
  D->n_tail = p->n_tail;
  D->group_max = p->group_max;
  D->digest_kind = p->digest_kind;
  D->s_shift = p->S == 16 ? 4 : (p->S == 32 ? 5 : 6);
  if (p->tile_stride != 0 && (p->tile_stride < p->S * p->d || p->tile_stride % 8 != 0)) return SCOUT_EINVAL;
  D->tile_stride = p->tile_stride != 0 ? p->tile_stride : p->S * p->d;
  D->share = 1;
  D->share_magic = 0;
  if (p->per_head) {  // every query head is a pair of its own that reads its KV head's digest and table rows
    D->share = D->G;
    D->share_magic = D->G > 1 ? (uint32_t)(((1ull << 32) + D->G - 1) / D->G) : 0;
    D->Hkv = D->Hq;
    D->G = 1;
  }
  D->ctx_len = p->ctx_len;
  if ((long long)D->B * D->Hkv > 65535) return SCOUT_EUNSUPPORTED;  // pairs are the second grid dimension
  return SCOUT_OK;
}

// For the entry points that work on the cache itself (one row per KV head whatever the selection mode).
static int check_problem_kv(const scout_problem* p, Dims* D) {
  if (p == nullptr) return SCOUT_EINVAL;
  scout_problem kv = *p;
  if (kv.per_head != 0 && kv.per_head != 1) return SCOUT_EINVAL;
  kv.per_head = 0;
  return check_problem(&kv, D);
}

static size_t round256(size_t x) { return (x + 255) & ~(size_t)255; }

struct WsLayout {
  size_t part_o, part_m, part_l, scores, total;
};

static WsLayout ws_layout(const Dims& D) {
  const size_t pairs = (size_t)D.B * D.Hkv;
  WsLayout L;
  size_t at = 0;
  L.part_o = at;
  at += round256(pairs * kMaxSplit * D.G * D.d * sizeof(float));
  L.part_m = at;
  at += round256(pairs * kMaxSplit * D.G * sizeof(float));
  L.part_l = at;
  at += round256(pairs * kMaxSplit * D.G * sizeof(float));
  L.scores = at;
  at += round256(pairs * D.max_blocks * sizeof(float));
  L.total = at > 0 ? at : 256;
  return L;
}

static int check_ws(const Dims& D, void* ws, size_t ws_bytes, WsLayout* L) {
  *L = ws_layout(D);
  if (ws == nullptr || (reinterpret_cast<uintptr_t>(ws) & 255u) != 0 || ws_bytes < L->total)
    return SCOUT_EWORKSPACE;
  return SCOUT_OK;
}

// Which attention kernel family, how many splits per pair, how many waves per workgroup.
struct AttnPlan {
  int family, nsplit, waves;
};

static int plan_attn(const Dims& D, int dtype, AttnPlan* out) {
  int fam = g_family;
  if (fam == 0) fam = mfma_supported(D, dtype) ? 2 : 1;
  if (fam == 2 && !mfma_supported(D, dtype)) return SCOUT_EUNSUPPORTED;
  const long long pairs = (long long)D.B * D.Hkv;
  int ns = g_nsplit, waves = 1;
  if (fam == 2) {
    // Eight waves per workgroup, one 16-token unit in flight per wave.  A compute unit sustains
    // only a fraction of the HBM rate on its own, so the launch should cover all 256 of them: a
    // pair's units are split over ceil(256 / pairs) workgroups (folded by the small combine pass)
    // unless the pairs alone nearly fill the chip.
    waves = g_waves ? g_waves : 8;
    if (ns == 0) {
      if (pairs >= 192) {
        ns = 1;
      } else {
        long long want = (256 + pairs - 1) / (pairs > 0 ? pairs : 1);
        const long long cap = ((long long)D.k * (D.S / 16) + waves - 1) / waves;
        ns = (int)(want > cap ? cap : want);
      }
    }
  } else if (ns == 0) {
    const long long chunks = (D.G + kValuHeadsPerWave - 1) / kValuHeadsPerWave;
    long long want = (4096 + pairs * chunks - 1) / (pairs > 0 ? pairs * chunks : 1);
    ns = (int)(want > D.k ? D.k : want);
  }
  if (ns < 1) ns = 1;
  if (ns > kMaxSplit) ns = kMaxSplit;
  out->family = fam;
  out->nsplit = ns;
  out->waves = waves;
  return SCOUT_OK;
}

// ceil(2^32 / waves that share a pair) for the MFMA family's division of a pair's units; 0 if one wave
static uint32_t waves_magic(const AttnPlan& A) {
  const uint32_t n_waves = (uint32_t)A.nsplit * (uint32_t)A.waves;
  return n_waves > 1 ? (uint32_t)(((1ull << 32) + n_waves - 1) / n_waves) : 0;
}

static Partials carve(void* ws, const WsLayout& L, const AttnPlan& A) {
  char* base = static_cast<char*>(ws);
  return Partials{reinterpret_cast<float*>(base + L.part_o), reinterpret_cast<float*>(base + L.part_m),
                  reinterpret_cast<float*>(base + L.part_l), A.nsplit, waves_magic(A)};
}

// Attention over the listed blocks, then what E asks for.  One launch when a single MFMA workgroup
// covers a pair, otherwise the split pass followed by the combine pass.
static int run_attn(const Dims& D, int dtype, const AttnPlan& A, const void* q, const void* k_pool,
                    const void* v_pool, long long n_slots, const int32_t* sel_gpu,
                    const int32_t* slot_gpu, const int32_t* n_gpu, void* ws, const WsLayout& L,
                    Epilogue E, hipStream_t st) {
  Partials P = carve(ws, L, A);
  if (A.family == 2 && A.nsplit == 1)  // one workgroup per pair finishes the pair itself
    return launch_attn(D, dtype, 2, A.waves, q, k_pool, v_pool, n_slots, sel_gpu, slot_gpu, n_gpu, P, E, st);
  Epilogue part{};
  part.mode = 0;
  int rc = launch_attn(D, dtype, A.family, A.waves, q, k_pool, v_pool, n_slots, sel_gpu, slot_gpu, n_gpu, P,
                       part, st);
  if (rc != SCOUT_OK) return rc;
  return launch_combine(D, P, E, st);
}

// ---- sparse_decode_attn_static: the per-split partials in a buffer the library image holds itself.
//
// `scratch` is device memory that exists on every GPU the library's code object is loaded on, from
// then until the process ends.  In host code the NAME below is only a stand-in for the symbol: the
// address a kernel may use comes from hipGetSymbolAddress, per device (each GPU has its own copy at
// its own address), and is what every launch gets as an argument.
static __device__ __align__(256) unsigned char scratch[SCOUT_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];  // zero-initialised; filled once per device, under the mutex

// Address of this device's copy of `scratch` (the current device), or nullptr with *rc set.
static void* static_scratch(int* rc) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    *rc = SCOUT_EHIP;
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
      *rc = SCOUT_EHIP;
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

// Partials of exactly A.nsplit splits, packed (the caller's workspace is laid out for the largest
// split count instead, so that its size does not depend on the plan).
static size_t static_layout(const Dims& D, const AttnPlan& A, size_t* off_m, size_t* off_l) {
  const size_t rows = (size_t)D.B * D.Hkv * A.nsplit * D.G;
  *off_m = round256(rows * D.d * sizeof(float));
  *off_l = *off_m + round256(rows * sizeof(float));
  return *off_l + round256(rows * sizeof(float));
}

}  // namespace scout

using namespace scout;

extern "C" {

int scout_version(void) { return 100; }

const char* scout_strerror(int code) {
  switch (code) {
    case SCOUT_OK: return "ok";
    case SCOUT_EINVAL: return "invalid argument";
    case SCOUT_EUNSUPPORTED: return "shape or type not supported by the kernels";
    case SCOUT_EWORKSPACE: return "workspace missing, misaligned or too small";
    case SCOUT_EHIP: return "HIP runtime error at launch";
    case SCOUT_ESCRATCH: return "problem needs more scratch than the library's static buffer holds";
    default: return "unknown error";
  }
}

int scout_set_attn_mode(int family, int nsplit, int waves) {
  // family 3 = MFMA family with select_topk as a launch of its own inside scout_layer_step;
  // family 4 = MFMA family with score_blocks as a launch of its own (selection still in the attention launch)
  g_fuse_select = family != 3;
  g_fuse_step = family != 3 && family != 4;
  if (family == 3 || family == 4) family = 2;
  if (family < 0 || family > 2 || nsplit < 0 || nsplit > kMaxSplit) return SCOUT_EINVAL;  // 3 and 4 were mapped to 2 above
  if (waves != 0 && waves != 4 && waves != 8 && waves != 16) return SCOUT_EINVAL;
  g_family = family;
  g_nsplit = nsplit;
  g_waves = waves;
  return SCOUT_OK;
}

int scout_workspace_bytes(const scout_problem* p, size_t* bytes) {
  Dims D;
  if (bytes == nullptr) return SCOUT_EINVAL;
  // ctx_len is not needed to size the workspace
  scout_problem tmp;
  if (p == nullptr) return SCOUT_EINVAL;
  tmp = *p;
  static const int32_t dummy = 0;
  if (tmp.ctx_len == nullptr) tmp.ctx_len = &dummy;
  const int rc = check_problem(&tmp, &D);
  if (rc != SCOUT_OK) return rc;
  *bytes = ws_layout(D).total;
  return SCOUT_OK;
}

int build_digests(const scout_problem* p, const void* k_blocks, void* digest, void* stream) {
  Dims D;
  int rc = check_problem_kv(p, &D);
  if (rc != SCOUT_OK) return rc;
  if (k_blocks == nullptr || digest == nullptr || !aligned16(k_blocks) || !aligned16(digest))
    return SCOUT_EINVAL;
  return launch_digest(D, p->dtype, k_blocks, digest, static_cast<hipStream_t>(stream));
}

int append_token(const scout_problem* p, int32_t* ctx_len, const void* k_new, const void* v_new,
                 const int32_t* new_slot, void* digest, int32_t* block_table, void* k_pool, void* v_pool,
                 int64_t n_slots, void* host_k, void* host_v, void* stream) {
  Dims D;
  int rc = check_problem_kv(p, &D);
  if (rc != SCOUT_OK) return rc;
  if (!ctx_len || !k_new || !v_new || !new_slot || !digest || !block_table || !k_pool || !v_pool)
    return SCOUT_EINVAL;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(digest) || !aligned16(k_pool) || !aligned16(v_pool))
    return SCOUT_EINVAL;
  if (n_slots < 0) return SCOUT_EINVAL;
  if ((host_k == nullptr) != (host_v == nullptr) || !aligned16(host_k) || !aligned16(host_v)) return SCOUT_EINVAL;
  return launch_append(D, p->dtype, ctx_len, k_new, v_new, new_slot, digest, block_table, k_pool, v_pool,
                       n_slots, host_k, host_v, static_cast<hipStream_t>(stream));
}

int score_blocks(const scout_problem* p, const void* q, const void* digest, float* scores, void* ws,
                 size_t ws_bytes, void* stream) {
  (void)ws;
  (void)ws_bytes;
  Dims D;
  int rc = check_problem(p, &D);
  if (rc != SCOUT_OK) return rc;
  if (q == nullptr || digest == nullptr || scores == nullptr) return SCOUT_EINVAL;
  if (!aligned16(q) || !aligned16(digest) || !aligned16(scores)) return SCOUT_EINVAL;
  return launch_score(D, p->dtype, q, digest, scores, static_cast<hipStream_t>(stream));
}

int select_topk(const scout_problem* p, const float* scores, const int32_t* block_table,
                int32_t* sel_all, int32_t* sel_gpu, int32_t* slot_gpu, int32_t* n_gpu,
                int32_t* sel_host, int32_t* n_host, void* ws, size_t ws_bytes, void* stream) {
  (void)ws;
  (void)ws_bytes;
  Dims D;
  int rc = check_problem(p, &D);
  if (rc != SCOUT_OK) return rc;
  if (!scores || !block_table || !sel_all || !sel_gpu || !slot_gpu || !n_gpu || !sel_host || !n_host)
    return SCOUT_EINVAL;
  return launch_topk(D, scores, block_table, sel_all, sel_gpu, slot_gpu, n_gpu, sel_host, n_host,
                     static_cast<hipStream_t>(stream));
}

int scout_attn_partials(const scout_problem* p, const void* q, const void* k_pool, const void* v_pool,
                        int64_t n_slots, const int32_t* sel_gpu, const int32_t* slot_gpu,
                        const int32_t* n_gpu, void* ws, size_t ws_bytes, void* stream) {
  Dims D;
  int rc = check_problem(p, &D);
  if (rc != SCOUT_OK) return rc;
  if (!q || !sel_gpu || !slot_gpu || !n_gpu || n_slots < 0) return SCOUT_EINVAL;
  if (n_slots > 0 && (!k_pool || !v_pool)) return SCOUT_EINVAL;
  if (!aligned16(q) || !aligned16(k_pool) || !aligned16(v_pool)) return SCOUT_EINVAL;
  WsLayout L;
  rc = check_ws(D, ws, ws_bytes, &L);
  if (rc != SCOUT_OK) return rc;
  AttnPlan A;
  rc = plan_attn(D, p->dtype, &A);
  if (rc != SCOUT_OK) return rc;
  Epilogue part{};
  part.mode = 0;
  return launch_attn(D, p->dtype, A.family, A.waves, q, k_pool, v_pool, n_slots, sel_gpu, slot_gpu, n_gpu,
                     carve(ws, L, A), part, static_cast<hipStream_t>(stream));
}

int scout_attn_finish(const scout_problem* p, const float* host_o, const float* host_m, const float* host_l,
                      void* out, float* lse, void* ws, size_t ws_bytes, void* stream) {
  Dims D;
  int rc = check_problem(p, &D);
  if (rc != SCOUT_OK) return rc;
  if (!out || !aligned16(out)) return SCOUT_EINVAL;
  const bool any_b = host_o || host_m || host_l, all_b = host_o && host_m && host_l;
  if (any_b && !all_b) return SCOUT_EINVAL;
  WsLayout L;
  rc = check_ws(D, ws, ws_bytes, &L);
  if (rc != SCOUT_OK) return rc;
  AttnPlan A;
  rc = plan_attn(D, p->dtype, &A);  // the same plan scout_attn_partials made: same split count
  if (rc != SCOUT_OK) return rc;
  Epilogue E{};
  E.mode = 2;
  E.host_o = host_o;
  E.host_m = host_m;
  E.host_l = host_l;
  E.out = out;
  E.lse = lse;
  E.dtype_out = p->dtype;
  return launch_combine(D, carve(ws, L, A), E, static_cast<hipStream_t>(stream));
}

int sparse_decode_attn(const scout_problem* p, const void* q, const void* k_pool, const void* v_pool,
                       int64_t n_slots, const int32_t* sel_gpu, const int32_t* slot_gpu,
                       const int32_t* n_gpu, float* o, float* m, float* l, void* ws, size_t ws_bytes,
                       void* stream) {
  Dims D;
  int rc = check_problem(p, &D);
  if (rc != SCOUT_OK) return rc;
  if (!q || !sel_gpu || !slot_gpu || !n_gpu || !o || !m || !l || n_slots < 0) return SCOUT_EINVAL;
  if (n_slots > 0 && (!k_pool || !v_pool)) return SCOUT_EINVAL;
  if (!aligned16(q) || !aligned16(k_pool) || !aligned16(v_pool) || !aligned16(o)) return SCOUT_EINVAL;
  WsLayout L;
  rc = check_ws(D, ws, ws_bytes, &L);
  if (rc != SCOUT_OK) return rc;
  AttnPlan A;
  rc = plan_attn(D, p->dtype, &A);
  if (rc != SCOUT_OK) return rc;
  Epilogue E{};
  E.mode = 1;
  E.o = o;
  E.m = m;
  E.l = l;
  return run_attn(D, p->dtype, A, q, k_pool, v_pool, n_slots, sel_gpu, slot_gpu, n_gpu, ws, L, E,
                  static_cast<hipStream_t>(stream));
}

int sparse_decode_attn_static(const scout_problem* p, const void* q, const void* k_pool, const void* v_pool,
                              int64_t n_slots, const int32_t* sel_gpu, const int32_t* slot_gpu,
                              const int32_t* n_gpu, float* o, float* m, float* l, void* stream) {
  Dims D;
  int rc = check_problem(p, &D);
  if (rc != SCOUT_OK) return rc;
  if (!q || !sel_gpu || !slot_gpu || !n_gpu || !o || !m || !l || n_slots < 0) return SCOUT_EINVAL;
  if (n_slots > 0 && (!k_pool || !v_pool)) return SCOUT_EINVAL;
  if (!aligned16(q) || !aligned16(k_pool) || !aligned16(v_pool) || !aligned16(o)) return SCOUT_EINVAL;
  AttnPlan A;
  rc = plan_attn(D, p->dtype, &A);
  if (rc != SCOUT_OK) return rc;
  Epilogue E{};
  E.mode = 1;
  E.o = o;
  E.m = m;
  E.l = l;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (A.family == 2 && A.nsplit == 1)  // one workgroup per pair finishes the pair itself: no scratch at all
    return launch_attn(D, p->dtype, 2, A.waves, q, k_pool, v_pool, n_slots, sel_gpu, slot_gpu, n_gpu,
                       Partials{nullptr, nullptr, nullptr, 1, waves_magic(A)}, E, st);
  size_t off_m, off_l;
  if (static_layout(D, A, &off_m, &off_l) > (size_t)SCOUT_STATIC_SCRATCH_BYTES) return SCOUT_ESCRATCH;
  char* base = static_cast<char*>(static_scratch(&rc));
  if (base == nullptr) return rc;
  // Nothing in the buffer has to start at zero: the first pass writes the partial of every (pair, split,
  // head) it was launched for, an empty share included, before the combine pass reads any of them.
  const Partials P{reinterpret_cast<float*>(base), reinterpret_cast<float*>(base + off_m),
                   reinterpret_cast<float*>(base + off_l), A.nsplit, waves_magic(A)};
  Epilogue part{};
  part.mode = 0;
  rc = launch_attn(D, p->dtype, A.family, A.waves, q, k_pool, v_pool, n_slots, sel_gpu, slot_gpu, n_gpu, P, part, st);
  if (rc != SCOUT_OK) return rc;
  return launch_combine(D, P, E, st);
}

int merge_partials(const scout_problem* p, const float* o_a, const float* m_a, const float* l_a,
                   const float* o_b, const float* m_b, const float* l_b, void* out, float* lse,
                   void* stream) {
  Dims D;
  int rc = check_problem(p, &D);
  if (rc != SCOUT_OK) return rc;
  if (!o_a || !m_a || !l_a || !out) return SCOUT_EINVAL;
  const bool any_b = o_b || m_b || l_b, all_b = o_b && m_b && l_b;
  if (any_b && !all_b) return SCOUT_EINVAL;
  return launch_merge(D, p->dtype, o_a, m_a, l_a, o_b, m_b, l_b, out, lse,
                      static_cast<hipStream_t>(stream));
}

int periodic_recall(const scout_problem* p, const void* q, const void* digest, int32_t* block_table,
                    int32_t* recall_blk, int32_t* recall_slot, int32_t* evict_blk, int32_t* n_recall,
                    void* ws, size_t ws_bytes, void* stream) {
  Dims D;
  int rc = check_problem(p, &D);
  if (rc != SCOUT_OK) return rc;
  if (p->per_head) return SCOUT_EUNSUPPORTED;  // a recall plans for the KV head; which heads' choices count is not defined
  if (!q || !digest || !block_table || !recall_blk || !recall_slot || !evict_blk || !n_recall)
    return SCOUT_EINVAL;
  if (!aligned16(q) || !aligned16(digest)) return SCOUT_EINVAL;
  WsLayout L;
  rc = check_ws(D, ws, ws_bytes, &L);
  if (rc != SCOUT_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  float* scores = reinterpret_cast<float*>(static_cast<char*>(ws) + L.scores);
  rc = launch_score(D, p->dtype, q, digest, scores, st);
  if (rc != SCOUT_OK) return rc;
  return launch_recall(D, scores, block_table, recall_blk, recall_slot, evict_blk, n_recall, st);
}

int recall_fetch(const scout_problem* p, const void* src_k, const void* src_v, const int32_t* recall_blk,
                 const int32_t* recall_slot, const int32_t* n_recall, void* k_pool, void* v_pool,
                 int64_t n_slots, void* stream) {
  Dims D;
  int rc = check_problem_kv(p, &D);
  if (rc != SCOUT_OK) return rc;
  if (!src_k || !src_v || !recall_blk || !recall_slot || !n_recall || !k_pool || !v_pool) return SCOUT_EINVAL;
  if (!aligned16(src_k) || !aligned16(src_v) || !aligned16(k_pool) || !aligned16(v_pool)) return SCOUT_EINVAL;
  if (n_slots < 0) return SCOUT_EINVAL;
  return launch_recall_fetch(D, p->dtype, src_k, src_v, recall_blk, recall_slot, n_recall, k_pool, v_pool,
                             n_slots, static_cast<hipStream_t>(stream));
}

int recall_scatter(const scout_problem* p, const void* staged, int64_t n_tiles, const int32_t* tile_off,
                   const int32_t* recall_blk, const int32_t* recall_slot, const int32_t* n_recall, void* k_pool,
                   void* v_pool, int64_t n_slots, void* stream) {
  Dims D;
  int rc = check_problem_kv(p, &D);
  if (rc != SCOUT_OK) return rc;
  if (!staged || !tile_off || !recall_blk || !recall_slot || !n_recall || !k_pool || !v_pool) return SCOUT_EINVAL;
  if (!aligned16(staged) || !aligned16(k_pool) || !aligned16(v_pool) || n_slots < 0 || n_tiles < 0) return SCOUT_EINVAL;
  return launch_recall_scatter(D, p->dtype, staged, (long long)n_tiles, tile_off, recall_blk, recall_slot, n_recall, k_pool, v_pool,
                               n_slots, static_cast<hipStream_t>(stream));
}

int scout_layer_step(const scout_problem* p, const void* q, const void* digest,
                     const int32_t* block_table, const void* k_pool, const void* v_pool,
                     int64_t n_slots, const float* host_o, const float* host_m, const float* host_l,
                     float* scores, int32_t* sel_all, int32_t* sel_gpu, int32_t* slot_gpu,
                     int32_t* n_gpu, int32_t* sel_host, int32_t* n_host, void* out, float* lse, void* ws,
                     size_t ws_bytes, void* stream) {
  Dims D;
  int rc = check_problem(p, &D);
  if (rc != SCOUT_OK) return rc;
  if (!q || !digest || !block_table || !sel_all || !sel_gpu || !slot_gpu || !n_gpu ||
      !sel_host || !n_host || !out || n_slots < 0)
    return SCOUT_EINVAL;
  if (n_slots > 0 && (!k_pool || !v_pool)) return SCOUT_EINVAL;
  const bool any_b = host_o || host_m || host_l, all_b = host_o && host_m && host_l;
  if (any_b && !all_b) return SCOUT_EINVAL;
  if (!aligned16(q) || !aligned16(digest) || !aligned16(k_pool) || !aligned16(v_pool) || !aligned16(scores))
    return SCOUT_EINVAL;
  WsLayout L;
  rc = check_ws(D, ws, ws_bytes, &L);
  if (rc != SCOUT_OK) return rc;
  AttnPlan A;
  rc = plan_attn(D, p->dtype, &A);
  if (rc != SCOUT_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  Epilogue E{};
  E.mode = 2;
  E.host_o = host_o;
  E.host_m = host_m;
  E.host_l = host_l;
  E.out = out;
  E.lse = lse;
  E.dtype_out = p->dtype;
  if (g_fuse_select && g_fuse_step && A.family == 2 && A.waves == 8 && A.nsplit == 1 && step_kernel_supported(D, p->dtype))
    // the pairs alone fill the chip: the whole step of a pair in one workgroup, one launch
    return launch_step(D, q, digest, block_table, k_pool, v_pool, n_slots, scores, sel_all, sel_gpu, slot_gpu, n_gpu,
                       sel_host, n_host, carve(ws, L, A), E, st);
  if (scores == nullptr) scores = reinterpret_cast<float*>(static_cast<char*>(ws) + L.scores);
  rc = launch_score(D, p->dtype, q, digest, scores, st);
  if (rc != SCOUT_OK) return rc;
  if (g_fuse_select && A.family == 2 && A.waves == 8 && select_attend_supported(D, p->dtype)) {
    // selection rides in the head of the attention kernel: two launches for the whole step
    Partials P = carve(ws, L, A);
    if (A.nsplit == 1)
      return launch_select_attend(D, q, scores, block_table, k_pool, v_pool, n_slots, sel_all, sel_gpu,
                                  slot_gpu, n_gpu, sel_host, n_host, P, E, st);
    Epilogue part{};
    part.mode = 0;
    rc = launch_select_attend(D, q, scores, block_table, k_pool, v_pool, n_slots, sel_all, sel_gpu, slot_gpu,
                              n_gpu, sel_host, n_host, P, part, st);
    if (rc != SCOUT_OK) return rc;
    return launch_combine(D, P, E, st);
  }
  rc = launch_topk(D, scores, block_table, sel_all, sel_gpu, slot_gpu, n_gpu, sel_host, n_host, st);
  if (rc != SCOUT_OK) return rc;
  return run_attn(D, p->dtype, A, q, k_pool, v_pool, n_slots, sel_gpu, slot_gpu, n_gpu, ws, L, E, st);
}

}  // extern "C"

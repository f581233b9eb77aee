// Host side of the co-attention (Sec. 3.2; Alg. 1 CPUAttn): partial attention over the selected
// blocks that live in host memory, by a pool of threads, asynchronous so that it can run a layer
// ahead of the GPU (Sec. 3.3).
//
// A job is the list of (sequence, KV head) pairs of one layer-step.  Threads take pairs from an atomic
// counter, heaviest pairs first would not pay here: pairs are small (a few blocks) and there are many
// more of them than threads.  A thread keeps one online-softmax stream per query head of the pair and
// walks the pair's blocks once: a block's K rows are widened to binary32 once and used by all G
// heads, then its V rows likewise.  Idle threads spin briefly on the job counter before they sleep:
// a layer-step is tens to hundreds of microseconds, a futex wake-up alone is of that order.
#include <atomic>
#include <chrono>
#include <cmath>
#include <condition_variable>
#include <cstring>
#include <limits>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "scout_host.h"

namespace {

constexpr int kMaxG = 16, kMaxD = 256, kMaxS = 64;

struct Job {
  scout_host_problem p{};
  const void* q = nullptr;
  const void* kb = nullptr;
  const void* vb = nullptr;
  const int32_t* sel = nullptr;
  const int32_t* n = nullptr;
  const int32_t* ctx = nullptr;
  float* o = nullptr;
  float* m = nullptr;
  float* l = nullptr;
  float scale = 0.0f;
  int pairs = 0;
};

inline float bf16_to_f32(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  std::memcpy(&f, &u, sizeof f);
  return f;
}

// Rows of a tile as binary32.  The loops are written for the auto-vectoriser; the clones let one
// build serve hosts with and without the wider vector units.
__attribute__((target_clones("default", "avx2", "avx512f"))) void widen_bf16(const uint16_t* src, float* dst,
                                                                               int n) {
  for (int i = 0; i < n; ++i) {
    uint32_t u = (uint32_t)src[i] << 16;
    std::memcpy(&dst[i], &u, sizeof(float));
  }
}

__attribute__((target_clones("default", "avx2,fma", "avx512f"))) void logits_of_block(
    const float* q, const float* kf, int G, int valid, int d, float scale, float* logit /*[G][kMaxS]*/) {
  for (int h = 0; h < G; ++h) {
    const float* qh = q + (size_t)h * d;
    for (int t = 0; t < valid; ++t) {
      const float* kr = kf + (size_t)t * d;
      float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      for (int c = 0; c < d; c += 8)
        for (int i = 0; i < 8; ++i) acc[i] += qh[c + i] * kr[c + i];
      logit[h * kMaxS + t] = scale * (((acc[0] + acc[4]) + (acc[2] + acc[6])) + ((acc[1] + acc[5]) + (acc[3] + acc[7])));
    }
  }
}

__attribute__((target_clones("default", "avx2,fma", "avx512f"))) void add_weighted_rows(
    const float* w /*[valid]*/, const float* vf, int valid, int d, float corr, float* acc /*[d]*/) {
  for (int c = 0; c < d; ++c) acc[c] *= corr;
  for (int t = 0; t < valid; ++t) {
    const float wt = w[t];
    const float* vr = vf + (size_t)t * d;
    for (int c = 0; c < d; ++c) acc[c] += wt * vr[c];
  }
}

void run_pair(const Job& J, int pair, float* kf, float* vf) {
  const scout_host_problem& P = J.p;
  const int G = P.Hq / P.Hkv, d = P.d, S = P.S;
  const int b = pair / P.Hkv, g = pair % P.Hkv;
  const size_t esz = P.dtype == 1 ? 2 : 4;
  float qf[kMaxG * kMaxD];
  float acc[kMaxG * kMaxD];
  float mx[kMaxG], sum[kMaxG];
  float logit[kMaxG * kMaxS];
  const size_t q_off = ((size_t)b * P.Hq + (size_t)g * G) * d;
  if (P.dtype == 1)
    widen_bf16(static_cast<const uint16_t*>(J.q) + q_off, qf, G * d);
  else
    std::memcpy(qf, static_cast<const float*>(J.q) + q_off, sizeof(float) * G * d);
  for (int h = 0; h < G; ++h) {
    mx[h] = -std::numeric_limits<float>::infinity();
    sum[h] = 0.0f;
  }
  std::memset(acc, 0, sizeof(float) * G * d);

  int n = J.n[pair];
  n = n < 0 ? 0 : (n > P.k ? P.k : n);
  const int ctx = J.ctx[b];
  const size_t tile = (size_t)S * d;
  for (int i = 0; i < n; ++i) {
    const int j = J.sel[(size_t)pair * P.k + i];
    if (j < 0 || j >= P.max_blocks) continue;
    int valid = ctx - j * S;
    valid = valid > S ? S : valid;
    if (valid <= 0) continue;
    const size_t off = ((size_t)pair * P.max_blocks + j) * tile;
    const float *kt, *vt;
    if (P.dtype == 1) {
      widen_bf16(static_cast<const uint16_t*>(J.kb) + off, kf, valid * d);
      widen_bf16(static_cast<const uint16_t*>(J.vb) + off, vf, valid * d);
      kt = kf;
      vt = vf;
    } else {
      kt = static_cast<const float*>(J.kb) + off;
      vt = static_cast<const float*>(J.vb) + off;
    }
    (void)esz;
    logits_of_block(qf, kt, G, valid, d, J.scale, logit);
    for (int h = 0; h < G; ++h) {
      float* lg = logit + h * kMaxS;
      float bm = lg[0];
      for (int t = 1; t < valid; ++t) bm = lg[t] > bm ? lg[t] : bm;
      const float m_new = bm > mx[h] ? bm : mx[h];
      // exp(-inf - finite) = 0 covers the first block; a block of -inf logits leaves the stream as it is
      if (m_new == -std::numeric_limits<float>::infinity()) continue;
      const float corr = std::exp(mx[h] - m_new);
      float s = 0.0f;
      for (int t = 0; t < valid; ++t) {
        lg[t] = std::exp(lg[t] - m_new);
        s += lg[t];
      }
      sum[h] = sum[h] * corr + s;
      mx[h] = m_new;
      add_weighted_rows(lg, vt, valid, d, corr, acc + (size_t)h * d);
    }
  }
  for (int h = 0; h < G; ++h) {
    const size_t hq = (size_t)b * P.Hq + (size_t)g * G + h;
    const float inv = sum[h] > 0.0f ? 1.0f / sum[h] : 0.0f;
    float* oo = J.o + hq * d;
    for (int c = 0; c < d; ++c) oo[c] = acc[(size_t)h * d + c] * inv;
    J.m[hq] = mx[h];
    J.l[hq] = sum[h];
  }
}

}  // namespace

struct scout_host_worker {
  std::vector<std::thread> threads;
  std::mutex mu;
  std::condition_variable cv_job, cv_done;
  Job job;
  std::atomic<uint64_t> generation{0};  // bumped at every submit
  std::atomic<uint64_t> ticket{0};      // (generation << 32) | next pair: a thread still leaving the
                                        // previous job can never take a pair of the next one
  std::atomic<int> pairs_left{0};
  std::atomic<bool> stop{false};
  std::atomic<bool> in_flight{false};
  std::chrono::steady_clock::time_point t_submit, t_done;

  void loop() {
    std::vector<float> kf((size_t)kMaxS * kMaxD), vf((size_t)kMaxS * kMaxD);
    uint64_t seen = 0;
    for (;;) {
      // wait for a new generation: spin for a short while, then sleep
      bool got = false;
      for (int spin = 0; spin < 20000 && !got; ++spin) {
        if (stop.load(std::memory_order_acquire)) return;
        got = generation.load(std::memory_order_acquire) != seen;
        if (!got) __builtin_ia32_pause();
      }
      if (!got) {
        std::unique_lock<std::mutex> lk(mu);
        cv_job.wait(lk, [&] { return stop.load() || generation.load() != seen; });
        if (stop.load()) return;
      }
      Job J;
      {
        std::lock_guard<std::mutex> lk(mu);  // submit writes the job under the same lock
        seen = generation.load(std::memory_order_acquire);
        J = job;
      }
      for (;;) {
        uint64_t t = ticket.load(std::memory_order_acquire);
        if ((t >> 32) != (seen & 0xffffffffu) || (int)(t & 0xffffffffu) >= J.pairs) break;
        if (!ticket.compare_exchange_weak(t, t + 1, std::memory_order_acq_rel)) continue;
        const int pair = (int)(t & 0xffffffffu);
        run_pair(J, pair, kf.data(), vf.data());
        if (pairs_left.fetch_sub(1, std::memory_order_acq_rel) == 1) {
          t_done = std::chrono::steady_clock::now();
          {
            std::lock_guard<std::mutex> lk(mu);
            in_flight.store(false, std::memory_order_release);
          }
          cv_done.notify_all();
        }
      }
    }
  }
};

extern "C" {

int scout_host_create(int n_threads, scout_host_worker** out) {
  if (out == nullptr || n_threads < 1 || n_threads > 1024) return -1;
  scout_host_worker* w = new (std::nothrow) scout_host_worker;
  if (w == nullptr) return -5;
  try {
    for (int i = 0; i < n_threads; ++i) w->threads.emplace_back([w] { w->loop(); });
  } catch (...) {
    scout_host_destroy(w);
    return -5;
  }
  *out = w;
  return 0;
}

void scout_host_destroy(scout_host_worker* w) {
  if (w == nullptr) return;
  scout_host_wait(w, nullptr);
  {
    std::lock_guard<std::mutex> lk(w->mu);
    w->stop.store(true, std::memory_order_release);
  }
  w->cv_job.notify_all();
  for (auto& t : w->threads)
    if (t.joinable()) t.join();
  delete w;
}

int scout_host_submit(scout_host_worker* w, const scout_host_problem* p, const void* q, const void* k_blocks,
                      const void* v_blocks, const int32_t* sel_host, const int32_t* n_host,
                      const int32_t* ctx_len, float* o, float* m, float* l) {
  if (!w || !p || !q || !k_blocks || !v_blocks || !sel_host || !n_host || !ctx_len || !o || !m || !l) return -1;
  if (p->B < 0 || p->Hq < 1 || p->Hkv < 1 || p->Hq % p->Hkv != 0 || p->Hq / p->Hkv > kMaxG) return -1;
  if (p->d < 8 || p->d % 8 != 0 || p->d > kMaxD || p->S < 1 || p->S > kMaxS) return -1;
  if ((p->dtype != 0 && p->dtype != 1) || p->max_blocks < 0 || p->k < 0) return -1;
  if (w->in_flight.load(std::memory_order_acquire)) return -6;
  Job J;
  J.p = *p;
  J.q = q; J.kb = k_blocks; J.vb = v_blocks; J.sel = sel_host; J.n = n_host; J.ctx = ctx_len;
  J.o = o; J.m = m; J.l = l;
  J.scale = p->sm_scale != 0.0f ? p->sm_scale : 1.0f / std::sqrt((float)p->d);
  J.pairs = p->B * p->Hkv;
  if (J.pairs == 0) return 0;
  {
    std::lock_guard<std::mutex> lk(w->mu);
    w->job = J;
    w->pairs_left.store(J.pairs, std::memory_order_relaxed);
    w->in_flight.store(true, std::memory_order_release);
    w->t_submit = std::chrono::steady_clock::now();
    const uint64_t gen = w->generation.load(std::memory_order_relaxed) + 1;
    w->ticket.store((gen & 0xffffffffu) << 32, std::memory_order_release);
    w->generation.store(gen, std::memory_order_release);
  }
  w->cv_job.notify_all();
  return 0;
}

int scout_host_wait(scout_host_worker* w, double* seconds) {
  if (w == nullptr) return -1;
  // spin first: the caller usually arrives when the job is nearly done
  for (int spin = 0; spin < 20000 && w->in_flight.load(std::memory_order_acquire); ++spin) __builtin_ia32_pause();
  if (w->in_flight.load(std::memory_order_acquire)) {
    std::unique_lock<std::mutex> lk(w->mu);
    w->cv_done.wait(lk, [&] { return !w->in_flight.load(); });
  }
  if (seconds != nullptr) *seconds = std::chrono::duration<double>(w->t_done - w->t_submit).count();
  return 0;
}

int scout_host_done(scout_host_worker* w) { return w == nullptr || !w->in_flight.load(std::memory_order_acquire) ? 1 : 0; }

}  // extern "C"

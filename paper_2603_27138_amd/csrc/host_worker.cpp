// Host side of the co-attention (Sec. 3.2; Alg. 1 CPUAttn): partial attention over the selected
// blocks that live in host memory, by a pool of threads, asynchronous so that it can run a layer
// ahead of the GPU (Sec. 3.3).
//
// A job is the list of (sequence, KV head) pairs of one layer-step.  Threads take pairs from an atomic
// counter, heaviest pairs first would not pay here: pairs are small (a few blocks) and there are many
// more of them than threads.  A thread keeps one online-softmax stream per query head of the pair and
// walks the pair's blocks once: a block's K rows are widened to binary32 once and used by all G
// heads, then its V rows likewise.  The query heads of the group are the vector lanes of the logits
// and of the softmax bookkeeping (no sums across lanes), the channels those of the value product.  Idle threads spin briefly on the job counter before they sleep:
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
  // kind 1 (packing the tiles of a recall plan): kb / vb are the block store, sel the planned block
  // indices, n their counts
  int kind = 0;
  char* staged = nullptr;
  const int32_t* tile_off = nullptr;
};

namespace scout_host_generic {
using ::Job;
#include "host_kernels.inc"
}  // namespace scout_host_generic

#if defined(__x86_64__)
#pragma GCC push_options
#pragma GCC target("avx2,fma")
namespace scout_host_avx2 {
using ::Job;
#include "host_kernels.inc"
}  // namespace scout_host_avx2
#pragma GCC pop_options
#endif

namespace {

// Recall staging (Sec. 3.4): the pair's planned tiles go to their places in the packed buffer.
void stage_pair(const Job& J, int pair) {
  const size_t tile = (size_t)J.p.S * J.p.d * (J.p.dtype == 1 ? 2 : 4);
  int n = J.n[pair];
  n = n < 0 ? 0 : (n > J.p.k ? J.p.k : n);
  const char* kb = static_cast<const char*>(J.kb) + (size_t)pair * J.p.max_blocks * tile;
  const char* vb = static_cast<const char*>(J.vb) + (size_t)pair * J.p.max_blocks * tile;
  char* out = J.staged + (size_t)J.tile_off[pair] * 2 * tile;
  for (int i = 0; i < n; ++i, out += 2 * tile) {
    const int blk = J.sel[(size_t)pair * J.p.k + i];
    if (blk < 0 || blk >= J.p.max_blocks) continue;
    std::memcpy(out, kb + (size_t)blk * tile, tile);
    std::memcpy(out + tile, vb + (size_t)blk * tile, tile);
  }
}

void run_pair(const Job& J, int pair, float* kf, float* vf) {
  if (J.kind == 1) return stage_pair(J, pair);
  const bool wide = J.p.Hq / J.p.Hkv > 8;
#if defined(__x86_64__)
  static const bool avx2 = __builtin_cpu_supports("avx2") && __builtin_cpu_supports("fma");
  if (avx2) {
    if (wide) scout_host_avx2::run_pair_nv<2>(J, pair, kf, vf);
    else scout_host_avx2::run_pair_nv<1>(J, pair, kf, vf);
    return;
  }
#endif
  if (wide) scout_host_generic::run_pair_nv<2>(J, pair, kf, vf);
  else scout_host_generic::run_pair_nv<1>(J, pair, kf, vf);
}

}  // namespace

struct scout_host_worker {
  std::vector<std::thread> threads;
  std::mutex mu;
  std::condition_variable cv_job, cv_done;
  Job job;
  // One job runs; one more may wait behind it (Alg. 1 spawns layer i+1's job while layer i's may still
  // be running).  The thread that finishes a job's last pair starts the queued one.  All under `mu`.
  Job queued;
  bool has_queued = false;
  uint64_t submitted = 0, completed = 0, waited = 0;  // jobs handed in, finished, reported by wait()
  std::chrono::steady_clock::time_point t_start[2], t_end[2];  // of job number n, at n % 2
  std::atomic<uint64_t> generation{0};  // bumped at every submit
  std::atomic<uint64_t> ticket{0};      // (generation << 32) | next pair: a thread still leaving the
                                        // previous job can never take a pair of the next one
  std::atomic<int> pairs_left{0};
  std::atomic<bool> stop{false};
  std::atomic<bool> in_flight{false};

  // Make J the running job.  Caller holds `mu` and notifies cv_job afterwards.
  void start_locked(const Job& J, uint64_t number) {
    job = J;
    pairs_left.store(J.pairs, std::memory_order_relaxed);
    in_flight.store(true, std::memory_order_release);
    t_start[number & 1] = std::chrono::steady_clock::now();
    const uint64_t gen = generation.load(std::memory_order_relaxed) + 1;
    ticket.store((gen & 0xffffffffu) << 32, std::memory_order_release);
    generation.store(gen, std::memory_order_release);
  }

  void loop() {
    std::vector<float> kf((size_t)(kMaxS + 4) * kMaxD), vf((size_t)kMaxS * kMaxD);
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
          const auto now = std::chrono::steady_clock::now();
          bool next = false;
          {
            std::lock_guard<std::mutex> lk(mu);
            t_end[completed & 1] = now;
            ++completed;
            if (has_queued) {  // the job that waited behind this one starts now
              has_queued = false;
              start_locked(queued, completed);
              next = true;
            } else {
              in_flight.store(false, std::memory_order_release);
            }
          }
          cv_done.notify_all();
          if (next) cv_job.notify_all();
        }
      }
    }
  }
};

// Hand a job to the threads: it starts at once if none is running, else it waits behind the running
// one.  -6 if one is waiting already.
static int publish(scout_host_worker* w, const Job& J) {
  bool started = false;
  {
    std::lock_guard<std::mutex> lk(w->mu);
    if (w->in_flight.load(std::memory_order_acquire)) {
      if (w->has_queued) return -6;
      w->queued = J;
      w->has_queued = true;
    } else {
      w->start_locked(J, w->submitted);
      started = true;
    }
    ++w->submitted;
  }
  if (started) w->cv_job.notify_all();
  return 0;
}

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
  scout_host_wait(w, nullptr);  // and the one that waited behind it
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
  Job J;
  J.p = *p;
  J.q = q; J.kb = k_blocks; J.vb = v_blocks; J.sel = sel_host; J.n = n_host; J.ctx = ctx_len;
  J.o = o; J.m = m; J.l = l;
  J.scale = p->sm_scale != 0.0f ? p->sm_scale : 1.0f / std::sqrt((float)p->d);
  J.pairs = p->B * p->Hkv;
  if (J.pairs == 0) return 0;
  return publish(w, J);
}

int scout_host_stage_recall(scout_host_worker* w, const scout_host_problem* p, const void* k_blocks,
                            const void* v_blocks, const int32_t* recall_blk, const int32_t* n_recall,
                            void* staged, size_t staged_bytes, int32_t* tile_off, int64_t* total_tiles) {
  if (!w || !p || !k_blocks || !v_blocks || !recall_blk || !n_recall || !tile_off || !total_tiles) return -1;
  if (p->B < 0 || p->Hkv < 1 || p->d < 1 || p->S < 1 || (p->dtype != 0 && p->dtype != 1) || p->max_blocks < 0 ||
      p->k < 0)
    return -1;
  {
    std::lock_guard<std::mutex> lk(w->mu);  // tile_off is written below: refuse before touching it
    if (w->in_flight.load(std::memory_order_acquire) && w->has_queued) return -6;
  }
  const int pairs = p->B * p->Hkv;
  const size_t tile = (size_t)p->S * p->d * (p->dtype == 1 ? 2 : 4);
  int64_t total = 0;
  for (int pair = 0; pair < pairs; ++pair) {
    const int n = n_recall[pair];
    if (total > std::numeric_limits<int32_t>::max()) return -1;
    tile_off[pair] = (int32_t)total;
    total += n < 0 ? 0 : (n > p->k ? p->k : n);
  }
  *total_tiles = total;
  if (total == 0) return 0;
  if (staged == nullptr || (size_t)total * 2 * tile > staged_bytes) return -1;
  Job J;
  J.p = *p;
  J.kind = 1;
  J.kb = k_blocks; J.vb = v_blocks; J.sel = recall_blk; J.n = n_recall;
  J.staged = static_cast<char*>(staged);
  J.tile_off = tile_off;
  J.pairs = pairs;
  return publish(w, J);
}

int scout_host_wait(scout_host_worker* w, double* seconds) {
  if (w == nullptr) return -1;
  uint64_t mine;
  {
    std::lock_guard<std::mutex> lk(w->mu);
    if (w->waited == w->submitted) {  // nothing outstanding
      if (seconds != nullptr) *seconds = 0.0;
      return 0;
    }
    mine = w->waited;
  }
  // the oldest job not yet reported.  Spin first: the caller usually arrives when it is nearly done
  auto finished = [&] {
    std::lock_guard<std::mutex> lk(w->mu);
    return w->completed > mine;
  };
  bool ok = false;
  for (int spin = 0; spin < 2000 && !(ok = finished()); ++spin)
    for (int i = 0; i < 10; ++i) __builtin_ia32_pause();
  std::unique_lock<std::mutex> lk(w->mu);
  if (!ok) w->cv_done.wait(lk, [&] { return w->completed > mine; });
  if (seconds != nullptr) *seconds = std::chrono::duration<double>(w->t_end[mine & 1] - w->t_start[mine & 1]).count();
  w->waited = mine + 1;
  return 0;
}

int scout_host_done(scout_host_worker* w) {
  if (w == nullptr) return 1;
  std::lock_guard<std::mutex> lk(w->mu);
  return w->completed == w->submitted ? 1 : 0;
}

}  // extern "C"

// Host pipeline around the generation entry points (see include/ernie_job.h): batch planning,
// preprocessing, inference and post-processing workers over two batch slots.  Host code only;
// all device work goes through ernie_prefill / ernie_decode_step and asynchronous copies.

#include "../../include/ernie_job.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <chrono>
#include <condition_variable>
#include <mutex>
#include <thread>
#include <vector>

namespace {

using Clock = std::chrono::steady_clock;
double since(Clock::time_point t0) { return std::chrono::duration<double>(Clock::now() - t0).count(); }

constexpr int kSlots = 2;
constexpr size_t kAlign = 256;
size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

enum SlotState { FREE = 0, READY = 1, INFLIGHT = 2 };

struct Slot {
  int32_t* ids_pinned = nullptr;      // [max_batch, l_cap] right-padded trimmed ids
  int32_t* lens_pinned = nullptr;     // [max_batch]
  int32_t* tok_pinned = nullptr;      // [n_gen, max_batch]
  int32_t* ids_dev = nullptr;
  int32_t* tok_dev = nullptr;
  hipEvent_t done = nullptr;
  int B = 0, Lmax = 0, batch = -1;
  SlotState state = FREE;
};

struct Run {
  ErnieHandle* h;
  const ErnieJob* job;
  ErnieConfig cfg;
  hipStream_t stream;
  int device;
  std::vector<int32_t> order, starts;
  int n_batches = 0;
  Slot slot[kSlots];
  std::mutex mu;
  std::condition_variable cv;
  std::atomic<int> error{ERNIE_OK};
  double pre_s = 0, enqueue_s = 0, post_s = 0;

  // Blocks until the slot reaches `want` (returns true) or the run has failed (false).
  bool wait_state(Slot& s, SlotState want) {
    std::unique_lock<std::mutex> lk(mu);
    cv.wait(lk, [&] { return s.state == want || error.load() != ERNIE_OK; });
    return error.load() == ERNIE_OK;
  }
  void set_state(Slot& s, SlotState st) {
    { std::lock_guard<std::mutex> lk(mu); s.state = st; }
    cv.notify_all();
  }
  void fail(int code) {
    {
      // under the mutex: a waiter that has just evaluated its predicate must not miss this wake-up
      std::lock_guard<std::mutex> lk(mu);
      int expected = ERNIE_OK;
      error.compare_exchange_strong(expected, code);
    }
    cv.notify_all();
  }

  // ---- the three stages of one batch ------------------------------------
  void stage_pre(int i, Slot& s) {
    const auto t0 = Clock::now();
    const int a = starts[i], b = starts[i + 1];
    s.B = b - a; s.batch = i;
    int lmax = 0;
    for (int r = a; r < b; ++r) {
      const int q = order[r];
      const int L = job->prompt_offsets_host[q + 1] - job->prompt_offsets_host[q];
      if (L > lmax) lmax = L;
    }
    s.Lmax = lmax;
    for (int r = a; r < b; ++r) {
      const int q = order[r];
      const int32_t* src = job->prompt_ids_host + job->prompt_offsets_host[q];
      const int L = job->prompt_offsets_host[q + 1] - job->prompt_offsets_host[q];
      int32_t* dst = s.ids_pinned + (size_t)(r - a) * lmax;
      for (int j = 0; j < L; ++j) dst[j] = job->full_to_trimmed_host[src[j]];
      for (int j = L; j < lmax; ++j) dst[j] = 0;
      s.lens_pinned[r - a] = L;
    }
    pre_s += since(t0);
  }

  bool stage_gpu(Slot& s) {
    const auto t0 = Clock::now();
    const int B = s.B, N = job->n_gen;
    bool ok = hipMemcpyAsync(s.ids_dev, s.ids_pinned, sizeof(int32_t) * (size_t)B * s.Lmax, hipMemcpyHostToDevice,
                             stream) == hipSuccess;
    int rc = ok ? ernie_prefill(h, B, s.Lmax, s.ids_dev, s.lens_pinned, nullptr, nullptr, s.tok_dev, stream) : ERNIE_EHIP;
    for (int t = 1; t < N && rc == ERNIE_OK; ++t)
      rc = ernie_decode_step(h, nullptr, nullptr, nullptr, s.tok_dev + (size_t)t * B, stream);
    if (rc == ERNIE_OK) {
      ok = hipMemcpyAsync(s.tok_pinned, s.tok_dev, sizeof(int32_t) * (size_t)N * B, hipMemcpyDeviceToHost, stream) ==
               hipSuccess &&
           hipEventRecord(s.done, stream) == hipSuccess;
      if (!ok) rc = ERNIE_EHIP;
    }
    enqueue_s += since(t0);
    if (rc != ERNIE_OK) { fail(rc); return false; }
    return true;
  }

  bool stage_post(Slot& s) {
    if (hipEventSynchronize(s.done) != hipSuccess) { fail(ERNIE_EHIP); return false; }
    // the batch has run: a decode kernel whose bounded wait gave up has left its mark by now
    if (const int rc = ernie_last_error(h); rc != ERNIE_OK) { fail(rc); return false; }
    const auto t0 = Clock::now();
    const int a = starts[s.batch], B = s.B, N = job->n_gen;
    for (int r = 0; r < B; ++r) {
      int32_t* dst = job->tokens_out_host + (size_t)order[a + r] * N;
      for (int t = 0; t < N; ++t) dst[t] = job->kept_ids_host[s.tok_pinned[(size_t)t * B + r]];
    }
    post_s += since(t0);
    return true;
  }
};

}  // namespace

extern "C" {

size_t ernie_job_workspace_bytes(const ErnieHandle* h, int32_t n_gen) {
  ErnieConfig c;
  if (!h || n_gen < 1 || ernie_get_config(h, &c) != ERNIE_OK) return 0;
  const size_t l_cap = (size_t)(c.max_seq < c.max_pos ? c.max_seq : c.max_pos);
  return kSlots * (align_up((size_t)c.max_batch * l_cap * 4) + align_up((size_t)n_gen * c.max_batch * 4));
}

int ernie_run_job(ErnieHandle* h, const ErnieJob* job, ErnieJobStats* stats_out, void* stream) {
  const auto t_wall = Clock::now();
  if (!h || !job) return ERNIE_EINVAL;
  Run run;
  run.h = h; run.job = job; run.stream = static_cast<hipStream_t>(stream);
  if (ernie_get_config(h, &run.cfg) != ERNIE_OK) return ERNIE_EINVAL;
  const ErnieConfig& c = run.cfg;
  const int n = job->n_requests, N = job->n_gen;
  if (n < 0 || N < 1 || job->max_batch < 1 || job->max_tokens < 1) return ERNIE_EINVAL;
  if (job->max_batch > c.max_batch) return ERNIE_ECAPACITY;
  if (!job->prompt_offsets_host || !job->full_to_trimmed_host || !job->kept_ids_host) return ERNIE_EINVAL;
  if (n > 0 && (!job->prompt_ids_host || !job->tokens_out_host)) return ERNIE_EINVAL;
  if (!job->workspace_dev || (uintptr_t)job->workspace_dev % kAlign != 0 ||
      job->workspace_bytes < ernie_job_workspace_bytes(h, N))
    return ERNIE_EINVAL;
  std::vector<int32_t> lens(n);
  for (int q = 0; q < n; ++q) {
    const int64_t L = (int64_t)job->prompt_offsets_host[q + 1] - job->prompt_offsets_host[q];
    if (L < 1) return ERNIE_EINVAL;
    if (L > c.max_seq || L > c.max_pos || L + N - 1 > c.max_seq || L + N - 1 > c.max_pos) return ERNIE_ECAPACITY;
    lens[q] = (int32_t)L;
  }
  for (int v = 0; v < c.vocab_full; ++v)
    if (job->full_to_trimmed_host[v] < 0 || job->full_to_trimmed_host[v] >= c.vocab_kept) return ERNIE_EINVAL;
  const int64_t total_ids = n > 0 ? job->prompt_offsets_host[n] - job->prompt_offsets_host[0] : 0;
  for (int64_t i = 0; i < total_ids; ++i) {
    const int32_t id = job->prompt_ids_host[job->prompt_offsets_host[0] + i];
    if (id < 0 || id >= c.vocab_full) return ERNIE_EINVAL;
  }

  // main: inference order and batch sizes
  run.order.resize(n > 0 ? n : 1); run.starts.resize(n + 1);
  int32_t nb = 0;
  const int prc = ernie_plan_batches(lens.data(), n, job->max_batch, job->max_tokens, run.order.data(), run.starts.data(), &nb);
  if (prc != ERNIE_OK) return prc;
  run.n_batches = nb;

  // staging: pinned host buffers + device slices of the caller's workspace
  if (hipGetDevice(&run.device) != hipSuccess) return ERNIE_EHIP;
  const size_t l_cap = (size_t)(c.max_seq < c.max_pos ? c.max_seq : c.max_pos);
  const size_t ids_bytes = align_up((size_t)c.max_batch * l_cap * 4), tok_bytes = align_up((size_t)N * c.max_batch * 4);
  bool alloc_ok = true;
  for (int k = 0; k < kSlots; ++k) {
    Slot& s = run.slot[k];
    unsigned char* base = static_cast<unsigned char*>(job->workspace_dev) + (size_t)k * (ids_bytes + tok_bytes);
    s.ids_dev = reinterpret_cast<int32_t*>(base);
    s.tok_dev = reinterpret_cast<int32_t*>(base + ids_bytes);
    alloc_ok &= hipHostMalloc(reinterpret_cast<void**>(&s.ids_pinned), ids_bytes, hipHostMallocDefault) == hipSuccess;
    alloc_ok &= hipHostMalloc(reinterpret_cast<void**>(&s.lens_pinned), (size_t)c.max_batch * 4, hipHostMallocDefault) == hipSuccess;
    alloc_ok &= hipHostMalloc(reinterpret_cast<void**>(&s.tok_pinned), tok_bytes, hipHostMallocDefault) == hipSuccess;
    alloc_ok &= hipEventCreateWithFlags(&s.done, hipEventDisableTiming) == hipSuccess;
  }
  if (!alloc_ok) run.fail(ERNIE_EHIP);

  if (run.error.load() == ERNIE_OK && nb > 0) {
    if (!job->overlap) {
      Slot& s = run.slot[0];
      for (int i = 0; i < nb; ++i) {
        run.stage_pre(i, s);
        if (!run.stage_gpu(s) || !run.stage_post(s)) break;
      }
    } else {
      // Every worker walks the batches in order over slot i % 2 and leaves as soon as the run has failed,
      // so no wait can outlive an error.
      std::thread pre([&] {
        (void)hipSetDevice(run.device);
        for (int i = 0; i < nb; ++i) {
          Slot& s = run.slot[i % kSlots];
          if (!run.wait_state(s, FREE)) return;
          run.stage_pre(i, s);
          run.set_state(s, READY);
        }
      });
      std::thread gpu([&] {
        (void)hipSetDevice(run.device);
        for (int i = 0; i < nb; ++i) {
          Slot& s = run.slot[i % kSlots];
          if (!run.wait_state(s, READY)) return;
          if (!run.stage_gpu(s)) return;
          run.set_state(s, INFLIGHT);
        }
      });
      std::thread post([&] {
        (void)hipSetDevice(run.device);
        for (int i = 0; i < nb; ++i) {
          Slot& s = run.slot[i % kSlots];
          if (!run.wait_state(s, INFLIGHT)) return;
          if (!run.stage_post(s)) return;
          run.set_state(s, FREE);
        }
      });
      pre.join(); gpu.join(); post.join();
    }
  }
  // nothing of this call may still be running on the stream when the staging goes away
  if (hipStreamSynchronize(run.stream) != hipSuccess) run.fail(ERNIE_EHIP);
  for (int k = 0; k < kSlots; ++k) {
    Slot& s = run.slot[k];
    if (s.ids_pinned) (void)hipHostFree(s.ids_pinned);
    if (s.lens_pinned) (void)hipHostFree(s.lens_pinned);
    if (s.tok_pinned) (void)hipHostFree(s.tok_pinned);
    if (s.done) (void)hipEventDestroy(s.done);
  }
  if (stats_out) {
    stats_out->pre_s = run.pre_s; stats_out->enqueue_s = run.enqueue_s; stats_out->post_s = run.post_s;
    stats_out->wall_s = since(t_wall); stats_out->n_batches = nb;
  }
  return run.error.load();
}

}  // extern "C"

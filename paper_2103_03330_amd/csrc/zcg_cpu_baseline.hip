// The DMA-based method the paper compares against (Section 4.1.2 (b)): CPU
// threads gather rows into a dense pinned staging buffer, then a host-to-device
// copy moves it. Host code only; a small persistent thread pool keeps thread
// start-up out of the timed region.
#include <hip/hip_runtime_api.h>

#include <atomic>
#include <condition_variable>
#include <cstring>
#include <functional>
#include <mutex>
#include <thread>
#include <vector>

#include "zcg_internal.h"

namespace {

class ForkJoinPool {
 public:
  ~ForkJoinPool() { stop(); }

  // Runs fn(t, n) for t in [0, n) on n threads (the caller is thread 0).
  void run(int n, const std::function<void(int, int)>& fn) {
    std::lock_guard<std::mutex> call_lock(call_mu_);
    if (n <= 1) {
      fn(0, 1);
      return;
    }
    resize(n - 1);
    {
      std::lock_guard<std::mutex> lk(mu_);
      job_ = &fn;
      n_ = n;
      pending_ = n - 1;
      ++generation_;
    }
    cv_.notify_all();
    fn(0, n);
    std::unique_lock<std::mutex> lk(mu_);
    done_cv_.wait(lk, [&] { return pending_ == 0; });
    job_ = nullptr;
  }

 private:
  void resize(int workers) {
    if ((int)threads_.size() == workers) return;
    stop();
    quit_ = false;
    for (int i = 0; i < workers; ++i) {
      const uint64_t born = generation_;
      threads_.emplace_back([this, i, born] { worker(i + 1, born); });
    }
  }

  void stop() {
    {
      std::lock_guard<std::mutex> lk(mu_);
      quit_ = true;
    }
    cv_.notify_all();
    for (auto& t : threads_) t.join();
    threads_.clear();
  }

  void worker(int tid, uint64_t seen) {
    for (;;) {
      const std::function<void(int, int)>* job;
      int n;
      {
        std::unique_lock<std::mutex> lk(mu_);
        cv_.wait(lk, [&] { return quit_ || generation_ != seen; });
        if (quit_) return;
        seen = generation_;
        job = job_;
        n = n_;
      }
      (*job)(tid, n);
      {
        std::lock_guard<std::mutex> lk(mu_);
        if (--pending_ == 0) done_cv_.notify_one();
      }
    }
  }

  std::mutex call_mu_, mu_;
  std::condition_variable cv_, done_cv_;
  std::vector<std::thread> threads_;
  const std::function<void(int, int)>* job_ = nullptr;
  int n_ = 0, pending_ = 0;
  uint64_t generation_ = 0;
  bool quit_ = false;
};

ForkJoinPool& pool() {
  static ForkJoinPool* p = new ForkJoinPool;  // never destroyed: no join at process exit
  return *p;
}

int resolve_threads(int n_threads) {
  if (n_threads > 0) return n_threads > 1024 ? 1024 : n_threads;
  unsigned hc = std::thread::hardware_concurrency();
  return hc ? (int)hc : 1;
}

// Rows [lo, hi) of the list into the staging buffer, split evenly over the threads. Every thread
// checks the indices it is about to use (so the check costs no pass of its own over the list);
// returns false, with some rows not gathered, if any index is outside [0, n_rows).
bool gather_rows_cpu(const char* table, int64_t n_rows, int64_t row_bytes, const int64_t* idx,
                     int64_t lo, int64_t hi, char* staging, int n_threads) {
  std::atomic<bool> bad(false);
  std::atomic<bool>* bad_p = &bad;
  pool().run(n_threads, [=](int t, int n) {
    const int64_t span = hi - lo;
    const int64_t a = lo + span * t / n, b = lo + span * (t + 1) / n;
    constexpr int64_t kAhead = 12;  // rows whose first lines are requested ahead of their copy
    for (int64_t i = a; i < b; ++i) {
      const int64_t r = idx[i];
      if (r < 0 || r >= n_rows) {
        bad_p->store(true, std::memory_order_relaxed);
        return;
      }
      if (i + kAhead < b) {
        const int64_t ra = idx[i + kAhead];
        if (ra >= 0 && ra < n_rows) {
          const char* p = table + ra * row_bytes;
          __builtin_prefetch(p, 0, 0);
          if (row_bytes > 64) __builtin_prefetch(p + 64, 0, 0);
        }
      }
      std::memcpy(staging + i * row_bytes, table + r * row_bytes, (size_t)row_bytes);
    }
  });
  return !bad.load();
}

int check_call(const zcg_table* t, const int64_t* idx_host, int64_t n_idx, void* staging,
               void* out_dev) {
  if (!zcg_is_live(t)) return ZCG_EHANDLE;
  if (!t->host_resident || !t->host) return ZCG_EINVAL;
  if (n_idx < 0) return ZCG_EINVAL;
  if (n_idx > 0 && (!idx_host || !staging || !out_dev)) return ZCG_EINVAL;
  return ZCG_OK;
}

}  // namespace

extern "C" {

int zcg_cpu_gather_memcpy(const zcg_table* t, const int64_t* idx_host, int64_t n_idx,
                          void* staging_pinned, void* out_dev, int n_threads, void* stream) {
  int rc = check_call(t, idx_host, n_idx, staging_pinned, out_dev);
  if (rc || n_idx == 0) return rc;
  if (!gather_rows_cpu(static_cast<const char*>(t->host), t->n_rows, t->row_bytes, idx_host, 0, n_idx,
                       static_cast<char*>(staging_pinned), resolve_threads(n_threads)))
    return ZCG_ERANGE;  // nothing has been copied to the GPU
  hipError_t e = hipMemcpyAsync(out_dev, staging_pinned, (size_t)(n_idx * t->row_bytes),
                                hipMemcpyHostToDevice, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ZCG_OK : zcg_fail_hip(e);
}

int zcg_cpu_gather_memcpy_chunked(const zcg_table* t, const int64_t* idx_host, int64_t n_idx,
                                  void* staging_pinned, void* out_dev, int n_threads,
                                  int64_t chunk_rows, void* stream) {
  if (chunk_rows < 1) return ZCG_EINVAL;
  int rc = check_call(t, idx_host, n_idx, staging_pinned, out_dev);
  if (rc || n_idx == 0) return rc;
  const int nt = resolve_threads(n_threads);
  char* staging = static_cast<char*>(staging_pinned);
  char* out = static_cast<char*>(out_dev);
  for (int64_t lo = 0; lo < n_idx; lo += chunk_rows) {
    const int64_t hi = lo + chunk_rows < n_idx ? lo + chunk_rows : n_idx;
    if (!gather_rows_cpu(static_cast<const char*>(t->host), t->n_rows, t->row_bytes, idx_host, lo, hi,
                         staging, nt))
      return ZCG_ERANGE;  // earlier chunks may already be on their way to the GPU
    // the copy of this chunk runs while the CPU gathers the next one
    hipError_t e = hipMemcpyAsync(out + lo * t->row_bytes, staging + lo * t->row_bytes,
                                  (size_t)((hi - lo) * t->row_bytes), hipMemcpyHostToDevice,
                                  static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return zcg_fail_hip(e);
  }
  return ZCG_OK;
}

}  // extern "C"

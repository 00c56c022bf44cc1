// Bounded ring of transfer units in pinned memory and the CPU threads that move data between the
// ring and ordinary (pageable) host memory, so that the pinned footprint of layer-wise offloading
// stays a few units instead of a whole KV cache (paper Section 4: a CPU thread takes the KV cache
// from pinned to pageable memory; Section 3.2.3: a transfer is cut into smaller units).
//
// Nothing here calls the GPU runtime: "the unit's bytes are final" is a callable handed in with the
// job, which lets the same code run under a thread sanitizer on a machine without a GPU.
#pragma once

#include <atomic>
#include <chrono>
#include <condition_variable>
#include <cstdint>
#include <cstring>
#include <deque>
#include <functional>
#include <memory>
#include <mutex>
#include <thread>
#include <vector>

namespace lkv {

class HostTier {
 public:
  struct Latch {
    std::mutex m;
    std::condition_variable cv;
    int left = 0;
  };
  struct Job {
    std::function<bool()> ready;  // blocks until the copy below may start; false = the wait failed
    void *dst = nullptr;          // copy done by the worker after ready(); bytes == 0: none
    const void *src = nullptr;
    int64_t bytes = 0;
    int unit = -1;                // ring unit handed back after the copy; -1: none
    int key = -1;                 // completion group (a layer); -1: none
    std::shared_ptr<Latch> latch; // counted down when the job is done
  };

  HostTier() = default;
  HostTier(const HostTier &) = delete;
  HostTier &operator=(const HostTier &) = delete;
  ~HostTier() { stop(); }

  // ring: units*unit_bytes bytes owned by the caller, which outlive stop().
  void start(char *ring, int64_t unit_bytes, int units, int threads, int num_keys) {
    stop();
    std::lock_guard<std::mutex> g(m_);
    ring_ = ring;
    unit_bytes_ = unit_bytes;
    free_.clear();
    for (int u = units - 1; u >= 0; --u) free_.push_back(u);  // unit 0 handed out first
    units_ = units;
    pending_.assign((size_t)num_keys, 0);
    pending_total_ = 0;
    failed_ = false;
    quit_ = false;
    for (int t = 0; t < threads; ++t) workers_.emplace_back([this] { work(); });
  }

  // Finishes every queued job, then joins the threads.
  void stop() {
    {
      std::lock_guard<std::mutex> g(m_);
      if (workers_.empty()) return;
      quit_ = true;
    }
    cv_job_.notify_all();
    for (auto &w : workers_) w.join();
    workers_.clear();
  }

  bool running() const { return !workers_.empty(); }
  int64_t unit_bytes() const { return unit_bytes_; }
  int units() const { return units_; }
  int threads() const { return (int)workers_.size(); }
  char *unit_ptr(int u) const { return ring_ + (int64_t)u * unit_bytes_; }

  // Takes a free unit, waiting for a worker to hand one back when all are in use.  Every unit taken
  // must come back through a submitted job or release(), or later callers wait for ever.
  int acquire() {
    std::unique_lock<std::mutex> lk(m_);
    if (free_.empty()) {
      auto t0 = std::chrono::steady_clock::now();
      cv_unit_.wait(lk, [this] { return !free_.empty(); });
      ring_wait_ns_ += std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now() - t0).count();
    }
    int u = free_.back();
    free_.pop_back();
    return u;
  }

  void release(int unit) {
    {
      std::lock_guard<std::mutex> g(m_);
      free_.push_back(unit);
    }
    cv_unit_.notify_one();
  }

  void submit(Job j) {
    {
      std::lock_guard<std::mutex> g(m_);
      if (j.key >= 0) pending_[(size_t)j.key] += 1;
      pending_total_ += 1;
      jobs_.push_back(std::move(j));
    }
    cv_job_.notify_one();
  }

  // Blocks until every job submitted so far under key has finished.  False once any job's wait failed.
  bool wait_key(int key) {
    std::unique_lock<std::mutex> lk(m_);
    cv_done_.wait(lk, [&] { return pending_[(size_t)key] == 0; });
    return !failed_;
  }
  bool busy_key(int key) {
    std::lock_guard<std::mutex> g(m_);
    return pending_[(size_t)key] != 0;
  }
  bool wait_all() {
    std::unique_lock<std::mutex> lk(m_);
    cv_done_.wait(lk, [&] { return pending_total_ == 0; });
    return !failed_;
  }
  bool failed() {
    std::lock_guard<std::mutex> g(m_);
    return failed_;
  }

  // memcpy split over the workers and the calling thread; returns when all of it is done.
  void copy_parallel(void *dst, const void *src, int64_t bytes) {
    const int64_t kPiece = (int64_t)4 << 20;
    int pieces = (int)((bytes + kPiece - 1) / kPiece);
    int lanes = threads() + 1;
    if (pieces < lanes) lanes = pieces < 1 ? 1 : pieces;
    if (lanes <= 1) {
      std::memcpy(dst, src, (size_t)bytes);
      return;
    }
    int64_t per = ((bytes + lanes - 1) / lanes + 63) & ~(int64_t)63;
    auto latch = std::make_shared<Latch>();
    int64_t off = per;
    for (int l = 1; l < lanes && off < bytes; ++l, off += per) {
      Job j;
      j.dst = (char *)dst + off;
      j.src = (const char *)src + off;
      j.bytes = bytes - off < per ? bytes - off : per;
      j.latch = latch;
      {
        std::lock_guard<std::mutex> g(latch->m);
        latch->left += 1;
      }
      submit(std::move(j));
    }
    std::memcpy(dst, src, (size_t)(per < bytes ? per : bytes));
    std::unique_lock<std::mutex> lk(latch->m);
    latch->cv.wait(lk, [&] { return latch->left == 0; });
  }

  int64_t copied_bytes() const { return copied_bytes_.load(); }
  int64_t copy_ns() const { return copy_ns_.load(); }
  int64_t ring_wait_ns() {
    std::lock_guard<std::mutex> g(m_);
    return ring_wait_ns_;
  }

 private:
  void work() {
    for (;;) {
      Job j;
      {
        std::unique_lock<std::mutex> lk(m_);
        cv_job_.wait(lk, [this] { return quit_ || !jobs_.empty(); });
        if (jobs_.empty()) return;  // quit_ and nothing left
        j = std::move(jobs_.front());
        jobs_.pop_front();
      }
      bool ok = !j.ready || j.ready();
      if (ok && j.bytes > 0) {
        auto t0 = std::chrono::steady_clock::now();
        std::memcpy(j.dst, j.src, (size_t)j.bytes);
        copy_ns_ += std::chrono::duration_cast<std::chrono::nanoseconds>(std::chrono::steady_clock::now() - t0).count();
        copied_bytes_ += j.bytes;
      }
      {
        std::lock_guard<std::mutex> g(m_);
        if (!ok) failed_ = true;
        if (j.unit >= 0) free_.push_back(j.unit);
        if (j.key >= 0) pending_[(size_t)j.key] -= 1;
        pending_total_ -= 1;
      }
      if (j.unit >= 0) cv_unit_.notify_one();
      cv_done_.notify_all();
      if (j.latch) {
        std::lock_guard<std::mutex> g(j.latch->m);
        j.latch->left -= 1;
        j.latch->cv.notify_all();
      }
    }
  }

  std::mutex m_;
  std::condition_variable cv_job_, cv_unit_, cv_done_;
  std::deque<Job> jobs_;
  std::vector<int> free_;
  std::vector<int> pending_;
  int64_t pending_total_ = 0;
  bool failed_ = false, quit_ = false;
  char *ring_ = nullptr;
  int64_t unit_bytes_ = 0;
  int units_ = 0;
  int64_t ring_wait_ns_ = 0;
  std::atomic<int64_t> copied_bytes_{0}, copy_ns_{0};
  std::vector<std::thread> workers_;
};

}  // namespace lkv

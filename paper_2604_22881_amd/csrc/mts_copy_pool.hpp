// Host-only helper of the transfer pipeline (no HIP): a pool of threads that splits one memcpy.
// Kept in a header of its own so that it also builds, alone, under the thread sanitizer.
#pragma once
#include <string.h>

#include <atomic>
#include <chrono>
#include <condition_variable>
#include <mutex>
#include <thread>
#include <vector>

namespace mts {

// n-way memcpy: the calling thread takes the first slice, n-1 helpers the others.  A run is a
// couple of megabytes, i.e. tens of microseconds per slice, so waking helpers through a
// condition variable would cost as much as the copy: between the copies of one task the helpers
// poll a generation counter (for at most kSpin), and only then go to sleep.
class CopyPool {
 public:
  explicit CopyPool(int n) : n_(n < 1 ? 1 : n) {
    for (int i = 1; i < n_; ++i) helpers_.emplace_back([this, i] { loop(i); });
  }
  ~CopyPool() {
    {
      std::lock_guard<std::mutex> g(mu_);
      stop_.store(true);
    }
    cv_.notify_all();
    for (auto& t : helpers_) t.join();
  }
  void copy(void* dst, const void* src, size_t bytes) {
    const size_t min_slice = 128 * 1024;
    int parts = (int)((bytes + min_slice - 1) / min_slice);
    if (parts > n_) parts = n_;
    if (parts <= 1) {
      memcpy(dst, src, bytes);
      return;
    }
    dst_ = static_cast<char*>(dst);
    src_ = static_cast<const char*>(src);
    bytes_ = bytes;
    parts_ = parts;
    left_.store(n_ - 1, std::memory_order_relaxed);   // every helper acknowledges every generation
    {
      std::lock_guard<std::mutex> g(mu_);          // pairs with the helpers' sleep: no lost wake-up
      gen_.fetch_add(1, std::memory_order_release);
    }
    cv_.notify_all();
    slice(0, parts, dst_, src_, bytes);
    while (left_.load(std::memory_order_acquire) != 0) cpu_relax();   // equal slices: a short wait
  }

 private:
  static void cpu_relax() {
#if defined(__x86_64__)
    __builtin_ia32_pause();
#endif
  }
  static void slice(int i, int parts, char* dst, const char* src, size_t bytes) {
    const size_t per = (bytes / parts + 63) & ~(size_t)63;
    const size_t lo = (size_t)i * per;
    if (lo >= bytes) return;
    const size_t n = (i == parts - 1 || lo + per > bytes) ? bytes - lo : per;
    memcpy(dst + lo, src + lo, n);
  }
  void loop(int i) {
    uint64_t seen = 0;
    for (;;) {
      // poll first, sleep if nothing comes
      const auto t0 = std::chrono::steady_clock::now();
      while (gen_.load(std::memory_order_acquire) == seen && !stop_.load(std::memory_order_relaxed)) {
        cpu_relax();
        if (std::chrono::steady_clock::now() - t0 > kSpin) {
          std::unique_lock<std::mutex> g(mu_);
          cv_.wait(g, [&] { return stop_.load() || gen_.load(std::memory_order_acquire) != seen; });
          break;
        }
      }
      if (stop_.load()) return;
      seen = gen_.load(std::memory_order_acquire);
      // The fields below were written before gen_ was bumped and stay put until left_ reaches
      // 0, which needs this helper's acknowledgement too: no helper is ever a generation behind.
      if (i < parts_) slice(i, parts_, dst_, src_, bytes_);
      left_.fetch_sub(1, std::memory_order_release);
    }
  }
  static constexpr std::chrono::microseconds kSpin{50};
  const int n_;
  std::vector<std::thread> helpers_;
  std::mutex mu_;
  std::condition_variable cv_;
  std::atomic<bool> stop_{false};
  std::atomic<uint64_t> gen_{0};
  std::atomic<int> left_{0};
  char* dst_ = nullptr;
  const char* src_ = nullptr;
  size_t bytes_ = 0;
  int parts_ = 0;
};

}  // namespace mts

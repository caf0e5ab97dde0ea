// The thread that makes a driver-mapped pool's driver calls, and the queue that feeds it.
//
// The paper takes its virtual-memory calls off the critical path (Sec. 3.1: chunks are mapped ahead
// of their first use, unmapping happens beside the computation). Here every such call is a job; the
// pool's thread works the jobs off strictly in the order they were pushed, so a chunk that leaves
// one tensor's range and enters another's is unmapped before it is mapped again, and "job n is
// done" implies that every job before it is done. The thread that pushes never calls the driver.
//
// The driver is a template parameter (the pool passes the HIP calls, the CPU tests a stand-in), so
// that the ordering and the waiting can be run under ThreadSanitizer without a GPU. It provides
//   int  wait_event(void* ev)           wait for, then dispose of, an event        (0 or an error code)
//   int  map(char* at, void* handle)    map the chunk at `at` and make it usable   (0 or an error code)
//   int  unmap(char* at)                                                           (0 or an error code)
//   const char* last_call()             name of the call that returned the last error
//   void thread_begin()                 called once on the new thread
#pragma once
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <cstdint>
#include <deque>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

namespace ellm {

struct MapJob {
  char* at;          // address in a tensor's range
  void* handle;      // chunk to map there (map jobs)
  bool unmap;
  void* after;       // not NULL: an event behind the kernels that may still read `at`; waited for first
};

template <class Driver>
class MapQueue {
 public:
  explicit MapQueue(Driver d) : drv_(d) {}
  MapQueue(const MapQueue&) = delete;
  MapQueue& operator=(const MapQueue&) = delete;
  ~MapQueue() { stop(); }

  void start() { thread_ = std::thread(&MapQueue::run, this); }
  bool running() const { return thread_.joinable(); }

  // Jobs go to the thread in the given order, numbered from last() + 1. Returns the number of the last one.
  uint64_t push(const std::vector<MapJob>& jobs) {
    {
      std::lock_guard<std::mutex> lk(mu_);
      for (const MapJob& j : jobs) queue_.push_back(j);
      pushed_ += jobs.size();
    }
    cv_work_.notify_one();
    return pushed_;
  }
  uint64_t last() const { return pushed_; }      // pushing thread only

  // jobs finished; once this is >= n, failed() tells whether any job up to n met an error
  uint64_t done() const { return done_.load(std::memory_order_acquire); }
  bool failed() const { return failed_.load(std::memory_order_acquire); }

  // Wait until job `seq` is done. Returns 0, or the first error any job has met so far (sticky) with
  // the name of the call in *where. After an error the queue is still worked off, so that nobody
  // waits for ever, but the driver is not asked for anything more.
  int wait(uint64_t seq, std::string* where) {
    if (done() < seq) {
      const auto t0 = std::chrono::steady_clock::now();
      std::unique_lock<std::mutex> lk(mu_);
      cv_done_.wait(lk, [&] { return done() >= seq; });
      waited_us_ += std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - t0).count();
    }
    std::lock_guard<std::mutex> lk(mu_);
    if (error_ && where) *where = error_where_;
    return error_;
  }

  // works off what is queued, then ends the thread
  void stop() {
    if (!thread_.joinable()) return;
    {
      std::lock_guard<std::mutex> lk(mu_);
      stop_ = true;
    }
    cv_work_.notify_one();
    thread_.join();
  }

  // The pushing thread met an error of its own that leaves mappings missing (it could not prepare a
  // job): recorded like a job's error, so that every later wait() reports it and failed() is set.
  void fail_now(int code, const char* where) {
    std::lock_guard<std::mutex> lk(mu_);
    if (!error_) {
      error_ = code;
      error_where_ = where;
    }
    failed_.store(true, std::memory_order_release);
  }

  // test hook: the n-th map job from now is not made and counts as refused by the driver (0: none)
  void fail_map_in(int n) { fail_in_.store(n); }

  // statistics: the first four are the thread's and are complete once wait(last()) has returned
  int64_t maps = 0, unmaps = 0;
  double map_us = 0, unmap_us = 0;
  double waited_us() const { return waited_us_; }   // time callers spent in wait() (pushing thread only)

 private:
  void run() {
    using clk = std::chrono::steady_clock;
    auto us_since = [](clk::time_point t0) { return std::chrono::duration<double, std::micro>(clk::now() - t0).count(); };
    drv_.thread_begin();
    uint64_t n = 0;
    for (;;) {
      MapJob job;
      {
        std::unique_lock<std::mutex> lk(mu_);
        cv_work_.wait(lk, [&] { return stop_ || !queue_.empty(); });
        if (queue_.empty()) return;          // asked to stop, nothing left to do
        job = queue_.front();
        queue_.pop_front();
      }
      int e = 0;
      const char* where = "";
      if (job.after) {
        e = drv_.wait_event(job.after);
        where = "wait for the kernels before an unmap";
      }
      if (e == 0 && !failed_.load(std::memory_order_relaxed)) {
        if (!job.unmap && fail_in_.load() > 0 && fail_in_.fetch_sub(1) == 1) {
          e = -1;
          where = "map: refused (debug hook)";
        } else {
          const auto t0 = clk::now();
          if (job.unmap) {
            e = drv_.unmap(job.at);
            unmap_us += us_since(t0);
            unmaps++;
          } else {
            e = drv_.map(job.at, job.handle);
            map_us += us_since(t0);
            maps++;
          }
          if (e) where = drv_.last_call();
        }
      }
      {
        std::lock_guard<std::mutex> lk(mu_);
        if (e && !error_) {
          error_ = e;
          error_where_ = where;
          failed_.store(true, std::memory_order_release);   // before the count below: see done()
        }
        done_.store(++n, std::memory_order_release);
      }
      cv_done_.notify_all();
    }
  }

  Driver drv_;
  std::thread thread_;
  std::mutex mu_;
  std::condition_variable cv_work_, cv_done_;
  std::deque<MapJob> queue_;           // guarded by mu_
  bool stop_ = false;                  // guarded by mu_
  int error_ = 0;                      // guarded by mu_
  std::string error_where_;            // guarded by mu_
  std::atomic<uint64_t> done_{0};
  std::atomic<bool> failed_{false};
  std::atomic<int> fail_in_{0};
  uint64_t pushed_ = 0;                // pushing thread only
  double waited_us_ = 0;               // pushing thread only
};

}  // namespace ellm

// The mapper thread of driver-mapped pools (csrc/map_queue.hpp) with a stand-in for the driver, built
// with ThreadSanitizer / AddressSanitizer by tests/test_sanitizers.py: jobs are carried out in the
// order they were pushed; wait(n) returns when job n is done and not before an event it depends on;
// an error is sticky, stops further driver calls and is visible to whoever sees the job as done;
// stopping works off what is queued.
#include <atomic>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <thread>
#include <vector>

#include "map_queue.hpp"

namespace {

struct Shared {                      // the stand-in driver's state: touched by the mapper thread only,
  std::map<char*, void*> mapped;     // read by the main thread after a full wait
  std::vector<char*> order;          // addresses in the order the calls were made
  int bad = 0;                       // calls that made no sense (map of a mapped address, ...)
  int events = 0;
};

struct FakeDriver {
  Shared* sh;
  unsigned state = 12345u;
  const char* call = "";
  void thread_begin() {}
  void dawdle() {
    state = state * 1664525u + 1013904223u;
    if ((state >> 28) == 0) std::this_thread::sleep_for(std::chrono::microseconds(50));
  }
  int wait_event(void* ev) {
    auto* flag = static_cast<std::atomic<int>*>(ev);
    while (!flag->load(std::memory_order_acquire)) std::this_thread::yield();
    sh->events++;
    call = "fake wait";
    return 0;
  }
  int map(char* at, void* handle) {
    dawdle();
    call = "fake map";
    if (handle == nullptr) return 7;                 // a handle the driver refuses
    if (sh->mapped.count(at)) sh->bad++;
    sh->mapped[at] = handle;
    sh->order.push_back(at);
    return 0;
  }
  int unmap(char* at) {
    dawdle();
    call = "fake unmap";
    if (!sh->mapped.count(at)) sh->bad++;
    sh->mapped.erase(at);
    sh->order.push_back(at);
    return 0;
  }
  const char* last_call() const { return call; }
};

void die(const char* what, long a = 0, long b = 0) {
  std::printf("FAILED: %s (%ld, %ld)\n", what, a, b);
  std::exit(1);
}

}  // namespace

int main(int argc, char** argv) {
  const unsigned seed = argc > 1 ? (unsigned)std::atoi(argv[1]) : 1u;
  const int rounds = argc > 2 ? std::atoi(argv[2]) : 400;
  unsigned rs = seed * 2654435761u + 1u;
  auto rnd = [&](unsigned n) { rs = rs * 1664525u + 1013904223u; return (rs >> 8) % n; };
  static char space[64];              // 64 addresses
  static int handles[64];
  static std::atomic<int> flags[4096];

  // 1. order, waits, events
  {
    Shared sh;
    ellm::MapQueue<FakeDriver> q(FakeDriver{&sh});
    q.start();
    std::map<char*, void*> model;                    // what the pushed jobs amount to
    std::vector<char*> pushed;
    std::vector<std::pair<uint64_t, std::atomic<int>*>> pending;   // (job number, its event) not yet signalled
    int n_flags = 0, n_events = 0;
    for (int r = 0; r < rounds; r++) {
      std::vector<ellm::MapJob> jobs;
      const int n = 1 + (int)rnd(5);
      for (int i = 0; i < n; i++) {
        char* at = space + rnd(64);
        if (model.count(at)) {
          void* ev = nullptr;
          if (rnd(3) == 0 && n_flags < 4096) { ev = &flags[n_flags++]; n_events++; }
          jobs.push_back({at, nullptr, true, ev});
          model.erase(at);
        } else {
          void* h = handles + rnd(64);
          jobs.push_back({at, h, false, nullptr});
          model[at] = h;
        }
        pushed.push_back(at);
      }
      const uint64_t before = q.last();
      const uint64_t last = q.push(jobs);
      if (last != before + jobs.size()) die("job numbers", (long)last, (long)before);
      for (size_t i = 0; i < jobs.size(); i++)
        if (jobs[i].after) pending.push_back({before + i + 1, static_cast<std::atomic<int>*>(jobs[i].after)});
      // a job behind an unsignalled event cannot be done yet
      if (!pending.empty() && q.done() >= pending.front().first) die("a job ran before its event", (long)q.done());
      if (rnd(2) == 0) {
        // signal the events ("the kernels have finished"), then wait for some job already pushed
        for (auto& pe : pending) pe.second->store(1, std::memory_order_release);
        pending.clear();
        const uint64_t target = last - rnd((unsigned)std::min<uint64_t>(last, 6));
        std::string where;
        if (q.wait(target, &where) != 0) die("unexpected error");
        if (q.done() < target) die("wait returned early", (long)q.done(), (long)target);
      }
    }
    for (auto& pe : pending) pe.second->store(1, std::memory_order_release);
    std::string where;
    if (q.wait(q.last(), &where) != 0 || q.failed()) die("unexpected error at the end");
    if (sh.bad) die("calls out of order", sh.bad);
    if (sh.order != pushed) die("order of the calls differs from the order of the pushes");
    if (sh.mapped != model) die("final mappings differ");
    if (sh.events != n_events) die("events waited for", sh.events, n_events);
    if (q.maps + q.unmaps != (int64_t)pushed.size()) die("statistics", (long)(q.maps + q.unmaps), (long)pushed.size());
    q.stop();
    if (q.running()) die("still running after stop");
  }
  // 2. an error: sticky, visible with the count, nothing more asked of the driver; stop drains
  {
    Shared sh;
    auto* q = new ellm::MapQueue<FakeDriver>(FakeDriver{&sh});
    q->start();
    std::vector<ellm::MapJob> jobs;
    for (int i = 0; i < 10; i++) jobs.push_back({space + i, i == 4 ? nullptr : (void*)(handles + i), false, nullptr});
    const uint64_t last = q->push(jobs);
    std::string where;
    const int early = q->wait(4, &where);             // 0, or 7 already if the thread has got to job 5 by now
    if (early != 0 && early != 7) die("wait(4)", early);
    if (q->wait(5, &where) != 7 || where != "fake map") die("error not reported");
    if (!q->failed()) die("failed() not set although the job counts as done");
    if (q->wait(last, &where) != 7) die("error not sticky");
    jobs.clear();
    for (int i = 10; i < 40; i++) jobs.push_back({space + i, (void*)(handles + i), false, nullptr});
    q->push(jobs);
    delete q;                                         // works the 30 jobs off (without calling the driver), joins
    if (sh.mapped.size() != 4) die("driver called after an error", (long)sh.mapped.size());
  }
  // 3. the hook that refuses the n-th mapping
  {
    Shared sh;
    ellm::MapQueue<FakeDriver> q(FakeDriver{&sh});
    q.start();
    q.fail_map_in(3);
    std::vector<ellm::MapJob> jobs;
    for (int i = 0; i < 6; i++) jobs.push_back({space + i, (void*)(handles + i), false, nullptr});
    std::string where;
    if (q.wait(q.push(jobs), &where) != -1 || where.find("refused") == std::string::npos) die("hook");
    if (sh.mapped.size() != 2) die("hook: mappings made", (long)sh.mapped.size());
  }
  // 4. an error of the pushing thread's own is reported like a job's
  {
    Shared sh;
    ellm::MapQueue<FakeDriver> q(FakeDriver{&sh});
    q.start();
    std::vector<ellm::MapJob> jobs = {{space, (void*)handles, false, nullptr}};
    std::string where;
    if (q.wait(q.push(jobs), &where) != 0 || q.failed()) die("clean start");
    q.fail_now(9, "reserve");
    if (!q.failed() || q.wait(0, &where) != 9 || where != "reserve") die("fail_now");
    jobs[0].at = space + 1;
    if (q.wait(q.push(jobs), &where) != 9 || sh.mapped.size() != 1) die("driver called after fail_now");
  }
  std::printf("mapper queue behaves\n");
  return 0;
}

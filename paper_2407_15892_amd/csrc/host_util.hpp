// Host-side helpers shared by the library sources: per-kernel event timing and small checks.
// Each shared library that includes this header owns its own profiler instance.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <mutex>
#include <vector>

namespace mst_host {

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) != 0; }

// Runs a set-up step once per HIP device and remembers whether it worked: kernel attributes such as the
// dynamic LDS limit belong to the device a kernel's code object is loaded on, not to the process.
struct PerDeviceOnce {
  static constexpr int kMaxDevices = 64;
  std::mutex mu;
  signed char state[kMaxDevices] = {};   // 0 = not run yet, 1 = done, -1 = failed
  template <class F>
  bool run(int dev, F step) {
    if (dev < 0 || dev >= kMaxDevices) return step();   // beyond the table: repeat the step on every call
    std::lock_guard<std::mutex> lk(mu);
    if (state[dev] == 0) state[dev] = step() ? 1 : -1;
    return state[dev] > 0;
  }
};

// Per-launch timing with HIP events.  `every` = n brackets every n-th launch of each kind (the first, the n + 1st, ...):
// events between launches cost a few microseconds each on the stream, about half a percent of a step made of 100
// GEMM launches when every launch carries them; `issued` counts all launches of a kind while timing is on.
struct Profiler {
  static constexpr int kMaxKinds = 32;
  std::mutex mu;
  std::atomic<int> every{0};               // 0 = off
  int64_t issued[kMaxKinds] = {};
  struct Rec { int kind; hipEvent_t a, b; };
  std::vector<Rec> recs;
  std::vector<hipEvent_t> pool;
  hipEvent_t get() {
    if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
  void enable(int n) {
    every.store(n > 0 ? n : 0);
  }
  // adds elapsed ms / counts of timed launches / counts of all launches per kind, clears the record; false if an
  // event could not be read
  bool collect(int n_kinds, double* ms_per_kind, int64_t* launches_per_kind, int64_t* issued_per_kind) {
    std::lock_guard<std::mutex> lk(mu);
    bool ok = true;
    for (int k = 0; k < n_kinds && k < kMaxKinds; ++k) {
      if (issued_per_kind) issued_per_kind[k] += issued[k];
      issued[k] = 0;
    }
    for (auto& r : recs) {
      float ms = 0.f;
      if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) ok = false;
      if (r.kind >= 0 && r.kind < n_kinds) {
        if (ms_per_kind) ms_per_kind[r.kind] += ms;
        if (launches_per_kind) launches_per_kind[r.kind] += 1;
      }
      pool.push_back(r.a);
      pool.push_back(r.b);
    }
    recs.clear();
    return ok;
  }
};

struct Scope {   // brackets one launch with events when profiling is on
  Profiler& pr; hipStream_t st; int kind; hipEvent_t a = nullptr, b = nullptr; bool on;
  Scope(Profiler& p, hipStream_t s, int k) : pr(p), st(s), kind(k), on(false) {
    const int every = p.every.load();
    if (every <= 0) return;
    std::lock_guard<std::mutex> lk(pr.mu);
    const int64_t seen = (k >= 0 && k < Profiler::kMaxKinds) ? pr.issued[k]++ : 0;
    on = seen % every == 0;
    if (!on) return;
    a = pr.get(); b = pr.get();
    if (a) (void)hipEventRecord(a, st);
  }
  ~Scope() {
    if (!on) return;
    if (b) (void)hipEventRecord(b, st);
    std::lock_guard<std::mutex> lk(pr.mu);
    if (a && b) pr.recs.push_back({kind, a, b});
    else {   // an event could not be created: this launch goes unrecorded
      if (a) pr.pool.push_back(a);
      if (b) pr.pool.push_back(b);
    }
  }
};

}  // namespace mst_host

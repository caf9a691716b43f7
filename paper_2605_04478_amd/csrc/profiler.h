// Optional per-kernel-class timing with HIP events on the context's stream.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <vector>

namespace ccld {

constexpr int PROF_NCLASS = 16;

struct Profiler {
  bool on = false;
  hipStream_t st = nullptr;
  std::vector<hipEvent_t> pool;
  struct Span { int cls; size_t e0, e1; };
  std::vector<Span> spans;
  size_t used = 0, cur = 0;
  double ms[PROF_NCLASS] = {0};
  uint64_t cnt[PROF_NCLASS] = {0};

  bool enable(hipStream_t stream, bool want) {
    st = stream;
    for (int i = 0; i < PROF_NCLASS; ++i) { ms[i] = 0; cnt[i] = 0; }
    spans.clear(); used = 0;
    if (want && pool.empty()) {
      pool.resize(1024);
      for (auto& e : pool) if (hipEventCreate(&e) != hipSuccess) { pool.clear(); on = false; return false; }
    }
    on = want;
    return true;
  }
  bool room() const { return on && used + 2 <= pool.size(); }
  void begin() { if (room()) { (void)hipEventRecord(pool[used], st); cur = used++; } }
  void end(int cls) {
    if (!room()) return;
    (void)hipEventRecord(pool[used], st);
    spans.push_back({cls, cur, used});
    ++used;
  }
  // ends the current span and begins the next one with a single event
  void split(int cls) {
    if (!room()) return;
    (void)hipEventRecord(pool[used], st);
    spans.push_back({cls, cur, used});
    cur = used++;
  }
  // after the stream has been synchronised
  void collect() {
    for (const Span& s : spans) {
      float t = 0;
      if (hipEventElapsedTime(&t, pool[s.e0], pool[s.e1]) == hipSuccess) { ms[s.cls] += t; cnt[s.cls] += 1; }
    }
    spans.clear(); used = 0;
  }
  void destroy() { for (auto& e : pool) (void)hipEventDestroy(e); pool.clear(); on = false; }
};

}  // namespace ccld

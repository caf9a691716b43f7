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
  bool open = false;
  int only = -1;             // -1: every class
  double ms[PROF_NCLASS] = {0};
  uint64_t cnt[PROF_NCLASS] = {0};

  bool enable(hipStream_t stream, bool want, int only_class = -1) {
    st = stream;
    only = only_class; open = false;
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
  bool wanted(int cls) const { return only < 0 || cls == only; }
  // A span is timed if its class is wanted (every class, or the one class asked for: a record costs
  // several microseconds on the stream, so a caller that needs one class does not pay for the others).
  void begin(int cls) {
    open = false;
    if (!room() || !wanted(cls)) return;
    (void)hipEventRecord(pool[used], st);
    cur = used++;
    open = true;
  }
  void end(int cls) {
    if (!open || !room()) { open = false; return; }
    (void)hipEventRecord(pool[used], st);
    spans.push_back({cls, cur, used});
    ++used;
    open = false;
  }
  // ends the span of cls_end and begins the span of cls_next with a single event
  void split(int cls_end, int cls_next) {
    const bool need_end = open, need_begin = wanted(cls_next);
    if (!need_end && !need_begin) return;
    if (!room()) { open = false; return; }
    (void)hipEventRecord(pool[used], st);
    if (need_end) spans.push_back({cls_end, cur, used});
    open = need_begin;
    if (need_begin) cur = used;
    ++used;
  }
  // after the stream has been synchronised
  void collect() {
    for (const Span& s : spans) {
      float t = 0;
      if (hipEventElapsedTime(&t, pool[s.e0], pool[s.e1]) == hipSuccess) { ms[s.cls] += t; cnt[s.cls] += 1; }
    }
    spans.clear(); used = 0;
  }
  // after an error return: the recorded spans are dropped unread
  void abandon() { spans.clear(); used = 0; open = false; }
  void destroy() { for (auto& e : pool) (void)hipEventDestroy(e); pool.clear(); on = false; }
};

}  // namespace ccld

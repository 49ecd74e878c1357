// Per-kernel timing with HIP events recorded on the launch stream.
#include <string.h>

#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "xsm_internal.h"

namespace xsm {
namespace {
struct Rec { const char* name; hipEvent_t a, b; };
struct Tracer {
  bool on = false;
  std::vector<Rec> recs;
  std::vector<hipEvent_t> pool;
  std::mutex mu;
} g_tr;

hipEvent_t take_event() {
  if (!g_tr.pool.empty()) { hipEvent_t e = g_tr.pool.back(); g_tr.pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}
}  // namespace

TraceScope::TraceScope(const char* name, hipStream_t s) : s_(s), idx_(-1) {
  if (!g_tr.on) return;
  std::lock_guard<std::mutex> lk(g_tr.mu);
  Rec r{name, take_event(), take_event()};
  if (!r.a || !r.b) return;
  (void)hipEventRecord(r.a, s);
  idx_ = (int)g_tr.recs.size();
  g_tr.recs.push_back(r);
}
TraceScope::~TraceScope() {
  if (idx_ < 0) return;
  std::lock_guard<std::mutex> lk(g_tr.mu);
  (void)hipEventRecord(g_tr.recs[idx_].b, s_);
}
}  // namespace xsm

extern "C" {

XSM_API void xsm_debug_trace_enable(int on) {
  std::lock_guard<std::mutex> lk(xsm::g_tr.mu);
  xsm::g_tr.on = on != 0;
}

// Synchronises the device, writes one line "name count total_ms" per kernel class
// into buf (NUL-terminated, truncated to cap), clears the records.  Returns the
// number of classes.
XSM_API int xsm_debug_trace_report(char* buf, size_t cap) {
  using namespace xsm;
  if (hipDeviceSynchronize() != hipSuccess) return -1;
  std::lock_guard<std::mutex> lk(g_tr.mu);
  std::map<std::string, std::pair<long, double>> agg;
  for (const Rec& r : g_tr.recs) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) {
      auto& e = agg[r.name];
      e.first += 1;
      e.second += ms;
    }
    g_tr.pool.push_back(r.a);
    g_tr.pool.push_back(r.b);
  }
  g_tr.recs.clear();
  std::string out;
  for (auto& kv : agg)
    out += kv.first + " " + std::to_string(kv.second.first) + " " + std::to_string(kv.second.second) + "\n";
  if (buf && cap > 0) {
    const size_t n = out.size() < cap - 1 ? out.size() : cap - 1;
    memcpy(buf, out.data(), n);
    buf[n] = 0;
  }
  return (int)agg.size();
}

}  // extern "C"

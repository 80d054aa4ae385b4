// Thread-local error message and the optional kernel timing aid of libumas.
#include <map>
#include <string>
#include <vector>

#include "umas_common.h"

namespace umas {
namespace {
thread_local char g_msg[512] = "";

struct Interval {
  const char* name;
  hipEvent_t begin, end;
};
std::vector<Interval> g_intervals;
std::vector<hipEvent_t> g_events;
hipEvent_t g_last = nullptr;
constexpr size_t kMaxIntervals = 1 << 16;

hipEvent_t new_event(hipStream_t st) {
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  g_events.push_back(e);
  if (hipEventRecord(e, st) != hipSuccess) return nullptr;
  return e;
}
void reset() {
  for (hipEvent_t e : g_events) (void)hipEventDestroy(e);
  g_events.clear();
  g_intervals.clear();
  g_last = nullptr;
}
}  // namespace

bool g_prof_on = false;

umas_status fail(umas_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_msg, sizeof(g_msg), fmt, ap);
  va_end(ap);
  return code;
}

void prof_mark(hipStream_t st) {
  if (!g_prof_on) return;
  g_last = new_event(st);
}

void prof_kernel(const char* name, hipStream_t st) {
  if (!g_prof_on || g_intervals.size() >= kMaxIntervals) return;
  hipEvent_t e = new_event(st);
  if (g_last && e) g_intervals.push_back(Interval{name, g_last, e});
  g_last = e;
}
}  // namespace umas

extern "C" const char* umas_last_error(void) { return umas::g_msg; }

extern "C" umas_status umas_profile_enable(int32_t on) {
  umas::reset();
  umas::g_prof_on = on != 0;
  return UMAS_OK;
}

extern "C" int32_t umas_profile_read(char* names, float* total_ms, int32_t* launches, int32_t cap) {
  using namespace umas;
  std::map<std::string, std::pair<double, int>> agg;
  std::vector<std::string> order;
  for (const Interval& iv : g_intervals) {
    if (hipEventSynchronize(iv.end) != hipSuccess) return -1;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, iv.begin, iv.end) != hipSuccess) return -1;
    auto it = agg.find(iv.name);
    if (it == agg.end()) {
      order.push_back(iv.name);
      agg[iv.name] = {ms, 1};
    } else {
      it->second.first += ms;
      it->second.second += 1;
    }
  }
  int32_t n = 0;
  for (const std::string& k : order) {
    if (n >= cap) break;
    snprintf(names + 32 * n, 32, "%s", k.c_str());
    total_ms[n] = static_cast<float>(agg[k].first);
    launches[n] = agg[k].second;
    ++n;
  }
  return n;
}

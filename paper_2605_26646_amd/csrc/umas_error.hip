// Thread-local error message, the pinned staging ring for thin host arrays and the optional kernel timing aid of libumas.
#include <string.h>

#include <map>
#include <mutex>
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

// ------------------------------------------------------------------ pinned staging ring
namespace {
struct StageSlot {
  char* host = nullptr;
  size_t cap = 0;
  hipEvent_t copied = nullptr;   // recorded behind the last copy issued from this block
  bool in_flight = false;
};
StageSlot g_slots[ThinStage::kSlots];
int g_next_slot = 0;
std::mutex g_stage_mutex;
}  // namespace

umas_status ThinStage::begin(size_t bytes) {
  g_stage_mutex.lock();
  slot_ = g_next_slot;
  g_next_slot = (g_next_slot + 1) % kSlots;
  StageSlot& s = g_slots[slot_];
  auto bail = [&](hipError_t e, const char* what) {
    slot_ = -1;
    cur_ = nullptr;
    g_stage_mutex.unlock();
    return fail(UMAS_EHIP, "%s failed: %s", what, hipGetErrorString(e));
  };
  if (s.in_flight) {             // the copy issued from this block kSlots calls ago must have read it
    const hipError_t e = hipEventSynchronize(s.copied);
    if (e != hipSuccess) return bail(e, "hipEventSynchronize");
    s.in_flight = false;
  }
  if (!s.copied) {
    const hipError_t e = hipEventCreateWithFlags(&s.copied, hipEventDisableTiming);
    if (e != hipSuccess) return bail(e, "hipEventCreateWithFlags");
  }
  if (s.cap < bytes) {
    if (s.host) (void)hipHostFree(s.host);
    s.host = nullptr;
    s.cap = 0;
    size_t cap = 1 << 16;
    while (cap < bytes) cap <<= 1;
    void* p = nullptr;
    const hipError_t e = hipHostMalloc(&p, cap, hipHostMallocDefault);
    if (e != hipSuccess) return bail(e, "hipHostMalloc");
    s.host = static_cast<char*>(p);
    s.cap = cap;
  }
  cur_ = s.host;
  return UMAS_OK;
}

void ThinStage::put(size_t off, const void* src, size_t n) {
  if (src && n) memcpy(cur_ + off, src, n);
}

void ThinStage::zero(size_t off, size_t n) {
  if (n) memset(cur_ + off, 0, n);
}

umas_status ThinStage::flush(void* dst, size_t bytes, hipStream_t st) {
  StageSlot& s = g_slots[slot_];
  hipError_t e = hipSuccess;
  if (bytes) {
    e = hipMemcpyAsync(dst, cur_, bytes, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipEventRecord(s.copied, st);
    if (e == hipSuccess) s.in_flight = true;
  }
  slot_ = -1;
  cur_ = nullptr;
  g_stage_mutex.unlock();
  if (e != hipSuccess) return fail(UMAS_EHIP, "staging copy failed: %s", hipGetErrorString(e));
  return UMAS_OK;
}

void ThinStage::abandon() {
  if (slot_ < 0) return;
  slot_ = -1;
  cur_ = nullptr;
  g_stage_mutex.unlock();
}

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

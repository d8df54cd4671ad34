// Optional per-kernel timing with HIP events on the launch stream (off by default).
// When enabled, every kernel launch of the library is bracketed by two events; reading the
// profile synchronises on them and returns, per kernel name, the launch count and total time.
#include <string.h>

#include <mutex>
#include <string>
#include <vector>

#include "fc_common.h"

namespace fc {

namespace {
struct Record { const char* name; hipEvent_t start, stop; };
std::mutex g_mu;
bool g_on = false;
std::vector<Record> g_records;
std::vector<hipEvent_t> g_pool;
constexpr size_t kMaxRecords = 1 << 16;

hipEvent_t take_event() {
  if (!g_pool.empty()) { hipEvent_t e = g_pool.back(); g_pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}
}  // namespace

bool profiling_on() { return g_on; }

ProfileScope::ProfileScope(const char* name, hipStream_t s) : stream_(s), idx_(-1) {
  if (!g_on) return;
  std::lock_guard<std::mutex> lock(g_mu);
  if (g_records.size() >= kMaxRecords) return;
  Record r{name, take_event(), take_event()};
  if (!r.start || !r.stop) return;
  if (hipEventRecord(r.start, stream_) != hipSuccess) return;   // this launch goes unrecorded
  g_records.push_back(r);
  idx_ = (long)g_records.size() - 1;
}

ProfileScope::~ProfileScope() {
  if (idx_ < 0) return;
  std::lock_guard<std::mutex> lock(g_mu);
  // (a failed record leaves the stop event unrecorded; flashcache_profile_read then reports FC_EHIP)
  if ((size_t)idx_ < g_records.size()) (void)hipEventRecord(g_records[idx_].stop, stream_);
}

}  // namespace fc

using namespace fc;

extern "C" {

fc_status flashcache_profile_enable(int32_t on) {
  std::lock_guard<std::mutex> lock(g_mu);
  for (auto& r : g_records) { g_pool.push_back(r.start); g_pool.push_back(r.stop); }
  g_records.clear();
  g_on = on != 0;
  return FC_OK;
}

fc_status flashcache_profile_read(int32_t max_entries, char* names, int32_t name_stride,
                                  int32_t* launches, float* total_ms, int32_t* n_entries) {
  if (!n_entries || max_entries < 0 || (max_entries > 0 && (!names || !launches || !total_ms)) ||
      name_stride < 2)
    return FC_EINVAL;
  std::lock_guard<std::mutex> lock(g_mu);
  std::vector<std::string> keys;
  std::vector<int32_t> cnt;
  std::vector<double> ms;
  for (auto& r : g_records) {
    if (hipEventSynchronize(r.stop) != hipSuccess) return FC_EHIP;
    float t = 0.f;
    if (hipEventElapsedTime(&t, r.start, r.stop) != hipSuccess) return FC_EHIP;
    size_t k = 0;
    for (; k < keys.size(); ++k)
      if (keys[k] == r.name) break;
    if (k == keys.size()) { keys.emplace_back(r.name); cnt.push_back(0); ms.push_back(0.0); }
    cnt[k] += 1;
    ms[k] += t;
  }
  int32_t n = (int32_t)keys.size() < max_entries ? (int32_t)keys.size() : max_entries;
  for (int32_t k = 0; k < n; ++k) {
    strncpy(names + (size_t)k * name_stride, keys[k].c_str(), name_stride - 1);
    names[(size_t)k * name_stride + name_stride - 1] = '\0';
    launches[k] = cnt[k];
    total_ms[k] = (float)ms[k];
  }
  *n_entries = (int32_t)keys.size();
  return FC_OK;
}

}  // extern "C"

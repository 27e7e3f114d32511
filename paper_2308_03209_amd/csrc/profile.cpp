// Optional per-kernel timing with HIP events on the launching stream, for roofline reports.
// Disabled by default; when disabled a launch pays one relaxed atomic load.
#include <atomic>
#include <cstring>
#include <map>
#include <mutex>

#include "common.h"

namespace cofree {

namespace {
struct Record {
  int cls;
  hipEvent_t start, stop;
};
struct ClassStat {
  std::string name;
  int64_t launches = 0;
  double ms = 0, bytes = 0, flops = 0;
};
std::atomic<int> g_enabled{0};
std::mutex g_mu;
std::vector<Record> g_records;
std::vector<hipEvent_t> g_pool;
std::vector<ClassStat> g_stats;
std::map<std::string, int> g_index;

hipEvent_t get_event() {
  if (!g_pool.empty()) {
    hipEvent_t e = g_pool.back();
    g_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}
}  // namespace

ProfScope::ProfScope(const char* name, hipStream_t stream, double alg_bytes, double alg_flops) {
  if (!g_enabled.load(std::memory_order_relaxed)) return;
  std::lock_guard<std::mutex> lk(g_mu);
  auto it = g_index.find(name);
  int cls;
  if (it == g_index.end()) {
    cls = (int)g_stats.size();
    g_index[name] = cls;
    ClassStat s;
    s.name = name;
    g_stats.push_back(s);
  } else {
    cls = it->second;
  }
  g_stats[cls].launches += 1;
  g_stats[cls].bytes += alg_bytes;
  g_stats[cls].flops += alg_flops;
  start_ = get_event();
  stop_ = get_event();
  if (!start_ || !stop_) return;
  stream_ = stream;
  cls_ = cls;
  active_ = hipEventRecord(start_, stream) == hipSuccess;
}

ProfScope::~ProfScope() {
  if (!active_) return;
  if (hipEventRecord(stop_, stream_) != hipSuccess) return;
  std::lock_guard<std::mutex> lk(g_mu);
  g_records.push_back(Record{cls_, start_, stop_});
}

}  // namespace cofree

using namespace cofree;

extern "C" {

int32_t cofree_profile_enable(int32_t on) {
  std::lock_guard<std::mutex> lk(g_mu);
  for (auto& r : g_records) {
    g_pool.push_back(r.start);
    g_pool.push_back(r.stop);
  }
  g_records.clear();
  g_stats.clear();
  g_index.clear();
  g_enabled.store(on ? 1 : 0);
  return COFREE_OK;
}

int32_t cofree_profile_read(cofree_kernel_stat* out, int32_t max_entries, int32_t* n_out) {
  COFREE_REQUIRE(out && n_out && max_entries >= 0, "profile_read: bad argument");
  std::lock_guard<std::mutex> lk(g_mu);
  for (auto& r : g_records) {
    COFREE_HIP_CHECK(hipEventSynchronize(r.stop));
    float ms = 0.f;
    COFREE_HIP_CHECK(hipEventElapsedTime(&ms, r.start, r.stop));
    g_stats[r.cls].ms += ms;
    g_pool.push_back(r.start);
    g_pool.push_back(r.stop);
  }
  g_records.clear();
  int32_t n = 0;
  for (auto& s : g_stats) {
    if (n >= max_entries) break;
    std::memset(&out[n], 0, sizeof(out[n]));
    std::strncpy(out[n].name, s.name.c_str(), sizeof(out[n].name) - 1);
    out[n].launches = s.launches;
    out[n].ms_total = s.ms;
    out[n].alg_bytes = s.bytes;
    out[n].alg_flops = s.flops;
    ++n;
  }
  *n_out = n;
  return COFREE_OK;
}

}  // extern "C"

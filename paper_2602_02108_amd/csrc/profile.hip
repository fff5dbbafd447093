// Host-side services shared by the kernel files: optional per-kernel timing for benchmarks (when
// enabled, every kernel launch of the library is bracketed by HIP events recorded on the caller's
// stream) and the once-per-device setup of a kernel's dynamic-LDS limit.
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "common.h"

namespace oomb {

namespace {
struct Entry {
  std::string name;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> pending;
  double total_ms = 0.0;
  int64_t launches = 0;
};
std::mutex g_mu;
int g_level = 0;  // 0 off, 1 every kernel, 2 only the four large kernels
std::vector<Entry> g_entries;
std::vector<hipEvent_t> g_free;

hipEvent_t get_event() {
  if (!g_free.empty()) {
    hipEvent_t e = g_free.back();
    g_free.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

void drain(Entry& en) {
  for (auto& pr : en.pending) {
    float ms = 0.f;
    if (hipEventSynchronize(pr.second) == hipSuccess && hipEventElapsedTime(&ms, pr.first, pr.second) == hipSuccess) {
      en.total_ms += ms;
      en.launches += 1;
    }
    g_free.push_back(pr.first);
    g_free.push_back(pr.second);
  }
  en.pending.clear();
}
}  // namespace

hipError_t ensure_max_dynamic_lds(DeviceOnce& once, const void* kernel, int bytes) {
  static std::mutex mu;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= DeviceOnce::MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(mu);
  if (once.done[dev]) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) once.done[dev] = 1;
  return e;
}

ProfScope::ProfScope(const char* name, hipStream_t st) : stream_(st), slot_(-1), start_(nullptr) {
  if (!g_level) return;
  if (g_level == 2 && std::strcmp(name, "attn_fwd_mfma") && std::strcmp(name, "bwd_dq_mfma") &&
      std::strcmp(name, "bwd_dkv_mfma") && std::strcmp(name, "page_score"))
    return;
  std::lock_guard<std::mutex> lk(g_mu);
  for (size_t i = 0; i < g_entries.size(); ++i)
    if (g_entries[i].name == name) slot_ = (int)i;
  if (slot_ < 0) {
    g_entries.push_back(Entry{});
    g_entries.back().name = name;
    slot_ = (int)g_entries.size() - 1;
  }
  start_ = get_event();
  if (start_) (void)hipEventRecord(start_, stream_);
}

ProfScope::~ProfScope() {
  if (slot_ < 0 || !start_) return;
  std::lock_guard<std::mutex> lk(g_mu);
  hipEvent_t stop = get_event();
  if (!stop) return;
  (void)hipEventRecord(stop, stream_);
  g_entries[slot_].pending.emplace_back(start_, stop);
}

}  // namespace oomb

extern "C" {

void oomb_profile_enable(int32_t on) {
  std::lock_guard<std::mutex> lk(oomb::g_mu);
  oomb::g_level = on;
}

void oomb_profile_reset(void) {
  std::lock_guard<std::mutex> lk(oomb::g_mu);
  for (auto& en : oomb::g_entries) oomb::drain(en);
  oomb::g_entries.clear();
}

int32_t oomb_profile_count(void) {
  std::lock_guard<std::mutex> lk(oomb::g_mu);
  return (int32_t)oomb::g_entries.size();
}

int32_t oomb_profile_read(int32_t idx, char* name, int32_t name_cap, double* total_ms, int64_t* launches) {
  std::lock_guard<std::mutex> lk(oomb::g_mu);
  if (idx < 0 || idx >= (int32_t)oomb::g_entries.size() || !name || name_cap <= 0 || !total_ms || !launches)
    return OOMB_ERR_INVALID_ARG;
  auto& en = oomb::g_entries[idx];
  oomb::drain(en);
  std::strncpy(name, en.name.c_str(), (size_t)name_cap - 1);
  name[name_cap - 1] = 0;
  *total_ms = en.total_ms;
  *launches = en.launches;
  return OOMB_OK;
}

}  // extern "C"

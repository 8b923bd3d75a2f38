// Library identification, launch error check and the optional per-kernel
// event timing used by benchmarks.
#include <string.h>
#include <string>
#include <vector>
#include "common.h"

namespace {
struct Entry {
  std::string name;
  std::vector<hipEvent_t> starts, stops;
};
bool g_on = false;
std::vector<Entry> g_entries;
std::vector<hipEvent_t> g_pool;

hipEvent_t take_event() {
  if (!g_pool.empty()) {
    hipEvent_t e = g_pool.back();
    g_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}
void clear_entries() {
  for (auto& en : g_entries) {
    for (auto e : en.starts) g_pool.push_back(e);
    for (auto e : en.stops) g_pool.push_back(e);
  }
  g_entries.clear();
}
}  // namespace

MoeLaunchScope::MoeLaunchScope(const char* name, hipStream_t s) : slot(-1), stream(s) {
  if (!g_on) return;
  int idx = -1;
  for (size_t i = 0; i < g_entries.size(); ++i)
    if (g_entries[i].name == name) { idx = static_cast<int>(i); break; }
  if (idx < 0) {
    g_entries.push_back(Entry{name, {}, {}});
    idx = static_cast<int>(g_entries.size()) - 1;
  }
  hipEvent_t a = take_event(), b = take_event();
  if (!a || !b) return;
  g_entries[idx].starts.push_back(a);
  g_entries[idx].stops.push_back(b);
  slot = idx;
  (void)hipEventRecord(a, stream);
}
MoeLaunchScope::~MoeLaunchScope() {
  if (slot < 0) return;
  (void)hipEventRecord(g_entries[slot].stops.back(), stream);
}

int moe_check_launch() { return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_LAUNCH; }

extern "C" {

const char* moe_version(void) { return "moe_hotpath 0.1 (gfx950, bf16 MFMA)"; }

int moe_prof_enable(int on) {
  clear_entries();
  g_on = on != 0;
  return MOE_OK;
}
int moe_prof_count(void) { return static_cast<int>(g_entries.size()); }

int moe_prof_read(int index, char* name, int name_cap, float* total_ms, int* launches) {
  if (index < 0 || index >= static_cast<int>(g_entries.size()) || !name || name_cap <= 0 || !total_ms || !launches)
    return MOE_ERR_INVALID;
  Entry& en = g_entries[index];
  float total = 0.f;
  for (size_t i = 0; i < en.starts.size(); ++i) {
    if (hipEventSynchronize(en.stops[i]) != hipSuccess) return MOE_ERR_LAUNCH;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, en.starts[i], en.stops[i]) != hipSuccess) return MOE_ERR_LAUNCH;
    total += ms;
  }
  strncpy(name, en.name.c_str(), static_cast<size_t>(name_cap) - 1);
  name[name_cap - 1] = '\0';
  *total_ms = total;
  *launches = static_cast<int>(en.starts.size());
  return MOE_OK;
}

}  // extern "C"

// Per-kernel timing registry (see timing.h) and its C entry points: part of the instrumented build only.
#include "timing.h"

#ifdef AFFMAE_TIMING
#include "../../include/affmae_timing.h"

#include <cstring>
#include <mutex>
#include <string>
#include <vector>

namespace affmae {
namespace {

struct Pending {
  int entry;
  hipEvent_t start, stop;
};
struct Entry {
  std::string name;
  double total_ms = 0.0;
  int count = 0;
};

std::mutex g_mu;
bool g_enabled = false;
std::vector<Entry> g_entries;
std::vector<Pending> g_pending;
std::vector<hipEvent_t> g_free;
int g_open = -1;  // index into g_pending of the scope being recorded

hipEvent_t get_event() {
  if (!g_free.empty()) {
    hipEvent_t e = g_free.back();
    g_free.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  (void)hipEventCreate(&e);
  return e;
}

// Folds finished event pairs into the totals.  Caller holds the mutex and has
// synchronised the streams involved.
void drain() {
  for (Pending& p : g_pending) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, p.start, p.stop) == hipSuccess) {
      g_entries[p.entry].total_ms += ms;
      g_entries[p.entry].count += 1;
    }
    g_free.push_back(p.start);
    g_free.push_back(p.stop);
  }
  g_pending.clear();
  g_open = -1;
}

}  // namespace

bool timing_enabled() { return g_enabled; }

void timing_begin(const char* name, hipStream_t stream) {
  std::lock_guard<std::mutex> lock(g_mu);
  int idx = -1;
  for (size_t i = 0; i < g_entries.size(); ++i)
    if (g_entries[i].name == name) idx = (int)i;
  if (idx < 0) {
    g_entries.push_back(Entry{name});
    idx = (int)g_entries.size() - 1;
  }
  Pending p{idx, get_event(), get_event()};
  (void)hipEventRecord(p.start, stream);
  g_pending.push_back(p);
  g_open = (int)g_pending.size() - 1;
}

void timing_end(hipStream_t stream) {
  std::lock_guard<std::mutex> lock(g_mu);
  if (g_open >= 0) (void)hipEventRecord(g_pending[g_open].stop, stream);
  g_open = -1;
}

}  // namespace affmae

extern "C" {

void affmae_timing_enable(int on) {
  std::lock_guard<std::mutex> lock(affmae::g_mu);
  affmae::g_enabled = on != 0;
}

void affmae_timing_reset(void) {
  (void)hipDeviceSynchronize();
  std::lock_guard<std::mutex> lock(affmae::g_mu);
  affmae::drain();
  affmae::g_entries.clear();
}

int affmae_timing_read(int index, char* name, int name_len, double* total_ms, int* count) {
  (void)hipDeviceSynchronize();
  std::lock_guard<std::mutex> lock(affmae::g_mu);
  affmae::drain();
  const int n = (int)affmae::g_entries.size();
  if (index >= 0 && index < n) {
    const affmae::Entry& e = affmae::g_entries[index];
    if (name && name_len > 0) {
      std::strncpy(name, e.name.c_str(), (size_t)name_len - 1);
      name[name_len - 1] = '\0';
    }
    if (total_ms) *total_ms = e.total_ms;
    if (count) *count = e.count;
  }
  return n;
}

}  // extern "C"
#endif  // AFFMAE_TIMING

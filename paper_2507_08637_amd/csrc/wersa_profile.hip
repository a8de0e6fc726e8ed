// Optional per-kernel timing with HIP events on the caller's stream (off by default).
// When enabled, every kernel launch of the library is bracketed by an event pair; reading
// the results synchronises those events.  Not thread-safe; meant for benchmarks and tools.
#include "wersa_internal.h"

#include <string.h>
#include <string>
#include <vector>

namespace wersa {
namespace {
struct Rec {
  const char *name;
  hipEvent_t a, b;
};
bool g_on = false;
bool g_open = false;        // the last prof_begin recorded an event pair
std::string g_only;         // when not empty: bracket only launches of this name
std::vector<Rec> g_recs;
std::vector<hipEvent_t> g_pool;
size_t g_pool_used = 0;
constexpr size_t kMaxEvents = 1 << 16;

hipEvent_t take_event() {
  if (g_pool_used == g_pool.size()) {
    if (g_pool.size() >= kMaxEvents) return nullptr;
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    g_pool.push_back(e);
  }
  return g_pool[g_pool_used++];
}
struct Agg {
  std::string name;
  double ms;
  int launches;
};
std::vector<Agg> g_agg;
}  // namespace

bool profiling() { return g_on; }

void prof_begin(const char *name, hipStream_t st) {
  g_open = false;
  if (!g_on) return;
  if (!g_only.empty() && g_only != name) return;
  hipEvent_t a = take_event(), b = take_event();
  if (!a || !b) return;
  g_recs.push_back(Rec{name, a, b});
  (void)hipEventRecord(a, st);
  g_open = true;
}
void prof_end(hipStream_t st) {
  if (!g_on || !g_open || g_recs.empty()) return;
  (void)hipEventRecord(g_recs.back().b, st);
  g_open = false;
}
}  // namespace wersa

using namespace wersa;

extern "C" {

void wersa_profile_enable(int on) {
  g_on = on != 0;
}

void wersa_profile_only(const char *name) {
  g_only = name ? name : "";
}

void wersa_profile_reset(void) {
  g_recs.clear();
  g_agg.clear();
  g_pool_used = 0;
}

int32_t wersa_profile_collect(void) {
  g_agg.clear();
  for (const Rec &r : g_recs) {
    if (hipEventSynchronize(r.b) != hipSuccess) continue;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) continue;
    bool found = false;
    for (Agg &a : g_agg)
      if (a.name == r.name) {
        a.ms += ms;
        a.launches += 1;
        found = true;
        break;
      }
    if (!found) g_agg.push_back(Agg{r.name, ms, 1});
  }
  g_recs.clear();
  g_pool_used = 0;
  return (int32_t)g_agg.size();
}

int32_t wersa_profile_get(int32_t index, char *name, int32_t name_len, double *total_ms,
                          int32_t *launches) {
  if (index < 0 || index >= (int32_t)g_agg.size() || !name || name_len < 1 || !total_ms || !launches)
    return 1;
  strncpy(name, g_agg[index].name.c_str(), (size_t)name_len - 1);
  name[name_len - 1] = 0;
  *total_ms = g_agg[index].ms;
  *launches = g_agg[index].launches;
  return 0;
}

}  // extern "C"

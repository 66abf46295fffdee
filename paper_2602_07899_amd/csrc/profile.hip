// Optional per-kernel timing: HIP events recorded on the launch stream around
// every kernel while profiling is enabled.  Host-side bookkeeping only.
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "common.h"

namespace tlq {
namespace {

struct Rec { int name_id; hipEvent_t start, stop; double work; };
// every tlq_profile_collect / reset starts a new generation: a scope that was opened before
// it must not touch the record list that was rebuilt in between
unsigned g_generation = 0;
struct Total { std::string name; int64_t launches; double ms; double work; };

std::mutex g_mu;
bool g_on = false;
std::vector<Rec> g_recs;
std::vector<Total> g_totals;
std::vector<hipEvent_t> g_free;

int name_id_locked(const char* name) {
  for (size_t i = 0; i < g_totals.size(); ++i)
    if (g_totals[i].name == name) return (int)i;
  g_totals.push_back({name, 0, 0.0, 0.0});
  return (int)g_totals.size() - 1;
}

hipEvent_t get_event_locked() {
  if (!g_free.empty()) { hipEvent_t e = g_free.back(); g_free.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

}  // namespace

ProfScope::ProfScope(const char* name, hipStream_t s, double work) : slot(-1), stream(s), generation(0) {
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_on) return;
  Rec r;
  r.name_id = name_id_locked(name);
  r.start = get_event_locked();
  r.stop = get_event_locked();
  r.work = work;
  if (!r.start || !r.stop) {          // hand back whichever event was obtained
    if (r.start) g_free.push_back(r.start);
    if (r.stop) g_free.push_back(r.stop);
    return;
  }
  (void)hipEventRecord(r.start, stream);
  g_recs.push_back(r);
  slot = (int)g_recs.size() - 1;
  generation = g_generation;
}

ProfScope::~ProfScope() {
  if (slot < 0) return;
  std::lock_guard<std::mutex> lk(g_mu);
  if (generation == g_generation && slot < (int)g_recs.size()) (void)hipEventRecord(g_recs[slot].stop, stream);
}

}  // namespace tlq

using namespace tlq;

extern "C" {

tlq_status tlq_profile_enable(int on) {
  std::lock_guard<std::mutex> lk(g_mu);
  g_on = on != 0;
  return TLQ_OK;
}

int tlq_profile_enabled(void) {
  std::lock_guard<std::mutex> lk(g_mu);
  return g_on ? 1 : 0;
}

tlq_status tlq_profile_collect(void) {
  std::lock_guard<std::mutex> lk(g_mu);
  for (Rec& r : g_recs) {
    float ms = 0.0f;
    if (hipEventSynchronize(r.stop) == hipSuccess &&
        hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess) {
      Total& t = g_totals[r.name_id];
      t.launches += 1; t.ms += ms; t.work += r.work;
    }
    g_free.push_back(r.start);
    g_free.push_back(r.stop);
  }
  g_recs.clear();
  ++g_generation;
  return TLQ_OK;
}

tlq_status tlq_profile_reset(void) {
  tlq_profile_collect();
  std::lock_guard<std::mutex> lk(g_mu);
  g_totals.clear();
  return TLQ_OK;
}

int tlq_profile_count(void) {
  std::lock_guard<std::mutex> lk(g_mu);
  return (int)g_totals.size();
}

tlq_status tlq_profile_get(int i, char* name, size_t name_cap, int64_t* launches,
                           double* total_ms, double* total_work) {
  std::lock_guard<std::mutex> lk(g_mu);
  if (i < 0 || i >= (int)g_totals.size()) return TLQ_ERR_SHAPE;
  const Total& t = g_totals[i];
  if (name && name_cap) {
    std::strncpy(name, t.name.c_str(), name_cap - 1);
    name[name_cap - 1] = 0;
  }
  if (launches) *launches = t.launches;
  if (total_ms) *total_ms = t.ms;
  if (total_work) *total_work = t.work;
  return TLQ_OK;
}

}  // extern "C"

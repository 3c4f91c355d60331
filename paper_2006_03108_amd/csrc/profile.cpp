// Optional per-kernel timing with HIP events on the stream the kernels are
// launched on, for the benchmark's roofline figures.  Off by default; when
// off the scopes cost one branch.
#include <cstring>
#include <map>
#include <string>

#include "common.h"
#include "profile.h"

namespace distdl {

struct ProfRecord {
  const char* name;
  hipEvent_t start, stop;
};
static bool g_prof_on = false;
static std::vector<ProfRecord> g_records;
static std::vector<hipEvent_t> g_free_events;

static hipEvent_t get_event() {
  if (!g_free_events.empty()) {
    hipEvent_t e = g_free_events.back();
    g_free_events.pop_back();
    return e;
  }
  // Timing-only events: without the system-scope fence a record does not write back and invalidate the caches
  // between two kernels, which would be charged to the kernel that follows.
  hipEvent_t e = nullptr;
  if (hipEventCreateWithFlags(&e, hipEventDisableSystemFence) != hipSuccess) {
    (void)hipGetLastError();
    (void)hipEventCreate(&e);
  }
  return e;
}

ProfScope::ProfScope(const char* name, hipStream_t st) : st_(st), active_(g_prof_on) {
  if (!active_) return;
  ProfRecord r{name, get_event(), get_event()};
  (void)hipEventRecord(r.start, st_);
  g_records.push_back(r);
}

ProfScope::~ProfScope() {
  if (!active_) return;
  (void)hipEventRecord(g_records.back().stop, st_);
}

}  // namespace distdl

using namespace distdl;

extern "C" {

int distdl_profile_enable(int on) {
  g_prof_on = on != 0;
  return DISTDL_OK;
}

int distdl_profile_report(char* out, size_t cap) {
  if (!out || cap == 0) return set_error(DISTDL_ERR_NULL, "profile_report: null buffer");
  struct Acc {
    int count = 0;
    double ms = 0;
  };
  std::map<std::string, Acc> acc;
  std::vector<std::string> order;
  for (ProfRecord& r : g_records) {
    DISTDL_HIP_TRY(hipEventSynchronize(r.stop));
    float ms = 0.f;
    DISTDL_HIP_TRY(hipEventElapsedTime(&ms, r.start, r.stop));
    if (!acc.count(r.name)) order.push_back(r.name);
    Acc& a = acc[r.name];
    a.count += 1;
    a.ms += ms;
    g_free_events.push_back(r.start);
    g_free_events.push_back(r.stop);
  }
  g_records.clear();
  std::string text;
  for (const std::string& n : order) {
    char line[160];
    snprintf(line, sizeof line, "%s %d %.6f\n", n.c_str(), acc[n].count, acc[n].ms);
    text += line;
  }
  if (text.size() + 1 > cap) return set_error(DISTDL_ERR_INVALID_ARG, "profile_report: buffer too small");
  std::memcpy(out, text.c_str(), text.size() + 1);
  return (int)text.size();
}

int distdl_plan_stats(const distdl_plan* plan, int64_t out[4]) {
  if (!plan || !out) return set_error(DISTDL_ERR_NULL, "plan_stats: null argument");
  out[0] = plan->fwd1.cells_copied;   // halo cells (in-domain, non-owned), all workers
  out[1] = plan->fwd1.cells_zeroed;   // zero-padding cells
  out[2] = plan->adj1.cells_band;     // bulk cells that some other worker holds a copy of
  out[3] = plan->adj1.cells_copied;   // halo cells gathered by the adjoint (== out[0])
  return DISTDL_OK;
}

}  // extern "C"

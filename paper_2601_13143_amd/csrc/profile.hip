// Optional per-kernel timing for benchmarks: HIP events recorded on the launch stream right before and
// after the launches of the selected kinds, accumulated per kind together with the algorithmic work
// (flops or bytes) of each launch.  Off by default; when off a ProfScope costs one load and a branch.
#include <mutex>
#include <vector>

#include "common.hpp"

namespace fastav {

namespace {
struct Rec { hipEvent_t a, b; int kind; double work; };
struct State {
  std::mutex mu;
  uint32_t mask = 0;
  std::vector<hipEvent_t> pool;
  std::vector<Rec> pending;
  double ms[FASTAV_PROF_KIND_COUNT] = {};
  double work[FASTAV_PROF_KIND_COUNT] = {};
  int64_t n[FASTAV_PROF_KIND_COUNT] = {};
};
State g_prof;

hipEvent_t get_event(State& st) {
  if (!st.pool.empty()) { hipEvent_t e = st.pool.back(); st.pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}
}  // namespace

ProfScope::ProfScope(int kind, double work, hipStream_t s) : rec_(nullptr), stream_(s) {
  if (!(g_prof.mask & (1u << kind))) return;
  std::lock_guard<std::mutex> lk(g_prof.mu);
  hipEvent_t a = get_event(g_prof), b = get_event(g_prof);
  if (!a || !b) return;
  g_prof.pending.push_back(Rec{a, b, kind, work});
  rec_ = (void*)b;                                         // the end event itself: a collect in between may reorder `pending`
  (void)hipEventRecord(a, s);
}

ProfScope::~ProfScope() {
  if (!rec_) return;
  (void)hipEventRecord((hipEvent_t)rec_, stream_);
}

}  // namespace fastav

using namespace fastav;

extern "C" {

fastav_status_t fastav_profile_enable(uint32_t kind_mask) {
  if (kind_mask >> FASTAV_PROF_KIND_COUNT) return fail(FASTAV_EINVAL, "profile: unknown kind bit");
  std::lock_guard<std::mutex> lk(g_prof.mu);
  g_prof.mask = kind_mask;
  return FASTAV_OK;
}

static fastav_status_t drain_locked() {
  for (Rec& r : g_prof.pending) {
    hipError_t e = hipEventSynchronize(r.b);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.a, r.b);
    if (e != hipSuccess) { g_prof.pending.clear(); return fail(FASTAV_EHIP, "profile: %s", hipGetErrorString(e)); }
    g_prof.ms[r.kind] += ms; g_prof.work[r.kind] += r.work; g_prof.n[r.kind] += 1;
    g_prof.pool.push_back(r.a); g_prof.pool.push_back(r.b);
  }
  g_prof.pending.clear();
  return FASTAV_OK;
}

fastav_status_t fastav_profile_collect(int32_t kind, double* total_ms, int64_t* launches, double* total_work) {
  if (kind < 0 || kind >= FASTAV_PROF_KIND_COUNT) return fail(FASTAV_EINVAL, "profile: bad kind");
  std::lock_guard<std::mutex> lk(g_prof.mu);
  fastav_status_t st = drain_locked();
  if (st != FASTAV_OK) return st;
  if (total_ms) *total_ms = g_prof.ms[kind];
  if (launches) *launches = g_prof.n[kind];
  if (total_work) *total_work = g_prof.work[kind];
  return FASTAV_OK;
}

fastav_status_t fastav_profile_reset(void) {
  std::lock_guard<std::mutex> lk(g_prof.mu);
  fastav_status_t st = drain_locked();
  for (int i = 0; i < FASTAV_PROF_KIND_COUNT; ++i) { g_prof.ms[i] = 0; g_prof.work[i] = 0; g_prof.n[i] = 0; }
  return st;
}

}  // extern "C"

// Per-kernel timing hook: when enabled, every launch site records a HIP event pair on the launch stream;
// ssa_profile_get() drains them into per-kernel totals.  Not thread-safe; meant for benchmarks.
#include "profile.h"

#include <vector>

#include "ssa_internal.h"

namespace {
const char *const kNames[PROF_COUNT] = {
    "prep_sort_pool", "cmp_fwd_scores_topk", "slc_fwd", "win_fwd", "slc_merge_combine",
    "bwd_prep", "bwd_pre_delta", "bwd_dq_cmp_win", "bwd_dq_slc", "bwd_invert_selection", "bwd_dkv_win", "bwd_dkv_slc", "bwd_dkv_cmp",
    "bwd_finish_unpool", "generic_path", "cmp_module_fwd", "cmp_module_bwd", "gate_fwd", "gate_bwd",
    "linear_fwd", "linear_bwd", "fwd_invert_selection", "bwd_dq_merge"};
struct Rec { int id; hipEvent_t a, b; };
bool g_on = false;
std::vector<Rec> g_pending;
std::vector<hipEvent_t> g_pool;
double g_ms[PROF_COUNT];
long long g_cnt[PROF_COUNT];
hipEvent_t g_open[PROF_COUNT];

hipEvent_t get_event() {
  if (!g_pool.empty()) { hipEvent_t e = g_pool.back(); g_pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  (void)hipEventCreate(&e);
  return e;
}
void drain() {
  for (const Rec &r : g_pending) {
    float ms = 0.f;
    if (hipEventSynchronize(r.b) == hipSuccess && hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) {
      g_ms[r.id] += ms;
      g_cnt[r.id] += 1;
    }
    g_pool.push_back(r.a);
    g_pool.push_back(r.b);
  }
  g_pending.clear();
}
}  // namespace

bool prof_enabled() { return g_on; }
void prof_begin(int id, hipStream_t s) {
  g_open[id] = get_event();
  (void)hipEventRecord(g_open[id], s);
}
void prof_end(int id, hipStream_t s) {
  hipEvent_t e = get_event();
  (void)hipEventRecord(e, s);
  g_pending.push_back(Rec{id, g_open[id], e});
}

extern "C" int ssa_profile_enable(int on) {
  drain();
  for (int i = 0; i < PROF_COUNT; ++i) { g_ms[i] = 0.0; g_cnt[i] = 0; }
  g_on = on != 0;
  return SSA_OK;
}
extern "C" int ssa_profile_num_kernels(void) { return PROF_COUNT; }
extern "C" int ssa_profile_get(int i, const char **name, double *total_ms, int64_t *launches) {
  if (i < 0 || i >= PROF_COUNT) return SSA_ERR_BAD_SHAPE;
  drain();
  if (name) *name = kNames[i];
  if (total_ms) *total_ms = g_ms[i];
  if (launches) *launches = g_cnt[i];
  return SSA_OK;
}

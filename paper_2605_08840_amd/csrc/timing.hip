// Optional per-kernel timing with HIP events on the caller's stream (off by default).
// Every kernel launch of a selected stage is bracketed by two events taken from a pool;
// restkv_timing_read() waits for them and returns the time per stage.  Each bracket costs a
// few microseconds of idle GPU between kernels, which is why stages can be selected one by one.
#include <mutex>
#include <vector>

#include "common.hpp"

namespace restkv {

namespace {
struct Rec { hipEvent_t a, b; int stage; };
std::mutex g_mu;
unsigned g_mask = 0;      // bit s: launches of stage s are timed
std::vector<Rec> g_pool;     // events are created once and reused
size_t g_used = 0;
}  // namespace

StageTimer::StageTimer(int stage, hipStream_t st) : st_(st), slot_(-1) {
  if (!((g_mask >> stage) & 1u)) return;
  std::lock_guard<std::mutex> lk(g_mu);
  if (g_used == g_pool.size()) {
    Rec r;
    r.stage = stage;
    if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) return;
    g_pool.push_back(r);
  }
  slot_ = (long)g_used++;
  g_pool[slot_].stage = stage;
  (void)hipEventRecord(g_pool[slot_].a, st_);
}

StageTimer::~StageTimer() {
  if (slot_ < 0) return;
  std::lock_guard<std::mutex> lk(g_mu);
  (void)hipEventRecord(g_pool[slot_].b, st_);
}

}  // namespace restkv

using namespace restkv;

extern "C" {

int restkv_timing_enable(int stage_mask) {
  std::lock_guard<std::mutex> lk(g_mu);
  g_mask = (unsigned)stage_mask;
  g_used = 0;
  return RESTKV_OK;
}

int restkv_timing_read(double* ms, int64_t* launches, int n_stages) {
  if (!ms || !launches || n_stages < RESTKV_N_STAGES) return RESTKV_EINVAL;
  std::lock_guard<std::mutex> lk(g_mu);
  for (int s = 0; s < n_stages; ++s) { ms[s] = 0.0; launches[s] = 0; }
  int rc = RESTKV_OK;
  for (size_t j = 0; j < g_used; ++j) {
    float t = 0.f;
    if (hipEventSynchronize(g_pool[j].b) != hipSuccess ||
        hipEventElapsedTime(&t, g_pool[j].a, g_pool[j].b) != hipSuccess) { rc = RESTKV_EHIP; continue; }
    ms[g_pool[j].stage] += (double)t;
    launches[g_pool[j].stage] += 1;
  }
  g_used = 0;
  return rc;
}

const char* restkv_stage_name(int stage) {
  static const char* names[RESTKV_N_STAGES] = {
      "gram", "attn_partial", "attn_combine", "vv", "score", "ema", "row_topk", "box", "select", "compact"};
  return (stage >= 0 && stage < RESTKV_N_STAGES) ? names[stage] : "?";
}

}  // extern "C"

// Optional per-stage timing with HIP events on the caller's stream.
// Off by default; when on, every kernel group enqueued by an entry point is
// bracketed by a pair of events so a benchmark can split the step time by stage
// without a profiler attached.
#include <mutex>
#include <vector>

#include "poetx_kernels.h"

namespace poetx {
namespace {
struct Record {
  int stage;
  hipEvent_t e0, e1;
};
std::mutex g_mu;
bool g_on = false;
size_t g_max = 0;
std::vector<Record> g_rec;
}  // namespace

StageTimer::StageTimer(int stage, hipStream_t st) : st_(st), idx_(-1) {
  if (!g_on) return;
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_on || g_rec.size() >= g_max) return;
  Record r;
  r.stage = stage;
  if (hipEventCreate(&r.e0) != hipSuccess) return;
  if (hipEventCreate(&r.e1) != hipSuccess) { (void)hipEventDestroy(r.e0); return; }
  (void)hipEventRecord(r.e0, st);
  g_rec.push_back(r);
  idx_ = (long)g_rec.size() - 1;
}

StageTimer::~StageTimer() {
  if (idx_ < 0) return;
  std::lock_guard<std::mutex> lk(g_mu);
  if ((size_t)idx_ < g_rec.size()) (void)hipEventRecord(g_rec[idx_].e1, st_);
}

}  // namespace poetx

using namespace poetx;

extern "C" {

int poetx_profile_begin(int32_t max_records) {
  if (max_records <= 0) return POETX_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lk(g_mu);
  for (auto& r : g_rec) { (void)hipEventDestroy(r.e0); (void)hipEventDestroy(r.e1); }
  g_rec.clear();
  g_max = (size_t)max_records;
  g_rec.reserve(g_max);
  g_on = true;
  return POETX_OK;
}

int poetx_profile_end(double* ms_by_stage, int64_t* launches_by_stage) {
  if (!ms_by_stage || !launches_by_stage) return POETX_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lk(g_mu);
  g_on = false;
  for (int s = 0; s < POETX_STAGE_COUNT; ++s) { ms_by_stage[s] = 0.0; launches_by_stage[s] = 0; }
  int rc = POETX_OK;
  for (auto& r : g_rec) {
    float ms = 0.f;
    if (hipEventSynchronize(r.e1) != hipSuccess || hipEventElapsedTime(&ms, r.e0, r.e1) != hipSuccess) rc = POETX_ERR_HIP;
    else if (r.stage >= 0 && r.stage < POETX_STAGE_COUNT) { ms_by_stage[r.stage] += ms; launches_by_stage[r.stage] += 1; }
    (void)hipEventDestroy(r.e0);
    (void)hipEventDestroy(r.e1);
  }
  g_rec.clear();
  return rc;
}

}  // extern "C"

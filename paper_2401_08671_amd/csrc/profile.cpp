// Optional per-kernel timing with HIP events (host-side state, off by default).
#include <vector>

#include "fsf_internal.h"
#include "fsf_measure.h"

namespace {

struct Rec {
  hipEvent_t start, stop;
  int phase;
};

bool g_on = false;
std::vector<Rec> g_recs;
std::vector<hipEvent_t> g_pool;

hipEvent_t get_event() {
  if (!g_pool.empty()) {
    hipEvent_t e = g_pool.back();
    g_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

}  // namespace

namespace fsf {

PhaseTimer::PhaseTimer(int phase, hipStream_t stream)
    : phase_(phase), stream_(stream), start_(nullptr), on_(g_on) {
  if (!on_) return;
  start_ = get_event();
  if (!start_ || hipEventRecord(start_, stream_) != hipSuccess) on_ = false;
}

PhaseTimer::~PhaseTimer() {
  if (!on_) return;
  hipEvent_t stop = get_event();
  if (!stop || hipEventRecord(stop, stream_) != hipSuccess) {  // drop the measurement, keep the events
    g_pool.push_back(start_);
    if (stop) g_pool.push_back(stop);
    return;
  }
  g_recs.push_back({start_, stop, phase_});
}

}  // namespace fsf

extern "C" int fsf_profile_enable(int on) {
  g_on = on != 0;
  return FSF_OK;
}

extern "C" int fsf_profile_read(double* ms_out, int64_t* launches_out) {
  if (!ms_out || !launches_out) return FSF_ERR_INVALID_ARG;
  for (int i = 0; i < FSF_N_PHASES; ++i) {
    ms_out[i] = 0.0;
    launches_out[i] = 0;
  }
  int status = FSF_OK;
  for (const Rec& r : g_recs) {
    float ms = 0.f;
    if (hipEventSynchronize(r.stop) != hipSuccess ||
        hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) {
      status = FSF_ERR_HIP;
    } else if (r.phase >= 0 && r.phase < FSF_N_PHASES) {
      ms_out[r.phase] += ms;
      launches_out[r.phase] += 1;
    }
    g_pool.push_back(r.start);
    g_pool.push_back(r.stop);
  }
  g_recs.clear();
  return status;
}

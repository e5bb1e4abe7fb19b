// Optional per-launch timing: HIP event pairs recorded on the launch stream around each kernel
// launch, summed per kernel class when the caller asks.  Measurement aid only.
#include <hip/hip_runtime.h>

#include <vector>

#include "../../include/mllm_stage.h"
#include "kernels.h"

namespace mllm_detail { void set_last_error(const char* msg); }

namespace {
struct Record { int cls; double work; };
bool g_on = false;
int g_used = 0;
int64_t g_dropped = 0;
std::vector<hipEvent_t> g_start, g_stop;
std::vector<Record> g_rec;
}  // namespace

namespace mllm {

ProfScope::ProfScope(int cls, double work, hipStream_t s) : slot(-1), stream(s) {
  if (!g_on) return;
  if (g_used >= (int)g_start.size()) { g_dropped++; return; }
  slot = g_used++;
  g_rec[slot] = {cls, work};
  (void)hipEventRecord(g_start[slot], s);
}
ProfScope::~ProfScope() {
  if (slot >= 0) (void)hipEventRecord(g_stop[slot], stream);
}

}  // namespace mllm

extern "C" {

mllm_status_t mllm_profile_begin(int32_t max_records) {
  if (max_records <= 0) { mllm_detail::set_last_error("max_records must be positive"); return MLLM_ERR_SHAPE; }
  while ((int)g_start.size() < max_records) {
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
      mllm_detail::set_last_error("hipEventCreate failed");
      return MLLM_ERR_HIP;
    }
    g_start.push_back(a);
    g_stop.push_back(b);
  }
  g_rec.resize(g_start.size());
  g_used = 0;
  g_dropped = 0;
  g_on = true;
  return MLLM_OK;
}

mllm_status_t mllm_profile_end(int64_t* launches, double* milliseconds, double* work, int64_t* dropped) {
  g_on = false;
  if (!launches || !milliseconds || !work) { mllm_detail::set_last_error("output array is NULL"); return MLLM_ERR_NULL; }
  for (int c = 0; c < mllm::PROF_N_CLASSES; c++) { launches[c] = 0; milliseconds[c] = 0; work[c] = 0; }
  for (int i = 0; i < g_used; i++) {
    if (hipEventSynchronize(g_stop[i]) != hipSuccess) { mllm_detail::set_last_error("hipEventSynchronize failed"); return MLLM_ERR_HIP; }
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, g_start[i], g_stop[i]) != hipSuccess) { mllm_detail::set_last_error("hipEventElapsedTime failed"); return MLLM_ERR_HIP; }
    launches[g_rec[i].cls]++;
    milliseconds[g_rec[i].cls] += ms;
    work[g_rec[i].cls] += g_rec[i].work;
  }
  if (dropped) *dropped = g_dropped;
  g_used = 0;
  return MLLM_OK;
}

}  // extern "C"

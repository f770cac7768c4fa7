// Optional per-kernel timing: when enabled, every launch site records a hipEvent pair on the
// launch stream; dsvt_prof_collect() turns the pairs into per-kernel totals.  Events are created
// when profiling is enabled, never on the launch path.
#include <vector>
#include "common.h"

namespace {
bool g_enabled = false;
std::vector<hipEvent_t> g_events;   // 2 per record: begin, end
std::vector<int> g_ids;
size_t g_used = 0;
const char* const kNames[DSVT_K_COUNT] = {
    "part_mark", "part_window_count", "part_scan_windows", "part_emit", "part_clear",
    "part_tiles", "layer", "pool_group", "pool_attention", "bev_clear", "bev_scatter", "vfe_group", "vfe_reduce"};
}  // namespace

void dsvt_prof_mark_begin(int id, hipStream_t s) {
  if (!g_enabled || g_used >= g_ids.size()) return;
  g_ids[g_used] = id;
  (void)hipEventRecord(g_events[2 * g_used], s);
}
void dsvt_prof_mark_end(int id, hipStream_t s) {
  if (!g_enabled || g_used >= g_ids.size()) return;
  (void)id;
  (void)hipEventRecord(g_events[2 * g_used + 1], s);
  ++g_used;
}

extern "C" int dsvt_prof_enable(int32_t max_launches) {
  if (max_launches <= 0) return DSVT_EINVAL;
  if (g_enabled) return DSVT_EINVAL;
  g_events.resize(2 * (size_t)max_launches);
  g_ids.assign((size_t)max_launches, -1);
  for (auto& e : g_events) DSVT_HIP_TRY(hipEventCreate(&e));
  g_used = 0;
  g_enabled = true;
  return DSVT_OK;
}

extern "C" int dsvt_prof_collect(float* total_ms, int32_t* launches, int32_t n_kernels) {
  if (!g_enabled || !total_ms || !launches || n_kernels < DSVT_K_COUNT) return DSVT_EINVAL;
  for (int k = 0; k < n_kernels; ++k) { total_ms[k] = 0.f; launches[k] = 0; }
  for (size_t r = 0; r < g_used; ++r) {
    DSVT_HIP_TRY(hipEventSynchronize(g_events[2 * r + 1]));
    float ms = 0.f;
    DSVT_HIP_TRY(hipEventElapsedTime(&ms, g_events[2 * r], g_events[2 * r + 1]));
    total_ms[g_ids[r]] += ms;
    launches[g_ids[r]] += 1;
  }
  for (auto& e : g_events) (void)hipEventDestroy(e);
  g_events.clear(); g_ids.clear(); g_used = 0; g_enabled = false;
  return DSVT_OK;
}

extern "C" int32_t dsvt_prof_kernel_count(void) { return DSVT_K_COUNT; }
extern "C" const char* dsvt_prof_kernel_name(int32_t id) { return (id >= 0 && id < DSVT_K_COUNT) ? kNames[id] : ""; }

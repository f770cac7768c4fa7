// Optional per-kernel timing: when enabled, every launch site records a hipEvent pair on the
// launch stream; dsvt_prof_collect() turns the pairs into per-kernel totals.  Launches of the same
// kernel that follow one another on one stream share one pair (begin before the first, end after
// the last), so that a run of back-to-back launches is charged the dispatch latency after an
// event once, as it is when the launches replay from a graph.  Events are created when profiling
// is enabled, never on the launch path.
#include <vector>
#include "common.h"

namespace {
bool g_enabled = false;
std::vector<hipEvent_t> g_events;   // 2 per record: begin, end
std::vector<int> g_ids, g_count;     // kernel and number of launches of each record
std::vector<hipStream_t> g_streams;
size_t g_used = 0;
bool g_extend = false;               // the launch being marked joins the previous record
const char* const kNames[DSVT_K_COUNT] = {
    "part_mark", "part_window_count", "part_scan_windows", "part_emit", "part_clear",
    "part_tiles", "layer", "pool_group", "pool_attention", "bev_clear", "bev_scatter", "vfe_group", "vfe_reduce"};
}  // namespace

void dsvt_prof_mark_begin(int id, hipStream_t s) {
  if (!g_enabled) return;
  g_extend = g_used > 0 && g_ids[g_used - 1] == id && g_streams[g_used - 1] == s;
  if (g_extend || g_used >= g_ids.size()) return;
  g_ids[g_used] = id;
  g_streams[g_used] = s;
  g_count[g_used] = 0;
  (void)hipEventRecord(g_events[2 * g_used], s);
}
void dsvt_prof_mark_end(int id, hipStream_t s) {
  if (!g_enabled) return;
  (void)id;
  if (g_extend) {                    // move the previous record's end behind this launch
    (void)hipEventRecord(g_events[2 * (g_used - 1) + 1], s);
    ++g_count[g_used - 1];
    return;
  }
  if (g_used >= g_ids.size()) return;
  (void)hipEventRecord(g_events[2 * g_used + 1], s);
  g_count[g_used] = 1;
  ++g_used;
}

extern "C" int dsvt_prof_enable(int32_t max_launches) {
  if (max_launches <= 0) return DSVT_EINVAL;
  if (g_enabled) return DSVT_EINVAL;
  g_events.resize(2 * (size_t)max_launches);
  g_ids.assign((size_t)max_launches, -1);
  g_count.assign((size_t)max_launches, 0);
  g_streams.assign((size_t)max_launches, nullptr);
  g_extend = false;
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
    launches[g_ids[r]] += g_count[r];
  }
  for (auto& e : g_events) (void)hipEventDestroy(e);
  g_events.clear(); g_ids.clear(); g_count.clear(); g_streams.clear(); g_used = 0; g_enabled = false;
  return DSVT_OK;
}

extern "C" int32_t dsvt_prof_kernel_count(void) { return DSVT_K_COUNT; }
extern "C" const char* dsvt_prof_kernel_name(int32_t id) { return (id >= 0 && id < DSVT_K_COUNT) ? kNames[id] : ""; }

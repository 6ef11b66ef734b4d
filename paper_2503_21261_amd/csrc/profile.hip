// Optional per-stage timing with HIP events, for the benchmark's roofline
// figures.  Off by default; when on, every kernel the library launches is
// bracketed by two events recorded on the launch stream.
#include <mutex>
#include <vector>

#include "hot_host.h"

namespace hot {

namespace {
struct Record {
  int stage;
  hipEvent_t start, stop;
};
std::mutex g_mu;
bool g_on = false;
std::vector<Record> g_records;
std::vector<hipEvent_t> g_pool;
std::vector<int> g_sequence;   // stages of the last finished recording, in launch order

hipEvent_t take_event() {
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

void stage_begin(int stage, hipStream_t s) {
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_on) return;
  Record r{stage, take_event(), take_event()};
  if (!r.start || !r.stop) return;
  (void)hipEventRecord(r.start, s);
  g_records.push_back(r);
}

void stage_end(int stage, hipStream_t s) {
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_on || g_records.empty() || g_records.back().stage != stage) return;
  (void)hipEventRecord(g_records.back().stop, s);
}

const char* const kStageNames[HOT_NUM_STAGES] = {
    "unused",        "act_col_absmax", "act_col_quant", "w_col_absmax",  "w_col_quant",
    "gy_row_quant",  "gy_row_absmax",  "gy_row_quant2", "gx_igemm",      "gyT_col_absmax",
    "gyT_col_quant", "gw_igemm",       "w_and_gy_row_quant", "gy_fused_absmax", "gy_fused_quant"};

}  // namespace hot

extern "C" {

hot_status hot_debug_profile_begin(void) {
  std::lock_guard<std::mutex> lock(hot::g_mu);
  for (auto& r : hot::g_records) {
    hot::g_pool.push_back(r.start);
    hot::g_pool.push_back(r.stop);
  }
  hot::g_records.clear();
  hot::g_on = true;
  return HOT_OK;
}

hot_status hot_debug_profile_end(float* stage_ms, int64_t* stage_launches) {
  std::lock_guard<std::mutex> lock(hot::g_mu);
  hot::g_on = false;
  if (!stage_ms || !stage_launches) return HOT_ERR_ARG;
  for (int i = 0; i < HOT_NUM_STAGES; ++i) {
    stage_ms[i] = 0.0f;
    stage_launches[i] = 0;
  }
  hot_status st = HOT_OK;
  hot::g_sequence.clear();
  for (auto& r : hot::g_records) {
    hot::g_sequence.push_back(r.stage);
    float ms = 0.0f;
    if (hipEventSynchronize(r.stop) != hipSuccess ||
        hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) {
      st = HOT_ERR_DEVICE;
    } else if (r.stage >= 0 && r.stage < HOT_NUM_STAGES) {
      stage_ms[r.stage] += ms;
      stage_launches[r.stage] += 1;
    }
    hot::g_pool.push_back(r.start);
    hot::g_pool.push_back(r.stop);
  }
  hot::g_records.clear();
  return st;
}

int64_t hot_debug_profile_sequence(int32_t* stages, int64_t capacity) {
  std::lock_guard<std::mutex> lock(hot::g_mu);
  const int64_t n = (int64_t)hot::g_sequence.size();
  for (int64_t i = 0; stages && i < n && i < capacity; ++i) stages[i] = hot::g_sequence[(size_t)i];
  return n;
}

const char* hot_debug_stage_name(int stage) {
  return (stage >= 0 && stage < HOT_NUM_STAGES) ? hot::kStageNames[stage] : "";
}

}  // extern "C"

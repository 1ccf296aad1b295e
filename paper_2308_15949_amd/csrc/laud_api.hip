// Status strings and ABI version of the dynamic-bottleneck library.
#include "laud_common.h"

#include <vector>

namespace laud {

bool g_stage_timing_on = false;

namespace {
struct StageRec { int stage; hipEvent_t e0, e1; };
std::vector<StageRec> g_recs;       // collected this round
std::vector<hipEvent_t> g_pool;     // events ready for reuse
constexpr size_t kMaxRecs = 65536;
bool g_open = false;                // a begin mark without its end

hipEvent_t take_event() {
  if (!g_pool.empty()) { hipEvent_t e = g_pool.back(); g_pool.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}
void recycle() {
  for (auto& r : g_recs) { if (r.e0) g_pool.push_back(r.e0); if (r.e1) g_pool.push_back(r.e1); }
  g_recs.clear();
  g_open = false;
}
}  // namespace

void stage_mark(int stage, hipStream_t stream, bool begin) {
  if (begin) {
    g_open = false;
    if (g_recs.size() >= kMaxRecs) return;
    StageRec r{stage, take_event(), take_event()};
    if (!r.e0 || !r.e1) return;
    if (hipEventRecord(r.e0, stream) != hipSuccess) return;
    g_recs.push_back(r);
    g_open = true;
  } else if (g_open) {
    (void)hipEventRecord(g_recs.back().e1, stream);
    g_open = false;
  }
}

}  // namespace laud

extern "C" const char* laud_status_string(int status) {
  switch (status) {
    case LAUD_OK: return "LAUD_OK";
    case LAUD_ERR_INVALID_ARG: return "LAUD_ERR_INVALID_ARG: null pointer, bad dimension, or S/D does not divide";
    case LAUD_ERR_UNSUPPORTED: return "LAUD_ERR_UNSUPPORTED: dtype or shape outside what the kernels cover";
    case LAUD_ERR_WORKSPACE: return "LAUD_ERR_WORKSPACE: workspace missing or too small";
    case LAUD_ERR_HIP: return "LAUD_ERR_HIP: kernel launch failed";
    case LAUD_ERR_SCRATCH_LIMIT:
      return "LAUD_ERR_SCRATCH_LIMIT: shapes need more scratch than the allocation-free entry point's fixed array";
    default: return "LAUD: unknown status";
  }
}

extern "C" int laud_abi_version(void) { return 4; }

extern "C" int laud_stage_timing_enable(int on) {
  laud::recycle();
  laud::g_stage_timing_on = on != 0;
  return LAUD_OK;
}

extern "C" int laud_stage_timing_read(double* total_ms, int64_t* launches) {
  if (!total_ms || !launches) return LAUD_ERR_INVALID_ARG;
  for (int i = 0; i < LAUD_STAGE_COUNT; ++i) { total_ms[i] = 0.0; launches[i] = 0; }
  int rc = LAUD_OK;
  for (auto& r : laud::g_recs) {
    float ms = 0.f;
    if (hipEventSynchronize(r.e1) != hipSuccess || hipEventElapsedTime(&ms, r.e0, r.e1) != hipSuccess) {
      rc = LAUD_ERR_HIP;
      continue;
    }
    if (r.stage >= 0 && r.stage < LAUD_STAGE_COUNT) { total_ms[r.stage] += ms; launches[r.stage] += 1; }
  }
  laud::recycle();
  return rc;
}

extern "C" const char* laud_stage_name(int stage) {
  static const char* names[LAUD_STAGE_COUNT] = {"mask_logits", "compact", "gather", "copy_inactive", "need",
                                               "conv1", "conv2", "conv3", "cs1", "cs2", "cs3", "scatter", "se"};
  return (stage >= 0 && stage < LAUD_STAGE_COUNT) ? names[stage] : "?";
}

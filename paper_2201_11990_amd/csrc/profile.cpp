// Optional per-kernel-class timing with HIP events on the launch stream.
#include <vector>

#include "common.h"

namespace mtnlg {

struct EventPair {
  int cls;
  hipEvent_t start, stop;
};

static bool g_enabled = false;
static std::vector<EventPair> g_records;
static std::vector<EventPair> g_pool;

LaunchScope::LaunchScope(int cls_, hipStream_t s) : cls(cls_), stream(s), idx(-1) {
  if (!g_enabled) return;
  EventPair ep;
  if (!g_pool.empty()) {
    ep = g_pool.back();
    g_pool.pop_back();
  } else {
    if (hipEventCreate(&ep.start) != hipSuccess) return;
    if (hipEventCreate(&ep.stop) != hipSuccess) {
      (void)hipEventDestroy(ep.start);
      return;
    }
  }
  ep.cls = cls;
  (void)hipEventRecord(ep.start, stream);
  g_records.push_back(ep);
  idx = (long)g_records.size() - 1;
}

LaunchScope::~LaunchScope() {
  if (idx >= 0 && idx < (long)g_records.size()) (void)hipEventRecord(g_records[idx].stop, stream);
}

}  // namespace mtnlg

using namespace mtnlg;

extern "C" int mtnlg_profile_enable(int on) {
  if (on) {
    g_enabled = true;
    return MTNLG_OK;
  }
  g_enabled = false;
  for (auto &ep : g_records) g_pool.push_back(ep);
  g_records.clear();
  for (auto &ep : g_pool) {
    (void)hipEventDestroy(ep.start);
    (void)hipEventDestroy(ep.stop);
  }
  g_pool.clear();
  return MTNLG_OK;
}

extern "C" int mtnlg_profile_read(int32_t *launches, float *ms) {
  if (!launches || !ms) return MTNLG_NULL_POINTER;
  for (int i = 0; i < MTNLG_K_CLASSES; ++i) {
    launches[i] = 0;
    ms[i] = 0.0f;
  }
  int status = MTNLG_OK;
  for (auto &ep : g_records) {
    float t = 0.0f;
    if (hipEventSynchronize(ep.stop) != hipSuccess || hipEventElapsedTime(&t, ep.start, ep.stop) != hipSuccess) {
      status = MTNLG_HIP_ERROR;
    } else if (ep.cls >= 0 && ep.cls < MTNLG_K_CLASSES) {
      launches[ep.cls] += 1;
      ms[ep.cls] += t;
    }
    g_pool.push_back(ep);
  }
  g_records.clear();
  return status;
}

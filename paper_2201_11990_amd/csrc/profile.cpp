// Optional per-kernel-class timing with HIP events on the launch stream.
//
// Every scope records one event when it closes.  A scope that opens on the stream on which the previous
// scope closed takes that event as its beginning (the two would sit back to back in the queue with the
// same time stamp), so a run of launches costs one event each instead of two; only the first scope after
// timing is switched on, after a read-out, or after a change of stream records a beginning of its own.
// A scope's time therefore runs from the end of the previous scope: whatever else the caller puts on the
// stream between two scopes is counted for the second.
#include <vector>

#include "common.h"

namespace mtnlg {

struct Record {
  int cls;
  hipEvent_t begin, end;
};

static bool g_enabled = false;
static std::vector<Record> g_records;
static std::vector<hipEvent_t> g_used;   // every event referenced by g_records, once
static std::vector<hipEvent_t> g_pool;
static hipEvent_t g_chain_end = nullptr;  // closing event of the latest scope, nullptr: chain broken
static hipStream_t g_chain_stream = nullptr;

static hipEvent_t take_event() {
  hipEvent_t e = nullptr;
  if (!g_pool.empty()) {
    e = g_pool.back();
    g_pool.pop_back();
  } else if (hipEventCreate(&e) != hipSuccess) {
    return nullptr;
  }
  g_used.push_back(e);
  return e;
}

LaunchScope::LaunchScope(int cls_, hipStream_t s) : cls(cls_), stream(s), idx(-1) {
  if (!g_enabled) return;
  Record r{cls, nullptr, nullptr};
  if (g_chain_end && g_chain_stream == stream) {
    r.begin = g_chain_end;
  } else {
    r.begin = take_event();
    if (!r.begin) return;
    (void)hipEventRecord(r.begin, stream);
  }
  r.end = take_event();
  if (!r.end) return;
  g_records.push_back(r);
  idx = (long)g_records.size() - 1;
}

LaunchScope::~LaunchScope() {
  if (idx < 0 || idx >= (long)g_records.size()) return;
  (void)hipEventRecord(g_records[idx].end, stream);
  g_chain_end = g_records[idx].end;
  g_chain_stream = stream;
}

}  // namespace mtnlg

using namespace mtnlg;

extern "C" int mtnlg_profile_enable(int on) {
  if (on) {
    if (!g_enabled) g_chain_end = nullptr;
    g_enabled = true;
    return MTNLG_OK;
  }
  g_enabled = false;
  g_chain_end = nullptr;
  g_records.clear();
  for (hipEvent_t e : g_used) g_pool.push_back(e);
  g_used.clear();
  for (hipEvent_t e : g_pool) (void)hipEventDestroy(e);
  g_pool.clear();
  return MTNLG_OK;
}

// Stop (paused != 0) or resume recording without touching what has been recorded: lets a caller bracket some of
// its steps and leave the others free of events.
extern "C" int mtnlg_profile_pause(int paused) {
  g_enabled = !paused;
  g_chain_end = nullptr;   // the next scope records a beginning of its own
  return MTNLG_OK;
}

extern "C" int mtnlg_profile_read(int32_t *launches, float *ms) {
  if (!launches || !ms) return MTNLG_NULL_POINTER;
  for (int i = 0; i < MTNLG_K_CLASSES; ++i) {
    launches[i] = 0;
    ms[i] = 0.0f;
  }
  int status = MTNLG_OK;
  for (auto &r : g_records) {
    float t = 0.0f;
    if (hipEventSynchronize(r.end) != hipSuccess || hipEventElapsedTime(&t, r.begin, r.end) != hipSuccess) {
      status = MTNLG_HIP_ERROR;
    } else if (r.cls >= 0 && r.cls < MTNLG_K_CLASSES) {
      launches[r.cls] += 1;
      ms[r.cls] += t;
    }
  }
  g_records.clear();
  g_chain_end = nullptr;
  for (hipEvent_t e : g_used) g_pool.push_back(e);
  g_used.clear();
  return status;
}

// Benchmark aids, linked into libla_verify_bench.so only: per-kernel event timing (the hooks the launchers call when
// they are present), and the self-test entry of the accept path's fp64 exponential.  The product library does not
// contain this translation unit; its launchers then find the hooks absent and do nothing.
#include <vector>

#include "la_internal.hpp"
#include "la_verify_bench.h"

namespace la {
namespace {

const char *kSlotNames[SLOT_COUNT] = {"attn_mfma",     "attn_merge",   "attn_f32",   "accept_stats", "accept_warp",
                                      "accept_decide", "accept_resid", "accept_pick", "kv_commit",
                                      "calib_mfma",    "calib_read"};
struct ProfileRecord {
  int slot;
  hipEvent_t start, stop;
};
// process-wide state of the timing aid (not thread-safe, as its header says)
bool g_profile_on = false;
uint32_t g_profile_mask = 0xffffffffu;      // slots that are timed
int g_profile_stride = 1;                   // of their launches, every stride-th one
int64_t g_seen[SLOT_COUNT];                 // launches of a slot seen while enabled
std::vector<ProfileRecord> g_records;       // pending (not yet collected)
std::vector<hipEvent_t> g_free_events;
int64_t g_launches[SLOT_COUNT];
double g_total_ms[SLOT_COUNT];

hipEvent_t take_event() {
  if (!g_free_events.empty()) {
    hipEvent_t e = g_free_events.back();
    g_free_events.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

}  // namespace

void *profile_before(int slot, hipStream_t stream) {
  if (!g_profile_on || !((g_profile_mask >> slot) & 1u)) return nullptr;
  if ((g_seen[slot]++ % g_profile_stride) != 0 || g_records.size() >= LA_PROFILE_MAX_RECORDS) return nullptr;
  hipEvent_t e = take_event();
  if (!e) return nullptr;
  if (hipEventRecord(e, stream) != hipSuccess) {
    g_free_events.push_back(e);
    return nullptr;
  }
  return e;
}

void profile_after(int slot, hipStream_t stream, void *start) {
  if (!start) return;
  hipEvent_t e = take_event();
  if (!e || hipEventRecord(e, stream) != hipSuccess) {
    if (e) g_free_events.push_back(e);
    g_free_events.push_back((hipEvent_t)start);
    return;
  }
  g_records.push_back({slot, (hipEvent_t)start, e});
}

}  // namespace la

using namespace la;

extern "C" {

la_status la_selftest_exp64(const double *y, double *out, size_t n, void *hip_stream) {
  if (!y || !out || n < 1 || n > ((size_t)1 << 30)) return LA_ERR_INVALID_ARG;
  return launch_exp64_probe(y, out, n, (hipStream_t)hip_stream) == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

la_status la_profile_select(uint32_t slot_mask, int32_t stride) {
  if (stride < 1) return LA_ERR_INVALID_ARG;
  g_profile_mask = slot_mask;
  g_profile_stride = stride;
  return LA_OK;
}

la_status la_profile_enable(int on) {
  g_profile_on = on != 0;
  return LA_OK;
}

la_status la_profile_collect(void) {
  la_status st = LA_OK;
  for (const ProfileRecord &r : g_records) {
    float ms = 0.f;
    if (hipEventSynchronize(r.stop) == hipSuccess && hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess) {
      g_launches[r.slot] += 1;
      g_total_ms[r.slot] += ms;
    } else {
      st = LA_ERR_LAUNCH;
    }
    g_free_events.push_back(r.start);
    g_free_events.push_back(r.stop);
  }
  g_records.clear();
  return st;
}

int32_t la_profile_num_kernels(void) { return SLOT_COUNT; }

la_status la_profile_get(int32_t slot, const char **name, int64_t *launches, double *total_ms) {
  if (slot < 0 || slot >= SLOT_COUNT) return LA_ERR_INVALID_ARG;
  if (name) *name = kSlotNames[slot];
  if (launches) *launches = g_launches[slot];
  if (total_ms) *total_ms = g_total_ms[slot];
  return LA_OK;
}

la_status la_profile_reset(void) {
  la_status st = la_profile_collect();
  for (int i = 0; i < SLOT_COUNT; ++i) g_launches[i] = 0, g_total_ms[i] = 0.0, g_seen[i] = 0;
  return st;
}

}  // extern "C"

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
int g_force_second_attempt = 0;
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

int selftest_force_second_attempt() { return g_force_second_attempt; }

}  // namespace la

using namespace la;

extern "C" {

la_status la_selftest_exp64(const double *y, double *out, size_t n, void *hip_stream) {
  if (!y || !out || n < 1 || n > ((size_t)1 << 30)) return LA_ERR_INVALID_ARG;
  return launch_exp64_probe(y, out, n, (hipStream_t)hip_stream) == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

la_status la_selftest_second_attempt(int on) {
  g_force_second_attempt = on != 0;
  return LA_OK;
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

// ---- index checks (debug aid) --------------------------------------------------------------------------------
namespace la {
namespace {

__global__ void check_reset_kernel(int32_t *report) {
  if (threadIdx.x == 0) report[0] = 0, report[1] = -1, report[2] = -1;
}

// entry (b, j) for j < used[b] (kMaxInline requests per launch: their block counts travel in the arguments)
struct CheckTables {
  const int32_t *tables;  // or null: identity
  int32_t *report;
  long long limit;        // ids must lie in [0, limit)
  int max_blocks, first_request, n_requests;
  int used[64];
};
__global__ __launch_bounds__(256) void check_tables_kernel(const CheckTables c) {
  const int r = blockIdx.y;
  if (r >= c.n_requests) return;
  const int b = c.first_request + r;
  for (int j = blockIdx.x * 256 + threadIdx.x; j < c.used[r]; j += gridDim.x * 256) {
    const long long id = c.tables ? (long long)c.tables[(size_t)b * c.max_blocks + j] : (long long)b * c.max_blocks + j;
    if (id < 0 || id >= c.limit) {
      atomicAdd(&c.report[0], 1);
      c.report[1] = b, c.report[2] = j;  // any one offender
    }
  }
}

__global__ __launch_bounds__(256) void check_tokens_kernel(const int32_t *tokens, int n, int k, int vocab,
                                                           int32_t *report) {
  for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += gridDim.x * 256) {
    const int t = tokens[i];
    if (t < 0 || t >= vocab) {
      atomicAdd(&report[0], 1);
      report[1] = i / k, report[2] = i % k;
    }
  }
}

}  // namespace
}  // namespace la

extern "C" {

la_status la_check_block_tables(const la_attn_desc *d, const int32_t *block_tables, const int32_t *prefix_lens_host,
                                int32_t extra_tokens, int64_t num_cache_blocks, int32_t *report, void *hip_stream) {
  if (!d || !prefix_lens_host || !report || extra_tokens < 0 || num_cache_blocks < 0) return LA_ERR_INVALID_ARG;
  if (d->num_requests < 1 || d->block_size < 16 || (d->block_size & (d->block_size - 1)) || d->max_blocks_per_request < 0)
    return LA_ERR_INVALID_ARG;
  for (int b = 0; b < d->num_requests; ++b) {
    const int64_t need = ((int64_t)prefix_lens_host[b] + extra_tokens + d->block_size - 1) / d->block_size;
    if (prefix_lens_host[b] < 0 || need > d->max_blocks_per_request) return LA_ERR_INVALID_ARG;
  }
  hipStream_t st = (hipStream_t)hip_stream;
  hipLaunchKernelGGL(la::check_reset_kernel, dim3(1), dim3(64), 0, st, report);
  for (int first = 0; first < d->num_requests; first += 64) {
    la::CheckTables c{};
    c.tables = block_tables, c.report = report, c.limit = num_cache_blocks, c.max_blocks = d->max_blocks_per_request;
    c.first_request = first, c.n_requests = d->num_requests - first < 64 ? d->num_requests - first : 64;
    int most = 0;
    for (int r = 0; r < c.n_requests; ++r) {
      c.used[r] = (int)(((int64_t)prefix_lens_host[first + r] + extra_tokens + d->block_size - 1) / d->block_size);
      most = c.used[r] > most ? c.used[r] : most;
    }
    if (most == 0) continue;
    const int gx = (most + 255) / 256 < 64 ? (most + 255) / 256 : 64;
    hipLaunchKernelGGL(la::check_tables_kernel, dim3(gx, c.n_requests), dim3(256), 0, st, c);
  }
  return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

la_status la_check_draft_tokens(const la_accept_desc *d, const int32_t *draft_tokens, int32_t *report,
                                void *hip_stream) {
  if (!d || !draft_tokens || !report || d->num_branches < 1 || d->num_draft < 1 || d->vocab < 1) return LA_ERR_INVALID_ARG;
  const int64_t n = (int64_t)d->num_branches * d->num_draft;
  if (n > ((int64_t)1 << 30)) return LA_ERR_UNSUPPORTED;
  hipStream_t st = (hipStream_t)hip_stream;
  hipLaunchKernelGGL(la::check_reset_kernel, dim3(1), dim3(64), 0, st, report);
  const int gx = (int)((n + 255) / 256 < 256 ? (n + 255) / 256 : 256);
  hipLaunchKernelGGL(la::check_tokens_kernel, dim3(gx), dim3(256), 0, st, draft_tokens, (int)n, d->num_draft, d->vocab,
                     report);
  return hipGetLastError() == hipSuccess ? LA_OK : LA_ERR_LAUNCH;
}

}  // extern "C"

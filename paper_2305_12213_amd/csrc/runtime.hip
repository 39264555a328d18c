// Error reporting and the per-kernel-class timing aid.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <mutex>
#include <vector>

#include "dynb_internal.h"

namespace dynb {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

namespace {
struct Pending {
  int cls;
  hipEvent_t start, stop;
};
struct ClassTotals {
  double ms = 0, flops = 0, bytes = 0;
  int64_t launches = 0;
};
std::mutex g_mu;
bool g_on = false;
std::vector<Pending> g_pending;
std::vector<hipEvent_t> g_free_events;
ClassTotals g_totals[KC_COUNT];

hipEvent_t get_event() {
  if (!g_free_events.empty()) {
    hipEvent_t e = g_free_events.back();
    g_free_events.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}
const char* kNames[KC_COUNT] = {"gemm_fwd",  "gemm_dgrad", "gemm_wgrad", "pack_input",
                                "transpose", "softmax_xent", "bias_grad", "finalize",
                                "weighted_aggregate", "sgd_update", "weight_cast", "conv_aux", "norm_add",
                                "gemm_wgrad_small_tiles", "gemm_small_tiles"};
}  // namespace

// The bracket holds its two events itself and hands them to the pending list only when both
// are recorded, so a dynb_profile_collect() on another thread in between cannot take them away.
Timed::Timed(KClass c, void* s, double flops, double bytes)
    : cls(-1), stream(s), start(nullptr), stop(nullptr) {
  if (!g_on) return;
  std::lock_guard<std::mutex> lk(g_mu);
  hipEvent_t a = get_event(), b = get_event();
  if (!a || !b) {
    if (a) g_free_events.push_back(a);
    if (b) g_free_events.push_back(b);
    return;
  }
  g_totals[c].flops += flops;
  g_totals[c].bytes += bytes;
  g_totals[c].launches += 1;
  (void)hipEventRecord(a, (hipStream_t)stream);
  cls = c;
  start = a;
  stop = b;
}

Timed::~Timed() {
  if (cls < 0) return;
  (void)hipEventRecord((hipEvent_t)stop, (hipStream_t)stream);
  std::lock_guard<std::mutex> lk(g_mu);
  Pending p;
  p.cls = cls;
  p.start = (hipEvent_t)start;
  p.stop = (hipEvent_t)stop;
  g_pending.push_back(p);
}

}  // namespace dynb

using namespace dynb;

extern "C" const char* dynb_last_error(void) { return g_err; }

extern "C" int dynb_profile_enable(int32_t on) {
  std::lock_guard<std::mutex> lk(g_mu);
  g_on = on != 0;
  return DYNB_OK;
}

extern "C" int dynb_profile_collect(void) {
  std::lock_guard<std::mutex> lk(g_mu);
  for (auto& p : g_pending) {
    if (hipEventSynchronize(p.stop) != hipSuccess)
      return fail(DYNB_ERR_HIP, "profile: hipEventSynchronize failed");
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, p.start, p.stop) == hipSuccess) g_totals[p.cls].ms += ms;
    g_free_events.push_back(p.start);
    g_free_events.push_back(p.stop);
  }
  g_pending.clear();
  return DYNB_OK;
}

extern "C" int dynb_profile_reset(void) {
  int rc = dynb_profile_collect();
  std::lock_guard<std::mutex> lk(g_mu);
  for (auto& t : g_totals) t = ClassTotals();
  return rc;
}

extern "C" int32_t dynb_profile_num_classes(void) { return KC_COUNT; }

extern "C" const char* dynb_profile_name(int32_t cls) {
  return (cls >= 0 && cls < KC_COUNT) ? kNames[cls] : "";
}

extern "C" int dynb_profile_get(int32_t cls, double* total_ms, int64_t* launches, double* flops,
                                double* bytes) {
  if (cls < 0 || cls >= KC_COUNT) return fail(DYNB_ERR_BADARG, "profile: class out of range");
  std::lock_guard<std::mutex> lk(g_mu);
  if (total_ms) *total_ms = g_totals[cls].ms;
  if (launches) *launches = g_totals[cls].launches;
  if (flops) *flops = g_totals[cls].flops;
  if (bytes) *bytes = g_totals[cls].bytes;
  return DYNB_OK;
}

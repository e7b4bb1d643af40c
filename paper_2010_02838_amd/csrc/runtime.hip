// Error reporting and the per-kernel-class timer of the codistillation-step library.
#include "common.h"
#include <cstdarg>
#include <cstdio>
#include <mutex>
#include <vector>

namespace cd {

static thread_local char g_err[512] = "";

int set_error(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(CD_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
  return CD_OK;
}

// ---- timer --------------------------------------------------------------------------------
struct ProfRec {
  int cls;
  hipEvent_t a, b;
};
struct ProfTotals {
  double ms = 0, flops = 0, bytes = 0;
  int64_t launches = 0;
};
static std::mutex g_prof_mu;
static bool g_prof_on = false;
static std::vector<ProfRec> g_prof_recs;
static std::vector<hipEvent_t> g_prof_free;
static ProfTotals g_prof_tot[CD_K_COUNT];

static hipEvent_t take_event() {
  if (!g_prof_free.empty()) {
    hipEvent_t e = g_prof_free.back();
    g_prof_free.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

ProfScope::ProfScope(int cls, hipStream_t s, double flops, double bytes) : idx(-1), stream(s) {
  if (!g_prof_on) return;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  ProfRec r;
  r.cls = cls;
  r.a = take_event();
  r.b = take_event();
  if (!r.a || !r.b) return;
  g_prof_tot[cls].flops += flops;
  g_prof_tot[cls].bytes += bytes;
  g_prof_tot[cls].launches += 1;
  (void)hipEventRecord(r.a, s);
  g_prof_recs.push_back(r);
  idx = static_cast<int>(g_prof_recs.size()) - 1;
}

ProfScope::~ProfScope() {
  if (idx < 0) return;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  (void)hipEventRecord(g_prof_recs[idx].b, stream);
}

bool timer_enabled() {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  return g_prof_on;
}

// ---- side stream --------------------------------------------------------------------------
static std::mutex g_side_mu;
static hipStream_t g_side_stream = nullptr;
static bool g_side_failed = false;
static std::vector<hipEvent_t> g_side_events;

hipStream_t side_stream() {
  std::lock_guard<std::mutex> lk(g_side_mu);
  if (!g_side_stream && !g_side_failed) {
    if (hipStreamCreateWithFlags(&g_side_stream, hipStreamNonBlocking) != hipSuccess) {
      g_side_stream = nullptr;
      g_side_failed = true;
      (void)hipGetLastError();
    }
  }
  return g_side_stream;
}

std::mutex& side_mutex() {
  static std::mutex mu;
  return mu;
}

hipEvent_t side_event(int i) {
  std::lock_guard<std::mutex> lk(g_side_mu);
  while ((int)g_side_events.size() <= i) {
    hipEvent_t e = nullptr;
    if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_side_events.push_back(e);
  }
  return g_side_events[i];
}

}  // namespace cd

using namespace cd;

// an empty launch, for measuring what a pair of events adds to a launch it brackets
__global__ void empty_kernel() {}

extern "C" int codistill_profile_event_overhead(double* microseconds, void* stream) {
  CD_REQUIRE(microseconds != nullptr, "profile_event_overhead: output pointer is NULL");
  hipStream_t s = static_cast<hipStream_t>(stream);
  constexpr int N = 200;
  std::vector<hipEvent_t> ev(2 * N, nullptr);
  int rc = CD_OK;
  for (auto& e : ev)
    if (hipEventCreate(&e) != hipSuccess) rc = set_error(CD_ERR_HIP, "profile_event_overhead: cannot create events");
  double total = 0;
  if (rc == CD_OK) {
    for (int i = 0; i < N; i++) {
      (void)hipEventRecord(ev[2 * i], s);
      hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, s);
      (void)hipEventRecord(ev[2 * i + 1], s);
    }
    if (hipStreamSynchronize(s) != hipSuccess) rc = set_error(CD_ERR_HIP, "profile_event_overhead: synchronise failed");
    for (int i = N / 2; i < N && rc == CD_OK; i++) {   // the second half: the first launches warm the path up
      float ms = 0;
      if (hipEventElapsedTime(&ms, ev[2 * i], ev[2 * i + 1]) != hipSuccess)
        rc = set_error(CD_ERR_HIP, "profile_event_overhead: elapsed time unavailable");
      total += ms;
    }
  }
  for (auto& e : ev)
    if (e) (void)hipEventDestroy(e);
  if (rc == CD_OK) *microseconds = total * 1e3 / (N / 2);
  return rc;
}

extern "C" int codistill_profile_enable(int on) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  g_prof_on = on != 0;
  return CD_OK;
}

extern "C" int codistill_profile_collect(void) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  int rc = CD_OK;
  for (auto& r : g_prof_recs) {
    float ms = 0;
    hipError_t e = hipEventSynchronize(r.b);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.a, r.b);
    if (e != hipSuccess)
      rc = set_error(CD_ERR_HIP, "profile_collect: %s", hipGetErrorString(e));
    else
      g_prof_tot[r.cls].ms += ms;
    g_prof_free.push_back(r.a);
    g_prof_free.push_back(r.b);
  }
  g_prof_recs.clear();
  return rc;
}

extern "C" int codistill_profile_get(int k, double* ms, int64_t* launches, double* flops, double* bytes) {
  CD_REQUIRE(k >= 0 && k < CD_K_COUNT, "profile_get: unknown kernel class %d", k);
  std::lock_guard<std::mutex> lk(g_prof_mu);
  if (ms) *ms = g_prof_tot[k].ms;
  if (launches) *launches = g_prof_tot[k].launches;
  if (flops) *flops = g_prof_tot[k].flops;
  if (bytes) *bytes = g_prof_tot[k].bytes;
  return CD_OK;
}

extern "C" int codistill_profile_reset(void) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  for (auto& t : g_prof_tot) t = ProfTotals();
  return CD_OK;
}

extern "C" const char* codistill_last_error(void) { return g_err; }
extern "C" const char* codistill_version(void) { return "codistill-gfx950 0.1"; }

// Per-launch kernel timing behind ftp_ktrace_begin / ftp_ktrace_end.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <map>
#include <string>
#include <vector>

#include "../../include/ftp.h"
#include "kernels.h"

void ftp_set_error(const char* fmt, ...);

namespace {
struct Rec { const char* name; double bytes, flops; long d[3]; hipEvent_t e0, e1; };
struct Trace {
  bool on = false;
  std::vector<Rec> recs;
  size_t used = 0;
  bool overflow = false;
  bool detail = false;   // one row per (kernel family, problem shape) instead of per family
  double bracket_overhead_ms = 0.0;   // what a pair of events adds to the launch it brackets (measured at begin)
} g_trace;

__global__ void ktrace_noop_k() {}

// The time between the two events around a launch is the kernel plus what the events themselves cost.  With e1 the
// bracket around one empty kernel and e2 the bracket around two of them, the second kernel costs e2 - e1 and the
// bracket alone 2*e1 - e2 (medians of 64 samples each on a stream of its own).
double measure_bracket_overhead_ms() {
  hipStream_t st = nullptr;
  hipEvent_t a = nullptr, b = nullptr;
  if (hipStreamCreateWithFlags(&st, hipStreamNonBlocking) != hipSuccess) return 0.0;
  double out = 0.0;
  if (hipEventCreate(&a) == hipSuccess && hipEventCreate(&b) == hipSuccess) {
    std::vector<float> t[2];
    for (int rep = 0; rep < 72; ++rep)
      for (int n = 1; n <= 2; ++n) {
        (void)hipEventRecord(a, st);
        for (int k = 0; k < n; ++k) hipLaunchKernelGGL(ktrace_noop_k, dim3(1), dim3(64), 0, st);
        (void)hipEventRecord(b, st);
        (void)hipStreamSynchronize(st);
        float ms = 0.f;
        if (rep >= 8 && hipEventElapsedTime(&ms, a, b) == hipSuccess) t[n - 1].push_back(ms);
      }
    if (!t[0].empty() && !t[1].empty()) {
      for (auto& v : t) std::nth_element(v.begin(), v.begin() + v.size() / 2, v.end());
      out = 2.0 * t[0][t[0].size() / 2] - t[1][t[1].size() / 2];
      if (out < 0.0) out = 0.0;
    }
  }
  if (a) (void)hipEventDestroy(a);
  if (b) (void)hipEventDestroy(b);
  (void)hipStreamDestroy(st);
  return out;
}
}  // namespace

namespace ftp {
// per thread, like the error text: the launcher that fails and the stage call that reports it run on one thread
static thread_local const char* g_plan_failure = nullptr;
void launch_plan_failed(const char* what) { g_plan_failure = what; }
const char* launch_plan_failure_take() { const char* w = g_plan_failure; g_plan_failure = nullptr; return w; }

KScope::KScope(hipStream_t s, const char* name, double alg_bytes, double flops, long d0, long d1, long d2) : slot(-1), st(s) {
  if (!g_trace.on) return;
  if (g_trace.used >= g_trace.recs.size()) { g_trace.overflow = true; return; }
  slot = (int)g_trace.used++;
  Rec& r = g_trace.recs[slot];
  r.name = name; r.bytes = alg_bytes; r.flops = flops; r.d[0] = d0; r.d[1] = d1; r.d[2] = d2;
  (void)hipEventRecord(r.e0, st);
}
KScope::~KScope() {
  if (slot >= 0) (void)hipEventRecord(g_trace.recs[slot].e1, st);
}
}  // namespace ftp

extern "C" int ftp_diag_fail_next_launch_plan(void) {
  ftp::launch_plan_failed("launch plan failure requested through ftp_diag_fail_next_launch_plan");
  return FTP_OK;
}

static void trace_release() {
  for (auto& r : g_trace.recs) { (void)hipEventDestroy(r.e0); (void)hipEventDestroy(r.e1); }
  g_trace.recs.clear();
  g_trace.used = 0;
  g_trace.on = false;
}

extern "C" int ftp_ktrace_begin(int max_launches) {
  g_trace.detail = max_launches < 0;      // negative: rows per problem shape ("name d0 d1 d2")
  if (max_launches < 0) max_launches = -max_launches;
  if (max_launches < 1 || max_launches > (1 << 20)) { ftp_set_error("ktrace_begin: max_launches out of range"); return FTP_ERR_ARG; }
  trace_release();
  g_trace.recs.resize(max_launches);
  for (auto& r : g_trace.recs) {
    if (hipEventCreate(&r.e0) != hipSuccess || hipEventCreate(&r.e1) != hipSuccess) {
      ftp_set_error("ktrace_begin: hipEventCreate failed");
      trace_release();
      return FTP_ERR_HIP;
    }
  }
  g_trace.overflow = false;
  g_trace.bracket_overhead_ms = measure_bracket_overhead_ms();
  g_trace.on = true;
  return FTP_OK;
}

extern "C" int ftp_ktrace_end(ftp_ktrace_row* rows, int max_rows, int* n_rows) {
  if (!rows || !n_rows || max_rows < 1) { ftp_set_error("ktrace_end: bad argument"); return FTP_ERR_ARG; }
  g_trace.on = false;
  if (hipDeviceSynchronize() != hipSuccess) { ftp_set_error("ktrace_end: synchronize failed"); trace_release(); return FTP_ERR_HIP; }
  std::map<std::string, ftp_ktrace_row> agg;
  for (size_t i = 0; i < g_trace.used; ++i) {
    Rec& r = g_trace.recs[i];
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.e0, r.e1) != hipSuccess) continue;
    char key[48];
    if (g_trace.detail && r.d[0] >= 0) snprintf(key, sizeof(key), "%s %ld %ld %ld", r.name, r.d[0], r.d[1], r.d[2]);
    else snprintf(key, sizeof(key), "%s", r.name);
    ftp_ktrace_row& row = agg[key];
    if (row.launches == 0) { memset(&row, 0, sizeof(row)); strncpy(row.name, key, sizeof(row.name) - 1); }
    row.launches += 1; row.total_ms += ms; row.alg_bytes += r.bytes; row.flops += r.flops;
  }
  int n = 0;
  for (auto& kv : agg) { if (n < max_rows) rows[n++] = kv.second; }
  if (n < max_rows) {      // what to take off every launch's time: the cost of the event pair itself
    ftp_ktrace_row& row = rows[n++];
    memset(&row, 0, sizeof(row));
    strncpy(row.name, "__event_pair_overhead", sizeof(row.name) - 1);
    row.launches = 1;
    row.total_ms = g_trace.bracket_overhead_ms;
  }
  *n_rows = n;
  bool ovf = g_trace.overflow;
  trace_release();
  if (ovf) { ftp_set_error("ktrace_end: more launches than max_launches; rows are incomplete"); return FTP_ERR_ARG; }
  return FTP_OK;
}

extern "C" int ftp_calibration_copy(void* dst_dev, const void* src_dev, size_t bytes, void* stream) {
  if (!dst_dev || !src_dev || bytes < 16 || (bytes % 16) != 0) { ftp_set_error("calibration_copy: need non-NULL buffers and a multiple of 16 bytes"); return FTP_ERR_ARG; }
  ftp::calibration_copy((hipStream_t)stream, src_dev, dst_dev, bytes);
  if (hipGetLastError() != hipSuccess) { ftp_set_error("calibration_copy: launch failed"); return FTP_ERR_HIP; }
  return FTP_OK;
}

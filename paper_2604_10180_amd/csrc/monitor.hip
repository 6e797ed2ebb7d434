// Online monitor (Sec. 3.4): queueing-aware switching between the latency-oriented and the
// throughput-oriented placement at fixed time windows.  Host code only.
//
// Per finished request the caller reports its completion time, its end-to-end latency (queueing
// included) and its pure execution latency as the paper's monitor collects it: one latency per kernel
// group (the kernels between two consecutive communication operations) plus the communication time.
// When a window closes, the ratio of the window's mean request latency to its mean execution latency
// is compared with the threshold beta: above it the throughput policy takes over, otherwise the
// latency policy; a window without completions leaves the policy unchanged.  State is O(1): two running
// sums and a count for the open window.
#include <cmath>
#include <new>

#include "common.hpp"

struct ts_monitor {
  double W, beta;
  int policy;
  int64_t open_window;        // index of the window still collecting
  double sum_req, sum_exec;
  int64_t count;
  int64_t windows_closed, switches;
  double last_ratio;          // NaN until a non-empty window has closed
};

namespace ts {
namespace {

// Index n of the window [n W, (n+1) W) that holds t, with the bounds evaluated as products so that a time
// that is exactly a multiple of W in floating point opens the next window.
int64_t window_of(double t, double W) {
  int64_t n = (int64_t)std::floor(t / W);
  while ((double)(n + 1) * W <= t) ++n;
  while (n > 0 && (double)n * W > t) --n;
  return n;
}

void close_windows_before(ts_monitor* m, int64_t window) {
  while (m->open_window < window) {
    if (m->count > 0) {
      const double ratio = (m->sum_req / (double)m->count) / (m->sum_exec / (double)m->count);
      const int next = ratio > m->beta ? TS_PLAN_THROUGHPUT : TS_PLAN_LATENCY;
      if (next != m->policy) ++m->switches;
      m->policy = next;
      m->last_ratio = ratio;
      m->sum_req = m->sum_exec = 0.0;
      m->count = 0;
      ++m->open_window;
      ++m->windows_closed;
    } else {                  // a run of empty windows changes nothing: skip it in one step
      m->windows_closed += window - m->open_window;
      m->open_window = window;
    }
  }
}

}  // namespace
}  // namespace ts

using namespace ts;

extern "C" {

int ts_monitor_create(double window_s, double beta, int initial_policy, ts_monitor** out) {
  TS_REQUIRE(out != nullptr, TS_ERR_INVALID_ARG, "ts_monitor_create: null output");
  TS_REQUIRE(window_s > 0.0 && std::isfinite(window_s) && beta > 0.0 && !std::isnan(beta), TS_ERR_INVALID_ARG,
             "ts_monitor_create: window %g s and threshold %g must be positive", window_s, beta);
  TS_REQUIRE(initial_policy == TS_PLAN_THROUGHPUT || initial_policy == TS_PLAN_LATENCY, TS_ERR_INVALID_ARG,
             "ts_monitor_create: unknown policy %d", initial_policy);
  ts_monitor* m = new (std::nothrow) ts_monitor();
  TS_REQUIRE(m != nullptr, TS_ERR_INVALID_ARG, "ts_monitor_create: out of host memory");
  m->W = window_s;
  m->beta = beta;
  m->policy = initial_policy;
  m->open_window = 0;
  m->sum_req = m->sum_exec = 0.0;
  m->count = 0;
  m->windows_closed = m->switches = 0;
  m->last_ratio = std::nan("");
  *out = m;
  return TS_OK;
}

void ts_monitor_destroy(ts_monitor* m) { delete m; }

int ts_monitor_record(ts_monitor* m, double t_complete_s, double request_latency_s, const double* group_latency_s,
                      int n_groups, double comm_s) {
  TS_REQUIRE(m != nullptr && n_groups >= 0 && (group_latency_s != nullptr || n_groups == 0), TS_ERR_INVALID_ARG,
             "ts_monitor_record: null argument");
  TS_REQUIRE(std::isfinite(t_complete_s) && t_complete_s >= 0.0 && std::isfinite(request_latency_s) &&
                 request_latency_s >= 0.0 && std::isfinite(comm_s) && comm_s >= 0.0,
             TS_ERR_INVALID_ARG, "ts_monitor_record: times must be finite and non-negative");
  double exec = 0.0;
  for (int i = 0; i < n_groups; ++i) {
    TS_REQUIRE(std::isfinite(group_latency_s[i]) && group_latency_s[i] >= 0.0, TS_ERR_INVALID_ARG,
               "ts_monitor_record: kernel group %d has a negative or non-finite latency", i);
    exec += group_latency_s[i];
  }
  exec += comm_s;
  TS_REQUIRE(exec > 0.0, TS_ERR_INVALID_ARG, "ts_monitor_record: a request needs a positive execution latency");
  const int64_t window = window_of(t_complete_s, m->W);
  TS_REQUIRE(window >= m->open_window, TS_ERR_INVALID_ARG,
             "ts_monitor_record: completion at %g s lies in window %lld, which has closed (open: %lld)", t_complete_s,
             (long long)window, (long long)m->open_window);
  close_windows_before(m, window);
  m->sum_req += request_latency_s;
  m->sum_exec += exec;
  ++m->count;
  return TS_OK;
}

int ts_monitor_advance(ts_monitor* m, double now_s, int* policy, int64_t* windows_closed, int64_t* n_switches,
                       double* last_ratio) {
  TS_REQUIRE(m != nullptr && std::isfinite(now_s) && now_s >= 0.0, TS_ERR_INVALID_ARG, "ts_monitor_advance: bad argument");
  const int64_t window = window_of(now_s, m->W);       // windows [nW, (n+1)W) with (n+1)W <= now are closed
  if (window > m->open_window) close_windows_before(m, window);
  if (policy) *policy = m->policy;
  if (windows_closed) *windows_closed = m->windows_closed;
  if (n_switches) *n_switches = m->switches;
  if (last_ratio) *last_ratio = m->last_ratio;
  return TS_OK;
}

}  // extern "C"

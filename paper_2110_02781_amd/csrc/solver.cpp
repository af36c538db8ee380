// Host-side partition solver and capacity estimate (paper, section "Dynamic
// Model Partition": capacity equation, per-layer estimate, DP base case and
// recurrence, transfer-time and last-stage-time equations).
//
// Capacity is a time multiplier (worker time / central-node time), so stage k
// holding layers [l, j) costs (P[j] - P[l]) * C[k] with P the running sum of the
// profiled layer costs.  best[n][j] is the optimum for the first j layers on
// devices 0..n-1; the last cut l runs over n-1 .. j-1 so that no stage is empty.
// Candidates are visited in ascending l and replace the incumbent only when
// strictly smaller.  All arithmetic is float64 with one rounding per operation
// (this file is compiled with floating-point contraction off).
#include <cmath>
#include <cstdio>
#include <vector>

#include "../../include/ftp.h"

void ftp_set_error(const char* fmt, ...);

extern "C" int ftp_solve_partition(const double* layer_costs, int L, const double* device_capacities, int N,
                                   const double* out_bytes, const double* bandwidth, int32_t* bounds,
                                   double* bottleneck) {
  if (!layer_costs || !device_capacities || !bounds) { ftp_set_error("solve_partition: NULL argument"); return FTP_ERR_ARG; }
  if (N < 1 || L < N) { ftp_set_error("solve_partition: need 1 <= N <= L (N=%d, L=%d)", N, L); return FTP_ERR_ARG; }
  for (int i = 0; i < L; ++i)
    if (!(std::isfinite(layer_costs[i]) && layer_costs[i] > 0.0)) {
      ftp_set_error("solve_partition: layer_costs[%d] must be finite and > 0", i);
      return FTP_ERR_VALUE;
    }
  for (int k = 0; k < N; ++k)
    if (!(std::isfinite(device_capacities[k]) && device_capacities[k] > 0.0)) {
      ftp_set_error("solve_partition: device_capacities[%d] must be finite and > 0", k);
      return FTP_ERR_VALUE;
    }
  const bool comm = out_bytes && bandwidth;
  if (comm) {
    for (int i = 0; i < L; ++i)
      if (!(std::isfinite(out_bytes[i]) && out_bytes[i] >= 0.0)) { ftp_set_error("solve_partition: bad out_bytes[%d]", i); return FTP_ERR_VALUE; }
    for (int k = 0; k + 1 < N; ++k)
      if (!(std::isfinite(bandwidth[k]) && bandwidth[k] > 0.0)) { ftp_set_error("solve_partition: bad bandwidth[%d]", k); return FTP_ERR_VALUE; }
  }
  std::vector<double> P(L + 1, 0.0);
  for (int i = 0; i < L; ++i) P[i + 1] = P[i] + layer_costs[i];
  const double INF = INFINITY;
  const int S = L + 1;
  std::vector<double> best((size_t)(N + 1) * S, INF);
  std::vector<int> arg((size_t)(N + 1) * S, 0);
  for (int j = 1; j <= L; ++j) best[(size_t)1 * S + j] = P[j] * device_capacities[0];
  for (int n = 2; n <= N; ++n) {
    const double cap = device_capacities[n - 1];
    for (int j = n; j <= L; ++j) {
      double b = INF;
      int a = -1;
      for (int l = n - 1; l < j; ++l) {
        double t = best[(size_t)(n - 1) * S + l];
        double last = (P[j] - P[l]) * cap;
        if (last > t) t = last;
        if (comm) {
          double c = 2.0 * (out_bytes[l - 1] / bandwidth[n - 2]);
          if (c > t) t = c;
        }
        if (t < b) { b = t; a = l; }
      }
      best[(size_t)n * S + j] = b;
      arg[(size_t)n * S + j] = a;
    }
  }
  std::vector<int32_t> out(N + 1);
  out[N] = L;
  int j = L;
  for (int n = N; n >= 2; --n) {
    j = arg[(size_t)n * S + j];
    out[n - 1] = j;
  }
  out[0] = 0;
  for (int k = 0; k <= N; ++k) bounds[k] = out[k];
  if (bottleneck) *bottleneck = best[(size_t)N * S + L];
  return FTP_OK;
}

extern "C" int ftp_estimate_capacity(double stage_time, const double* layer_costs, int L, int start, int end,
                                     double* capacity) {
  if (!layer_costs || !capacity || start < 0 || end < start || end >= L) {
    ftp_set_error("estimate_capacity: bad argument");
    return FTP_ERR_ARG;
  }
  if (!(std::isfinite(stage_time) && stage_time > 0.0)) { ftp_set_error("estimate_capacity: bad stage_time"); return FTP_ERR_VALUE; }
  double s = 0.0;
  for (int i = start; i <= end; ++i) s += layer_costs[i];
  if (!(s > 0.0)) { ftp_set_error("estimate_capacity: non-positive cost sum"); return FTP_ERR_VALUE; }
  *capacity = stage_time / s;
  return FTP_OK;
}

// Which stage of `bounds` (n stages, half-open) holds layer l; -1 if none.
static int stage_of(const int32_t* bounds, int n, int l) {
  for (int k = 0; k < n; ++k)
    if (bounds[k] <= l && l < bounds[k + 1]) return k;
  return -1;
}

static bool bounds_ok(const int32_t* b, int n) {
  if (!b || n < 1 || b[0] != 0) return false;
  for (int k = 0; k < n; ++k)
    if (b[k + 1] <= b[k]) return false;
  return true;
}

extern "C" int ftp_redistribution_plan(const int32_t* bounds_new, int n_new, const int32_t* bounds_cur, int n_cur, int i_fail,
                                       int i_cur, int i_new, int32_t* source) {
  if (!bounds_ok(bounds_new, n_new) || !bounds_ok(bounds_cur, n_cur) || !source) {
    ftp_set_error("redistribution_plan: bounds must start at 0 and increase strictly; source must not be NULL");
    return FTP_ERR_ARG;
  }
  if (bounds_new[n_new] != bounds_cur[n_cur]) {
    ftp_set_error("redistribution_plan: both partitions must cover the same %d layers", (int)bounds_cur[n_cur]);
    return FTP_ERR_ARG;
  }
  if (i_cur < 0 || i_cur >= n_cur || i_new < 0 || i_new >= n_new || i_fail < -1 || i_fail >= n_cur || i_fail == i_cur) {
    ftp_set_error("redistribution_plan: worker index out of range (i_cur=%d of %d, i_new=%d of %d, i_fail=%d)", i_cur, n_cur,
                  i_new, n_new, i_fail);
    return FTP_ERR_ARG;
  }
  const int lo = bounds_new[i_new], hi = bounds_new[i_new + 1];
  const int have_lo = bounds_cur[i_cur], have_hi = bounds_cur[i_cur + 1];
  for (int l = lo; l < hi; ++l) {
    if (have_lo <= l && l < have_hi) { source[l - lo] = -1; continue; }     // held already
    int t = stage_of(bounds_cur, n_cur, l);
    if (i_fail >= 0) {
      if (t > i_fail) t -= 1;                                  // the numbering behind the failed worker moved up
      else if (t == i_fail && i_fail == n_cur - 1) t = 0;      // backup of the last stage lives on the central node
      // t == i_fail otherwise: the chain successor holds the backup and now carries this index
    }
    source[l - lo] = t;
  }
  return FTP_OK;
}

// Worker list after failures (section "Fault Tolerance Mechanism"): the failed entries leave the list and the alive
// ones keep their order.  With one failure that lowers every index behind it by one; with several, each failed
// place is taken by the next alive worker behind it, one by one.  Worker 0 is the central node, which runs the
// fault handler and therefore is never among the failed.
extern "C" int ftp_renumber_workers(const int32_t* worker_ids, int n, const int32_t* failed, int n_failed, int32_t* new_ids,
                                    int32_t* new_index, int* n_new) {
  if (!worker_ids || !new_ids || !n_new || n < 1 || n_failed < 0 || (n_failed > 0 && !failed)) {
    ftp_set_error("renumber_workers: NULL argument or empty worker list");
    return FTP_ERR_ARG;
  }
  for (int f = 0; f < n_failed; ++f) {
    if (failed[f] < 1 || failed[f] >= n) {
      ftp_set_error("renumber_workers: failed index %d is not a worker index 1..%d (0 is the central node)", (int)failed[f], n - 1);
      return FTP_ERR_ARG;
    }
    for (int q = 0; q < f; ++q)
      if (failed[q] == failed[f]) { ftp_set_error("renumber_workers: index %d listed twice", (int)failed[f]); return FTP_ERR_ARG; }
  }
  int m = 0;
  for (int i = 0; i < n; ++i) {
    bool dead = false;
    for (int f = 0; f < n_failed; ++f) dead = dead || failed[f] == i;
    if (new_index) new_index[i] = dead ? -1 : m;
    if (!dead) new_ids[m++] = worker_ids[i];
  }
  *n_new = m;
  return FTP_OK;
}

// Re-partition schedule (section "Dynamic Model Partition"): first after 10 trained batches, then every 100.
extern "C" int ftp_repartition_due(int64_t batches_done, int* due) {
  if (!due || batches_done < 0) { ftp_set_error("repartition_due: batches_done >= 0 and a non-NULL result required"); return FTP_ERR_ARG; }
  *due = batches_done == 10 || (batches_done > 10 && (batches_done - 10) % 100 == 0);
  return FTP_OK;
}

// Capacities for the next re-partition from the workers' reported mean execution times (capacity equations): the
// central node keeps 1.0; with a report missing from any other worker all are taken equal.
extern "C" int ftp_repartition_capacities(const double* mean_times, const double* layer_costs, int L, const int32_t* bounds_cur,
                                          int n, double* capacities) {
  if (!mean_times || !layer_costs || !capacities || !bounds_ok(bounds_cur, n) || bounds_cur[n] != L) {
    ftp_set_error("repartition_capacities: NULL argument or bounds that do not cover the %d layers", L);
    return FTP_ERR_ARG;
  }
  bool all = true;
  for (int i = 1; i < n; ++i) all = all && std::isfinite(mean_times[i]) && mean_times[i] > 0.0;
  capacities[0] = 1.0;
  for (int i = 1; i < n; ++i) {
    capacities[i] = 1.0;
    if (!all) continue;
    int rc = ftp_estimate_capacity(mean_times[i], layer_costs, L, bounds_cur[i], bounds_cur[i + 1] - 1, &capacities[i]);
    if (rc) return rc;
  }
  return FTP_OK;
}

// NPFP** scheduling decisions of CF-DETR (Sec. IV): host code only, no GPU work.
//
//   cfdetr_sched_response_times  offline test of individually executed coarse subtasks
//                                (Lemma 1, Eq. 3-4)
//   cfdetr_sched_coarse_batch    coarse batch assignment (Algo. 2, P1, P2, Eq. 5)
//   cfdetr_sched_fine_batches    dynamic batch assignment (Algo. 3, Lemma 3, Eq. 6)
//   cfdetr_sched_decide          the decision at a scheduling instant (Algo. 1)
//
// The runtime decisions are O(n) and O(n^2) over at most kMaxTasks tasks with table
// look-ups for the WCETs, as the paper requires of anything that runs at a scheduling
// instant; nothing here allocates.
#include <cmath>
#include <cstdint>
#include <limits>

#include "../../include/cfdetr.h"

namespace {

constexpr int kMaxTasks = 64;
constexpr double kInf = std::numeric_limits<double>::infinity();

// Stable insertion sort of 0..n-1 by workload (n <= 64).
void sort_by_workload(int n, const int32_t* workload, int32_t* order) {
  for (int i = 0; i < n; ++i) {
    int pos = i;
    while (pos > 0 && workload[order[pos - 1]] > workload[i]) {
      order[pos] = order[pos - 1];
      --pos;
    }
    order[pos] = i;
  }
}

struct FineTable {
  const double* c;
  int n_levels, max_size;
  double at(int level, int size) const { return c[(size_t)level * (max_size + 1) + size]; }
};

// DBA[0..n] and, for every k, the start (1-based j) of the last batch of the best
// partition of the first k sorted subtasks.  A batch (j..k) starts at t + DBA[j-1]; it
// must end by every deadline in it and by the next coarse release, else it costs
// infinity.  Ties go to the first minimum met when j runs k, k-1, ..., 1.
void dba_table(int n, const int32_t* w, const double* dl, double t, double next_release,
               const FineTable& tab, double* dba, int32_t* arg) {
  dba[0] = 0.0;
  arg[0] = 0;
  for (int k = 1; k <= n; ++k) {
    dba[k] = kInf;
    arg[k] = 0;
    double min_dl = kInf;   // earliest deadline among subtasks j..k
    for (int j = k; j >= 1; --j) {
      min_dl = std::fmin(min_dl, dl[j - 1]);
      if (dba[j - 1] == kInf) continue;
      const double c = tab.at(w[k - 1], k - j + 1);
      const double end = t + dba[j - 1] + c;
      if (end > next_release || end > min_dl) continue;
      const double cost = dba[j - 1] + c;
      if (cost < dba[k]) {
        dba[k] = cost;
        arg[k] = j;
      }
    }
  }
}

int coarse_batch(int n_active, double t, double next_release, const double* c_by_size) {
  if (n_active >= 2)
    for (int x = n_active; x >= 2; --x)
      if (c_by_size[x] <= next_release - t) return x;
  return n_active >= 1 ? 1 : 0;
}

// Sorted order, and the batches of the longest schedulable prefix as end indices.
int fine_batches(int n, const int32_t* workload, const double* deadline, double t,
                 double next_release, const FineTable& tab, int32_t* order, int32_t* batch_end,
                 double* dba_out) {
  int32_t w[kMaxTasks];
  double dl[kMaxTasks], dba[kMaxTasks + 1];
  int32_t arg[kMaxTasks + 1];
  sort_by_workload(n, workload, order);
  for (int i = 0; i < n; ++i) {
    w[i] = workload[order[i]];
    dl[i] = deadline[order[i]];
  }
  dba_table(n, w, dl, t, next_release, tab, dba, arg);
  if (dba_out)
    for (int k = 0; k <= n; ++k) dba_out[k] = dba[k];
  int k = n;
  while (k > 0 && dba[k] == kInf) --k;
  int nb = 0;
  for (int e = k; e > 0; e = arg[e] - 1) ++nb;
  int slot = nb;
  for (int e = k; e > 0; e = arg[e] - 1) batch_end[--slot] = e;
  return nb;
}

}  // namespace

extern "C" {

CFDETR_API cfdetr_status cfdetr_sched_response_times(int32_t n, const double* period,
                                                     const double* c_coarse, double* response,
                                                     int32_t* schedulable) {
  if (n < 1 || n > kMaxTasks || !period || !c_coarse || !response || !schedulable)
    return CFDETR_EINVAL;
  for (int i = 0; i < n; ++i)
    if (!(period[i] > 0.0) || !(c_coarse[i] > 0.0)) return CFDETR_EINVAL;
  bool ok = true;
  for (int i = 0; i < n; ++i) {
    double blocking = 0.0;
    for (int j = i + 1; j < n; ++j) blocking = std::fmax(blocking, c_coarse[j]);
    double r = c_coarse[i] + blocking;
    for (int it = 0; it < 100000; ++it) {
      double hp = 0.0;
      for (int h = 0; h < i; ++h) hp += std::ceil(r / period[h]) * c_coarse[h];
      const double nxt = c_coarse[i] + blocking + hp;
      if (nxt == r) break;
      r = nxt;
      if (r > period[i]) {
        r = kInf;
        break;
      }
    }
    response[i] = r;
    ok = ok && r <= period[i];
  }
  *schedulable = ok ? 1 : 0;
  return CFDETR_OK;
}

CFDETR_API int32_t cfdetr_sched_coarse_batch(int32_t n_active, double t, double next_release,
                                             const double* c_batch_by_size) {
  if (n_active < 0 || n_active > kMaxTasks || !c_batch_by_size) return -1;
  return coarse_batch(n_active, t, next_release, c_batch_by_size);
}

CFDETR_API cfdetr_status cfdetr_sched_fine_batches(int32_t n, const int32_t* workload,
                                                   const double* deadline, double t,
                                                   double next_coarse_release,
                                                   const double* c_batch, int32_t n_levels,
                                                   int32_t max_size, int32_t* order,
                                                   int32_t* batch_end, int32_t* n_batches,
                                                   double* dba) {
  if (n < 0 || n > kMaxTasks || n_levels < 1 || max_size < n || !c_batch || !n_batches ||
      (n > 0 && (!workload || !deadline || !order || !batch_end)))
    return CFDETR_EINVAL;
  for (int i = 0; i < n; ++i)
    if (workload[i] < 0 || workload[i] >= n_levels) return CFDETR_EINVAL;
  const FineTable tab{c_batch, n_levels, max_size};
  *n_batches = fine_batches(n, workload, deadline, t, next_coarse_release, tab, order, batch_end, dba);
  return CFDETR_OK;
}

CFDETR_API cfdetr_status cfdetr_sched_decide(cfdetr_policy policy, double t, int32_t n_coarse,
                                             const int32_t* active_coarse, int32_t n_fine,
                                             const int32_t* active_fine,
                                             const int32_t* fine_workload,
                                             const double* fine_deadline, double next_release,
                                             const double* c_coarse_by_size, const double* c_fine,
                                             int32_t n_levels, int32_t max_size,
                                             cfdetr_sched_action* kind, int32_t* tasks,
                                             int32_t* batch_end, int32_t* n_batches) {
  if (policy < CFDETR_POLICY_C || policy > CFDETR_POLICY_BC_BF || n_coarse < 0 ||
      n_coarse > kMaxTasks || n_fine < 0 || n_fine > kMaxTasks || !kind || !tasks || !batch_end ||
      !n_batches || !c_coarse_by_size || (n_coarse > 0 && !active_coarse) ||
      (n_fine > 0 && (!active_fine || !fine_workload || !fine_deadline || !c_fine)))
    return CFDETR_EINVAL;
  if (n_fine > 0) {
    if (n_levels < 1 || max_size < n_fine) return CFDETR_EINVAL;
    for (int i = 0; i < n_fine; ++i)
      if (fine_workload[i] < 0 || fine_workload[i] >= n_levels) return CFDETR_EINVAL;
  }
  const bool batched_c = policy == CFDETR_POLICY_BC_F || policy == CFDETR_POLICY_BC_BF;
  const bool any_f = policy != CFDETR_POLICY_C;
  const bool batched_f = policy == CFDETR_POLICY_C_BF || policy == CFDETR_POLICY_BC_BF;
  *kind = CFDETR_SCHED_IDLE;
  *n_batches = 0;
  if (n_coarse > 0) {   // coarse subtasks always come first (Algo. 1, line 1)
    const int x = batched_c ? coarse_batch(n_coarse, t, next_release, c_coarse_by_size) : 1;
    for (int i = 0; i < x; ++i) tasks[i] = active_coarse[i];
    batch_end[0] = x;
    *n_batches = 1;
    *kind = CFDETR_SCHED_COARSE;
    return CFDETR_OK;
  }
  if (n_fine > 0 && any_f) {
    const FineTable tab{c_fine, n_levels, max_size};
    if (batched_f && n_fine >= 2) {
      int32_t order[kMaxTasks];
      const int nb = fine_batches(n_fine, fine_workload, fine_deadline, t, next_release, tab, order,
                                  batch_end, nullptr);
      if (nb > 0) {
        for (int i = 0; i < batch_end[nb - 1]; ++i) tasks[i] = active_fine[order[i]];
        *n_batches = nb;
        *kind = CFDETR_SCHED_FINE;
      }
      return CFDETR_OK;
    }
    // one fine subtask: the highest-priority one, if it ends before the next coarse release
    if (t + tab.at(fine_workload[0], 1) <= next_release) {
      tasks[0] = active_fine[0];
      batch_end[0] = 1;
      *n_batches = 1;
      *kind = CFDETR_SCHED_FINE;
    }
  }
  return CFDETR_OK;
}

}  // extern "C"

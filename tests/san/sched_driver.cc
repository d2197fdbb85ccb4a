// Replays scheduling cases from a text file through the library's host code (Sec. IV of
// the paper: Lemma 1, Algo. 1-3), built with AddressSanitizer and UndefinedBehaviorSanitizer
// by tests/test_host_sanitizers.py.  Output buffers are heap arrays of exactly the size the
// header promises, so that a write past one is caught.  One result line per case.
//
// Case lines (numbers separated by blanks):
//   R n  period[n]  c[n]
//   B n_active t next  m  c[m]
//   F n  workload[n]  deadline[n]  t next  n_levels max_size  table[n_levels*(max_size+1)]
//   D policy t  nc ac[nc]  nf af[nf] w[nf] dl[nf]  next  m cc[m]  n_levels max_size table[...]
#include <cstdio>
#include <cstdlib>
#include <fstream>
#include <iostream>
#include <sstream>
#include <string>
#include <vector>

#include "../../include/cfdetr.h"

namespace {
template <typename T>
std::vector<T> take(std::istringstream& in, int n) {
  std::vector<T> v(n);
  for (int i = 0; i < n; ++i) in >> v[i];
  return v;
}
void put(double x) { std::printf(" %.17g", x); }
}  // namespace

int main(int argc, char** argv) {
  if (argc != 2) return 2;
  std::ifstream f(argv[1]);
  std::string line;
  while (std::getline(f, line)) {
    std::istringstream in(line);
    char kind;
    if (!(in >> kind)) continue;
    if (kind == 'R') {
      int n;
      in >> n;
      auto period = take<double>(in, n), c = take<double>(in, n);
      double* R = new double[n];
      int32_t ok = -1;
      const int st = cfdetr_sched_response_times(n, period.data(), c.data(), R, &ok);
      std::printf("R %d %d", st, ok);
      for (int i = 0; i < n; ++i) put(R[i]);
      std::printf("\n");
      delete[] R;
    } else if (kind == 'B') {
      int n, m;
      double t, nxt;
      in >> n >> t >> nxt >> m;
      auto c = take<double>(in, m);
      std::printf("B %d\n", cfdetr_sched_coarse_batch(n, t, nxt, c.data()));
    } else if (kind == 'F') {
      int n, levels, max_size;
      in >> n;
      auto w = take<int32_t>(in, n);
      auto dl = take<double>(in, n);
      double t, nxt;
      in >> t >> nxt >> levels >> max_size;
      auto tab = take<double>(in, levels * (max_size + 1));
      int32_t* order = new int32_t[n > 0 ? n : 1];
      int32_t* ends = new int32_t[n > 0 ? n : 1];
      double* dba = new double[n + 1];
      int32_t nb = -1;
      const int st = cfdetr_sched_fine_batches(n, w.data(), dl.data(), t, nxt, tab.data(), levels,
                                               max_size, order, ends, &nb, dba);
      std::printf("F %d %d |", st, nb);
      if (st == 0) {
        for (int i = 0; i < n; ++i) std::printf(" %d", order[i]);
        std::printf(" |");
        for (int b = 0; b < nb; ++b) std::printf(" %d", ends[b]);
        std::printf(" |");
        for (int i = 0; i <= n; ++i) put(dba[i]);
      }
      std::printf("\n");
      delete[] order;
      delete[] ends;
      delete[] dba;
    } else if (kind == 'D') {
      int policy, nc, nf, m, levels, max_size;
      double t, nxt;
      in >> policy >> t >> nc;
      auto ac = take<int32_t>(in, nc);
      in >> nf;
      auto af = take<int32_t>(in, nf);
      auto w = take<int32_t>(in, nf);
      auto dl = take<double>(in, nf);
      in >> nxt >> m;
      auto cc = take<double>(in, m);
      in >> levels >> max_size;
      auto tab = take<double>(in, levels * (max_size + 1));
      const int cap = nc > nf ? nc : nf;
      int32_t* tasks = new int32_t[cap > 0 ? cap : 1];
      int32_t* ends = new int32_t[cap > 0 ? cap : 1];
      cfdetr_sched_action act = CFDETR_SCHED_IDLE;
      int32_t nb = -1;
      const int st = cfdetr_sched_decide((cfdetr_policy)policy, t, nc, ac.data(), nf, af.data(),
                                         w.data(), dl.data(), nxt, cc.data(), tab.data(), levels,
                                         max_size, &act, tasks, ends, &nb);
      std::printf("D %d %d %d |", st, (int)act, nb);
      if (st == 0) {
        int a = 0;
        for (int b = 0; b < nb; ++b) {
          for (; a < ends[b]; ++a) std::printf(" %d", tasks[a]);
          std::printf(" /");
        }
      }
      std::printf("\n");
      delete[] tasks;
      delete[] ends;
    } else {
      return 3;
    }
  }
  return 0;
}

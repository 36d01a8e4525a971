#include "planner.h"

#include <algorithm>
#include <numeric>

namespace vte {

namespace {
int min_width(const Pool& pool) {
  int w = pool.total_cus();
  for (int i = 0; i < pool.size(); ++i) w = std::min(w, pool.at(i).width);
  return w;
}
}  // namespace

double plan_progress(const Pool& pool, const PlanTime& time, int op, int width) {
  const int m0 = min_width(pool);
  const double t0 = time(op, m0), t = time(op, width);
  if (t0 > 0 && t > 0) return t0 / t;
  return static_cast<double>(width) / m0;  // no profile: perfect scaling
}

std::vector<int> tput_plan(const Pool& pool, const std::vector<PlanOp>& ops, const PlanTime& time) {
  const int n = static_cast<int>(ops.size());
  std::vector<int> A(n, -1);
  std::vector<int> order(n);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return ops[a].age < ops[b].age; });

  auto free_of_others = [&](int o, int p) {
    for (int q = 0; q < n; ++q)
      if (q != o && A[q] >= 0 && pool.overlaps(A[q], p)) return false;
    return true;
  };

  // progress on `p` counts half when its queue shares a dispatch pipe with another tenant
  auto shares_pipe = [&](int o, int p) {
    const int pipe = pool.at(p).pipe;
    if ((ops[o].busy_pipes >> pipe) & 1u) return true;
    for (int q = 0; q < n; ++q)
      if (q != o && A[q] >= 0 && pool.at(A[q]).pipe == pipe) return true;
    return false;
  };
  auto progress = [&](int o, int p) {
    return plan_progress(pool, time, o, pool.at(p).width) * (shares_pipe(o, p) ? 0.5 : 1.0);
  };

  // MinBind: oldest first, the narrowest eligible pCtx that overlaps nothing assigned so far
  // (equal widths: a free pipe, the predecessor's pCtx, then the lowest id, which packs leaves from one side)
  for (int o : order) {
    int best = -1;
    for (int p : ops[o].eligible) {
      if (!free_of_others(o, p)) continue;
      if (best < 0) { best = p; continue; }
      const int wb = pool.at(best).width, wp = pool.at(p).width;
      if (wp != wb) { if (wp < wb) best = p; continue; }
      const bool sb = shares_pipe(o, best), sp = shares_pipe(o, p);
      if (sp != sb) { if (!sp) best = p; continue; }
      if (p == ops[o].pred_pctx && best != ops[o].pred_pctx) best = p;
    }
    A[o] = best;
  }

  // greedy expansion by the largest positive marginal gain
  while (true) {
    double best_g = 0;
    int best_o = -1, best_p = -1;
    for (int o : order) {
      if (A[o] < 0) continue;
      const int m = pool.at(A[o]).width;
      const double P = progress(o, A[o]);
      auto consider = [&](int p) {
        const int m2 = pool.at(p).width;
        if (m2 <= m || !free_of_others(o, p)) return;
        const double g = (progress(o, p) - P) / (m2 - m);
        if (g > best_g * (1 + 1e-12) && g > 0) { best_g = g; best_o = o; best_p = p; }
      };
      for (int p : ops[o].eligible) consider(p);
      for (int p : ops[o].later) consider(p);
    }
    if (best_o < 0) break;
    A[best_o] = best_p;
  }
  return A;
}

}  // namespace vte

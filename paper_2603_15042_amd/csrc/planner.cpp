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

  // Buddy packing: how far up the tree from p one has to go to find a block that is already broken
  // up (the other child of that ancestor holds something leased, reserved or assigned in this plan).
  // Taking the candidate with the smallest such distance completes a broken block instead of
  // breaking a whole one, so that whole halves stay free for a tenant that scales.
  auto broken_distance = [&](int o, int p) {
    int d = 1, x = p;
    while (pool.at(x).kind == kNode && pool.at(x).parent >= 0) {
      const Pctx& par = pool.at(pool.at(x).parent);
      const int sib = par.child[0] == x ? par.child[1] : par.child[0];
      if (sib >= 0) {
        if (pool.is_active(sib) || pool.at(sib).active_below > 0) return d;
        for (int q = 0; q < n; ++q)
          if (q != o && A[q] >= 0 && pool.overlaps(A[q], sib)) return d;
      }
      x = pool.at(x).parent;
      ++d;
    }
    return 1 << 20;
  };

  // MinBind: oldest first.  An op whose predecessor is still in flight starts where that predecessor
  // runs (its vstream's lease is open there: a seat elsewhere would hold two allocations for one
  // stream and fragment the pool).  Otherwise the narrowest eligible pCtx that overlaps nothing
  // assigned so far; equal widths: a free pipe, the one nearest to a block that is already broken up, then the lowest id.
  for (int o : order) {
    const int pred = ops[o].pred_pctx;
    if (pred >= 0 && std::find(ops[o].eligible.begin(), ops[o].eligible.end(), pred) != ops[o].eligible.end() &&
        free_of_others(o, pred)) {
      A[o] = pred;
      continue;
    }
    int best = -1;
    for (int p : ops[o].eligible) {
      if (!free_of_others(o, p)) continue;
      if (best < 0) { best = p; continue; }
      const int wb = pool.at(best).width, wp = pool.at(p).width;
      if (wp != wb) { if (wp < wb) best = p; continue; }
      const bool sb = shares_pipe(o, best), sp = shares_pipe(o, p);
      if (sp != sb) { if (!sp) best = p; continue; }
      const int db = broken_distance(o, best), dp = broken_distance(o, p);
      if (dp != db) { if (dp < db) best = p; continue; }
    }
    A[o] = best;
  }

  // greedy expansion by the largest positive marginal gain; equal gains: the op on the narrower seat,
  // the pCtx that contains the current seat (growing in place), then the one nearest to a block that
  // is already broken up
  while (true) {
    double best_g = 0;
    int best_o = -1, best_p = -1, best_d = 0, best_m = 0;
    bool best_in_place = false;
    for (int o : order) {
      if (A[o] < 0) continue;
      const int m = pool.at(A[o]).width;
      const double P = progress(o, A[o]);
      auto consider = [&](int p) {
        const int m2 = pool.at(p).width;
        if (m2 <= m || !free_of_others(o, p)) return;
        const double g = (progress(o, p) - P) / (m2 - m);
        if (g <= 0) return;
        if (best_o >= 0 && g < best_g * (1 - 1e-12)) return;
        const bool in_place = pool.overlaps(p, A[o]);
        const int d = broken_distance(o, p);
        if (best_o >= 0 && g <= best_g * (1 + 1e-12)) {  // a tie: the narrower seat grows first (ties fill evenly)
          if (m != best_m) { if (m > best_m) return; }
          else if (in_place != best_in_place) { if (!in_place) return; }
          else if (d >= best_d) return;
        }
        best_g = g; best_o = o; best_p = p; best_in_place = in_place; best_d = d; best_m = m;
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

// Throughput-Oriented resource assignment (Sec. 5, Algorithm 1 of the paper) as a
// pure function of the ready set, the pool and the width profiles: MinBind gives
// the largest number of ready ops a minimum-size, non-overlapping pCtx in age
// order, then the feasible expansion with the largest marginal gain
//   G_o(p, p') = (P_o(m(p')) - P_o(m(p))) / (m(p') - m(p)),  P_o(m) = T^_o(m_min) / T^_o(m)
// is applied until none has positive gain.  An op whose pCtx shares a dispatch pipe
// with another tenant takes turns with it, so its progress there counts half.
// Host logic only (no HIP).
#pragma once
#include <cstdint>
#include <functional>
#include <vector>

#include "pool.h"

namespace vte {

struct PlanOp {
  uint64_t age = 0;            // smaller = older
  int pred_pctx = -1;          // preferred among equals (keeps a stream edge in stream order)
  std::vector<int> eligible;   // pCtxs the op can take now
  std::vector<int> later;      // pCtxs blocked only by leases of the op's own vstream
  uint32_t busy_pipes = 0;     // dispatch pipes that leases of other vstreams are using
};

// time(op index, width) = profiled seconds, or <= 0 when unknown (then the op is
// taken to scale perfectly: T ~ 1 / m).
typedef std::function<double(int, int)> PlanTime;

// Returns one pCtx id per op, -1 = not assigned.  An id out of `later` means: leave
// the op ready until its own lease has drained.
std::vector<int> tput_plan(const Pool& pool, const std::vector<PlanOp>& ops, const PlanTime& time);

// Normalised progress P_o(m) used by the plan (exposed for tests).
double plan_progress(const Pool& pool, const PlanTime& time, int op, int width);

}  // namespace vte

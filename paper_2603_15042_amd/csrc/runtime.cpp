// The late-binding runtime: pool realisation, virtual streams with token
// chains, the policy-driven dispatcher with validation, lease state machine and
// completion propagation (Sec. 4.2 - 4.5 of the paper), behind the C ABI.
#include "runtime.h"
#include "planner.h"

#include <algorithm>
#include <cstring>
#include <new>

#include "backend_fake.h"

namespace vte {

static thread_local std::string g_err;
static thread_local int g_hip_err = 0;
void set_error(const std::string& msg, int hip_code) {
  g_err = msg;
  g_hip_err = hip_code;
}

namespace {

using Lock = std::unique_lock<std::mutex>;

constexpr int kMaxSubmitRetries = 8;    // backend submissions of one op that may fail before the op is failed
constexpr int kMaxRecordRetries = 8;    // the same for completion records on one pCtx
constexpr size_t kMaxFailedKept = 1u << 16;

// Runtime lock held, on the thread where the backend call just failed: the message and HIP code
// that set_error left there are copied into the context, under the token they belong to.
void note_failure(vte_ctx* c, vte_token tok, int rc, const char* fallback = nullptr) {
  vte_ctx::Failure f{rc, rc == VTE_EHIP ? g_hip_err : 0, fallback ? std::string(fallback) : g_err};
  c->failed[tok] = f;
  if (c->failed.size() > kMaxFailedKept) c->failed.erase(c->failed.begin());  // oldest token first
  if (!c->failure_unreported) { c->failure_unreported = true; c->first_unreported = tok; }
  ++c->stats.failed;
}

// Hands the failure recorded for `tok` to the calling thread; VTE_OK if there is none.
int report_failure(vte_ctx* c, vte_token tok) {
  auto it = c->failed.find(tok);
  if (it == c->failed.end()) return VTE_OK;
  set_error(it->second.msg, it->second.hip);
  return it->second.rc;
}

void bump(vte_ctx* c) {  // runtime lock held: something changed from outside
  ++c->change_seq;
  c->cv_work.notify_all();
}

void notify_done(vte_ctx* c) {  // runtime lock held: launches retired, were bound, or the dispatcher went quiet
  c->done_epoch.fetch_add(1, std::memory_order_release);
  c->cv_done.notify_all();
}

inline void cpu_relax() {
#if defined(__x86_64__)
  __builtin_ia32_pause();
#else
  std::this_thread::yield();
#endif
}

// A condition-variable wake lies on the path of every burst twice (the idle dispatcher at its start,
// the caller at its end) and costs from a microsecond or two to tens of them, depending on the host
// and its load (measured here: 1.5 us of the 17 us that a single small launch takes from submission to
// the caller's return).  Both sides therefore poll for a bounded time where the event they wait for
// is close, and sleep otherwise.
constexpr double kWaiterPollSeconds = 20e-3;     // per wait call, while what it waits for is on the device
constexpr double kDispatcherPollSeconds = 2e-3;  // after the dispatcher ran out of work, before it sleeps

// Runtime lock held.  Returns when done() holds.  While on_device() says that everything awaited has
// been handed to the device the caller polls the notification epoch without the lock (up to
// kWaiterPollSeconds in total); before that, and past the budget, it sleeps on cv_done.
template <class Done, class OnDevice>
void wait_done(vte_ctx* c, Lock& lk, Done done, OnDevice on_device) {
  double polled = 0;
  while (!done()) {
    if (c->backend->is_fake() || polled >= kWaiterPollSeconds || !on_device()) {
      c->cv_done.wait(lk);  // every state change that done() or on_device() look at is notified with the lock held
      continue;
    }
    const uint64_t e = c->done_epoch.load(std::memory_order_acquire);
    lk.unlock();
    const auto t0 = std::chrono::steady_clock::now();
    double dt = 0;
    while (c->done_epoch.load(std::memory_order_acquire) == e && dt < 500e-6) {
      for (int i = 0; i < 32; ++i) cpu_relax();
      dt = std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
    }
    polled += dt;
    lk.lock();
  }
}

bool token_done(vte_ctx* c, vte_token t) {
  if (t == 0) return true;
  return c->live.find(t) == c->live.end();
}

void fill_info(const Pool& pool, int id, vte_pctx_info* o) {
  const Pctx& p = pool.at(id);
  std::memset(o, 0, sizeof *o);
  o->id = p.id; o->kind = p.kind; o->width = p.width; o->level = p.level; o->parent = p.parent;
  o->child[0] = p.child[0]; o->child[1] = p.child[1]; o->remainder = p.remainder;
  o->state = p.state; o->gate_open = p.gate_open ? 1 : 0; o->outstanding = p.outstanding;
  o->reserved_for = p.reserved_for;
  for (size_t w = 0; w < p.mask.size() && w < 8; ++w) o->mask[w] = p.mask[w];
  o->pipe = p.pipe;
}

// ---- lease state machine (Sec. 4.3 "pCtx Lifecycle") ---------------------------

// Can `vs` (or an explicit launch, vs = -1) put one more op on pCtx `id` now?
// `quiet`: the eligibility scan of a dispatch round asks about every pCtx; it wants the answer, not a message.
int can_admit(vte_ctx* c, int id, int vs, bool quiet = false) {
  const Pctx& p = c->pool.at(id);
  const char* why = nullptr;
  if (p.state == kDraining || !p.gate_open) why = "pCtx gate is closed (draining)";
  else if (p.reserved_for >= 0 && p.reserved_for != vs) why = "pCtx is reserved for another vstream";
  else if (p.state == kLeased) {  // lease reuse by its holder: conflicts were excluded when it was opened
    if (p.holder != vs) why = "pCtx is leased to another vstream";
  } else if (c->pool.conflicts_with_active(id, vs)) why = "pCtx overlaps an active lease or reservation";
  if (!why) return VTE_OK;
  if (!quiet) set_error(why);
  return VTE_EBUSY;
}

void admit(vte_ctx* c, int id, int vs) {
  Pctx& p = c->pool.at(id);
  if (p.state == kIdle || p.state == kReserved) {
    p.state = kLeased;
    p.holder = vs;
    p.gate_open = true;
    p.reservation_pending = false;
    c->pool.set_active(id, true);
    ++c->stats.leases_opened;
  } else {
    ++c->stats.leases_reused;
  }
  ++p.outstanding;
}

// A pending reservation takes effect once nothing else overlapping is active.
void settle_reservations(vte_ctx* c) {
  for (int id = 0; id < c->pool.size(); ++id) {
    Pctx& p = c->pool.at(id);
    if (!p.reservation_pending || p.state != kIdle) continue;
    if (!c->pool.conflicts_with_active(id, p.reserved_for)) {
      p.reservation_pending = false;
      p.state = kReserved;
    }
  }
}

void retire_one(vte_ctx* c, int id) {
  Pctx& p = c->pool.at(id);
  --p.outstanding;
  if (p.outstanding > 0) return;
  // lease released: back to idle, or to reserved when held for a vstream
  p.gate_open = true;
  if (p.reserved_for >= 0) {
    if (c->pool.conflicts_with_active(id, p.reserved_for)) {
      p.state = kIdle;
      p.reservation_pending = true;  // stays active so nothing unrelated moves in
    } else {
      p.state = kReserved;
      p.reservation_pending = false;
    }
  } else {
    p.state = kIdle;
    c->pool.set_active(id, false);
  }
  settle_reservations(c);
}

// ---- lease control with the runtime lock held (Sec. 4.3) -------------------------

void close_gate_locked(vte_ctx* c, int id) {
  Pctx& p = c->pool.at(id);
  if (p.state == kLeased) {
    p.state = kDraining;  // outstanding work continues, no new admissions
    p.gate_open = false;
    ++c->stats.gates_closed;
  }
}

int reserve_locked(vte_ctx* c, int id, int vs) {
  Pctx& p = c->pool.at(id);
  if (p.reserved_for >= 0 && p.reserved_for != vs) { set_error("pCtx is reserved for another vstream"); return VTE_EBUSY; }
  std::vector<int> ov;
  c->pool.active_overlapping(id, &ov);
  for (int o : ov) {
    const Pctx& q = c->pool.at(o);
    if (q.reserved_for >= 0 && q.reserved_for != vs) { set_error("overlaps a reservation of another vstream"); return VTE_EBUSY; }
  }
  p.reserved_for = vs;
  ++c->stats.reservations;
  if (p.state == kIdle) {
    c->pool.set_active(id, true);  // from now on unrelated leases are excluded
    if (ov.empty()) { p.state = kReserved; p.reservation_pending = false; }
    else p.reservation_pending = true;  // waits for overlapping work to drain
  }
  // leased / draining: becomes RESERVED when its outstanding count reaches zero
  return VTE_OK;
}

void unreserve_locked(vte_ctx* c, int id) {
  Pctx& p = c->pool.at(id);
  p.reserved_for = -1;
  p.reservation_pending = false;
  if (p.state == kReserved) p.state = kIdle;
  if (p.state == kIdle) c->pool.set_active(id, false);
  settle_reservations(c);
}

double tpot_token_time(vte_ctx* c, const vte_vstream* vs, int width);

// ---- completion propagation (Sec. 4.4) -------------------------------------------

void record_op(vte_ctx* c, const Op* op) {
  if (c->ring.empty()) return;
  vte_op_record& r = c->ring[(c->ring_head + c->ring_count) % c->ring.size()];
  if (c->ring_count == c->ring.size()) c->ring_head = (c->ring_head + 1) % c->ring.size();
  else ++c->ring_count;
  r.token = op->tok; r.vstream = op->vs; r.klass = op->klass; r.kernel = op->desc->kernel;
  r.pctx = op->pctx; r.width = c->pool.at(op->pctx).width;
  r.t_submit = op->t_submit; r.t_ready = op->t_ready; r.t_bound = op->t_bound; r.t_done = op->t_done;
  r.gpu_seconds = op->gpu_seconds; r.gpu_begin = op->gpu_begin; r.gpu_end = op->gpu_end;
}

void complete_op(vte_ctx* c, Op* op, int rc = VTE_OK) {
  op->state = kDone;
  op->t_done = c->now();
  if (rc != VTE_OK) note_failure(c, op->tok, rc);
  if (op->completion) {
    op->gpu_seconds = c->backend->elapsed(op->completion);
    if (op->gpu_seconds >= 0) {
      op->gpu_begin = c->backend->device_time(op->completion, false);
      op->gpu_end = c->backend->device_time(op->completion, true);
    }
    c->backend->release(op->completion);
    op->completion = nullptr;
  }
  if (c->lazy_tail[op->pctx] == op) c->lazy_tail[op->pctx] = nullptr;
  retire_one(c, op->pctx);
  if (op->vs >= 0) {
    vte_vstream* vs = c->vstreams[op->vs];
    --vs->unfinished_bound;
    if (vs->tpot > 0) {
      ++vs->ops_done;
      if (vs->ops_done % static_cast<uint64_t>(vs->ops_per_token) == 0) {  // a token is out
        ++vs->tokens_done;
        if (vs->t_ref >= 0 && op->t_done > vs->t_ref + vs->tpot) ++vs->deadline_misses;
        if (vs->t_ref >= 0 && vs->standing >= 0) {
          // how much slower than its solo profile the token ran (co-tenants share HBM and caches)
          const double solo = tpot_token_time(c, vs, c->pool.at(vs->standing).width);
          if (solo > 0) {
            const double f = std::min(8.0, std::max(1.0, (op->t_done - vs->t_ref) / solo));
            vs->slowdown += 0.25 * (f - vs->slowdown);
          }
        }
        vs->t_ref = op->t_done;
      }
      if (vs->queue.empty() && vs->unfinished_bound == 0) vs->t_idle = op->t_done;
    }
  }
  --c->inflight_by_class[op->klass];
  ++c->stats.completed;
  record_op(c, op);
  c->live.erase(op->tok);  // the token is now satisfied
  delete op;
}

// Poll completions.  Within a pCtx launches finish in submission order, so the
// newest completion record that is done retires every older launch of that pCtx,
// recorded or not, and nothing behind a record that is not done is looked at.
bool poll_completions(vte_ctx* c) {
  if (c->inflight.empty()) return false;
  const int np = c->pool.size();
  std::vector<int>&frontier = c->scratch.frontier, &first_bad = c->scratch.first_bad;
  std::vector<char>& blocked = c->scratch.blocked;
  frontier.assign(np, -1);
  first_bad.assign(np, -1);
  blocked.assign(np, 0);
  std::string bad_msg;
  int bad_hip = 0;
  for (size_t i = 0; i < c->inflight.size(); ++i) {
    Op* op = c->inflight[i];
    if (blocked[op->pctx] || !op->completion) continue;
    const int st = c->backend->status(op->completion);
    if (st == 0) { blocked[op->pctx] = 1; continue; }
    frontier[op->pctx] = static_cast<int>(i);
    if (st < 0 && first_bad[op->pctx] < 0) {
      // The device reported an error behind this record.  The record covers this launch and the
      // unrecorded ones of its pCtx in front of it (back to the record before): all of them are
      // retired as failed, since which one faulted is not known.
      int lo = static_cast<int>(i);
      for (int k = static_cast<int>(i) - 1; k >= 0; --k) {
        if (c->inflight[k]->pctx != op->pctx) continue;
        if (c->inflight[k]->completion) break;
        lo = k;
      }
      first_bad[op->pctx] = lo;
      if (bad_msg.empty()) { bad_msg = g_err; bad_hip = g_hip_err; }
    }
  }
  bool any = false;
  bool none_done = true;
  for (int p = 0; p < np; ++p) none_done = none_done && frontier[p] < 0;
  if (none_done) return false;  // the common answer while a launch is running
  std::vector<Op*>&keep = c->scratch.keep, &done = c->scratch.done;
  keep.clear();
  done.clear();
  for (size_t i = 0; i < c->inflight.size(); ++i) {
    Op* op = c->inflight[i];
    if (static_cast<int>(i) <= frontier[op->pctx]) done.push_back(op);
    else keep.push_back(op);
  }
  if (!done.empty()) {
    std::vector<int>& rcs = c->scratch.rcs;
    rcs.clear();
    for (size_t i = 0; i < c->inflight.size(); ++i) {
      const Op* op = c->inflight[i];
      if (static_cast<int>(i) > frontier[op->pctx]) continue;
      rcs.push_back(first_bad[op->pctx] >= 0 && static_cast<int>(i) >= first_bad[op->pctx] ? VTE_EHIP : VTE_OK);
    }
    c->inflight.swap(keep);
    for (size_t i = 0; i < done.size(); ++i) {
      if (rcs[i] != VTE_OK) set_error(bad_msg, bad_hip);  // what note_failure copies
      complete_op(c, done[i], rcs[i]);
    }
    any = true;
    notify_done(c);
  }
  return any;
}

// Retires every in-flight launch of pCtx `p` as failed (its stream no longer takes a completion
// record, so nothing would ever be observed).  The calling thread's error is what gets recorded.
void fail_inflight_on(vte_ctx* c, int p, int rc) {
  std::vector<Op*> keep, bad;
  for (Op* op : c->inflight) (op->pctx == p ? bad : keep).push_back(op);
  if (bad.empty()) return;
  const std::string msg = g_err;
  const int hip = g_hip_err;
  c->inflight.swap(keep);
  for (Op* op : bad) { set_error(msg, hip); complete_op(c, op, rc); }
  notify_done(c);
}

// Give the newest unrecorded launch of a pCtx a completion record when it is
// needed to observe progress: nothing recorded is pending on that pCtx, a quarter
// of the lookahead window (at least eight launches) has piled up behind the last
// record, or a caller waits for a launch that no pending record covers.  A record
// idles its stream for a few microseconds, so none is made without such a reason.
void flush_records(vte_ctx* c) {
  const int np = c->pool.size();
  std::vector<int> recorded(np, 0), lazy(np, 0);
  std::vector<char> covered(np, 0), urgent(np, 0);
  for (size_t i = c->inflight.size(); i-- > 0;) {  // newest first: a record covers everything older on its pCtx
    const Op* op = c->inflight[i];
    if (op->completion) { ++recorded[op->pctx]; covered[op->pctx] = 1; continue; }
    if (covered[op->pctx]) continue;
    ++lazy[op->pctx];  // launches behind the newest record only
    if (urgent[op->pctx]) continue;
    if (c->waiters_all > 0 || std::find(c->awaited.begin(), c->awaited.end(), op->tok) != c->awaited.end())
      urgent[op->pctx] = 1;
  }
  const int pile = std::max(8, c->cfg.lookahead / 4);
  for (int p = 0; p < np; ++p) {
    Op* op = c->lazy_tail[p];
    if (!op) continue;
    if (recorded[p] > 0 && lazy[p] < pile && !urgent[p]) continue;
    void* comp = nullptr;
    const int rc = c->backend->record(c->pool.at(p).stream, &comp);
    if (rc == VTE_OK) {
      op->completion = comp;
      c->lazy_tail[p] = nullptr;
      ++c->stats.completion_records;
      c->record_failures[p] = 0;
    } else if (rc == VTE_EHIP && ++c->record_failures[p] >= kMaxRecordRetries) {
      c->record_failures[p] = 0;
      fail_inflight_on(c, p, rc);  // the stream is dead: its launches are reported as failed instead of never
    }
  }
}

// ---- readiness (Sec. 4.4 "Readiness Before Binding") -----------------------------

// STRICT: every predecessor token satisfied.  PIPELINED: every predecessor is
// satisfied or already bound to a backend stream, and the vstream has fewer than
// `lookahead` bound-but-unfinished ops.
bool bindable(vte_ctx* c, const vte_vstream* vs, const Op* op, int* pred_pctx) {
  *pred_pctx = -1;
  const bool pipelined = c->cfg.mode == VTE_MODE_PIPELINED;
  if (pipelined && vs && vs->unfinished_bound >= c->cfg.lookahead) return false;
  for (vte_token t : op->deps) {
    if (t == 0) continue;
    auto it = c->live.find(t);
    if (it == c->live.end()) continue;  // satisfied
    if (!pipelined) return false;
    if (it->second->state != kInflight) return false;
    *pred_pctx = it->second->pctx;
  }
  return true;
}

// ---- built-in policies (Sec. 5) -----------------------------------------------------

double profile_time(vte_ctx* c, uint64_t key, int width) {
  auto it = c->profiles.find({key, width});
  return it == c->profiles.end() ? -1.0 : it->second;
}

int builtin_pick(vte_ctx*, const vte_ready_op* ready, int n, const vte_pool_view*) {
  int best = -1;
  for (int i = 0; i < n; ++i) {
    if (best < 0) { best = i; continue; }
    // latency class first, then oldest
    if (ready[i].klass < ready[best].klass || (ready[i].klass == ready[best].klass && ready[i].age < ready[best].age)) best = i;
  }
  return best;
}

int widest(const vte_ready_op* op, const int* el, int n, const vte_pool_view* S, int max_width) {
  int best = -1;
  for (int i = 0; i < n; ++i) {
    const vte_pctx_info& p = S->pctx[el[i]];
    if (p.width > max_width) continue;
    if (best < 0) { best = el[i]; continue; }
    const vte_pctx_info& b = S->pctx[best];
    if (p.width > b.width || (p.width == b.width && el[i] == op->pred_pctx)) best = el[i];
  }
  return best;
}

// True when pCtx `id` could take an op of `op`'s vstream were it not for leases
// that this same vstream holds on overlapping pCtxs: those drain on their own.
bool blocked_by_own_leases_only(vte_ctx* c, int id, const vte_ready_op* op) {
  const Pctx& p = c->pool.at(id);
  if (op->pinned_pctx >= 0 && id != op->pinned_pctx) return false;
  if (p.reserved_for >= 0 && p.reserved_for != op->vstream) return false;
  if (p.state == kDraining || p.state == kLeased || !p.gate_open) return false;
  std::vector<int> ov;
  c->pool.active_overlapping(id, &ov);
  bool own_lease = false;
  for (int o : ov) {
    const Pctx& q = c->pool.at(o);
    const bool only_reservation = q.state == kReserved || (q.state == kIdle && q.reservation_pending);
    if (only_reservation && q.reserved_for == op->vstream) continue;  // its own reservation does not block it
    if (!(q.state == kLeased && q.holder == op->vstream)) return false;
    own_lease = true;
  }
  return own_lease;
}

// Profiled time at `width` of the recurring chain the op belongs to: the sum over
// the descriptors its vstream submitted lately (Sec. 5 "Performance Profiles").
// A width that lacks a profile for any of them gives -1.
double chain_time(vte_ctx* c, const vte_ready_op* op, int width) {
  double sum = 0;
  bool own = false;
  if (op->vstream >= 0 && op->vstream < static_cast<int>(c->vstreams.size()) && c->vstreams[op->vstream]) {
    for (uint64_t key : c->vstreams[op->vstream]->recent_keys) {
      const double t = profile_time(c, key, width);
      if (key == op->desc.profile_key) { own = true; if (t <= 0) return -1.0; }
      if (t > 0) sum += t;
    }
  }
  if (!own) {
    const double t = profile_time(c, op->desc.profile_key, width);
    if (t <= 0) return -1.0;
    sum += t;
  }
  return sum;
}

int builtin_select(vte_ctx* c, const vte_ready_op* op, const int* el, int n, const vte_pool_view* S) {
  if (n == 0) return -1;
  const int total = c->pool.total_cus();
  if (c->builtin == VTE_POLICY_WIDEST) return widest(op, el, n, S, total);
  // QUEUE_STATE
  if (op->klass == VTE_CLASS_LATENCY) {
    // best chain time over what is eligible now or will be once this vstream's own leases drain
    double best_t = -1;
    for (int i = 0; i < n; ++i) {
      const double t = chain_time(c, op, S->pctx[el[i]].width);
      if (t > 0 && (best_t < 0 || t < best_t)) best_t = t;
    }
    if (best_t < 0) return widest(op, el, n, S, total);  // no profile: take what scales best
    double best_later = -1;
    for (int id = 0; id < c->pool.size(); ++id) {
      if (!blocked_by_own_leases_only(c, id, op)) continue;
      const double t = chain_time(c, op, c->pool.at(id).width);
      if (t > 0 && (best_later < 0 || t < best_later)) best_later = t;
    }
    if (best_later > 0 && best_later < best_t) best_t = best_later;
    // alone on the device the chain takes the fastest width; sharing it, the narrowest within `slack`
    const bool sharing = S->ready_by_class[VTE_CLASS_BEST_EFFORT] + S->inflight_by_class[VTE_CLASS_BEST_EFFORT] > 0;
    const double limit = best_t * (1.0 + (sharing ? c->slack : 0.02));
    int pick = -1;
    for (int i = 0; i < n; ++i) {
      const vte_pctx_info& p = S->pctx[el[i]];
      const double t = chain_time(c, op, p.width);
      if (t <= 0 || t > limit) continue;
      if (el[i] == op->pred_pctx) return el[i];  // good enough and keeps the edge in stream order
      if (pick < 0 || (sharing ? p.width < S->pctx[pick].width : t < chain_time(c, op, S->pctx[pick].width))) pick = el[i];
    }
    if (pick >= 0) return pick;
    if (best_later > 0 && best_later <= limit) return -1;  // a good pCtx frees up as soon as this vstream's in-flight ops retire
    return widest(op, el, n, S, total);
  }
  const bool latency_active = S->ready_by_class[VTE_CLASS_LATENCY] + S->inflight_by_class[VTE_CLASS_LATENCY] > 0;
  const int cap = latency_active ? total - c->keep_free : total;
  const int now = widest(op, el, n, S, cap);
  // A wider allocation may be blocked only by this vstream's own (narrower) lease:
  // then leave the op ready until that lease has drained rather than renewing it.
  for (int id = 0; id < c->pool.size(); ++id) {
    const Pctx& p = c->pool.at(id);
    if (p.width > cap || (now >= 0 && p.width <= S->pctx[now].width)) continue;
    if (blocked_by_own_leases_only(c, id, op)) return -1;
  }
  return now;
}

// ---- binding and submission (Sec. 4.4) ----------------------------------------------

bool compatible(const vte_desc* d, const Pctx& p) {
  // every pCtx is a CU subset of the same device: a descriptor runs unchanged on
  // any of them as long as one workgroup fits one CU
  const uint64_t threads = static_cast<uint64_t>(d->block[0]) * d->block[1] * d->block[2];
  return p.width >= 1 && threads >= 1 && threads <= 1024 && d->lds_bytes <= 160u * 1024u;
}

// Validate the proposal, open or reuse the lease, submit the descriptor
// unchanged, record it as outstanding.  Commit only after a successful submit.
int bind_and_submit(vte_ctx* c, Op* op, int pctx, bool record_now) {
  if (pctx < 0 || pctx >= c->pool.size()) { set_error("no such pCtx"); return VTE_EINVAL; }
  Pctx& p = c->pool.at(pctx);
  if (!compatible(op->desc, p)) { set_error("pCtx cannot run the descriptor unchanged"); return VTE_EINCOMPAT; }
  int rc = can_admit(c, pctx, op->vs);
  if (rc != VTE_OK) { ++c->stats.lease_conflicts; return rc; }
  // device-side edges for predecessors still running on other pCtxs (PIPELINED)
  for (vte_token t : op->deps) {
    auto it = c->live.find(t);
    if (it == c->live.end() || it->second->state != kInflight) continue;
    Op* pred = it->second;
    if (pred->pctx == pctx) continue;  // same backend stream: stream order
    if (!pred->completion) {  // not recorded yet: record the predecessor stream's current end
      Op* tail = c->lazy_tail[pred->pctx] ? c->lazy_tail[pred->pctx] : pred;
      void* comp = nullptr;
      rc = c->backend->record(c->pool.at(pred->pctx).stream, &comp);
      if (rc != VTE_OK) return rc;
      tail->completion = comp;
      ++c->stats.completion_records;
      c->lazy_tail[pred->pctx] = nullptr;
      pred = tail;
    }
    rc = c->backend->wait_on(p.stream, pred->completion, pred->pctx);
    if (rc != VTE_OK) return rc;
  }
  void* completion = nullptr;
  bool timed = (c->cfg.device_timing_mask >> op->desc->kernel) & 1u;
  if (timed && c->cfg.device_timing_stride > 1)
    timed = c->timing_seen[op->desc->kernel & 31]++ % static_cast<unsigned>(c->cfg.device_timing_stride) == 0;
  rc = c->backend->submit(op->desc, p.stream, pctx, op->tok, timed, record_now, &completion);
  if (rc != VTE_OK) { ++c->stats.submit_failures; return rc; }  // op stays ready
  admit(c, pctx, op->vs);
  if (completion) ++c->stats.completion_records;
  op->pctx = pctx;
  op->completion = completion;
  c->lazy_tail[pctx] = completion ? nullptr : op;  // a record also covers older launches of the pCtx
  op->state = kInflight;
  op->t_bound = c->now();
  c->inflight.push_back(op);
  ++c->inflight_by_class[op->klass];
  if (op->vs >= 0) ++c->vstreams[op->vs]->unfinished_bound;
  return VTE_OK;
}

// E: non-conflicting pCtxs that can run the op unchanged
void eligible_set(vte_ctx* c, const Op* op, int pinned, std::vector<int>* out) {
  out->clear();
  for (int id = 0; id < c->pool.size(); ++id) {
    if (pinned >= 0 && id != pinned) continue;
    if (!compatible(op->desc, c->pool.at(id))) continue;
    if (can_admit(c, id, op->vs, true) != VTE_OK) continue;
    out->push_back(id);
  }
}

bool planned_round(vte_ctx* c, const std::vector<vte_ready_op>& ready, const std::vector<Op*>& ready_ops);

// Takes the head of a vstream's queue out as failed: its token is retired with the error, whoever
// waits for it is woken.  The calling thread's error is what gets recorded unless `why` is given.
void fail_head(vte_ctx* c, vte_vstream* vs, int rc, const char* why = nullptr) {
  Op* op = vs->queue.front();
  vs->queue.pop_front();
  note_failure(c, op->tok, rc, why);
  c->live.erase(op->tok);
  delete op;
  if (vs->tpot > 0 && vs->queue.empty() && vs->unfinished_bound == 0) vs->t_idle = c->now();
  notify_done(c);
}

// An op whose predecessor failed fails with it (Sec. 4.2: it may run only after its predecessors
// completed, and they never will).  Returns true if anything was taken out.
bool purge_failed_dependants(vte_ctx* c) {
  if (c->failed.empty()) return false;
  bool any = false;
  for (vte_vstream* vs : c->vstreams) {
    if (!vs) continue;
    while (!vs->queue.empty()) {
      const Op* op = vs->queue.front();
      const vte_ctx::Failure* cause = nullptr;
      for (vte_token t : op->deps) {
        auto it = c->failed.find(t);
        if (it != c->failed.end()) { cause = &it->second; break; }
      }
      if (!cause) break;
      const std::string why = "a predecessor failed: " + cause->msg;
      set_error(why, cause->hip);
      fail_head(c, vs, cause->rc);
      any = true;
    }
  }
  return any;
}

// A backend submission of the head of `vs` failed: it stays ready (Sec. 4.4) until it has failed
// kMaxSubmitRetries times, then it is failed for good so that its waiters return.
void submission_failed(vte_ctx* c, Op* op, int rc) {
  if (rc != VTE_EHIP || op->vs < 0) return;
  if (++op->submit_failures < kMaxSubmitRetries) return;
  vte_vstream* vs = c->vstreams[op->vs];
  if (!vs->queue.empty() && vs->queue.front() == op) fail_head(c, vs, rc);
}

// One dispatch round: gather the ready heads, let the policy pick and select,
// validate, submit.  Returns true if something was bound.
bool dispatch_round(vte_ctx* c) {
  if (purge_failed_dependants(c)) return true;
  std::vector<vte_ready_op>& ready = c->scratch.ready;
  std::vector<Op*>& ready_ops = c->scratch.ready_ops;
  ready.clear();
  ready_ops.clear();
  for (vte_vstream* vs : c->vstreams) {
    if (!vs || vs->queue.empty()) continue;
    Op* op = vs->queue.front();
    int pred = -1;
    if (!bindable(c, vs, op, &pred)) continue;
    if (!op->ready_marked) { op->ready_marked = true; op->t_ready = c->now(); }
    vte_ready_op r;
    std::memset(&r, 0, sizeof r);
    r.token = op->tok; r.vstream = vs->id; r.klass = vs->klass; r.pinned_pctx = vs->pinned;
    r.age = op->age; r.pred_pctx = pred;
    vte_desc_info(op->desc, &r.desc);
    ready.push_back(r);
    ready_ops.push_back(op);
  }
  if (ready.empty()) return false;
  if (!c->custom_policy && c->builtin >= VTE_POLICY_TPUT_PLAN) return planned_round(c, ready, ready_ops);

  std::vector<vte_pctx_info>& infos = c->scratch.infos;
  infos.resize(c->pool.size());
  for (int i = 0; i < c->pool.size(); ++i) fill_info(c->pool, i, &infos[i]);
  vte_pool_view S;
  S.count = c->pool.size();
  S.pctx = infos.data();
  S.ready_by_class[0] = S.ready_by_class[1] = 0;
  for (auto& r : ready) ++S.ready_by_class[r.klass];
  S.inflight_by_class[0] = c->inflight_by_class[0];
  S.inflight_by_class[1] = c->inflight_by_class[1];

  bool bound_any = false;
  // each ready op gets at most one proposal per round
  std::vector<char>& tried = c->scratch.tried;
  tried.assign(ready.size(), 0);
  std::vector<vte_ready_op>& q = c->scratch.q;
  std::vector<int>& qi = c->scratch.qi;
  for (size_t round = 0; round < ready.size(); ++round) {
    q.clear();
    qi.clear();
    for (size_t i = 0; i < ready.size(); ++i)
      if (!tried[i]) { q.push_back(ready[i]); qi.push_back(static_cast<int>(i)); }
    if (q.empty()) break;
    int pick = c->custom_policy && c->policy.pick
                   ? c->policy.pick(c->policy_user, q.data(), static_cast<int>(q.size()), &S)
                   : builtin_pick(c, q.data(), static_cast<int>(q.size()), &S);
    if (pick < 0 || pick >= static_cast<int>(q.size())) break;  // policy defers
    const int ri = qi[pick];
    tried[ri] = 1;
    Op* op = ready_ops[ri];
    const vte_ready_op& ro = ready[ri];
    std::vector<int>& eligible = c->scratch.eligible;
    eligible.clear();
    eligible_set(c, op, ro.pinned_pctx, &eligible);
    if (eligible.empty()) continue;
    int sel = c->custom_policy && c->policy.select
                  ? c->policy.select(c->policy_user, &ro, eligible.data(), static_cast<int>(eligible.size()), &S)
                  : builtin_select(c, &ro, eligible.data(), static_cast<int>(eligible.size()), &S);
    if (sel < 0) continue;
    // the proposal is tentative: it must be one of E and still valid
    if (std::find(eligible.begin(), eligible.end(), sel) == eligible.end()) { ++c->stats.stale_proposals; continue; }
    int rc = bind_and_submit(c, op, sel, c->cfg.mode != VTE_MODE_PIPELINED);
    if (rc != VTE_OK) { submission_failed(c, op, rc); continue; }  // op remains ready for rescheduling (a bounded number of times)
    c->vstreams[op->vs]->queue.pop_front();
    bound_any = true;
    for (int i = 0; i < c->pool.size(); ++i) fill_info(c->pool, i, &infos[i]);
    --S.ready_by_class[ro.klass];
    S.inflight_by_class[0] = c->inflight_by_class[0];
    S.inflight_by_class[1] = c->inflight_by_class[1];
  }
  return bound_any;
}

// ---- plan-driven policies (Sec. 5: Throughput-Oriented, TPOT-First) ---------------------

// Seconds the ops of `vs` that belong to its current token are predicted to need
// from now: ops already in flight at the width they run on, queued ones at
// `width`.  Ops the application has not submitted yet are unknown and count as 0.
double tpot_remaining(vte_ctx* c, const vte_vstream* vs, int width) {
  int left = vs->ops_per_token - static_cast<int>(vs->ops_done % static_cast<uint64_t>(vs->ops_per_token));
  double sum = 0;
  for (const Op* op : c->inflight) {
    if (left <= 0) break;
    if (op->vs != vs->id) continue;
    const double t = profile_time(c, op->desc->profile_key, c->pool.at(op->pctx).width);
    if (t > 0) sum += t;
    --left;
  }
  for (const Op* op : vs->queue) {
    if (left <= 0) break;
    const double t = profile_time(c, op->desc->profile_key, width);
    if (t > 0) sum += t;
    --left;
  }
  return sum * vs->slowdown;  // profiles are solo times; the factor is what sharing has cost lately
}

// Profiled time of one token of `vs` at `width`: the sum over the last
// ops_per_token ops it submitted; -1 while any of them lacks a profile.
double tpot_token_time(vte_ctx* c, const vte_vstream* vs, int width) {
  if (vs->token_keys.empty()) return -1.0;
  double sum = 0;
  for (uint64_t key : vs->token_keys) {
    const double t = profile_time(c, key, width);
    if (t <= 0) return -1.0;
    sum += t;
  }
  return sum;
}

bool reservable_for(vte_ctx* c, int id, int vs) {
  const Pctx& p = c->pool.at(id);
  if (p.reserved_for >= 0 && p.reserved_for != vs) return false;
  std::vector<int> ov;
  c->pool.active_overlapping(id, &ov);
  for (int o : ov) {
    const Pctx& q = c->pool.at(o);
    if (q.reserved_for >= 0 && q.reserved_for != vs) return false;
  }
  return true;
}

// TPOT-First bookkeeping, run by the dispatcher before every dispatch round: the
// standing reservation, the next-token deadline d_o = (previous token's
// completion) + target, the prediction on the standing pCtx including queued
// decode work, and Prepare when the token is at risk.
void tpot_maintain(vte_ctx* c) {
  const double now = c->now();
  for (vte_vstream* vs : c->vstreams) {
    if (!vs || !vs->alive || vs->tpot <= 0) continue;
    // standing pCtx: the narrowest width whose profiled token time meets the target
    if (vs->standing < 0) {
      if (vs->ops_submitted < static_cast<uint64_t>(vs->ops_per_token)) continue;  // the chain of one token is not known yet
      if (vs->queue.empty() && vs->unfinished_bound == 0) continue;                // idle: holds nothing
      int want = -1;
      std::vector<int> widths;
      for (int id = 0; id < c->pool.size(); ++id)
        if (c->pool.at(id).kind == kNode) widths.push_back(c->pool.at(id).width);
      std::sort(widths.begin(), widths.end());
      widths.erase(std::unique(widths.begin(), widths.end()), widths.end());
      bool profiled = false;
      for (int w : widths) {
        const double t = tpot_token_time(c, vs, w);
        if (t <= 0) continue;
        profiled = true;
        if (t * (1.0 + c->slack) <= vs->tpot) { want = w; break; }
      }
      if (!profiled) continue;                 // nothing to size it from yet
      if (want < 0) want = c->pool.total_cus();  // no width meets the target: the whole device
      // a pipe no other vstream will be dispatching on beside it, then the lowest id: standing pCtxs
      // pack from one side, so a pre-created remainder covers the rest.  Leases that overlap the
      // candidate do not count: the reservation closes their gates and they drain.
      auto pipe_taken = [&](int cand) {
        for (int id = 0; id < c->pool.size(); ++id) {
          const Pctx& q = c->pool.at(id);
          const bool mine = q.reserved_for == vs->id || (q.state == kLeased && q.holder == vs->id);
          if (q.active_self && !mine && q.pipe == c->pool.at(cand).pipe && !c->pool.overlaps(id, cand)) return true;
        }
        return false;
      };
      for (int pass = 0; pass < 2 && vs->standing < 0; ++pass)
        for (int id = 0; id < c->pool.size() && vs->standing < 0; ++id) {
          const Pctx& p = c->pool.at(id);
          if (p.kind != kNode || p.width != want || !reservable_for(c, id, vs->id)) continue;
          if (pass == 0 && pipe_taken(id)) continue;
          if (reserve_locked(c, id, vs->id) == VTE_OK) vs->standing = id;
        }
      if (vs->standing < 0) continue;
      // exclusive: leases of other vstreams that overlap it take nothing new and drain
      std::vector<int> ov;
      c->pool.active_overlapping(vs->standing, &ov);
      for (int o : ov) {
        const Pctx& q = c->pool.at(o);
        if (q.state == kLeased && q.holder != vs->id) close_gate_locked(c, o);
      }
    }
    const bool idle = vs->queue.empty() && vs->unfinished_bound == 0;
    if (idle && vs->escalated < 0 && vs->t_idle >= 0 && now - vs->t_idle > 2 * vs->tpot) {
      // nothing for two token periods: the CUs go back until the next submission sizes it again
      unreserve_locked(c, vs->standing);
      vs->standing = -1;
      continue;
    }
    const uint64_t token_now = vs->ops_done / static_cast<uint64_t>(vs->ops_per_token);
    const int w_st = c->pool.at(vs->standing).width;
    const double deadline = vs->t_ref + vs->tpot;
    const bool at_risk = !idle && vs->t_ref >= 0 && now + tpot_remaining(c, vs, w_st) > deadline;
    vs->at_risk = at_risk;
    if (vs->escalated >= 0) {
      // give the wider pCtx back at a token boundary once the standing one suffices again
      if (idle || (!at_risk && token_now > vs->escalated_token)) {
        unreserve_locked(c, vs->escalated);
        vs->escalated = -1;
      }
      continue;
    }
    if (!at_risk) continue;
    // Prepare: the smallest wider pCtx predicted to meet the deadline (the widest if none does)
    int target = -1;
    bool target_meets = false;
    for (int id = 0; id < c->pool.size(); ++id) {
      const Pctx& p = c->pool.at(id);
      if (p.width <= w_st || !c->pool.overlaps(id, vs->standing) || !reservable_for(c, id, vs->id)) continue;
      const bool meets = now + tpot_remaining(c, vs, p.width) <= deadline;
      bool better;
      if (target < 0) better = true;
      else if (meets != target_meets) better = meets;
      else better = meets ? p.width < c->pool.at(target).width : p.width > c->pool.at(target).width;
      if (better) { target = id; target_meets = meets; }
    }
    if (target < 0) continue;
    std::vector<int> ov;
    c->pool.active_overlapping(target, &ov);
    for (int o : ov) {
      const Pctx& q = c->pool.at(o);
      if (q.state == kLeased && q.holder != vs->id) close_gate_locked(c, o);  // drain overlapping best-effort work
    }
    if (reserve_locked(c, target, vs->id) == VTE_OK) {
      vs->escalated = target;
      vs->escalated_token = token_now;
      ++vs->escalations;
    }
  }
}

// One dispatch round of the plan-driven policies.  TPOT-First places the decode
// ops of vstreams with a target first (earliest deadline, at-risk first) on their
// prepared or standing pCtx; everything else follows the Throughput-Oriented plan:
// Pick returns the next planned op in age order, Select returns A[o].
bool planned_round(vte_ctx* c, const std::vector<vte_ready_op>& ready, const std::vector<Op*>& ready_ops) {
  const int n = static_cast<int>(ready.size());
  bool bound_any = false;
  std::vector<char> handled(n, 0);
  auto bind = [&](int i, int pctx) {
    Op* op = ready_ops[i];
    const int rc = bind_and_submit(c, op, pctx, c->cfg.mode != VTE_MODE_PIPELINED);
    if (rc != VTE_OK) { submission_failed(c, op, rc); return false; }
    c->vstreams[op->vs]->queue.pop_front();
    bound_any = true;
    return true;
  };

  if (c->builtin == VTE_POLICY_TPOT_FIRST) {
    std::vector<int> dec;
    for (int i = 0; i < n; ++i) {
      const vte_vstream* vs = c->vstreams[ready[i].vstream];
      if (vs->tpot > 0 && vs->standing >= 0 && ready[i].pinned_pctx < 0) dec.push_back(i);
    }
    std::stable_sort(dec.begin(), dec.end(), [&](int a, int b) {
      const vte_vstream* va = c->vstreams[ready[a].vstream];
      const vte_vstream* vb = c->vstreams[ready[b].vstream];
      if (va->at_risk != vb->at_risk) return va->at_risk;
      return va->t_ref + va->tpot < vb->t_ref + vb->tpot;
    });
    for (int i : dec) {
      handled[i] = 1;
      const vte_vstream* vs = c->vstreams[ready[i].vstream];
      std::vector<int> el;
      eligible_set(c, ready_ops[i], -1, &el);
      auto has = [&](int id) { return id >= 0 && std::find(el.begin(), el.end(), id) != el.end(); };
      if (vs->escalated >= 0) {
        if (has(vs->escalated)) { bind(i, vs->escalated); continue; }
        // blocked only by this vstream's own in-flight ops: it frees up as they retire
        if (blocked_by_own_leases_only(c, vs->escalated, &ready[i])) continue;
        // preparation incomplete (overlapping work still drains): use what is available
      }
      if (has(vs->standing)) bind(i, vs->standing);
      // else defer: the standing pCtx is exclusive, so this only waits for the vstream's own work
    }
  }

  std::vector<int> idx;
  std::vector<PlanOp> ops;
  for (int i = 0; i < n; ++i) {
    if (handled[i]) continue;
    PlanOp po;
    po.age = ready[i].age;
    po.pred_pctx = ready[i].pred_pctx;
    eligible_set(c, ready_ops[i], ready[i].pinned_pctx, &po.eligible);
    for (int id = 0; id < c->pool.size(); ++id) {
      if (blocked_by_own_leases_only(c, id, &ready[i])) po.later.push_back(id);
      const Pctx& q = c->pool.at(id);  // pipes other vstreams are dispatching on
      if ((q.state == kLeased || q.state == kDraining) && q.holder != ready[i].vstream) po.busy_pipes |= 1u << q.pipe;
    }
    idx.push_back(i);
    ops.push_back(po);
  }
  if (ops.empty()) return bound_any;
  // age-aware: while an older op has nowhere to go, a younger one does not renew its vstream's
  // lease; the lease drains and the next round plans both together
  uint64_t oldest_starved = ~0ull;
  for (size_t o = 0; o < ops.size(); ++o)
    if (ops[o].eligible.empty() && ops[o].later.empty() && ready[idx[o]].pinned_pctx < 0)
      oldest_starved = std::min(oldest_starved, ops[o].age);
  // An op stands for the recurring chain its vstream runs (Sec. 5 "Performance Profiles"): the plan
  // weighs the chain's profiled time at a width, not the time of the launch that happens to be ready
  // when the plan is made.  Planned per launch, a stream whose ready op was a norm (flat profile) or
  // a small projection was left on a leaf while the co-tenant took the remainder, and the leases
  // then kept it there: decode on 32 + 32 CUs beside a GEMM on 192, sum 1.10 against 1.21 for the
  // fixed split at 80 requests/s.
  const std::vector<int> A = tput_plan(c->pool, ops, [&](int o, int width) {
    const double t = chain_time(c, &ready[idx[o]], width);
    return t > 0 ? t : profile_time(c, ready[idx[o]].desc.profile_key, width);
  });
  std::vector<int> order(ops.size());
  for (size_t o = 0; o < order.size(); ++o) order[o] = static_cast<int>(o);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return ops[a].age < ops[b].age; });
  for (int o : order) {
    if (A[o] < 0) continue;
    if (std::find(ops[o].eligible.begin(), ops[o].eligible.end(), A[o]) == ops[o].eligible.end()) continue;  // waits for its own lease
    if (ops[o].age > oldest_starved && c->pool.at(A[o]).state == kLeased) continue;
    bind(idx[o], A[o]);
  }
  return bound_any;
}

void dispatcher_main(vte_ctx* c) {
  c->backend->make_current();
  Lock lk(c->mu);
  while (true) {
    const uint64_t seen = c->change_seq;
    bool progress = poll_completions(c);
    if (!c->custom_policy && c->builtin == VTE_POLICY_TPOT_FIRST) tpot_maintain(c);
    // keep binding while ops become bindable (PIPELINED chains, freed leases)
    bool bound = false;
    while (dispatch_round(c)) bound = true;
    progress = progress || bound;
    flush_records(c);  // PIPELINED: one completion record per burst and pCtx instead of one per launch
    if (bound && (!c->awaited.empty() || c->waiters_all)) notify_done(c);  // a waiter may start polling now
    if (c->stop && c->live.empty()) break;
    if (progress) continue;
    if (c->change_seq == seen) {
      c->quiesced_seq = seen;
      c->cv_done.notify_all();  // for vte_dispatcher_quiesce only: no launch changed state, pollers need not look
    }
    if (!c->inflight.empty() && !c->backend->is_fake()) {
      // device work outstanding: poll again soon, letting callers in
      lk.unlock();
      std::this_thread::yield();
      lk.lock();
    } else if (c->change_seq == seen) {
      // nothing can change without outside input (or a policy that deferred)
      bool pending = false;
      for (vte_vstream* vs : c->vstreams) if (vs && !vs->queue.empty()) pending = true;
      if (pending && c->inflight.empty()) {
        c->cv_work.wait_for(lk, std::chrono::microseconds(200));
      } else {
        if (!c->backend->is_fake() && !c->stop) {
          // just ran out of work: the next submission often follows within the millisecond (the caller
          // synchronised and submits the next burst); poll for it before going to sleep
          lk.unlock();
          const auto t0 = std::chrono::steady_clock::now();
          while (c->change_seq.load(std::memory_order_acquire) == seen &&
                 std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count() < kDispatcherPollSeconds)
            for (int i = 0; i < 32; ++i) cpu_relax();
          lk.lock();
        }
        c->cv_work.wait(lk, [&] { return c->change_seq != seen || c->stop; });
      }
    }
  }
}

vte_ctx* ctx_of(vte_vstream* vs) { return vs ? vs->ctx : nullptr; }

}  // namespace
}  // namespace vte

using namespace vte;

extern "C" {

const char* vte_last_error(void) { return g_err.c_str(); }
int vte_last_hip_error(void) { return g_hip_err; }

int vte_pool_cfg_default(vte_pool_cfg* cfg) {
  if (!cfg) { set_error("null cfg"); return VTE_EINVAL; }
  std::memset(cfg, 0, sizeof *cfg);
  cfg->backend = VTE_BACKEND_HIP;
  cfg->leaf_cus = 32;
  cfg->layout = VTE_LAYOUT_STRIPED;
  cfg->with_remainders = VTE_REMAINDERS_PER_LEVEL;
  cfg->mode = VTE_MODE_STRICT;
  cfg->lookahead = 16;
  cfg->stats_capacity = 65536;
  return VTE_OK;
}

int vte_init(vte_ctx** out, int device, const vte_pool_cfg* user_cfg) {
  if (!out) { set_error("null out"); return VTE_EINVAL; }
  vte_pool_cfg cfg;
  vte_pool_cfg_default(&cfg);
  if (user_cfg) cfg = *user_cfg;
  if (cfg.leaf_cus <= 0) cfg.leaf_cus = 32;
  if (cfg.lookahead <= 0) cfg.lookahead = 16;
  if (cfg.stats_capacity <= 0) cfg.stats_capacity = 65536;
  if (cfg.layout != VTE_LAYOUT_STRIPED) { set_error("only VTE_LAYOUT_STRIPED is offered"); return VTE_EINVAL; }
  if (cfg.mode != VTE_MODE_STRICT && cfg.mode != VTE_MODE_PIPELINED) { set_error("unknown mode"); return VTE_EINVAL; }
  if (cfg.backend != VTE_BACKEND_HIP && cfg.backend != VTE_BACKEND_FAKE) { set_error("unknown backend"); return VTE_EINVAL; }
  vte_ctx* c = new (std::nothrow) vte_ctx;
  if (!c) { set_error("out of host memory"); return VTE_ENOMEM; }
  c->cfg = cfg;
  c->device = device;
  c->t0 = std::chrono::steady_clock::now();
  c->backend = cfg.backend == VTE_BACKEND_FAKE ? make_fake_backend() : make_hip_backend();
  int cus = cfg.total_cus;
  int rc = c->backend->init(device, &cus);
  if (rc == VTE_OK && cfg.backend == VTE_BACKEND_HIP) rc = static_scratch_setup(device);  // the device is current here
  if (rc != VTE_OK) { delete c->backend; delete c; return rc; }
  c->cfg.total_cus = cus;
  std::string err;
  if (cus > 256) { set_error("more than 256 CUs are not supported"); delete c->backend; delete c; return VTE_EINVAL; }
  if (cfg.with_remainders < 0 || cfg.with_remainders > 2) { set_error("with_remainders must be 0, 1 or 2"); delete c->backend; delete c; return VTE_EINVAL; }
  if (!c->pool.build(cus, cfg.leaf_cus, cfg.with_remainders, &err)) {
    set_error(err); delete c->backend; delete c; return VTE_EINVAL;
  }
  // pre-create every pCtx's backend stream: nothing is created on the dispatch path.
  // The device deals queues to its dispatch pipes in creation order, so the order
  // decides which pCtxs can dispatch side by side.
  if (cfg.device_timing_stride < 0) { set_error("device_timing_stride must not be negative"); delete c->backend; delete c; return VTE_EINVAL; }
  if (cfg.dispatch_pipes < 0 || cfg.dispatch_pipes > 32) { set_error("dispatch_pipes must be in [0,32]"); delete c->backend; delete c; return VTE_EINVAL; }
  c->pool.assign_pipes(cfg.dispatch_pipes == 0 ? 4 : cfg.dispatch_pipes);
  c->cfg.dispatch_pipes = c->pool.pipes();
  for (int id : c->pool.creation_order()) {
    void* s = nullptr;
    if (id >= 0) {
      Pctx& p = c->pool.at(id);
      rc = c->backend->create_stream(p.mask.data(), static_cast<int>(p.mask.size()), &s);
      if (rc == VTE_OK) p.stream = s;
    } else {  // placeholder that keeps the rotation in step; never used
      const Pctx& p = c->pool.at(c->pool.root());
      rc = c->backend->create_stream(p.mask.data(), static_cast<int>(p.mask.size()), &s);
      if (rc == VTE_OK) c->placeholder_streams.push_back(s);
    }
    if (rc != VTE_OK) {
      for (int j = 0; j < c->pool.size(); ++j) if (c->pool.at(j).stream) c->backend->destroy_stream(c->pool.at(j).stream);
      for (void* d : c->placeholder_streams) c->backend->destroy_stream(d);
      delete c->backend; delete c; return rc;
    }
  }
  c->ring.resize(static_cast<size_t>(cfg.stats_capacity));
  c->lazy_tail.assign(c->pool.size(), nullptr);
  c->record_failures.assign(c->pool.size(), 0);
  c->dispatcher = std::thread(dispatcher_main, c);
  *out = c;
  return VTE_OK;
}

int vte_device_sync(vte_ctx* c) {
  if (!c) { set_error("null ctx"); return VTE_EINVAL; }
  Lock lk(c->mu);
  // waits on every token issued so far (all vstream tails and explicit launches)
  const vte_token upto = c->next_token;
  ++c->waiters_all;
  bump(c);  // the dispatcher records a completion behind every pCtx's newest launch while somebody waits for all
  wait_done(c, lk,
            [&] {
              for (auto& kv : c->live) if (kv.first < upto) return false;
              return true;
            },
            [&] { return c->live.size() == c->inflight.size(); });  // nothing is left unbound
  --c->waiters_all;
  if (c->failure_unreported) {  // something failed since the last device-wide wait: say so once, here
    c->failure_unreported = false;
    return report_failure(c, c->first_unreported);
  }
  return VTE_OK;
}

int vte_shutdown(vte_ctx* c) {
  if (!c) { set_error("null ctx"); return VTE_EINVAL; }
  if (!c->backend->is_fake()) vte_device_sync(c);
  {
    Lock lk(c->mu);
    if (c->backend->is_fake()) {
      // nothing will complete by itself: finish what is in flight, drop the rest
      auto* fb = static_cast<FakeBackend*>(c->backend);
      fb->autocomplete = true;
      for (Op* op : c->inflight) fb->complete(op->tok);
      for (vte_vstream* vs : c->vstreams) {
        if (!vs) continue;
        for (Op* op : vs->queue) { c->live.erase(op->tok); delete op; }
        vs->queue.clear();
      }
    }
    c->stop = true;
    bump(c);
  }
  c->dispatcher.join();
  for (int id = 0; id < c->pool.size(); ++id) c->backend->destroy_stream(c->pool.at(id).stream);
  for (void* d : c->placeholder_streams) c->backend->destroy_stream(d);
  for (vte_vstream* vs : c->vstreams) delete vs;
  for (vte_desc* d : c->descs) delete d;
  delete c->backend;
  delete c;
  return VTE_OK;
}

int vte_pool_count(vte_ctx* c, int* count) {
  if (!c || !count) { set_error("null argument"); return VTE_EINVAL; }
  *count = c->pool.size();
  return VTE_OK;
}

int vte_pool_info(vte_ctx* c, int id, vte_pctx_info* info) {
  if (!c || !info || id < 0 || id >= c->pool.size()) { set_error("pool_info: bad argument"); return VTE_EINVAL; }
  Lock lk(c->mu);
  fill_info(c->pool, id, info);
  return VTE_OK;
}

int vte_pool_creation_order(vte_ctx* c, int* ids, int cap, int* n_out) {
  if (!c || !ids || cap < 0 || !n_out) { set_error("creation_order: bad argument"); return VTE_EINVAL; }
  const std::vector<int> order = c->pool.creation_order();
  *n_out = static_cast<int>(order.size());
  for (int i = 0; i < cap && i < *n_out; ++i) ids[i] = order[i];
  return VTE_OK;
}

int vte_pool_find(vte_ctx* c, int kind, int width, int index, int* pctx_id) {
  if (!c || !pctx_id || index < 0) { set_error("pool_find: bad argument"); return VTE_EINVAL; }
  for (int id = 0; id < c->pool.size(); ++id) {
    const Pctx& p = c->pool.at(id);
    if (p.kind == kind && p.width == width && index-- == 0) { *pctx_id = id; return VTE_OK; }
  }
  set_error("pool_find: no such pCtx");
  return VTE_EINVAL;
}

int vte_pool_conflict(vte_ctx* c, int a, int b, int* conflict) {
  if (!c || !conflict || a < 0 || b < 0 || a >= c->pool.size() || b >= c->pool.size()) { set_error("pool_conflict: bad argument"); return VTE_EINVAL; }
  *conflict = c->pool.overlaps(a, b) ? 1 : 0;
  return VTE_OK;
}

int vte_pctx_native_stream(vte_ctx* c, int id, void** s) {
  if (!c || !s || id < 0 || id >= c->pool.size()) { set_error("native_stream: bad argument"); return VTE_EINVAL; }
  *s = c->pool.at(id).stream;
  return VTE_OK;
}

int vte_desc_destroy(vte_desc* d) {
  if (!d) { set_error("null desc"); return VTE_EINVAL; }
  vte_ctx* c = d->ctx;
  {
    Lock lk(c->mu);
    for (auto& kv : c->live)
      if (kv.second->desc == d) { set_error("descriptor still has launches in flight"); return VTE_EBUSY; }
    c->descs.erase(std::remove(c->descs.begin(), c->descs.end(), d), c->descs.end());
  }
  delete d;
  return VTE_OK;
}

int vte_bind_and_launch(vte_ctx* c, const vte_desc* d, int pctx, vte_token* tok_out) {
  if (!c || !d) { set_error("bind_and_launch: null argument"); return VTE_EINVAL; }
  if (d->ctx != c) { set_error("descriptor belongs to another context"); return VTE_EINVAL; }
  Lock lk(c->mu);
  Op* op = new (std::nothrow) Op;
  if (!op) { set_error("out of host memory"); return VTE_ENOMEM; }
  op->tok = c->next_token;
  op->desc = d;
  op->vs = -1;
  op->klass = VTE_CLASS_LATENCY;
  op->age = c->next_age;
  op->t_submit = op->t_ready = c->now();
  c->backend->make_current();
  int rc = bind_and_submit(c, op, pctx, true);
  if (rc != VTE_OK) { delete op; return rc; }
  ++c->next_token;
  ++c->next_age;
  c->live[op->tok] = op;
  ++c->stats.submitted;
  if (tok_out) *tok_out = op->tok;
  bump(c);
  return VTE_OK;
}

int vte_vstream_create(vte_ctx* c, int klass, vte_vstream** out) {
  if (!c || !out || (klass != VTE_CLASS_LATENCY && klass != VTE_CLASS_BEST_EFFORT)) { set_error("vstream_create: bad argument"); return VTE_EINVAL; }
  vte_vstream* vs = new (std::nothrow) vte_vstream;
  if (!vs) { set_error("out of host memory"); return VTE_ENOMEM; }
  Lock lk(c->mu);
  vs->ctx = c;
  vs->klass = klass;
  vs->id = static_cast<int>(c->vstreams.size());
  c->vstreams.push_back(vs);
  *out = vs;
  return VTE_OK;
}

int vte_vstream_id(const vte_vstream* vs, int* id) {
  if (!vs || !id) { set_error("null argument"); return VTE_EINVAL; }
  *id = vs->id;
  return VTE_OK;
}

int vte_vstream_pin(vte_vstream* vs, int pctx) {
  vte_ctx* c = ctx_of(vs);
  if (!c || pctx < -1 || pctx >= c->pool.size()) { set_error("vstream_pin: bad argument"); return VTE_EINVAL; }
  Lock lk(c->mu);
  vs->pinned = pctx;
  bump(c);
  return VTE_OK;
}

// runtime lock held
static int submit_locked(vte_ctx* c, vte_vstream* vs, const vte_desc* d, const vte_token* deps, int n_deps, vte_token* tok_out) {
  if (!vs->alive) { set_error("vstream was destroyed"); return VTE_EINVAL; }
  for (int i = 0; i < n_deps; ++i)
    if (deps[i] >= c->next_token) { set_error("dependency on a token that was never issued"); return VTE_EINVAL; }
  Op* op = new (std::nothrow) Op;
  if (!op) { set_error("out of host memory"); return VTE_ENOMEM; }
  op->tok = c->next_token++;
  op->desc = d;
  op->vs = vs->id;
  op->klass = vs->klass;
  op->age = c->next_age++;
  op->t_submit = c->now();
  op->deps.push_back(vs->tail);  // stream order: depends on the tail, becomes the tail
  for (int i = 0; i < n_deps; ++i) op->deps.push_back(deps[i]);
  for (vte_token t : vs->waited_events) op->deps.push_back(t);  // stream-level waits: this op carries them, later ops follow it
  vs->waited_events.clear();
  if (vs->tpot > 0 && vs->queue.empty() && vs->unfinished_bound == 0) vs->t_ref = op->t_submit;  // the clock of an idle stream starts now
  ++vs->ops_submitted;
  if (vs->tpot > 0) {
    vs->token_keys.push_back(d->profile_key);
    if (vs->token_keys.size() > static_cast<size_t>(vs->ops_per_token)) vs->token_keys.pop_front();
  }
  vs->tail = op->tok;
  vs->queue.push_back(op);
  auto& rk = vs->recent_keys;  // move-to-front list of the chain's distinct descriptors
  auto kit = std::find(rk.begin(), rk.end(), d->profile_key);
  if (kit != rk.end()) rk.erase(kit);
  rk.insert(rk.begin(), d->profile_key);
  if (rk.size() > 16) rk.pop_back();
  c->live[op->tok] = op;
  ++c->stats.submitted;
  if (tok_out) *tok_out = op->tok;
  return VTE_OK;
}

int vte_submit_after(vte_vstream* vs, const vte_desc* d, const vte_token* deps, int n_deps, vte_token* tok_out) {
  vte_ctx* c = ctx_of(vs);
  if (!c || !d || n_deps < 0 || (n_deps > 0 && !deps)) { set_error("submit: bad argument"); return VTE_EINVAL; }
  if (d->ctx != c) { set_error("descriptor belongs to another context"); return VTE_EINVAL; }
  Lock lk(c->mu);
  const int rc = submit_locked(c, vs, d, deps, n_deps, tok_out);
  if (rc == VTE_OK) bump(c);
  return rc;
}

int vte_submit(vte_vstream* vs, const vte_desc* d, vte_token* tok_out) {
  return vte_submit_after(vs, d, nullptr, 0, tok_out);
}

int vte_submit_batch(vte_vstream* vs, const vte_desc* const* descs, int n, vte_token* last_out) {
  vte_ctx* c = ctx_of(vs);
  if (!c || !descs || n < 1) { set_error("submit_batch: bad argument"); return VTE_EINVAL; }
  for (int i = 0; i < n; ++i)
    if (!descs[i] || descs[i]->ctx != c) { set_error("submit_batch: null descriptor or one of another context"); return VTE_EINVAL; }
  Lock lk(c->mu);  // the dispatcher sees the whole batch at once
  if (!vs->alive) { set_error("vstream was destroyed"); return VTE_EINVAL; }
  vte_token last = 0;
  for (int i = 0; i < n; ++i) {
    const int rc = submit_locked(c, vs, descs[i], nullptr, 0, &last);
    if (rc != VTE_OK) { if (i > 0) bump(c); return rc; }  // out of memory: earlier ops stay submitted
    if (last_out) *last_out = last;
  }
  bump(c);
  return VTE_OK;
}

int vte_event_record(vte_vstream* vs, vte_token* event_out) {
  vte_ctx* c = ctx_of(vs);
  if (!c || !event_out) { set_error("event_record: bad argument"); return VTE_EINVAL; }
  Lock lk(c->mu);
  *event_out = vs->tail;
  return VTE_OK;
}

int vte_vstream_wait_event(vte_vstream* vs, vte_token event) {
  vte_ctx* c = ctx_of(vs);
  if (!c) { set_error("wait_event: null vstream"); return VTE_EINVAL; }
  Lock lk(c->mu);
  if (!vs->alive) { set_error("vstream was destroyed"); return VTE_EINVAL; }
  if (event >= c->next_token) { set_error("wait_event: token was never issued"); return VTE_EINVAL; }
  if (event != 0 && !token_done(c, event)) vs->waited_events.push_back(event);
  return VTE_OK;
}

int vte_token_query(vte_ctx* c, vte_token t, int* done) {
  if (!c || !done) { set_error("null argument"); return VTE_EINVAL; }
  Lock lk(c->mu);
  if (t >= c->next_token) { set_error("token was never issued"); return VTE_EINVAL; }
  *done = token_done(c, t) ? 1 : 0;
  return *done ? report_failure(c, t) : VTE_OK;
}

int vte_token_wait(vte_ctx* c, vte_token t) {
  if (!c) { set_error("null ctx"); return VTE_EINVAL; }
  Lock lk(c->mu);
  if (t >= c->next_token) { set_error("token was never issued"); return VTE_EINVAL; }
  if (token_done(c, t)) return report_failure(c, t);
  c->awaited.push_back(t);
  bump(c);  // the dispatcher sees to it that a completion record covers the awaited launch
  wait_done(c, lk, [&] { return token_done(c, t); },
            [&] {
              auto it = c->live.find(t);
              return it != c->live.end() && it->second->state == kInflight;
            });
  c->awaited.erase(std::find(c->awaited.begin(), c->awaited.end(), t));
  return report_failure(c, t);
}

int vte_vstream_sync(vte_vstream* vs) {
  vte_ctx* c = ctx_of(vs);
  if (!c) { set_error("null vstream"); return VTE_EINVAL; }
  vte_token t;
  {
    Lock lk(c->mu);
    t = vs->tail;
  }
  const int rc = vte_token_wait(c, t);
  if (rc != VTE_OK && rc != VTE_EINVAL) {
    // the failure has been handed to the caller: the stream starts again from an empty tail, so
    // that what is submitted from now on does not inherit it
    Lock lk(c->mu);
    if (vs->tail == t) vs->tail = 0;
  }
  return rc;
}

int vte_vstream_destroy(vte_vstream* vs) {
  vte_ctx* c = ctx_of(vs);
  if (!c) { set_error("null vstream"); return VTE_EINVAL; }
  if (!c->backend->is_fake()) vte_vstream_sync(vs);
  Lock lk(c->mu);
  if (!vs->queue.empty() || vs->unfinished_bound > 0) { set_error("vstream still has work"); return VTE_EBUSY; }
  vs->alive = false;  // the slot stays so ids remain stable; freed at shutdown
  for (int id = 0; id < c->pool.size(); ++id) {
    Pctx& p = c->pool.at(id);
    if (p.reserved_for == vs->id) {
      p.reserved_for = -1; p.reservation_pending = false;
      if (p.state == kReserved) p.state = kIdle;
      if (p.state == kIdle) c->pool.set_active(id, false);
    }
  }
  settle_reservations(c);
  bump(c);
  return VTE_OK;
}

// ---- lease control ------------------------------------------------------------------

int vte_pctx_close_gate(vte_ctx* c, int id) {
  if (!c || id < 0 || id >= c->pool.size()) { set_error("close_gate: bad argument"); return VTE_EINVAL; }
  Lock lk(c->mu);
  close_gate_locked(c, id);
  bump(c);
  return VTE_OK;
}

int vte_pctx_reserve(vte_ctx* c, int id, vte_vstream* vs) {
  if (!c || !vs || vs->ctx != c || id < 0 || id >= c->pool.size()) { set_error("reserve: bad argument"); return VTE_EINVAL; }
  Lock lk(c->mu);
  const int rc = reserve_locked(c, id, vs->id);
  if (rc == VTE_OK) bump(c);
  return rc;
}

int vte_pctx_unreserve(vte_ctx* c, int id) {
  if (!c || id < 0 || id >= c->pool.size()) { set_error("unreserve: bad argument"); return VTE_EINVAL; }
  Lock lk(c->mu);
  unreserve_locked(c, id);
  bump(c);
  return VTE_OK;
}

// ---- TPOT target of a decode vstream (Sec. 5, TPOT-First) ----------------------------------

int vte_vstream_set_tpot(vte_vstream* vs, double tpot_seconds, int ops_per_token) {
  vte_ctx* c = ctx_of(vs);
  if (!c || tpot_seconds < 0 || (tpot_seconds > 0 && ops_per_token < 1)) { set_error("set_tpot: bad argument"); return VTE_EINVAL; }
  Lock lk(c->mu);
  if (!vs->alive) { set_error("vstream was destroyed"); return VTE_EINVAL; }
  if (!vs->queue.empty() || vs->unfinished_bound > 0) { set_error("set_tpot: the vstream has work"); return VTE_EBUSY; }
  if (vs->escalated >= 0) { unreserve_locked(c, vs->escalated); vs->escalated = -1; }
  if (vs->standing >= 0) { unreserve_locked(c, vs->standing); vs->standing = -1; }
  vs->tpot = tpot_seconds;
  vs->ops_per_token = tpot_seconds > 0 ? ops_per_token : 0;
  vs->ops_done = vs->ops_submitted = vs->tokens_done = vs->deadline_misses = vs->escalations = 0;
  vs->t_ref = -1;
  vs->at_risk = false;
  vs->slowdown = 1.0;
  vs->t_idle = -1;
  vs->token_keys.clear();
  bump(c);
  return VTE_OK;
}

int vte_vstream_tpot_info(vte_vstream* vs, vte_tpot_info* out) {
  vte_ctx* c = ctx_of(vs);
  if (!c || !out) { set_error("tpot_info: bad argument"); return VTE_EINVAL; }
  Lock lk(c->mu);
  std::memset(out, 0, sizeof *out);
  out->tpot_seconds = vs->tpot;
  out->ops_per_token = vs->ops_per_token;
  out->standing_pctx = vs->standing;
  out->escalated_pctx = vs->escalated;
  out->at_risk = vs->at_risk ? 1 : 0;
  out->tokens_done = vs->tokens_done;
  out->deadline_misses = vs->deadline_misses;
  out->escalations = vs->escalations;
  return VTE_OK;
}

// ---- policy -----------------------------------------------------------------------------

int vte_set_policy(vte_ctx* c, const vte_policy_vtbl* vtbl, void* user) {
  if (!c) { set_error("null ctx"); return VTE_EINVAL; }
  Lock lk(c->mu);
  if (vtbl) { c->policy = *vtbl; c->policy_user = user; c->custom_policy = true; }
  else { c->custom_policy = false; std::memset(&c->policy, 0, sizeof c->policy); c->policy_user = nullptr; }
  bump(c);
  return VTE_OK;
}

int vte_set_builtin_policy(vte_ctx* c, int which, double slack, int keep_free_cus) {
  if (!c || which < VTE_POLICY_WIDEST || which > VTE_POLICY_TPOT_FIRST || slack < 0 || keep_free_cus < 0) {
    set_error("set_builtin_policy: bad argument"); return VTE_EINVAL;
  }
  Lock lk(c->mu);
  c->custom_policy = false;
  c->builtin = which;
  c->slack = slack;
  c->keep_free = keep_free_cus;
  bump(c);
  return VTE_OK;
}

int vte_set_device_timing(vte_ctx* c, unsigned mask, int stride) {
  if (!c || stride < 0) { set_error("set_device_timing: bad argument"); return VTE_EINVAL; }
  Lock lk(c->mu);
  c->cfg.device_timing_mask = mask;
  c->cfg.device_timing_stride = stride;
  for (auto& n : c->timing_seen) n = 0;
  return VTE_OK;
}

int vte_hint_submit(vte_ctx* c, const vte_hint* hint) {
  if (!c || !hint) { set_error("null argument"); return VTE_EINVAL; }
  Lock lk(c->mu);
  if (hint->vstream < 0 || hint->vstream >= static_cast<int>(c->vstreams.size())) { set_error("hint: no such vstream"); return VTE_EINVAL; }
  std::vector<vte_pctx_info> infos(c->pool.size());
  for (int i = 0; i < c->pool.size(); ++i) fill_info(c->pool, i, &infos[i]);
  vte_pool_view S{};
  S.count = c->pool.size();
  S.pctx = infos.data();
  S.inflight_by_class[0] = c->inflight_by_class[0];
  S.inflight_by_class[1] = c->inflight_by_class[1];
  vte_prepare_plan plan;
  std::memset(&plan, 0, sizeof plan);
  plan.target_pctx = -1;
  if (c->custom_policy && c->policy.prepare) {
    c->policy.prepare(c->policy_user, hint, &S, &plan);
  } else {
    // default Prepare: the narrowest pCtx at least as wide as wanted with the
    // fewest overlapping active leases; close those gates, reserve the target
    int best = -1; size_t best_ov = 0;
    for (int id = 0; id < c->pool.size(); ++id) {
      const Pctx& p = c->pool.at(id);
      if (p.width < hint->want_width) continue;
      if (p.reserved_for >= 0 && p.reserved_for != hint->vstream) continue;
      std::vector<int> ov; c->pool.active_overlapping(id, &ov);
      if (best < 0 || p.width < c->pool.at(best).width || (p.width == c->pool.at(best).width && ov.size() < best_ov)) { best = id; best_ov = ov.size(); }
    }
    if (best >= 0) {
      plan.target_pctx = best; plan.reserve = 1;
      std::vector<int> ov; c->pool.active_overlapping(best, &ov);
      for (int o : ov) if (plan.n_close < 32 && c->pool.at(o).state == kLeased && o != best) plan.close[plan.n_close++] = o;
    }
  }
  // validate the plan before touching physical state
  if (plan.target_pctx < 0) return VTE_OK;
  if (plan.target_pctx >= c->pool.size() || plan.n_close < 0 || plan.n_close > 32) { ++c->stats.stale_proposals; set_error("prepare: plan rejected"); return VTE_EINVAL; }
  vte_vstream* vs = c->vstreams[hint->vstream];
  for (int i = 0; i < plan.n_close; ++i) {
    const int o = plan.close[i];
    if (o < 0 || o >= c->pool.size() || !c->pool.overlaps(o, plan.target_pctx)) { ++c->stats.stale_proposals; continue; }
    Pctx& q = c->pool.at(o);
    if (q.state == kLeased && o != plan.target_pctx) { q.state = kDraining; q.gate_open = false; ++c->stats.gates_closed; }
  }
  lk.unlock();
  if (plan.reserve) return vte_pctx_reserve(c, plan.target_pctx, vs);
  return VTE_OK;
}

// ---- profiles --------------------------------------------------------------------------

int vte_profile_set(vte_ctx* c, uint64_t key, int width, double seconds) {
  if (!c || width <= 0 || !(seconds > 0)) { set_error("profile_set: bad argument"); return VTE_EINVAL; }
  Lock lk(c->mu);
  c->profiles[{key, width}] = seconds;
  return VTE_OK;
}

int vte_profile_get(vte_ctx* c, uint64_t key, int width, double* seconds) {
  if (!c || !seconds) { set_error("null argument"); return VTE_EINVAL; }
  Lock lk(c->mu);
  const double t = profile_time(c, key, width);
  if (t < 0) { set_error("no profile for this key and width"); return VTE_EINVAL; }
  *seconds = t;
  return VTE_OK;
}

int vte_profile_measure(vte_ctx* c, const vte_desc* d, int warmup, int reps) {
  if (!c || !d || d->ctx != c || warmup < 0 || reps < 1) { set_error("profile_measure: bad argument"); return VTE_EINVAL; }
  if (c->backend->is_fake()) { set_error("profiles cannot be measured on the fake backend"); return VTE_ESTATE; }
  vte_device_sync(c);
  Lock lk(c->mu);
  if (!c->inflight.empty()) { set_error("profile_measure needs an idle device"); return VTE_EBUSY; }
  c->backend->make_current();
  std::vector<int> seen;
  for (int id = 0; id < c->pool.size(); ++id) {
    const Pctx& p = c->pool.at(id);
    if (std::find(seen.begin(), seen.end(), p.width) != seen.end()) continue;
    seen.push_back(p.width);
    double sec = 0;
    int rc = c->backend->time_launches(d, p.stream, warmup, reps, &sec);
    if (rc != VTE_OK) return rc;
    c->profiles[{d->profile_key, p.width}] = sec;
  }
  return VTE_OK;
}

int vte_profile_measure_on(vte_ctx* c, const vte_desc* d, int pctx, int warmup, int reps, double* seconds) {
  if (!c || !d || d->ctx != c || !seconds || warmup < 0 || reps < 1 || pctx < 0 || pctx >= c->pool.size()) {
    set_error("profile_measure_on: bad argument"); return VTE_EINVAL;
  }
  if (c->backend->is_fake()) { set_error("profiles cannot be measured on the fake backend"); return VTE_ESTATE; }
  vte_device_sync(c);
  Lock lk(c->mu);
  if (!c->inflight.empty()) { set_error("profile_measure needs an idle device"); return VTE_EBUSY; }
  c->backend->make_current();
  int rc = c->backend->time_launches(d, c->pool.at(pctx).stream, warmup, reps, seconds);
  if (rc == VTE_OK) c->profiles[{d->profile_key, c->pool.at(pctx).width}] = *seconds;
  return rc;
}

// ---- statistics -----------------------------------------------------------------------

int vte_stats(vte_ctx* c, vte_stats_t* out) {
  if (!c || !out) { set_error("null argument"); return VTE_EINVAL; }
  Lock lk(c->mu);
  *out = c->stats;
  return VTE_OK;
}

int vte_stats_read(vte_ctx* c, vte_op_record* dst, int cap, int* n_out) {
  if (!c || !dst || cap < 0 || !n_out) { set_error("stats_read: bad argument"); return VTE_EINVAL; }
  Lock lk(c->mu);
  const size_t n = std::min<size_t>(static_cast<size_t>(cap), c->ring_count);
  const size_t first = c->ring_count - n;
  for (size_t i = 0; i < n; ++i) dst[i] = c->ring[(c->ring_head + first + i) % c->ring.size()];
  *n_out = static_cast<int>(n);
  return VTE_OK;
}

int vte_stats_reset(vte_ctx* c) {
  if (!c) { set_error("null ctx"); return VTE_EINVAL; }
  Lock lk(c->mu);
  std::memset(&c->stats, 0, sizeof c->stats);
  c->ring_head = c->ring_count = 0;
  return VTE_OK;
}

// ---- fake backend hooks ------------------------------------------------------------------

static FakeBackend* fake_of(vte_ctx* c) {
  if (!c) { set_error("null ctx"); return nullptr; }
  if (!c->backend->is_fake()) { set_error("only valid with the fake backend"); return nullptr; }
  return static_cast<FakeBackend*>(c->backend);
}

int vte_fake_complete(vte_ctx* c, vte_token t) {
  FakeBackend* fb = fake_of(c);
  if (!fb) return c ? VTE_ESTATE : VTE_EINVAL;
  Lock lk(c->mu);
  if (!fb->complete(t)) { set_error("fake_complete: token is not in flight"); return VTE_EINVAL; }
  bump(c);
  return VTE_OK;
}

int vte_fake_complete_error(vte_ctx* c, vte_token t) {
  FakeBackend* fb = fake_of(c);
  if (!fb) return c ? VTE_ESTATE : VTE_EINVAL;
  Lock lk(c->mu);
  if (!fb->complete(t, true)) { set_error("fake_complete_error: token is not in flight"); return VTE_EINVAL; }
  bump(c);
  return VTE_OK;
}

int vte_fake_set_autocomplete(vte_ctx* c, int on) {
  FakeBackend* fb = fake_of(c);
  if (!fb) return c ? VTE_ESTATE : VTE_EINVAL;
  Lock lk(c->mu);
  fb->autocomplete = on != 0;
  return VTE_OK;
}

int vte_fake_fail_next_submits(vte_ctx* c, int n) {
  FakeBackend* fb = fake_of(c);
  if (!fb) return c ? VTE_ESTATE : VTE_EINVAL;
  Lock lk(c->mu);
  fb->fail_next = n;
  return VTE_OK;
}

int vte_fake_log(vte_ctx* c, vte_fake_log_entry* dst, int cap, int* n_out) {
  FakeBackend* fb = fake_of(c);
  if (!fb) return c ? VTE_ESTATE : VTE_EINVAL;
  if (!dst || !n_out || cap < 0) { set_error("fake_log: bad argument"); return VTE_EINVAL; }
  Lock lk(c->mu);
  const int n = std::min<int>(cap, static_cast<int>(fb->log.size()));
  for (int i = 0; i < n; ++i) dst[i] = fb->log[i];
  *n_out = n;
  return VTE_OK;
}

int vte_dispatcher_quiesce(vte_ctx* c) {
  if (!c) { set_error("null ctx"); return VTE_EINVAL; }
  Lock lk(c->mu);
  bump(c);  // force one more full pass after everything the caller did
  const uint64_t want = c->change_seq;
  c->cv_done.wait(lk, [&] { return c->quiesced_seq >= want && c->quiesced_seq != ~0ull; });
  return VTE_OK;
}

int vte_now(vte_ctx* c, double* seconds) {
  if (!c || !seconds) { set_error("null argument"); return VTE_EINVAL; }
  *seconds = c->now();
  return VTE_OK;
}

}  // extern "C"

// Internal types of the late-binding runtime: descriptors, backends, ops,
// virtual streams and the context that ties them to the pCtx pool.
#pragma once
#include <atomic>
#include <chrono>
#include <condition_variable>
#include <cstdint>
#include <deque>
#include <map>
#include <mutex>
#include <string>
#include <thread>
#include <unordered_map>
#include <vector>

#include "../../include/vte.h"
#include "pool.h"

// Immutable launch descriptor D_k (Sec. 4.2).  Every field is written once by a
// constructor in desc.cpp; the dispatcher and the backends only ever see it
// through a pointer to const.
struct vte_desc {
  vte_ctx* ctx;
  int kernel;
  const void* entry;  // kernel entry (host stub address)
  uint32_t grid[3];
  uint32_t block[3];
  uint32_t lds_bytes;
  uint32_t arg_bytes;
  alignas(16) unsigned char args[192];
  uint64_t hash;
  uint64_t profile_key;
  uint64_t bytes;
  uint64_t flops;
};

namespace vte {

void set_error(const std::string& msg, int hip_code = 0);
uint64_t fnv1a(const void* data, size_t n, uint64_t h = 1469598103934665603ull);
uint64_t desc_hash(const vte_desc* d);

// What a pCtx needs from the device side.  HIP: CU-masked streams and events.
// FAKE: a log, with completions driven by the test.
class Backend {
 public:
  virtual ~Backend() {}
  virtual bool is_fake() const = 0;
  virtual int init(int device, int* cu_count) = 0;
  virtual int make_current() = 0;  // bind the device to the calling thread
  virtual int create_stream(const uint32_t* mask, int words, void** stream) = 0;
  virtual void destroy_stream(void* stream) = 0;
  // Submit the descriptor unchanged on `stream`, then record a completion.
  // `timed`: bracket the launch with timing events; elapsed() then gives its device time.
  // `record_now` false: no completion is recorded (*completion = nullptr); a later record() on
  // the same stream covers this launch too, since a stream completes in order.
  virtual int submit(const vte_desc* d, void* stream, int pctx, vte_token tok, bool timed, bool record_now,
                     void** completion) = 0;
  virtual int record(void* stream, void** completion) = 0;
  virtual double elapsed(void* completion) = 0;  // seconds, -1 if the launch was not timed
  // Device-clock time of a timed launch's begin (end = false) or end, in seconds since the backend's
  // init; -1 if the launch was not timed.
  virtual double device_time(void* completion, bool end) = 0;
  // Make later work on `stream` wait (on the device) for `completion`.
  virtual int wait_on(void* stream, void* completion, int completion_pctx) = 0;
  // 0: not finished yet; 1: finished; < 0: the device reported an error for it (VTE_EHIP, message and
  // HIP code left with set_error on the calling thread).  Never blocks.
  virtual int status(void* completion) = 0;
  virtual void release(void* completion) = 0;
  virtual int sync_stream(void* stream) = 0;
  // Seconds per launch of `d` on `stream`, device-timed.
  virtual int time_launches(const vte_desc* d, void* stream, int warmup, int reps, double* sec) = 0;
  virtual int prepare_kernel(const vte_desc* d) = 0;  // one-time per-kernel attributes
};

// Looks up, once per device, the device address of the library's static scratch array
// (the calling thread's current device must be `device`).
int static_scratch_setup(int device);

Backend* make_hip_backend();
Backend* make_fake_backend();

enum OpState { kWaiting = 0, kInflight = 1, kDone = 2 };

struct Op {
  vte_token tok = 0;
  const vte_desc* desc = nullptr;
  int vs = -1;
  int klass = 0;
  uint64_t age = 0;
  std::vector<vte_token> deps;
  int state = kWaiting;
  int pctx = -1;
  void* completion = nullptr;
  bool ready_marked = false;
  int submit_failures = 0;  // backend submissions of this op that failed so far
  double t_submit = 0, t_ready = 0, t_bound = 0, t_done = 0, gpu_seconds = -1, gpu_begin = -1, gpu_end = -1;
};

}  // namespace vte

struct vte_vstream {
  vte_ctx* ctx;
  int id;
  int klass;
  int pinned = -1;
  vte_token tail = 0;
  std::deque<vte::Op*> queue;  // submitted, not yet bound, in order
  std::vector<vte_token> waited_events;  // events waited on since the last submission: the next op depends on them
  int unfinished_bound = 0;    // bound (in flight) ops of this stream
  std::vector<uint64_t> recent_keys;  // profile keys of the last distinct descriptors submitted (newest first)
  // TPOT-First (Sec. 5): per-token deadline bookkeeping; tpot <= 0: none
  double tpot = 0;
  int ops_per_token = 0;
  int standing = -1;          // exclusive standing pCtx (reserved for this vstream), or -1
  int escalated = -1;         // wider pCtx reserved while a token is at risk, or -1
  uint64_t ops_submitted = 0; // ops submitted since the target was set
  std::deque<uint64_t> token_keys;  // profile keys of the last ops_per_token ops submitted: one token's chain
  uint64_t ops_done = 0;      // completed ops since the target was set
  double t_ref = -1;          // completion of the previous token (or submission into an idle stream)
  uint64_t escalations = 0;
  uint64_t escalated_token = 0;  // token index at which `escalated` was reserved
  uint64_t tokens_done = 0, deadline_misses = 0;
  double slowdown = 1.0;      // EWMA of observed token time / solo-profiled token time, in [1, 8]
  double t_idle = -1;         // when the stream last ran out of work
  bool at_risk = false;       // the current token is predicted to miss its deadline on the standing pCtx
  bool alive = true;
};

struct vte_ctx {
  vte_pool_cfg cfg;
  int device = 0;
  vte::Backend* backend = nullptr;
  vte::Pool pool;
  std::vector<void*> placeholder_streams;  // queues created only to keep the pipe rotation in step

  std::mutex mu;
  std::condition_variable cv_work;  // dispatcher sleeps here
  std::condition_variable cv_done;  // waiters sleep here
  std::thread dispatcher;
  bool stop = false;
  std::atomic<uint64_t> change_seq{0};  // bumped by every outside input (written with the lock held; the idle dispatcher polls it without)
  std::atomic<uint64_t> done_epoch{0};  // bumped with every cv_done notification: what a polling waiter watches without the lock
  uint64_t quiesced_seq = ~0ull;

  vte_token next_token = 1;
  uint64_t next_age = 0;
  std::unordered_map<vte_token, vte::Op*> live;  // not yet done
  std::vector<vte::Op*> inflight;                // in bind order
  // Working storage of the dispatcher thread (poll_completions, dispatch_round): kept between rounds so
  // that the dispatch path makes no heap allocation of its own per launch.  Dispatcher thread only, lock held.
  struct Scratch {
    std::vector<int> frontier, first_bad, rcs, qi, eligible;
    std::vector<char> blocked, tried;
    std::vector<vte::Op*> keep, done, ready_ops;
    std::vector<vte_ready_op> ready, q;
    std::vector<vte_pctx_info> infos;
  } scratch;
  unsigned timing_seen[32] = {};                 // launches of each kernel id that device_timing_mask selected so far
  std::vector<vte::Op*> lazy_tail;               // per pCtx: newest in-flight op without a completion record
  std::vector<vte_vstream*> vstreams;
  std::vector<vte_desc*> descs;
  int inflight_by_class[2] = {0, 0};
  std::vector<vte_token> awaited;  // tokens callers are blocked on (one entry per caller)
  int waiters_all = 0;             // callers blocked in a wait for everything submitted so far

  vte_policy_vtbl policy{};
  void* policy_user = nullptr;
  bool custom_policy = false;
  int builtin = VTE_POLICY_WIDEST;
  double slack = 0.1;
  int keep_free = 0;

  std::map<std::pair<uint64_t, int>, double> profiles;

  // Failures observed by the dispatcher (a completion that reports a device error, a submission
  // that keeps failing): the token is retired as failed, the error is kept here and handed to
  // whoever waits for the token, its vstream or the device, on that caller's thread.
  struct Failure { int rc; int hip; std::string msg; };
  std::map<vte_token, Failure> failed;
  bool failure_unreported = false;   // a failure no vte_device_sync has returned yet
  vte_token first_unreported = 0;
  std::vector<int> record_failures;  // per pCtx: consecutive completion records that could not be made

  vte_stats_t stats{};
  std::vector<vte_op_record> ring;
  size_t ring_head = 0, ring_count = 0;

  // fake backend state lives in the backend; log mirrored here for the API
  std::chrono::steady_clock::time_point t0;
  double now() const {
    return std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
  }
};

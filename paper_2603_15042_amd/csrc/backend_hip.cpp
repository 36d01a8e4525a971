// HIP backend: a pCtx is a stream created with a CU mask; a completion is an
// event recorded right after the launch (Sec. 3.4: CU-masked queues are the AMD
// primitive; Sec. 6: events polled in batches).
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "runtime.h"

namespace vte {
namespace {

#define VTE_HIP(call)                                                        \
  do {                                                                       \
    hipError_t e_ = (call);                                                  \
    if (e_ != hipSuccess) {                                                  \
      set_error(std::string(#call) + ": " + hipGetErrorString(e_), (int)e_); \
      return VTE_EHIP;                                                       \
    }                                                                        \
  } while (0)

// With VTE_TRACE_SLOW_CALLS=<microseconds> in the environment, any HIP call made on
// the dispatch path that takes longer is reported on stderr.
struct SlowCall {
  const char* what;
  std::chrono::steady_clock::time_point t0;
  static double limit_us() {
    static const double v = [] { const char* e = getenv("VTE_TRACE_SLOW_CALLS"); return e ? atof(e) : 0.0; }();
    return v;
  }
  explicit SlowCall(const char* w) : what(w) { if (limit_us() > 0) t0 = std::chrono::steady_clock::now(); }
  ~SlowCall() {
    if (limit_us() <= 0) return;
    const double us = std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - t0).count();
    if (us > limit_us()) fprintf(stderr, "[vte] %s took %.1f us\n", what, us);
  }
};

class HipBackend : public Backend {
 public:
  ~HipBackend() override {
    for (hipEvent_t e : free_events_) (void)hipEventDestroy(e);
    for (hipEvent_t e : free_timing_events_) (void)hipEventDestroy(e);
    if (ref_) (void)hipEventDestroy(ref_);
  }
  bool is_fake() const override { return false; }
  int init(int device, int* cu_count) override {
    device_ = device;
    int n = 0;
    VTE_HIP(hipGetDeviceCount(&n));
    if (device < 0 || device >= n) { set_error("no such device"); return VTE_EINVAL; }
    VTE_HIP(hipSetDevice(device));
    hipDeviceProp_t prop;
    VTE_HIP(hipGetDeviceProperties(&prop, device));
    if (cu_count && *cu_count <= 0) *cu_count = prop.multiProcessorCount;
    max_lds_ = static_cast<uint32_t>(prop.sharedMemPerBlock);
    // origin of the device clock that device_time() reports against
    VTE_HIP(hipEventCreate(&ref_));
    VTE_HIP(hipEventRecord(ref_, nullptr));
    VTE_HIP(hipEventSynchronize(ref_));
    return VTE_OK;
  }
  int make_current() override { VTE_HIP(hipSetDevice(device_)); return VTE_OK; }
  int create_stream(const uint32_t* mask, int words, void** stream) override {
    hipStream_t s;
    VTE_HIP(hipExtStreamCreateWithCUMask(&s, static_cast<uint32_t>(words), mask));
    *stream = s;
    return VTE_OK;
  }
  void destroy_stream(void* stream) override { (void)hipStreamDestroy(static_cast<hipStream_t>(stream)); }

  // A completion is an event recorded behind the launch; a timed launch carries a
  // start and a done event itself, both with timing enabled.
  struct Completion {
    hipEvent_t done = nullptr;
    hipEvent_t start = nullptr;  // timed launches only
  };
  int get_event(bool timing, hipEvent_t* ev) {
    std::vector<hipEvent_t>& pool = timing ? free_timing_events_ : free_events_;
    if (!pool.empty()) { *ev = pool.back(); pool.pop_back(); return VTE_OK; }
    VTE_HIP(hipEventCreateWithFlags(ev, timing ? hipEventDefault : hipEventDisableTiming));
    return VTE_OK;
  }
  void put_event(bool timing, hipEvent_t ev) { (timing ? free_timing_events_ : free_events_).push_back(ev); }

  int submit(const vte_desc* d, void* stream, int, vte_token, bool timed, bool record_now,
             void** completion) override {
    hipStream_t s = static_cast<hipStream_t>(stream);
    *completion = nullptr;
    if (!timed && !record_now) return launch(d, s);
    Completion* c = new Completion;
    int rc = get_event(timed, &c->done);
    if (rc == VTE_OK && timed) rc = get_event(true, &c->start);
    auto fail = [&](int code) {
      if (c->done) put_event(timed, c->done);
      if (c->start) put_event(true, c->start);
      delete c;
      return code;
    };
    if (rc != VTE_OK) return fail(rc);
    // The events ride on the kernel's own dispatch: a timed launch takes its begin and
    // end timestamps from it, and no marker is queued in front of or behind the kernel
    // (a recorded event costs the stream about 5 us of idle time).
    void* params[1] = {const_cast<unsigned char*>(d->args)};
    SlowCall sc("hipExtLaunchKernel");
    hipError_t e = hipExtLaunchKernel(d->entry, dim3(d->grid[0], d->grid[1], d->grid[2]),
                                      dim3(d->block[0], d->block[1], d->block[2]), params, d->lds_bytes, s,
                                      c->start, c->done, 0);
    if (e != hipSuccess) { set_error(std::string("hipExtLaunchKernel: ") + hipGetErrorString(e), (int)e); return fail(VTE_EHIP); }
    *completion = c;
    return VTE_OK;
  }
  int record(void* stream, void** completion) override {
    Completion* c = new Completion;
    int rc = get_event(false, &c->done);
    if (rc != VTE_OK) { delete c; return rc; }
    SlowCall sc("hipEventRecord");
    hipError_t e = hipEventRecord(c->done, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) {
      put_event(false, c->done);
      delete c;
      set_error(std::string("hipEventRecord: ") + hipGetErrorString(e), (int)e);
      return VTE_EHIP;
    }
    *completion = c;
    return VTE_OK;
  }
  double elapsed(void* completion) override {
    Completion* c = static_cast<Completion*>(completion);
    if (!c->start) return -1.0;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, c->start, c->done) != hipSuccess) return -1.0;
    return static_cast<double>(ms) * 1e-3;
  }
  double device_time(void* completion, bool end) override {
    Completion* c = static_cast<Completion*>(completion);
    if (!c->start || !ref_) return -1.0;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, ref_, end ? c->done : c->start) != hipSuccess) return -1.0;
    return static_cast<double>(ms) * 1e-3;
  }
  int wait_on(void* stream, void* completion, int) override {
    VTE_HIP(hipStreamWaitEvent(static_cast<hipStream_t>(stream), static_cast<Completion*>(completion)->done, 0));
    return VTE_OK;
  }
  int status(void* completion) override {
    SlowCall sc("hipEventQuery");
    const hipError_t e = hipEventQuery(static_cast<Completion*>(completion)->done);
    if (e == hipSuccess) return 1;
    if (e == hipErrorNotReady) return 0;
    // a launch failure or a fault behind this event: the work will not finish, and says why
    set_error(std::string("hipEventQuery: ") + hipGetErrorString(e), (int)e);
    return VTE_EHIP;
  }
  void release(void* completion) override {
    Completion* c = static_cast<Completion*>(completion);
    const bool timed = c->start != nullptr;
    put_event(timed, c->done);
    if (c->start) put_event(true, c->start);
    delete c;
  }
  int sync_stream(void* stream) override { VTE_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream))); return VTE_OK; }

  int time_launches(const vte_desc* d, void* stream, int warmup, int reps, double* sec) override {
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipEvent_t a, b;
    VTE_HIP(hipEventCreate(&a));
    VTE_HIP(hipEventCreate(&b));
    int rc = VTE_OK;
    for (int i = 0; i < warmup && rc == VTE_OK; ++i) rc = launch(d, s);
    if (rc == VTE_OK) {
      VTE_HIP(hipEventRecord(a, s));
      for (int i = 0; i < reps && rc == VTE_OK; ++i) rc = launch(d, s);
      VTE_HIP(hipEventRecord(b, s));
      VTE_HIP(hipStreamSynchronize(s));
      float ms = 0.f;
      VTE_HIP(hipEventElapsedTime(&ms, a, b));
      *sec = static_cast<double>(ms) * 1e-3 / (reps > 0 ? reps : 1);
    }
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    return rc;
  }

  int prepare_kernel(const vte_desc* d) override {
    if (d->lds_bytes > max_lds_) { set_error("descriptor needs more LDS than a workgroup may have"); return VTE_EINCOMPAT; }
    if (d->lds_bytes > 48 * 1024) {
      VTE_HIP(hipFuncSetAttribute(d->entry, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(d->lds_bytes)));
    }
    return VTE_OK;
  }

 private:
  // The one place a kernel is launched: entry, dimensions and the argument bytes
  // come from the descriptor as they are.
  int launch(const vte_desc* d, hipStream_t s) {
    void* params[1] = {const_cast<unsigned char*>(d->args)};
    SlowCall sc("hipLaunchKernel");
    hipError_t e = hipLaunchKernel(d->entry, dim3(d->grid[0], d->grid[1], d->grid[2]),
                                   dim3(d->block[0], d->block[1], d->block[2]), params, d->lds_bytes, s);
    if (e != hipSuccess) {
      set_error(std::string("hipLaunchKernel: ") + hipGetErrorString(e), (int)e);
      return VTE_EHIP;
    }
    return VTE_OK;
  }
  int device_ = 0;
  hipEvent_t ref_ = nullptr;
  uint32_t max_lds_ = 65536;
  std::vector<hipEvent_t> free_events_;
  std::vector<hipEvent_t> free_timing_events_;
};

}  // namespace

Backend* make_hip_backend() { return new HipBackend(); }

}  // namespace vte

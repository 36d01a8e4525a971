// Fake backend: no device.  A submission is appended to a log and stays in
// flight until the test completes it (or at once in autocomplete mode); the next
// n submissions can be made to fail.  Lets every rule of the dispatcher be
// exercised on a CPU.
#pragma once
#include <set>
#include <vector>
#include "runtime.h"

namespace vte {
class FakeBackend : public Backend {
 public:
  struct Completion { vte_token tok; bool done; bool error = false; };
  bool is_fake() const override { return true; }
  int init(int, int* cu_count) override { if (cu_count && *cu_count <= 0) *cu_count = 256; return VTE_OK; }
  int make_current() override { return VTE_OK; }
  int create_stream(const uint32_t*, int, void** stream) override {
    *stream = reinterpret_cast<void*>(static_cast<uintptr_t>(++streams_)); return VTE_OK;
  }
  void destroy_stream(void*) override {}
  int submit(const vte_desc* d, void* stream, int pctx, vte_token tok, bool timed, bool record_now,
             void** completion) override;  // always records: tests complete launches one by one
  int record(void*, void**) override { return VTE_ESTATE; }
  double elapsed(void*) override { return -1.0; }
  double device_time(void*, bool) override { return -1.0; }
  int wait_on(void* stream, void* completion, int completion_pctx) override;
  int status(void* c) override {
    const Completion* k = static_cast<Completion*>(c);
    if (!k->done) return 0;
    if (!k->error) return 1;
    set_error("fake backend: injected device error", 719);
    return VTE_EHIP;
  }
  void release(void* c) override { delete static_cast<Completion*>(c); }
  int sync_stream(void*) override { return VTE_OK; }
  int time_launches(const vte_desc*, void*, int, int, double* sec) override { *sec = 0; return VTE_ESTATE; }
  int prepare_kernel(const vte_desc*) override { return VTE_OK; }

  // driven by the vte_fake_* calls (runtime lock held)
  bool complete(vte_token tok, bool with_error = false);
  bool autocomplete = false;
  int fail_next = 0;
  std::vector<vte_fake_log_entry> log;
 private:
  int streams_ = 0;
  int pending_wait_ = -1;
  std::vector<Completion*> open_;
};
}  // namespace vte

#include "backend_fake.h"

namespace vte {

int FakeBackend::wait_on(void*, void*, int completion_pctx) {
  pending_wait_ = completion_pctx;  // attached to the next submission's log entry
  return VTE_OK;
}

int FakeBackend::submit(const vte_desc* d, void*, int pctx, vte_token tok, bool, bool, void** completion) {
  if (fail_next > 0) {
    --fail_next;
    pending_wait_ = -1;
    set_error("fake backend: injected submission failure");
    return VTE_EHIP;
  }
  vte_fake_log_entry e;
  e.token = tok;
  e.pctx = pctx;
  e.desc_hash = desc_hash(d);  // recomputed from the bytes the backend sees
  e.waited_on_pctx = pending_wait_;
  pending_wait_ = -1;
  log.push_back(e);
  auto* c = new Completion{tok, autocomplete};
  if (!autocomplete) open_.push_back(c);
  *completion = c;
  return VTE_OK;
}

bool FakeBackend::complete(vte_token tok, bool with_error) {
  for (size_t i = 0; i < open_.size(); ++i) {
    if (open_[i]->tok == tok) {
      open_[i]->done = true;
      open_[i]->error = with_error;
      open_.erase(open_.begin() + i);
      return true;
    }
  }
  return false;
}

Backend* make_fake_backend() { return new FakeBackend(); }

}  // namespace vte

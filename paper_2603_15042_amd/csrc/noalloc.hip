// The LM head + greedy token as one call that allocates nothing: for callers that may not
// allocate device memory where they stand (a stream under graph capture, a tight serving loop,
// a harness that forbids it).  The per-workgroup (value, index) candidates that the ordinary
// descriptor keeps in a caller-supplied workspace live here in a fixed array inside the
// library's device image; the kernels, their default plan and therefore every output bit are
// those of vte_desc_lmhead_argmax + vte_desc_argmax_finish.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>

#include "kargs.h"
#include "runtime.h"

extern "C" const void* vte_fill_entry();

namespace vte {
int fill_lmhead_pair(const void* W, const void* H, int32_t* tok, float* logits_or_null, void* ws, int B, int V, int K,
                     vte_desc* lm, vte_desc* fin, size_t* ticket_words, size_t* ws_words);
}

namespace {

constexpr size_t kScratchBytes = 1u << 20;  // 1 MiB per device, held until the process ends
constexpr int kMaxDevices = 64;

// On the host this name is only a handle for hipGetSymbolAddress; the device address it stands
// for is looked up once per device and kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

std::mutex g_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// The address of the array on `device`, which must be the calling thread's current device.
int scratch_on(int device, void** out) {
  if (device < 0 || device >= kMaxDevices) { vte::set_error("static scratch: device index out of range"); return VTE_EINVAL; }
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_scratch_ptr[device]) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      vte::set_error(std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(e), static_cast<int>(e));
      return VTE_EHIP;
    }
    g_scratch_ptr[device] = p;
  }
  *out = g_scratch_ptr[device];
  return VTE_OK;
}

int launch(const vte_desc& d, hipStream_t s, const char* what) {
  void* params[1] = {const_cast<unsigned char*>(d.args)};
  hipError_t e = hipLaunchKernel(d.entry, dim3(d.grid[0], d.grid[1], d.grid[2]), dim3(d.block[0], d.block[1], d.block[2]),
                                 params, d.lds_bytes, s);
  if (e != hipSuccess) {
    vte::set_error(std::string(what) + ": " + hipGetErrorString(e), static_cast<int>(e));
    return VTE_EHIP;
  }
  return VTE_OK;
}

}  // namespace

namespace vte {
// Called by vte_init with its device current, so the lookup is done before any launch path runs.
int static_scratch_setup(int device) {
  void* p = nullptr;
  return scratch_on(device, &p);
}
}  // namespace vte

extern "C" {

int vte_static_scratch_bytes(size_t* bytes) {
  if (!bytes) { vte::set_error("null bytes"); return VTE_EINVAL; }
  *bytes = kScratchBytes;
  return VTE_OK;
}

int vte_lmhead_argmax_static(void* hip_stream, const void* W, const void* H, int32_t* tok, float* logits_or_null,
                             int B, int V, int K) {
  int device = -1;
  hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) { vte::set_error(std::string("hipGetDevice: ") + hipGetErrorString(e), static_cast<int>(e)); return VTE_EHIP; }
  void* ws = nullptr;
  int rc = scratch_on(device, &ws);
  if (rc != VTE_OK) return rc;
  vte_desc lm, fin;
  size_t ticket_words = 0, ws_words = 0;
  rc = vte::fill_lmhead_pair(W, H, tok, logits_or_null, ws, B, V, K, &lm, &fin, &ticket_words, &ws_words);
  if (rc != VTE_OK) return rc;
  if (ws_words * 4 > kScratchBytes) {
    char msg[160];
    snprintf(msg, sizeof msg, "lmhead_argmax_static: this shape needs %zu bytes of scratch, the static array holds %zu",
             ws_words * 4, kScratchBytes);
    vte::set_error(msg);
    return VTE_EINVAL;
  }
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  // The array keeps the previous call's contents.  The candidates are rewritten in full by every
  // launch; the ticket words in front of them must be zero, so they are cleared by a fill
  // launch on the same stream (a kernel, not a memset node: safe to record into a graph).
  vte_desc fill;
  std::memset(&fill, 0, sizeof fill);
  FillArgs fa{static_cast<unsigned char*>(ws), (ticket_words * 4 + 15) & ~static_cast<size_t>(15), 0u};
  fill.entry = vte_fill_entry();
  fill.grid[0] = static_cast<uint32_t>((fa.bytes + 16383) / 16384);
  fill.grid[1] = fill.grid[2] = 1;
  fill.block[0] = 256; fill.block[1] = fill.block[2] = 1;
  fill.arg_bytes = sizeof fa;
  std::memcpy(fill.args, &fa, sizeof fa);
  if ((rc = launch(fill, s, "lmhead_argmax_static: fill launch")) != VTE_OK) return rc;
  if ((rc = launch(lm, s, "lmhead_argmax_static: LM-head launch")) != VTE_OK) return rc;
  return launch(fin, s, "lmhead_argmax_static: finish launch");
}

}  // extern "C"

// Embedding gather: H[b,:] = E[tok[b],:], 128-bit copies.  Grid and block depend
// on (B, K) only.
#include "dev_util.h"
#include "kargs.h"

__global__ __launch_bounds__(256) void gather_kernel(const GatherArgs a) {
  const int b = blockIdx.y;
  const int c = blockIdx.x * 256 + threadIdx.x;  // 8-element chunk within the row
  if (b >= a.B || c * 8 >= a.K) return;
  int t = a.tok[b];
  t = t < 0 ? 0 : (t >= a.V ? a.V - 1 : t);
  st16(a.H + static_cast<size_t>(b) * a.K + c * 8, ld16(a.E + static_cast<size_t>(t) * a.K + c * 8));
}

extern "C" const void* vte_gather_entry() { return (const void*)gather_kernel; }

// Matrix-core GEMV, one column tile (batch <= 16): the instantiations (see gemv_mfma_kernel.h).
#include "gemv_mfma_kernel.h"
#define VTE_MFMA_CT 1

#define VTE_MFMA_EPI(NBK, G, NB, MAXW, AF, OC)                                                       \
  {                                                                                                 \
    if (epi == 0) return (const void*)gemv_mfma_kernel<NBK, G, NB, MAXW, AF, OC, EPI_NONE, VTE_MFMA_CT>;         \
    if (epi == 1) return (const void*)gemv_mfma_kernel<NBK, G, NB, MAXW, AF, OC, EPI_SILU, VTE_MFMA_CT>;         \
    if (epi == 2) return (const void*)gemv_mfma_kernel<NBK, G, NB, MAXW, AF, OC, EPI_ARGMAX, VTE_MFMA_CT>;       \
  }
#define VTE_MFMA_CASE(NBK, G, NB, MAXW)                                  \
  if (nbk == NBK && g == G && nb == NB && maxw == MAXW) {                \
    if (allfull && onechunk) VTE_MFMA_EPI(NBK, G, NB, MAXW, true, true)  \
    if (allfull && !onechunk) VTE_MFMA_EPI(NBK, G, NB, MAXW, true, false) \
    if (!allfull) VTE_MFMA_EPI(NBK, G, NB, MAXW, false, false)           \
  }

// nbk = 128-element blocks per K chunk, g = row tiles per workgroup, nb = blocks the
// loads run ahead, maxw = most waves per workgroup, allfull = K / S is a multiple of
// the chunk, onechunk = no more chunks than waves; nullptr when the combination is not built.
extern "C" const void* vte_gemv_entry_mfma(int nbk, int g, int nb, int maxw, int allfull, int onechunk, int epi) {
  VTE_MFMA_CASE(4, 1, 2, 8)
  VTE_MFMA_CASE(4, 1, 4, 8)
  VTE_MFMA_CASE(4, 2, 2, 8)
  VTE_MFMA_CASE(4, 2, 4, 8)
  VTE_MFMA_CASE(4, 4, 2, 8)
  VTE_MFMA_CASE(4, 4, 4, 8)
  VTE_MFMA_CASE(4, 8, 4, 8)
  VTE_MFMA_CASE(4, 8, 2, 8)
  VTE_MFMA_CASE(4, 8, 4, 4)
  VTE_MFMA_CASE(4, 2, 2, 4)
  VTE_MFMA_CASE(4, 4, 2, 4)
  VTE_MFMA_CASE(4, 1, 4, 4)
  VTE_MFMA_CASE(4, 2, 4, 4)
  VTE_MFMA_CASE(4, 4, 4, 4)
  VTE_MFMA_CASE(8, 1, 2, 4)  // 1024-element chunks: K = 4096 is one chunk for each of four waves
  VTE_MFMA_CASE(8, 2, 2, 4)
  return nullptr;
}

// The same kernel with the decode loop's step boundary in its prologue (K = 4096, batch <= 16):
// g = row tiles per workgroup (1 or 2); nullptr otherwise.
extern "C" const void* vte_gemv_entry_mfma_norm(int g) {
  if (g == 1) return (const void*)gemv_mfma_kernel<8, 1, 2, 4, true, true, EPI_NONE, 1, true>;
  if (g == 2) return (const void*)gemv_mfma_kernel<8, 2, 2, 4, true, true, EPI_NONE, 1, true>;
  return nullptr;
}

#ifdef VTE_TRACE_STAMPS
// Trace build only: copies the stamp table of this file's kernels (most recent launch) to the host.
extern "C" int vte_trace_stamps_read(unsigned long long* host, size_t count) {
  if (count > static_cast<size_t>(kTraceWorkgroups) * kTraceWaves * kTracePoints) return -1;
  return static_cast<int>(hipMemcpyFromSymbol(host, HIP_SYMBOL(vte_trace_stamps), count * sizeof(unsigned long long)));
}
#endif

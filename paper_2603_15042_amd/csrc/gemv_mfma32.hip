// Matrix-core GEMV, two column tiles (batch 17 to 32): the instantiations (see gemv_mfma_kernel.h).
#include "gemv_mfma_kernel.h"
#define VTE_MFMA_CT 2

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
// Two column tiles (batch 17 to 32).  X for 32 batch rows and a 512-element chunk takes 128
// registers of a wave: with four waves a wave may have 512; with eight (one chunk per wave at
// K = 4096, so X is loaded once per workgroup) the rest has to fit into the other 128.
extern "C" const void* vte_gemv_entry_mfma32(int nbk, int g, int nb, int maxw, int allfull, int onechunk, int epi) {
  VTE_MFMA_CASE(4, 1, 4, 4)
  VTE_MFMA_CASE(4, 2, 2, 4)
  VTE_MFMA_CASE(4, 2, 4, 4)
  VTE_MFMA_CASE(4, 4, 2, 4)
  VTE_MFMA_CASE(4, 4, 4, 4)
  VTE_MFMA_CASE(4, 1, 2, 8)
  VTE_MFMA_CASE(4, 2, 2, 8)
  return nullptr;
}

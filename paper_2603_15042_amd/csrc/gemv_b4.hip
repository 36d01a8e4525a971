// GEMV kernels for a batch tile of 4 rows (see gemv_kernels.h).
#include "gemv_kernels.h"
#define VTE_GEMV_CASES(BT) \
  VTE_GEMV_CASE(4, 8, 2, 1, 8) \
  VTE_GEMV_CASE(4, 4, 4, 1, 8) \
  VTE_GEMV_CASE(4, 4, 4, 0, 8) \
  VTE_GEMV_CASE(4, 16, 1, 1, 8) \
  VTE_GEMV_CASE(4, 8, 1, 1, 16) \
  VTE_GEMV_CASE(4, 4, 2, 1, 16)
VTE_GEMV_ENTRY_FOR_BT(4)

// GEMV kernels for a batch tile of 1 rows (see gemv_kernels.h).
#include "gemv_kernels.h"
#define VTE_GEMV_CASES(BT) \
  VTE_GEMV_CASE(1, 16, 1, 1, 8) \
  VTE_GEMV_CASE(1, 16, 1, 1, 16) \
  VTE_GEMV_CASE(1, 16, 2, 0, 8)
VTE_GEMV_ENTRY_FOR_BT(1)

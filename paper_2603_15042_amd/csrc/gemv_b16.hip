// GEMV kernels for a batch tile of 16 rows (see gemv_kernels.h).
#include "gemv_kernels.h"
#define VTE_GEMV_CASES(BT) \
  VTE_GEMV_CASE(16, 4, 2, 1, 8) \
  VTE_GEMV_CASE(16, 4, 1, 1, 8) \
  VTE_GEMV_CASE(16, 2, 2, 1, 8) \
  VTE_GEMV_CASE(16, 2, 2, 1, 16) \
  VTE_GEMV_CASE(16, 4, 1, 1, 16) \
  VTE_GEMV_CASE(16, 2, 1, 1, 16)
VTE_GEMV_ENTRY_FOR_BT(16)

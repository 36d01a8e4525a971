// GEMV kernels for a batch tile of 8 rows (see gemv_kernels.h).
#include "gemv_kernels.h"
#define VTE_GEMV_CASES(BT) \
  VTE_GEMV_CASE(8, 2, 4, 0) \
  VTE_GEMV_CASE(8, 2, 4, 1) \
  VTE_GEMV_CASE(8, 2, 4, 2) \
  VTE_GEMV_CASE(8, 2, 8, 0) \
  VTE_GEMV_CASE(8, 2, 8, 1) \
  VTE_GEMV_CASE(8, 2, 8, 2) \
  VTE_GEMV_CASE(8, 2, 16, 0) \
  VTE_GEMV_CASE(8, 2, 16, 1) \
  VTE_GEMV_CASE(8, 2, 16, 2) \
  VTE_GEMV_CASE(8, 4, 4, 0) \
  VTE_GEMV_CASE(8, 4, 4, 1) \
  VTE_GEMV_CASE(8, 4, 4, 2) \
  VTE_GEMV_CASE(8, 4, 8, 0) \
  VTE_GEMV_CASE(8, 4, 8, 1) \
  VTE_GEMV_CASE(8, 4, 8, 2) \
  VTE_GEMV_CASE(8, 4, 16, 0) \
  VTE_GEMV_CASE(8, 4, 16, 1) \
  VTE_GEMV_CASE(8, 4, 16, 2) \
  VTE_GEMV_CASE(8, 8, 4, 0) \
  VTE_GEMV_CASE(8, 8, 4, 1) \
  VTE_GEMV_CASE(8, 8, 4, 2) \
  VTE_GEMV_CASE(8, 8, 8, 0) \
  VTE_GEMV_CASE(8, 8, 8, 1) \
  VTE_GEMV_CASE(8, 8, 8, 2) \
  VTE_GEMV_CASE(8, 8, 16, 0) \
  VTE_GEMV_CASE(8, 8, 16, 1) \
  VTE_GEMV_CASE(8, 8, 16, 2)
VTE_GEMV_ENTRY_FOR_BT(8)

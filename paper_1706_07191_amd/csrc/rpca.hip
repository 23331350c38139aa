// Robust PCA by inexact ALM (Alg. 3): elementwise kernels and the fixed-iteration loop.
#include "common.h"

extern "C" int brsvd_rpca_ialm(brsvd_handle, const float*, const float*, int32_t, float, float, float, double,
                               float*, float*, float*, double*, brsvd_stats*) {
  return BRSVD_ERR_ARG;   // filled in by a later change
}

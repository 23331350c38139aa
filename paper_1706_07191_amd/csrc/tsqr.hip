// TSQR route of the panel orthonormaliser (placeholder until the Householder tree lands).
#include "common.h"

namespace brsvd {

uint64_t tsqr_work_bytes(int64_t, int) { return 0; }

int tsqr_panel(float*, float*, int64_t, int, int, OrthWork&, double*, float**, hipStream_t) {
  return BRSVD_ERR_ORTH_BREAKDOWN;
}

}  // namespace brsvd

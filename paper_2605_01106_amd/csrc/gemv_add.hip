// Instantiations of the skinny-GEMM kernel for one epilogue (see gemv.hip).
#include "gemv_kernel.h"

namespace hh {
hipError_t gemv_dispatch_add(const GemvArgs& a, int m0, const GemvPlan& p, hipStream_t s) {
  return a.bf16 ? gemv_dispatch<1, EPI_ADD>(a, m0, p, s) : gemv_dispatch<0, EPI_ADD>(a, m0, p, s);
}
}  // namespace hh

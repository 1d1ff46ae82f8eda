// bf16 GEMM instantiations contracting over the token dimension (both operands [K x *]):
// Gy^T T of Eq. (2) (split-K partials or direct store) and the exact weight gradient.
#include "gemm_bf16_launch.hip.h"
namespace mecefo {
hipError_t launch_gemm_bf16_tn(GemmLaunch& g, hipStream_t s) {
  switch (g.epi) {
    case EPI_STORE: return run_bf16_auto<false, false, EPI_STORE>(g, s);
    case EPI_SPLIT_F32: return run_bf16_auto<false, false, EPI_SPLIT_F32>(g, s);
    case EPI_GRAD: return run_bf16_auto<false, false, EPI_GRAD>(g, s);
    default: return hipErrorInvalidValue;
  }
}
hipError_t prepare_gemm_bf16_tn() {
  hipError_t e = hipSuccess;
  if (e == hipSuccess) e = prepare_bf16<false, false, EPI_STORE>();
  if (e == hipSuccess) e = prepare_bf16<false, false, EPI_SPLIT_F32>();
  if (e == hipSuccess) e = prepare_bf16<false, false, EPI_GRAD>();
  return e;
}
}  // namespace mecefo

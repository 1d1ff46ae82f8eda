// bf16 GEMM instantiations with A K-contiguous and B given as [K x N]: the exact Dgrad
// products (dY Wd, dG Wg + dZ Wu) and the projection step X P of Eq. (2).
#include "gemm_bf16_launch.hip.h"
namespace mecefo {
hipError_t launch_gemm_bf16_nn(GemmLaunch& g, hipStream_t s) {
  switch (g.epi) {
    case EPI_STORE: return run_bf16_auto<true, false, EPI_STORE>(g, s);
    case EPI_GRAD: return run_bf16_auto<true, false, EPI_GRAD>(g, s);
    case EPI_SPLIT_F32: return run_bf16_auto<true, false, EPI_SPLIT_F32>(g, s);
    default: return hipErrorInvalidValue;
  }
}
hipError_t prepare_gemm_bf16_nn() {
  hipError_t e = hipSuccess;
  if (e == hipSuccess) e = prepare_bf16<true, false, EPI_STORE>();
  if (e == hipSuccess) e = prepare_bf16<true, false, EPI_GRAD>();
  if (e == hipSuccess) e = prepare_bf16<true, false, EPI_SPLIT_F32>();
  return e;
}
}  // namespace mecefo

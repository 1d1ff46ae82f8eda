// bf16 GEMM instantiations with both operands K-contiguous: FFN recompute (U Wg^T, U Wu^T
// with SwiGLU epilogues), the down projection, the expand step C P^T of Eq. (2), and the
// attention-score products Q K^T and dO V^T of the standard-mode backward.
#include "gemm_bf16_launch.hip.h"
namespace mecefo {
hipError_t launch_gemm_bf16_nt(GemmLaunch& g, hipStream_t s) {
  switch (g.epi) {
    case EPI_STORE: return run_bf16_auto<true, true, EPI_STORE>(g, s);
    case EPI_GRAD: return run_bf16_auto<true, true, EPI_GRAD>(g, s);
    case EPI_SPLIT_F32: return run_bf16_auto<true, true, EPI_SPLIT_F32>(g, s);
    case EPI_SWIGLU_FWD: return run_bf16_auto<true, true, EPI_SWIGLU_FWD>(g, s);
    case EPI_SWIGLU_BWD: return run_bf16_auto<true, true, EPI_SWIGLU_BWD>(g, s);
    case EPI_ATTN_P: return run_bf16_auto<true, true, EPI_ATTN_P>(g, s);
    case EPI_ATTN_DS: return run_bf16_auto<true, true, EPI_ATTN_DS>(g, s);
    default: return hipErrorInvalidValue;
  }
}
hipError_t prepare_gemm_bf16_nt() {
  hipError_t e = hipSuccess;
  if (e == hipSuccess) e = prepare_bf16<true, true, EPI_STORE>();
  if (e == hipSuccess) e = prepare_bf16<true, true, EPI_GRAD>();
  if (e == hipSuccess) e = prepare_bf16<true, true, EPI_SPLIT_F32>();
  if (e == hipSuccess) e = prepare_bf16<true, true, EPI_SWIGLU_FWD>();
  if (e == hipSuccess) e = prepare_bf16<true, true, EPI_SWIGLU_BWD>();
  if (e == hipSuccess) e = prepare_bf16<true, true, EPI_ATTN_P>();
  if (e == hipSuccess) e = prepare_bf16<true, true, EPI_ATTN_DS>();
  return e;
}
}  // namespace mecefo

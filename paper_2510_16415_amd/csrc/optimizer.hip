// Steps that follow the backward pass of a layer in Alg. 1: the gradient average of Eq. (1) over the
// ranks that contribute to a parameter group (here over gradient buffers that live on one GPU: the
// cross-rank exchange itself is not part of this library) and the AdamW update.  Both are HBM-bound
// elementwise kernels: 16-byte accesses, one pass over every operand.
#include <math.h>

#include "../../include/mecefo.h"
#include "mecefo_internal.h"

namespace mecefo {
namespace {

constexpr int kMaxRanks = 16;

struct RankPtrs { const void* g[kMaxRanks]; };

// out = (1 / count) * sum of the contributing buffers, summed in rank order.
template <typename T>
__global__ __launch_bounds__(256) void grad_average_kernel(RankPtrs in, int n_in, float inv_count,
                                                           T* __restrict__ out, int64_t n) {
  const int64_t i4 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i4 >= n) return;
  if (i4 + 4 <= n) {
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int r = 0; r < n_in; ++r) {
      const T* g = (const T*)in.g[r] + i4;
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[e] += (float)g[e];
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) out[i4 + e] = (T)(acc[e] * inv_count);
  } else {
    for (int64_t i = i4; i < n; ++i) {
      float acc = 0.f;
      for (int r = 0; r < n_in; ++r) acc += (float)((const T*)in.g[r])[i];
      out[i] = (T)(acc * inv_count);
    }
  }
}

// AdamW with decoupled weight decay; m, v fp32; W in its storage type; G fp32 or the storage type.
template <typename TW, typename TG>
__global__ __launch_bounds__(256) void adamw_kernel(TW* __restrict__ W, const TG* __restrict__ G,
                                                    float* __restrict__ M, float* __restrict__ V, int64_t n,
                                                    float lr, float beta1, float beta2, float eps, float decay,
                                                    float inv_bc1, float inv_bc2) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const float g = (float)G[i];
    const float m = beta1 * M[i] + (1.f - beta1) * g;
    const float v = beta2 * V[i] + (1.f - beta2) * g * g;
    M[i] = m;
    V[i] = v;
    const float w = (float)W[i];
    W[i] = (TW)(w * decay - lr * (m * inv_bc1) / (sqrtf(v * inv_bc2) + eps));
  }
}

inline unsigned grid_for(int64_t n) { int64_t g = (n + 255) / 256; return (unsigned)(g < 1 ? 1 : (g > 262144 ? 262144 : g)); }

}  // namespace
}  // namespace mecefo

using namespace mecefo;

extern "C" {

mecefo_status_t mecefo_grad_average(mecefo_dtype_t grad_dtype, const void* const* grads, const int32_t* contributes,
                                    int n_ranks, void* out, int64_t n_elems, void* hip_stream) {
  if (grad_dtype != MECEFO_F32 && grad_dtype != MECEFO_BF16) return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "grad_dtype must be MECEFO_F32 or MECEFO_BF16");
  if (!grads || !contributes || !out) return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "grads, contributes and out are required");
  if (n_ranks < 1 || n_ranks > kMaxRanks) return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "n_ranks must be in [1, %d]", kMaxRanks);
  if (n_elems < 0) return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "n_elems must be >= 0");
  RankPtrs in;
  int cnt = 0;
  for (int r = 0; r < n_ranks; ++r) {
    if (!contributes[r]) continue;
    if (!grads[r]) return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "gradient buffer of contributing rank %d is NULL", r);
    if ((uintptr_t)grads[r] % 16) return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "gradient buffers must be 16-byte aligned");
    in.g[cnt++] = grads[r];
  }
  if ((uintptr_t)out % 16) return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "out must be 16-byte aligned");
  for (int r = cnt; r < kMaxRanks; ++r) in.g[r] = nullptr;
  if (n_elems == 0) return MECEFO_OK;
  hipStream_t s = (hipStream_t)hip_stream;
  const float inv = cnt > 0 ? 1.0f / (float)cnt : 0.f;   // no contributing rank: zero gradient
  const unsigned grid = grid_for((n_elems + 3) / 4);
  if (grad_dtype == MECEFO_F32)
    hipLaunchKernelGGL(grad_average_kernel<float>, dim3(grid), dim3(256), 0, s, in, cnt, inv, (float*)out, n_elems);
  else
    hipLaunchKernelGGL(grad_average_kernel<__bf16>, dim3(grid), dim3(256), 0, s, in, cnt, inv, (__bf16*)out, n_elems);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return (mecefo_status_t)fail(MECEFO_ERR_LAUNCH, "grad_average: %s", hipGetErrorString(e));
  return MECEFO_OK;
}

mecefo_status_t mecefo_adamw_step(mecefo_dtype_t w_dtype, mecefo_dtype_t grad_dtype, void* W, const void* G,
                                  float* M, float* V, int64_t n_elems, int64_t step, float lr, float beta1,
                                  float beta2, float eps, float weight_decay, void* hip_stream) {
  if ((w_dtype != MECEFO_F32 && w_dtype != MECEFO_BF16) || (grad_dtype != MECEFO_F32 && grad_dtype != w_dtype))
    return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "w_dtype must be F32 or BF16, grad_dtype F32 or equal to w_dtype");
  if (!W || !G || !M || !V) return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "W, G, M and V are required");
  if (n_elems < 0 || step < 1) return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "n_elems >= 0 and step >= 1 required");
  if (!(beta1 >= 0.f && beta1 < 1.f && beta2 >= 0.f && beta2 < 1.f)) return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "betas must be in [0, 1)");
  if (n_elems == 0) return MECEFO_OK;
  const float inv_bc1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)step)));
  const float inv_bc2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)step)));
  const float decay = 1.0f - lr * weight_decay;
  hipStream_t s = (hipStream_t)hip_stream;
  const unsigned grid = grid_for(n_elems);
  if (w_dtype == MECEFO_F32)
    hipLaunchKernelGGL((adamw_kernel<float, float>), dim3(grid), dim3(256), 0, s, (float*)W, (const float*)G, M, V, n_elems, lr, beta1, beta2, eps, decay, inv_bc1, inv_bc2);
  else if (grad_dtype == MECEFO_F32)
    hipLaunchKernelGGL((adamw_kernel<__bf16, float>), dim3(grid), dim3(256), 0, s, (__bf16*)W, (const float*)G, M, V, n_elems, lr, beta1, beta2, eps, decay, inv_bc1, inv_bc2);
  else
    hipLaunchKernelGGL((adamw_kernel<__bf16, __bf16>), dim3(grid), dim3(256), 0, s, (__bf16*)W, (const __bf16*)G, M, V, n_elems, lr, beta1, beta2, eps, decay, inv_bc1, inv_bc2);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return (mecefo_status_t)fail(MECEFO_ERR_LAUNCH, "adamw_step: %s", hipGetErrorString(e));
  return MECEFO_OK;
}

}  // extern "C"

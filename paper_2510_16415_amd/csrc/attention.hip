// HBM-bound helpers of the standard-mode attention backward (Alg. 3, first branch): the rotary
// angle tables, the inverse rotation applied to dQ and dK, and the per-row dot product
// D = rowsum(dO * O) that the softmax backward subtracts.  The matrix products of the attention
// backward run in the GEMM core as batched products.
#include "mecefo_internal.h"

namespace mecefo {
namespace {

template <typename T, int VEC> struct alignas(sizeof(T) * VEC) Vec { T e[VEC]; };

// cos / sin of position * theta^(-2j/dh), j < dh/2, evaluated in fp64 and stored as fp32.
__global__ __launch_bounds__(256) void rope_table_kernel(float* __restrict__ cs, float* __restrict__ sn,
                                                         int seq, int half, double theta) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= seq * half) return;
  const int s = i / half, j = i - s * half;
  const double inv = pow(theta, -(double)j / (double)half);   // 2j / dh with dh = 2 * half
  const double ang = (double)s * inv;
  cs[i] = (float)cos(ang);
  sn[i] = (float)sin(ang);
}

// In-place inverse rotation of the pairs (x[j], x[j + dh/2]) of every head of a token-major
// [tokens x d] gradient: the transpose of the forward rotation by the position angle.
// One thread per VEC consecutive pairs.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void rope_bwd_kernel(T* __restrict__ X, int64_t ldx,
                                                       const float* __restrict__ cs,
                                                       const float* __restrict__ sn, int64_t tokens, int seq,
                                                       int heads, int half) {
  const int per_head = half / VEC;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t per_tok = (int64_t)heads * per_head;
  if (i >= tokens * per_tok) return;
  const int64_t t = i / per_tok;
  const int r = (int)(i - t * per_tok);
  const int h = r / per_head, j0 = (r - h * per_head) * VEC;
  const int s = (int)(t % seq);
  T* x1p = X + t * ldx + (int64_t)h * 2 * half + j0;
  T* x2p = x1p + half;
  const Vec<T, VEC> a = *(const Vec<T, VEC>*)x1p;
  const Vec<T, VEC> b = *(const Vec<T, VEC>*)x2p;
  const float* c = cs + (int64_t)s * half + j0;
  const float* sv = sn + (int64_t)s * half + j0;
  Vec<T, VEC> o1, o2;
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    const float x1 = (float)a.e[e], x2 = (float)b.e[e];
    o1.e[e] = (T)(x1 * c[e] + x2 * sv[e]);
    o2.e[e] = (T)(x2 * c[e] - x1 * sv[e]);
  }
  *(Vec<T, VEC>*)x1p = o1;
  *(Vec<T, VEC>*)x2p = o2;
}

// D[(seq_index * heads + h) * seq + s] = sum_j dO[t, h*dh + j] * O[t, h*dh + j], t = seq_index*seq + s.
// One workgroup per token: products of VEC-element chunks go to LDS, then one thread per head adds
// its chunks in a fixed order (results do not depend on scheduling).
template <typename T, int VEC>
__global__ __launch_bounds__(256) void attn_rowdot_kernel(const T* __restrict__ dO, int64_t lddo,
                                                          const T* __restrict__ O, int64_t ldo,
                                                          float* __restrict__ D, int seq, int heads, int dh) {
  extern __shared__ float part[];
  const int64_t t = blockIdx.x;
  const int d = heads * dh;
  const int nchunk = d / VEC;
  const T* a = dO + t * lddo;
  const T* b = O + t * ldo;
  for (int c = threadIdx.x; c < nchunk; c += 256) {
    const Vec<T, VEC> x = *(const Vec<T, VEC>*)(a + c * VEC);
    const Vec<T, VEC> y = *(const Vec<T, VEC>*)(b + c * VEC);
    float acc = 0.f;
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc += (float)x.e[e] * (float)y.e[e];
    part[c] = acc;
  }
  __syncthreads();
  const int cph = dh / VEC;
  const int64_t bi = t / seq;
  const int s = (int)(t - bi * seq);
  for (int h = threadIdx.x; h < heads; h += 256) {
    float acc = 0.f;
    for (int c = 0; c < cph; ++c) acc += part[h * cph + c];
    D[(bi * heads + h) * seq + s] = acc;
  }
}

}  // namespace

hipError_t launch_rope_tables(float* cs, float* sn, int seq, int dh, double theta, hipStream_t s) {
  const int half = dh / 2;
  const int n = seq * half;
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, s, cs, sn, seq, half, theta);
  return hipGetLastError();
}

hipError_t launch_rope_bwd(bool bf16, void* X, int64_t ldx, const float* cs, const float* sn, int64_t tokens,
                           int seq, int heads, int dh, hipStream_t s) {
  const int half = dh / 2;
  if (tokens == 0 || half == 0) return hipSuccess;
  auto grid = [&](int vec) { return dim3((unsigned)((tokens * heads * (half / vec) + 255) / 256)); };
  if (bf16) {
    if (half % 8 == 0 && ldx % 8 == 0)
      hipLaunchKernelGGL((rope_bwd_kernel<__bf16, 8>), grid(8), dim3(256), 0, s, (__bf16*)X, ldx, cs, sn, tokens, seq, heads, half);
    else
      hipLaunchKernelGGL((rope_bwd_kernel<__bf16, 1>), grid(1), dim3(256), 0, s, (__bf16*)X, ldx, cs, sn, tokens, seq, heads, half);
  } else {
    if (half % 4 == 0 && ldx % 4 == 0)
      hipLaunchKernelGGL((rope_bwd_kernel<float, 4>), grid(4), dim3(256), 0, s, (float*)X, ldx, cs, sn, tokens, seq, heads, half);
    else
      hipLaunchKernelGGL((rope_bwd_kernel<float, 1>), grid(1), dim3(256), 0, s, (float*)X, ldx, cs, sn, tokens, seq, heads, half);
  }
  return hipGetLastError();
}

hipError_t launch_attn_rowdot(bool bf16, const void* dO, int64_t lddo, const void* O, int64_t ldo, float* D,
                              int64_t tokens, int seq, int heads, int dh, hipStream_t s) {
  if (tokens == 0) return hipSuccess;
  const int d = heads * dh;
  const dim3 grid((unsigned)tokens), block(256);
  if (bf16) {
    if (dh % 8 == 0 && lddo % 8 == 0 && ldo % 8 == 0)
      hipLaunchKernelGGL((attn_rowdot_kernel<__bf16, 8>), grid, block, (size_t)(d / 8) * 4, s, (const __bf16*)dO, lddo, (const __bf16*)O, ldo, D, seq, heads, dh);
    else
      hipLaunchKernelGGL((attn_rowdot_kernel<__bf16, 1>), grid, block, (size_t)d * 4, s, (const __bf16*)dO, lddo, (const __bf16*)O, ldo, D, seq, heads, dh);
  } else {
    if (dh % 4 == 0 && lddo % 4 == 0 && ldo % 4 == 0)
      hipLaunchKernelGGL((attn_rowdot_kernel<float, 4>), grid, block, (size_t)(d / 4) * 4, s, (const float*)dO, lddo, (const float*)O, ldo, D, seq, heads, dh);
    else
      hipLaunchKernelGGL((attn_rowdot_kernel<float, 1>), grid, block, (size_t)d * 4, s, (const float*)dO, lddo, (const float*)O, ldo, D, seq, heads, dh);
  }
  return hipGetLastError();
}

}  // namespace mecefo

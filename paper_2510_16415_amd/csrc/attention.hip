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

// In-place rotation of the pairs (x[j], x[j + dh/2]) of every head of a token-major [tokens x d]
// tensor by the position angle (sgn = +1: the forward rotation of Q and K) or by its negative
// (sgn = -1: the transpose, applied to the gradients dQ and dK).  One thread per VEC consecutive pairs.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void rope_kernel(T* __restrict__ X, int64_t ldx,
                                                   const float* __restrict__ cs,
                                                   const float* __restrict__ sn, int64_t tokens, int seq,
                                                   int heads, int half, float sgn) {
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
    o1.e[e] = (T)(x1 * c[e] - sgn * x2 * sv[e]);
    o2.e[e] = (T)(x2 * c[e] + sgn * x1 * sv[e]);
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

// Causal softmax of one chunk of score matrices.  S [nprod][seq x lds] fp32 holds the raw dot
// products q.k; row q of a product uses keys 0..q: x = scale * s, L = log sum exp(x), P = exp(x - L).
// P (storage type, row stride ldp) gets zeros from key q+1 up to the end of the 256-block that
// contains the diagonal, which is as far as the products that consume P read.  One workgroup per row.
template <typename T, bool PRECISE>
__global__ __launch_bounds__(256) void softmax_rows_kernel(const float* __restrict__ S, int64_t lds,
                                                           T* __restrict__ P, int64_t ldp,
                                                           float* __restrict__ L, int seq, float scale) {
  __shared__ float red[4];
  const int q = blockIdx.x;
  const int64_t z = blockIdx.y;
  const float* s = S + (z * seq + q) * lds;
  T* p = P + (z * seq + q) * ldp;
  const int n = q + 1;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float m = -INFINITY;
  for (int k = threadIdx.x; k < n; k += 256) m = fmaxf(m, s[k] * scale);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
  if (lane == 0) red[wave] = m;
  __syncthreads();
  m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float sum = 0.f;
  for (int k = threadIdx.x; k < n; k += 256) {
    const float x = s[k] * scale - m;
    sum += PRECISE ? expf(x) : __builtin_amdgcn_exp2f(1.44269504088896341f * x);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
  if (lane == 0) red[wave] = sum;
  __syncthreads();
  sum = (red[0] + red[1]) + (red[2] + red[3]);
  const float lse = m + logf(sum);
  if (threadIdx.x == 0) L[z * seq + q] = lse;
  const int zero_to = min(seq, ((q >> 8) + 1) << 8);
  for (int k = threadIdx.x; k < zero_to; k += 256) {
    float v = 0.f;
    if (k < n) {
      const float x = s[k] * scale - lse;
      v = PRECISE ? expf(x) : __builtin_amdgcn_exp2f(1.44269504088896341f * x);
    }
    p[k] = (T)v;
  }
}

}  // namespace

hipError_t launch_softmax_rows(bool bf16, const float* S, int64_t lds, void* P, int64_t ldp, float* L, int nprod,
                               int seq, float scale, hipStream_t s) {
  if (nprod == 0 || seq == 0) return hipSuccess;
  const dim3 grid((unsigned)seq, (unsigned)nprod);
  if (bf16) hipLaunchKernelGGL((softmax_rows_kernel<__bf16, false>), grid, dim3(256), 0, s, S, lds, (__bf16*)P, ldp, L, seq, scale);
  else hipLaunchKernelGGL((softmax_rows_kernel<float, true>), grid, dim3(256), 0, s, S, lds, (float*)P, ldp, L, seq, scale);
  return hipGetLastError();
}

hipError_t launch_rope_tables(float* cs, float* sn, int seq, int dh, double theta, hipStream_t s) {
  const int half = dh / 2;
  const int n = seq * half;
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, s, cs, sn, seq, half, theta);
  return hipGetLastError();
}

hipError_t launch_rope(bool bf16, void* X, int64_t ldx, const float* cs, const float* sn, int64_t tokens,
                       int seq, int heads, int dh, bool inverse, hipStream_t s) {
  const float sgn = inverse ? -1.f : 1.f;
  const int half = dh / 2;
  if (tokens == 0 || half == 0) return hipSuccess;
  auto grid = [&](int vec) { return dim3((unsigned)((tokens * heads * (half / vec) + 255) / 256)); };
  if (bf16) {
    if (half % 8 == 0 && ldx % 8 == 0)
      hipLaunchKernelGGL((rope_kernel<__bf16, 8>), grid(8), dim3(256), 0, s, (__bf16*)X, ldx, cs, sn, tokens, seq, heads, half, sgn);
    else
      hipLaunchKernelGGL((rope_kernel<__bf16, 1>), grid(1), dim3(256), 0, s, (__bf16*)X, ldx, cs, sn, tokens, seq, heads, half, sgn);
  } else {
    if (half % 4 == 0 && ldx % 4 == 0)
      hipLaunchKernelGGL((rope_kernel<float, 4>), grid(4), dim3(256), 0, s, (float*)X, ldx, cs, sn, tokens, seq, heads, half, sgn);
    else
      hipLaunchKernelGGL((rope_kernel<float, 1>), grid(1), dim3(256), 0, s, (float*)X, ldx, cs, sn, tokens, seq, heads, half, sgn);
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

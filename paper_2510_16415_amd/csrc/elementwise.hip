// HBM-bound kernels of the degraded block backward: RMSNorm recompute and backward with
// the residual add (the skip: dX = dOut + normbwd(dU)), the gain-gradient column
// reduction, the split-K reduction of the Eq. (2) token contraction, and the standalone
// SwiGLU backward used when saved activations are supplied.
// One wavefront (64 lanes) owns a row; row reductions are DPP/shuffle butterflies.
#include <type_traits>

#include "mecefo_internal.h"

namespace mecefo {
namespace {

template <typename T> __device__ inline float ldf(const T* p) { return (float)*p; }

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Vector of VEC elements of T, loaded/stored with one instruction when VEC > 1.
template <typename T, int VEC> struct alignas(sizeof(T) * VEC) Vec { T e[VEC]; };

template <typename T, int VEC>
__global__ __launch_bounds__(256) void rmsnorm_fwd_kernel(const T* __restrict__ H, int64_t ldh,
                                                          const T* __restrict__ gamma, float eps,
                                                          T* __restrict__ U, int64_t ldu,
                                                          float* __restrict__ rstd, int64_t b, int d) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= b) return;
  const T* h = H + row * ldh;
  const int nv = d / VEC;
  float ss = 0.f;
  for (int i = lane; i < nv; i += 64) {
    const Vec<T, VEC> x = *(const Vec<T, VEC>*)(h + i * VEC);
#pragma unroll
    for (int e = 0; e < VEC; ++e) { const float f = (float)x.e[e]; ss += f * f; }
  }
  ss = wave_sum(ss);
  const float rs = 1.0f / sqrtf(ss / (float)d + eps);
  if (lane == 0) rstd[row] = rs;
  T* u = U + row * ldu;
  for (int i = lane; i < nv; i += 64) {
    const Vec<T, VEC> x = *(const Vec<T, VEC>*)(h + i * VEC);
    const Vec<T, VEC> g = *(const Vec<T, VEC>*)(gamma + i * VEC);
    Vec<T, VEC> o;
#pragma unroll
    for (int e = 0; e < VEC; ++e) o.e[e] = (T)((float)x.e[e] * rs * (float)g.e[e]);
    *(Vec<T, VEC>*)(u + i * VEC) = o;
  }
}

// The same with the row held in registers between the two passes (ITERS vectors per lane cover the
// row): one read of H from memory, nothing re-read through the caches.
template <typename T, int VEC, int ITERS>
__global__ __launch_bounds__(256) void rmsnorm_fwd_row_kernel(const T* __restrict__ H, int64_t ldh,
                                                              const T* __restrict__ gamma, float eps,
                                                              T* __restrict__ U, int64_t ldu,
                                                              float* __restrict__ rstd, int64_t b, int d) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= b) return;
  const T* h = H + row * ldh;
  const int nv = d / VEC;
  Vec<T, VEC> x[ITERS];
  float ss = 0.f;
#pragma unroll
  for (int k = 0; k < ITERS; ++k) {
    const int i = k * 64 + lane;
    if (i < nv) {
      x[k] = *(const Vec<T, VEC>*)(h + i * VEC);
#pragma unroll
      for (int e = 0; e < VEC; ++e) { const float f = (float)x[k].e[e]; ss += f * f; }
    }
  }
  ss = wave_sum(ss);
  const float rs = 1.0f / sqrtf(ss / (float)d + eps);
  if (lane == 0) rstd[row] = rs;
  T* u = U + row * ldu;
#pragma unroll
  for (int k = 0; k < ITERS; ++k) {
    const int i = k * 64 + lane;
    if (i < nv) {
      const Vec<T, VEC> g = *(const Vec<T, VEC>*)(gamma + i * VEC);
      Vec<T, VEC> o;
#pragma unroll
      for (int e = 0; e < VEC; ++e) o.e[e] = (T)((float)x[k].e[e] * rs * (float)g.e[e]);
      *(Vec<T, VEC>*)(u + i * VEC) = o;
    }
  }
}

// dX_i = dOut_i + rstd_i * (dN_i - N_i * mean_j(dN_ij N_ij)),  dN = dU*gamma, N = H*rstd.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void rmsnorm_bwd_kernel(const T* __restrict__ dU, int64_t lddu,
                                                          const T* __restrict__ H, int64_t ldh,
                                                          const float* __restrict__ rstd,
                                                          const T* __restrict__ gamma,
                                                          const T* dOut, int64_t lddo, T* dX, int64_t lddx,
                                                          int64_t b, int d) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= b) return;
  const T* du = dU + row * lddu;
  const T* h = H + row * ldh;
  const float rs = rstd[row];
  const int nv = d / VEC;
  float dot = 0.f;
  for (int i = lane; i < nv; i += 64) {
    const Vec<T, VEC> a = *(const Vec<T, VEC>*)(du + i * VEC);
    const Vec<T, VEC> x = *(const Vec<T, VEC>*)(h + i * VEC);
    const Vec<T, VEC> g = *(const Vec<T, VEC>*)(gamma + i * VEC);
#pragma unroll
    for (int e = 0; e < VEC; ++e) dot += (float)a.e[e] * (float)g.e[e] * ((float)x.e[e] * rs);
  }
  const float c = wave_sum(dot) / (float)d;
  const T* go = dOut + row * lddo;
  T* dx = dX + row * lddx;
  for (int i = lane; i < nv; i += 64) {
    const Vec<T, VEC> a = *(const Vec<T, VEC>*)(du + i * VEC);
    const Vec<T, VEC> x = *(const Vec<T, VEC>*)(h + i * VEC);
    const Vec<T, VEC> g = *(const Vec<T, VEC>*)(gamma + i * VEC);
    const Vec<T, VEC> r = *(const Vec<T, VEC>*)(go + i * VEC);
    Vec<T, VEC> o;
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const float n = (float)x.e[e] * rs;
      o.e[e] = (T)((float)r.e[e] + rs * ((float)a.e[e] * (float)g.e[e] - n * c));
    }
    *(Vec<T, VEC>*)(dx + i * VEC) = o;
  }
}

// Norm backward, residual add and the gain-gradient partials in one pass over dU, H and dOut: a
// workgroup owns rows_per_block consecutive rows, its four waves take them in turn with the rows of
// dU and H in registers (ITERS vectors per lane), and every lane sums dU * N of its columns over
// the wave's rows.  The four waves' sums are combined through LDS in a fixed order into
// partial[block][col] (results do not depend on scheduling).  partial may be NULL.
template <typename T, int VEC, int ITERS>
__global__ __launch_bounds__(256, 2) void rmsnorm_bwd_fused_kernel(const T* __restrict__ dU, int64_t lddu,
                                                                   const T* __restrict__ H, int64_t ldh,
                                                                   const float* __restrict__ rstd,
                                                                   const T* __restrict__ gamma,
                                                                   const T* dOut, int64_t lddo, T* dX, int64_t lddx,
                                                                   float* __restrict__ partial, int64_t b, int d,
                                                                   int rows_per_block) {
  extern __shared__ float comb[];      // [3][d]: the column sums of waves 1-3
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nv = d / VEC;
  Vec<T, VEC> g[ITERS];
  float acc[ITERS][VEC];
#pragma unroll
  for (int k = 0; k < ITERS; ++k) {
    const int i = k * 64 + lane;
    if (i < nv) g[k] = *(const Vec<T, VEC>*)(gamma + i * VEC);
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[k][e] = 0.f;
  }
  const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
  const int64_t r1 = r0 + rows_per_block < b ? r0 + rows_per_block : b;
  for (int64_t row = r0 + wave; row < r1; row += 4) {
    const T* du = dU + row * lddu;
    const T* h = H + row * ldh;
    const T* go = dOut + row * lddo;
    Vec<T, VEC> a[ITERS], x[ITERS];
#pragma unroll
    for (int k = 0; k < ITERS; ++k) {
      const int i = k * 64 + lane;
      if (i < nv) {
        a[k] = *(const Vec<T, VEC>*)(du + i * VEC);
        x[k] = *(const Vec<T, VEC>*)(h + i * VEC);
      }
    }
    const float rs = rstd[row];
    float dot = 0.f;
#pragma unroll
    for (int k = 0; k < ITERS; ++k)
      if (k * 64 + lane < nv) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) dot += (float)a[k].e[e] * (float)g[k].e[e] * ((float)x[k].e[e] * rs);
      }
    const float c = wave_sum(dot) / (float)d;
    T* dx = dX + row * lddx;
#pragma unroll
    for (int k = 0; k < ITERS; ++k) {
      const int i = k * 64 + lane;
      if (i < nv) {
        const Vec<T, VEC> r = *(const Vec<T, VEC>*)(go + i * VEC);    // read before the store: dX may alias dOut
        Vec<T, VEC> o;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const float n = (float)x[k].e[e] * rs;
          o.e[e] = (T)((float)r.e[e] + rs * ((float)a[k].e[e] * (float)g[k].e[e] - n * c));
          acc[k][e] += (float)a[k].e[e] * n;
        }
        *(Vec<T, VEC>*)(dx + i * VEC) = o;
      }
    }
  }
  if (!partial) return;      // kernel argument: the whole workgroup takes the same branch
  if (wave > 0) {
#pragma unroll
    for (int k = 0; k < ITERS; ++k) {
      const int i = k * 64 + lane;
      if (i < nv) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) comb[(wave - 1) * d + i * VEC + e] = acc[k][e];
      }
    }
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int k = 0; k < ITERS; ++k) {
      const int i = k * 64 + lane;
      if (i < nv) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const int col = i * VEC + e;
          partial[(int64_t)blockIdx.x * d + col] = ((acc[k][e] + comb[col]) + comb[d + col]) + comb[2 * d + col];
        }
      }
    }
  }
}

// The same for long rows: the whole workgroup works on one row at a time (thread t owns vectors
// t, t + 256, ...), the row dot product is combined across the four waves through LDS (one barrier
// per row, alternating slots), and the next row's dU and H are fetched while the current row is
// finished.  Every thread owns its columns for all rows of the block, so its sums go straight to
// partial[block][col].
template <typename T, int VEC, int ITERS>
__global__ __launch_bounds__(256) void rmsnorm_bwd_block_kernel(const T* __restrict__ dU, int64_t lddu,
                                                                const T* __restrict__ H, int64_t ldh,
                                                                const float* __restrict__ rstd,
                                                                const T* __restrict__ gamma,
                                                                const T* dOut, int64_t lddo, T* dX, int64_t lddx,
                                                                float* __restrict__ partial, int64_t b, int d,
                                                                int rows_per_block) {
  __shared__ float red[2][4];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int nv = d / VEC;
  Vec<T, VEC> g[ITERS], a[ITERS], x[ITERS], r[ITERS];
  float acc[ITERS][VEC];
#pragma unroll
  for (int k = 0; k < ITERS; ++k) {
    const int i = k * 256 + t;
    if (i < nv) g[k] = *(const Vec<T, VEC>*)(gamma + i * VEC);
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[k][e] = 0.f;
  }
  const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
  const int64_t r1 = r0 + rows_per_block < b ? r0 + rows_per_block : b;
  // dOut of a row is read a whole row ahead of the store of that row's dX, which may be the same memory
  auto fetch = [&](int64_t row, Vec<T, VEC> (&aa)[ITERS], Vec<T, VEC> (&xx)[ITERS], Vec<T, VEC> (&rr)[ITERS]) {
#pragma unroll
    for (int k = 0; k < ITERS; ++k) {
      const int i = k * 256 + t;
      if (i < nv) {
        aa[k] = *(const Vec<T, VEC>*)(dU + row * lddu + i * VEC);
        xx[k] = *(const Vec<T, VEC>*)(H + row * ldh + i * VEC);
        rr[k] = *(const Vec<T, VEC>*)(dOut + row * lddo + i * VEC);
      }
    }
  };
  // Two register sets take turns (no copies between them: a copy would have to wait for the loads
  // it moves): one row is finished from the first while the second receives the row after it.
  Vec<T, VEC> a2[ITERS], x2[ITERS], r2[ITERS];
  float rs = 0.f, rs2 = 0.f;
  auto finish_row = [&](int64_t row, int slot, const Vec<T, VEC> (&aa)[ITERS], const Vec<T, VEC> (&xx)[ITERS],
                        const Vec<T, VEC> (&rr)[ITERS], float rsv) {
    float dot = 0.f;
#pragma unroll
    for (int k = 0; k < ITERS; ++k)
      if (k * 256 + t < nv) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) dot += (float)aa[k].e[e] * (float)g[k].e[e] * ((float)xx[k].e[e] * rsv);
      }
    dot = wave_sum(dot);
    if (lane == 0) red[slot][wave] = dot;
    __syncthreads();
    const float c = ((red[slot][0] + red[slot][1]) + (red[slot][2] + red[slot][3])) / (float)d;
    T* dx = dX + row * lddx;
#pragma unroll
    for (int k = 0; k < ITERS; ++k) {
      const int i = k * 256 + t;
      if (i < nv) {
        Vec<T, VEC> o;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const float n = (float)xx[k].e[e] * rsv;
          o.e[e] = (T)((float)rr[k].e[e] + rsv * ((float)aa[k].e[e] * (float)g[k].e[e] - n * c));
          acc[k][e] += (float)aa[k].e[e] * n;
        }
        *(Vec<T, VEC>*)(dx + i * VEC) = o;
      }
    }
  };
  if (r0 < r1) { fetch(r0, a, x, r); rs = rstd[r0]; }
  for (int64_t row = r0; row < r1; row += 2) {      // bounds are the same for the whole workgroup
    if (row + 1 < r1) { fetch(row + 1, a2, x2, r2); rs2 = rstd[row + 1]; }
    finish_row(row, 0, a, x, r, rs);
    if (row + 1 < r1) {
      if (row + 2 < r1) { fetch(row + 2, a, x, r); rs = rstd[row + 2]; }
      finish_row(row + 1, 1, a2, x2, r2, rs2);
    }
  }
  if (!partial) return;
#pragma unroll
  for (int k = 0; k < ITERS; ++k) {
    const int i = k * 256 + t;
    if (i < nv) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) partial[(int64_t)blockIdx.x * d + i * VEC + e] = acc[k][e];
    }
  }
}

// Partial column sums of dU * N over a chunk of rows: partial[chunk][col].
template <typename T, int VEC>
__global__ __launch_bounds__(256) void dgamma_partial_kernel(const T* __restrict__ dU, int64_t lddu,
                                                             const T* __restrict__ H, int64_t ldh,
                                                             const float* __restrict__ rstd,
                                                             float* __restrict__ partial, int64_t b, int d,
                                                             int rows_per_chunk) {
  const int cv = blockIdx.x * 256 + threadIdx.x;
  if (cv * VEC >= d) return;
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_chunk;
  const int64_t r1 = r0 + rows_per_chunk < b ? r0 + rows_per_chunk : b;
  float acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
  for (int64_t r = r0; r < r1; ++r) {
    const Vec<T, VEC> a = *(const Vec<T, VEC>*)(dU + r * lddu + cv * VEC);
    const Vec<T, VEC> x = *(const Vec<T, VEC>*)(H + r * ldh + cv * VEC);
    const float rs = rstd[r];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] += (float)a.e[e] * ((float)x.e[e] * rs);
  }
#pragma unroll
  for (int e = 0; e < VEC; ++e) partial[(int64_t)blockIdx.y * d + cv * VEC + e] = acc[e];
}

// dgamma[c] = sum over chunks of partial[chunk][c].  A block owns 32 columns; its 32 groups of 32
// threads each sum a strided part of the chunks (coalesced 128-byte rows), then combine in LDS
// in a fixed order.
template <typename T>
__global__ __launch_bounds__(1024) void dgamma_reduce_kernel(const float* __restrict__ partial, int nblk, int d,
                                                             void* dgamma, int out_f32, int accumulate) {
  __shared__ float red[32][32];
  const int cl = threadIdx.x & 31, g = threadIdx.x >> 5;
  const int c = blockIdx.x * 32 + cl;
  float s = 0.f;
  if (c < d) {
#pragma unroll 16
    for (int k = g; k < nblk; k += 32) s += partial[(int64_t)k * d + c];
  }
  red[g][cl] = s;
  __syncthreads();
  if (g != 0 || c >= d) return;
#pragma unroll
  for (int k = 1; k < 32; ++k) s += red[k][cl];
  if (out_f32) {
    float* o = (float*)dgamma;
    o[c] = accumulate ? o[c] + s : s;
  } else {
    T* o = (T*)dgamma;
    o[c] = (T)(accumulate ? (float)o[c] + s : s);
  }
}

template <typename T, int VEC>
__global__ __launch_bounds__(256) void add_kernel(const T* a, int64_t lda, const T* __restrict__ bsrc,
                                                  int64_t ldb, T* out, int64_t ldo, int64_t rows, int cols) {
  const int nv = cols / VEC;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= rows * nv) return;
  const int64_t r = idx / nv;
  const int cv = (int)(idx - r * nv);
  const Vec<T, VEC> x = *(const Vec<T, VEC>*)(a + r * lda + cv * VEC);
  const Vec<T, VEC> y = *(const Vec<T, VEC>*)(bsrc + r * ldb + cv * VEC);
  Vec<T, VEC> o;
#pragma unroll
  for (int e = 0; e < VEC; ++e) o.e[e] = (T)((float)x.e[e] + (float)y.e[e]);
  *(Vec<T, VEC>*)(out + r * ldo + cv * VEC) = o;
}

// C[i] = sum_s partial[s][i], fixed summation order (bit-reproducible).
template <typename T>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, int splits,
                                                            int64_t mn, T* __restrict__ C) {
  const int64_t i4 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i4 >= mn) return;
  if (i4 + 4 <= mn) {
    float4 s = *(const float4*)(partial + i4);
    for (int k = 1; k < splits; ++k) {
      const float4 v = *(const float4*)(partial + (int64_t)k * mn + i4);
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    C[i4] = (T)s.x; C[i4 + 1] = (T)s.y; C[i4 + 2] = (T)s.z; C[i4 + 3] = (T)s.w;
  } else {
    for (int64_t i = i4; i < mn; ++i) {
      float s = 0.f;
      for (int k = 0; k < splits; ++k) s += partial[(int64_t)k * mn + i];
      C[i] = (T)s;
    }
  }
}

template <bool PRECISE> __device__ inline float sigm(float g) {
  if constexpr (PRECISE) return 1.0f / (1.0f + expf(-g));
  else return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896341f * g));
}

// dA (in DG), saved G, Z  ->  DG = dG, DZ = dZ, AA = silu(G)*Z.  VEC columns per thread.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const T* __restrict__ G, const T* __restrict__ Z,
                                                         int64_t ldgz, T* DG, T* __restrict__ DZ,
                                                         T* __restrict__ AA, int64_t ldf, int64_t b, int f,
                                                         int pad_cols) {
  const int nv = (pad_cols + VEC - 1) / VEC;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= b * nv) return;
  const int64_t r = idx / nv;
  const int c0 = (int)(idx - r * nv) * VEC;
  Vec<T, VEC> g, z, da, odg, odz, oa;
  if (c0 < f) {
    g = *(const Vec<T, VEC>*)(G + r * ldgz + c0);
    z = *(const Vec<T, VEC>*)(Z + r * ldgz + c0);
    da = *(const Vec<T, VEC>*)(DG + r * ldf + c0);
  }
#pragma unroll
  for (int e = 0; e < VEC; ++e) {
    float vdg = 0.f, vdz = 0.f, va = 0.f;
    if (c0 + e < f) {
      const float gg = (float)g.e[e], zz = (float)z.e[e], d = (float)da.e[e];
      const float sg = sigm<sizeof(T) == 4>(gg);
      const float s = gg * sg;
      va = s * zz;
      vdz = d * s;
      vdg = d * zz * (sg * (1.0f + gg * (1.0f - sg)));
    }
    odg.e[e] = (T)vdg; odz.e[e] = (T)vdz; oa.e[e] = (T)va;
  }
  *(Vec<T, VEC>*)(DG + r * ldf + c0) = odg;
  *(Vec<T, VEC>*)(DZ + r * ldf + c0) = odz;
  *(Vec<T, VEC>*)(AA + r * ldf + c0) = oa;
}

inline unsigned blocks_for(int64_t n) { return (unsigned)((n + 255) / 256); }
constexpr int kDgammaRows = 16;

// The register-resident row kernels (bf16, eight elements per lane and step) cover rows of up to
// 8 * 64 * 8 = 4096 elements whose strides keep every 16-byte vector aligned.
bool row_fits(int d, int64_t l0, int64_t l1, int64_t l2, int64_t l3) {
  return d % 8 == 0 && d <= 4096 && l0 % 8 == 0 && l1 % 8 == 0 && l2 % 8 == 0 && l3 % 8 == 0;
}
template <typename F> void dispatch_iters(int nv, F&& f) {
  if (nv <= 64) f(std::integral_constant<int, 1>{});
  else if (nv <= 128) f(std::integral_constant<int, 2>{});
  else if (nv <= 256) f(std::integral_constant<int, 4>{});
  else f(std::integral_constant<int, 8>{});
}

}  // namespace

hipError_t launch_rmsnorm_fwd(bool bf16, const void* H, int64_t ldh, const void* gamma, float eps, void* U,
                              int64_t ldu, float* rstd, int64_t b, int d, hipStream_t s) {
  const unsigned grid = (unsigned)((b + 3) / 4);
  if (bf16 && row_fits(d, ldh, ldu, ldu, ldu)) {
    auto go = [&](auto iters) {
      hipLaunchKernelGGL((rmsnorm_fwd_row_kernel<__bf16, 8, decltype(iters)::value>), dim3(grid), dim3(256), 0, s,
                         (const __bf16*)H, ldh, (const __bf16*)gamma, eps, (__bf16*)U, ldu, rstd, b, d);
    };
    dispatch_iters(d / 8, go);
  } else if (bf16)
    hipLaunchKernelGGL((rmsnorm_fwd_kernel<__bf16, 8>), dim3(grid), dim3(256), 0, s, (const __bf16*)H, ldh,
                       (const __bf16*)gamma, eps, (__bf16*)U, ldu, rstd, b, d);
  else
    hipLaunchKernelGGL((rmsnorm_fwd_kernel<float, 1>), dim3(grid), dim3(256), 0, s, (const float*)H, ldh,
                       (const float*)gamma, eps, (float*)U, ldu, rstd, b, d);
  return hipGetLastError();
}

int rmsnorm_bwd_blocks(int64_t b) { return (int)((b + kDgammaRows - 1) / kDgammaRows); }

hipError_t launch_rmsnorm_bwd(bool bf16, const void* dU, int64_t lddu, const void* H, int64_t ldh,
                              const float* rstd, const void* gamma, const void* dOut, int64_t lddo, void* dX,
                              int64_t lddx, float* dg_partial, int nblk, int64_t b, int d, hipStream_t s) {
  if (bf16 && d % 8 == 0 && d <= 8192 && lddu % 8 == 0 && ldh % 8 == 0 && lddo % 8 == 0 && lddx % 8 == 0) {
    const int nv = d / 8;
    const dim3 grid((unsigned)rmsnorm_bwd_blocks(b));
#define MECEFO_NORM_BWD(KERNEL, ITERS, LDS)                                                                          \
  hipLaunchKernelGGL((KERNEL<__bf16, 8, ITERS>), grid, dim3(256), LDS, s, (const __bf16*)dU, lddu,                 \
                     (const __bf16*)H, ldh, rstd, (const __bf16*)gamma, (const __bf16*)dOut, lddo, (__bf16*)dX, lddx, \
                     dg_partial, b, d, kDgammaRows)
    const size_t comb = (size_t)3 * d * 4;
    if (nv <= 64) MECEFO_NORM_BWD(rmsnorm_bwd_fused_kernel, 1, comb);         // a wave per row
    else if (nv <= 128) MECEFO_NORM_BWD(rmsnorm_bwd_fused_kernel, 2, comb);
    else if (nv <= 256) MECEFO_NORM_BWD(rmsnorm_bwd_block_kernel, 1, 0);      // the workgroup per row
    else if (nv <= 512) MECEFO_NORM_BWD(rmsnorm_bwd_block_kernel, 2, 0);
    else MECEFO_NORM_BWD(rmsnorm_bwd_block_kernel, 4, 0);
#undef MECEFO_NORM_BWD
    return hipGetLastError();
  }
  // The gain-gradient partials read dU and H before dX is written (dX may alias dOut only).
  if (dg_partial) {
    if (bf16)
      hipLaunchKernelGGL((dgamma_partial_kernel<__bf16, 8>), dim3(blocks_for(d / 8), nblk), dim3(256), 0, s,
                         (const __bf16*)dU, lddu, (const __bf16*)H, ldh, rstd, dg_partial, b, d, kDgammaRows);
    else
      hipLaunchKernelGGL((dgamma_partial_kernel<float, 1>), dim3(blocks_for(d), nblk), dim3(256), 0, s,
                         (const float*)dU, lddu, (const float*)H, ldh, rstd, dg_partial, b, d, kDgammaRows);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const unsigned grid = (unsigned)((b + 3) / 4);
  if (bf16)
    hipLaunchKernelGGL((rmsnorm_bwd_kernel<__bf16, 8>), dim3(grid), dim3(256), 0, s, (const __bf16*)dU, lddu,
                       (const __bf16*)H, ldh, rstd, (const __bf16*)gamma, (const __bf16*)dOut, lddo,
                       (__bf16*)dX, lddx, b, d);
  else
    hipLaunchKernelGGL((rmsnorm_bwd_kernel<float, 1>), dim3(grid), dim3(256), 0, s, (const float*)dU, lddu,
                       (const float*)H, ldh, rstd, (const float*)gamma, (const float*)dOut, lddo, (float*)dX,
                       lddx, b, d);
  return hipGetLastError();
}

hipError_t launch_dgamma_reduce(const float* dg_partial, int nblk, int d, void* dgamma, bool out_f32,
                                bool bf16, int accumulate, hipStream_t s) {
  if (bf16)
    hipLaunchKernelGGL(dgamma_reduce_kernel<__bf16>, dim3((d + 31) / 32), dim3(1024), 0, s, dg_partial, nblk, d,
                       dgamma, (int)out_f32, accumulate);
  else
    hipLaunchKernelGGL(dgamma_reduce_kernel<float>, dim3((d + 31) / 32), dim3(1024), 0, s, dg_partial, nblk, d,
                       dgamma, 1, accumulate);
  return hipGetLastError();
}

hipError_t launch_add(bool bf16, const void* a, int64_t lda, const void* bsrc, int64_t ldb, void* out,
                      int64_t ldo, int64_t rows, int cols, hipStream_t s) {
  if (bf16)
    hipLaunchKernelGGL((add_kernel<__bf16, 8>), dim3(blocks_for(rows * (cols / 8))), dim3(256), 0, s,
                       (const __bf16*)a, lda, (const __bf16*)bsrc, ldb, (__bf16*)out, ldo, rows, cols);
  else
    hipLaunchKernelGGL((add_kernel<float, 1>), dim3(blocks_for(rows * cols)), dim3(256), 0, s, (const float*)a,
                       lda, (const float*)bsrc, ldb, (float*)out, ldo, rows, cols);
  return hipGetLastError();
}

hipError_t launch_splitk_reduce(bool bf16, const float* partial, int splits, int64_t mn, void* C,
                                hipStream_t s) {
  const unsigned grid = blocks_for((mn + 3) / 4);
  if (bf16)
    hipLaunchKernelGGL(splitk_reduce_kernel<__bf16>, dim3(grid), dim3(256), 0, s, partial, splits, mn,
                       (__bf16*)C);
  else
    hipLaunchKernelGGL(splitk_reduce_kernel<float>, dim3(grid), dim3(256), 0, s, partial, splits, mn,
                       (float*)C);
  return hipGetLastError();
}

hipError_t launch_swiglu_bwd(bool bf16, const void* G, const void* Z, int64_t ldgz, void* DG, void* DZ,
                             void* AA, int64_t ldf, int64_t b, int f, int pad_cols, hipStream_t s) {
  if (bf16) {
    const int nv = (pad_cols + 7) / 8;
    hipLaunchKernelGGL((swiglu_bwd_kernel<__bf16, 8>), dim3(blocks_for(b * nv)), dim3(256), 0, s,
                       (const __bf16*)G, (const __bf16*)Z, ldgz, (__bf16*)DG, (__bf16*)DZ, (__bf16*)AA, ldf, b,
                       f, pad_cols);
  } else {
    hipLaunchKernelGGL((swiglu_bwd_kernel<float, 1>), dim3(blocks_for(b * pad_cols)), dim3(256), 0, s,
                       (const float*)G, (const float*)Z, ldgz, (float*)DG, (float*)DZ, (float*)AA, ldf, b, f,
                       pad_cols);
  }
  return hipGetLastError();
}

}  // namespace mecefo

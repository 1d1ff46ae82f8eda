// Projection refresh of Alg. 3: an orthonormal basis of (an approximation to) the span of the
// top-r right (or left) singular vectors of a weight matrix, computed without an SVD or a QR:
// subspace iteration X <- W^T (W X) on the GEMM core, with Newton-Schulz steps X <- X q(X^T X)
// in between.  A right-multiplication by an invertible r x r matrix changes the basis but not its
// span, so the Newton-Schulz steps only control the conditioning of the basis (they push every
// singular value of X towards 1); the final steps use the form X + X E, E = (I - X^T X)/2, whose
// small correction keeps full relative precision in the storage type.
#include <math.h>
#include <string.h>

#include "../../include/mecefo.h"
#include "mecefo_internal.h"

namespace mecefo {
namespace {

constexpr int kNormBlocks = 256;
constexpr int kMaxSplits = 8;

// The iterate is kept as an fp32 master copy.  For bf16 weights it enters the MFMA products as the
// sum of two bf16 matrices (hi = bf16(x), lo = bf16(x - hi): 16 mantissa bits), contracted as two K
// segments of one launch: a single bf16 rounding of the iterate would drown the weakest of the r
// directions, whose share of X after one application of W^T W is (s_r/s_1)^2.
__global__ __launch_bounds__(256) void split_kernel(const float* __restrict__ X, __bf16* __restrict__ hi,
                                                    __bf16* __restrict__ lo, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const float x = X[i];
    const __bf16 h = (__bf16)x;
    hi[i] = h;
    lo[i] = (__bf16)(x - (float)h);
  }
}

__global__ __launch_bounds__(256) void sumsq_partial_kernel(const float* __restrict__ X, int64_t ld, int64_t rows,
                                                            int cols, float* __restrict__ partial) {
  // block b sums rows b, b + gridDim.x, ... in a fixed order
  __shared__ float red[256];
  float acc = 0.f;
  for (int64_t row = blockIdx.x; row < rows; row += gridDim.x)
    for (int c = threadIdx.x; c < cols; c += 256) {
      const float v = X[row * ld + c];
      acc += v * v;
    }
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

// X *= 1 / sqrt(sum of the partial sums); a zero matrix is left unchanged.
__global__ __launch_bounds__(256) void scale_by_inv_norm_kernel(float* __restrict__ X, int64_t ld, int64_t rows,
                                                                int cols, const float* __restrict__ partial,
                                                                int nparts) {
  __shared__ float inv;
  if (threadIdx.x == 0) {
    float s = 0.f;
    for (int i = 0; i < nparts; ++i) s += partial[i];
    inv = s > 0.f ? 1.0f / sqrtf(s) : 1.0f;
  }
  __syncthreads();
  const float k = inv;
  for (int64_t row = blockIdx.x; row < rows; row += gridDim.x)
    for (int c = threadIdx.x; c < cols; c += 256) X[row * ld + c] *= k;
}

// out[i, j] = a * (i == j) + b * A[i, j] + c * A2[i, j]   (A2 may be NULL), r x r, fp32 in, T out.
template <typename T>
__global__ __launch_bounds__(256) void poly_kernel(T* __restrict__ out, int64_t ldo, const float* __restrict__ A,
                                                   const float* __restrict__ A2, int64_t lda, int r, float a,
                                                   float b, float c) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (int64_t)r * r) return;
  const int row = (int)(i / r), col = (int)(i - (int64_t)row * r);
  float v = b * A[row * lda + col];
  if (A2) v += c * A2[row * lda + col];
  if (row == col) v += a;
  out[row * ldo + col] = (T)v;
}

// dst[rows x cols] (row stride ldd) = src (row stride lds), converting the element type;
// columns [cols, ldd_fill) of dst are set to zero.
template <typename D, typename S>
__global__ __launch_bounds__(256) void convert2d_kernel(D* __restrict__ dst, int64_t ldd, const S* __restrict__ src,
                                                        int64_t lds, int64_t rows, int cols, int fill_to) {
  const int64_t n = rows * fill_to;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int64_t row = i / fill_to;
    const int c = (int)(i - row * fill_to);
    dst[row * ldd + c] = c < cols ? (D)(float)src[row * lds + c] : (D)0.f;
  }
}

inline int64_t up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }
inline unsigned grid_for(int64_t n) { int64_t g = (n + 255) / 256; return (unsigned)(g < 1 ? 1 : (g > 65536 ? 65536 : g)); }

struct Plan {
  bool bf16;
  int esz;
  int m, n, r;       // W is [m x n]; the basis has `dim` rows (n for right, m for left vectors)
  int dim, other;
  int64_t ldx;       // row stride of every internal [* x r] buffer
  size_t X32[2], Y32, Xh, Xl, Yh, Yl, A32, B32, M16, A16, part, partial, total;
};

Plan make_plan(bool bf16, int m, int n, int r, int left) {
  Plan p;
  p.bf16 = bf16; p.esz = bf16 ? 2 : 4;
  p.m = m; p.n = n; p.r = r;
  p.dim = left ? m : n; p.other = left ? n : m;
  p.ldx = up(r, 8);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += (size_t)up((int64_t)bytes, 256); return o; };
  p.X32[0] = take((size_t)p.dim * p.ldx * 4);
  p.X32[1] = take((size_t)p.dim * p.ldx * 4);
  p.Y32 = take((size_t)p.other * p.ldx * 4);
  const size_t hx = bf16 ? (size_t)p.dim * p.ldx * 2 : 0, hy = bf16 ? (size_t)p.other * p.ldx * 2 : 0;
  p.Xh = take(hx); p.Xl = take(hx); p.Yh = take(hy); p.Yl = take(hy);
  p.A32 = take((size_t)r * p.ldx * 4);
  p.B32 = take((size_t)r * p.ldx * 4);
  p.M16 = take((size_t)r * p.ldx * p.esz);
  p.A16 = take((size_t)r * p.ldx * p.esz);
  p.part = take(kNormBlocks * 4);
  // split-K partials of the products with few output tiles and a long contraction
  const int64_t big = (p.dim > p.other ? p.dim : p.other);
  p.partial = take(bf16 ? (size_t)kMaxSplits * big * p.ldx * 4 : 0);
  p.total = off + 256;
  return p;
}

// An iterate as GEMM operand: fp32 path: the master copy; bf16 path: the hi and lo halves.
struct Operand { const void* hi; const void* lo; };

// C (fp32, row stride ldx) (+)= opA * opB, where exactly one of the two sides may be an iterate
// split into hi + lo (then the launch has two K segments over the same other operand).
GemmLaunch product(const Plan& pl, bool akc, bool bkc, const void* A_hi, const void* A_lo, int64_t lda,
                   const void* B_hi, const void* B_lo, int64_t ldb, float* C, int M, int N, int K, int accumulate) {
  GemmLaunch g;
  memset(&g, 0, sizeof(g));
  g.a_kcontig = akc; g.b_kcontig = bkc; g.epi = EPI_GRAD; g.bf16 = pl.bf16; g.out_f32 = true;
  g.accumulate = accumulate; g.splits = 1; g.nprob = 1;
  GemmProblem& p = g.p[0];
  const bool two = A_lo != nullptr || B_lo != nullptr;
  p.A[0] = A_hi; p.A[1] = A_lo ? A_lo : A_hi; p.A[2] = A_hi;
  p.B[0] = B_hi; p.B[1] = B_lo ? B_lo : B_hi; p.B[2] = B_hi;
  p.C[0] = C;
  p.lda = lda; p.ldb = ldb; p.ldc = pl.ldx; p.M = M; p.N = N; p.K = K; p.nseg = two ? 2 : 1;
  return g;
}

// Products with fewer than 160 tiles of 256 x 256 and a long contraction are cut along K so that
// every CU gets a block; the fp32 partials are then summed in a fixed order.
hipError_t run_product(const Plan& pl, char* base, GemmLaunch& g, hipStream_t s) {
  GemmProblem& p = g.p[0];
  const int tiles = ((p.M + 255) / 256) * ((p.N + 255) / 256);
  const int stages = ((p.K + 63) / 64) * p.nseg;
  int splits = 1;
  if (pl.bf16 && !g.accumulate && tiles < 160 && stages >= 64) {
    splits = (256 + tiles - 1) / tiles;
    if (splits > stages / 8) splits = stages / 8;
    if (splits > kMaxSplits) splits = kMaxSplits;
    while (splits > 1 && (int64_t)splits * p.M * p.ldc * 4 > (int64_t)kMaxSplits * (pl.dim > pl.other ? pl.dim : pl.other) * pl.ldx * 4) --splits;
  }
  if (splits <= 1) return launch_gemm(g, s);
  float* C = (float*)p.C[0];
  g.epi = EPI_SPLIT_F32;
  g.splits = splits;
  g.partial = (float*)(base + pl.partial);
  g.partial_off[0] = 0;
  g.force_large = true;
  hipError_t e = launch_gemm(g, s);
  if (e != hipSuccess) return e;
  return launch_splitk_reduce(false, g.partial, splits, (int64_t)p.M * p.ldc, C, s);
}

#define HIP_TRY(x) do { hipError_t e__ = (x); if (e__ != hipSuccess) return (mecefo_status_t)fail(MECEFO_ERR_LAUNCH, "%s: %s", #x, hipGetErrorString(e__)); } while (0)

template <typename T>
hipError_t run_poly(void* out, int64_t ldo, const float* A, const float* A2, int64_t lda, int r, float a, float b,
                    float c, hipStream_t s) {
  hipLaunchKernelGGL(poly_kernel<T>, dim3(grid_for((int64_t)r * r)), dim3(256), 0, s, (T*)out, ldo, A, A2, lda, r, a, b, c);
  return hipGetLastError();
}

struct Refresh {
  Plan pl;
  char* base;
  hipStream_t s;
  int cur = 0;

  float* X32(int i) const { return (float*)(base + pl.X32[i]); }
  float* Y32() const { return (float*)(base + pl.Y32); }
  Operand opX() const { return pl.bf16 ? Operand{base + pl.Xh, base + pl.Xl} : Operand{X32(cur), nullptr}; }
  Operand opY() const { return pl.bf16 ? Operand{base + pl.Yh, base + pl.Yl} : Operand{Y32(), nullptr}; }

  hipError_t split(const float* src, size_t hi, size_t lo, int rows) const {
    if (!pl.bf16) return hipSuccess;
    const int64_t n = (int64_t)rows * pl.ldx;
    hipLaunchKernelGGL(split_kernel, dim3(grid_for(n)), dim3(256), 0, s, src, (__bf16*)(base + hi), (__bf16*)(base + lo), n);
    return hipGetLastError();
  }
  hipError_t split_x() const { return split(X32(cur), pl.Xh, pl.Xl, pl.dim); }
  hipError_t split_y() const { return split(Y32(), pl.Yh, pl.Yl, pl.other); }

  hipError_t normalise() const {  // X /= ||X||_F, so that every singular value is <= 1
    float* part = (float*)(base + pl.part);
    hipLaunchKernelGGL(sumsq_partial_kernel, dim3(kNormBlocks), dim3(256), 0, s, X32(cur), pl.ldx, (int64_t)pl.dim, pl.r, part);
    hipLaunchKernelGGL(scale_by_inv_norm_kernel, dim3(pl.dim < 4096 ? pl.dim : 4096), dim3(256), 0, s, X32(cur), pl.ldx, (int64_t)pl.dim, pl.r, part, kNormBlocks);
    return hipGetLastError();
  }

  // One Newton-Schulz step X <- X (a I + b A + c A^2), A = X^T X; `additive` (c == 0): X <- X + X E
  // with E = (a - 1) I + b A.  A, A^2 and the polynomial only shape the conditioning and are taken
  // in the storage type; the product with X keeps the split operand.
  mecefo_status_t ns_step(float a, float b, float c, bool additive) {
    const int r = pl.r, dim = pl.dim;
    float* A32 = (float*)(base + pl.A32);
    float* B32 = (float*)(base + pl.B32);
    void* M16 = base + pl.M16;
    void* A16 = base + pl.A16;
    const Operand x = opX();
    {  // A = X^T X  [r x r], contraction over the rows of X (hi part only)
      GemmLaunch g = product(pl, false, false, x.hi, nullptr, pl.ldx, x.hi, nullptr, pl.ldx, A32, r, r, dim, 0);
      HIP_TRY(run_product(pl, base, g, s));
    }
    const float* A2 = nullptr;
    if (c != 0.f) {  // A^2 = A A^T (A is symmetric)
      HIP_TRY(pl.bf16 ? run_poly<__bf16>(A16, pl.ldx, A32, nullptr, pl.ldx, r, 0.f, 1.f, 0.f, s)
                      : run_poly<float>(A16, pl.ldx, A32, nullptr, pl.ldx, r, 0.f, 1.f, 0.f, s));
      GemmLaunch g = product(pl, true, true, A16, nullptr, pl.ldx, A16, nullptr, pl.ldx, B32, r, r, r, 0);
      HIP_TRY(run_product(pl, base, g, s));
      A2 = B32;
    }
    const float da = additive ? a - 1.f : a;
    HIP_TRY(pl.bf16 ? run_poly<__bf16>(M16, pl.ldx, A32, A2, pl.ldx, r, da, b, c, s)
                    : run_poly<float>(M16, pl.ldx, A32, A2, pl.ldx, r, da, b, c, s));
    float* out = X32(cur ^ 1);
    if (additive) HIP_TRY(hipMemcpyAsync(out, X32(cur), (size_t)dim * pl.ldx * 4, hipMemcpyDeviceToDevice, s));
    // the polynomial of the symmetric A is symmetric: X M = X M^T, so M is the K-contiguous operand
    GemmLaunch g = product(pl, true, true, x.hi, x.lo, pl.ldx, M16, nullptr, pl.ldx, out, dim, r, r, additive ? 1 : 0);
    HIP_TRY(run_product(pl, base, g, s));
    cur ^= 1;
    HIP_TRY(split_x());
    return MECEFO_OK;
  }

  // Quintic steps with slope 3.4445 at zero: a small singular value grows by that factor per step,
  // values near 1 stay within about [0.7, 1.2] (the odd quintic used for low-precision
  // orthogonalisation; it does not converge to exactly 1, the cubic steps do).
  mecefo_status_t condition(int steps) {
    HIP_TRY(normalise());
    HIP_TRY(split_x());
    for (int i = 0; i < steps; ++i) {
      mecefo_status_t e = ns_step(3.4445f, -4.7750f, 2.0315f, false);
      if (e != MECEFO_OK) return e;
    }
    return MECEFO_OK;
  }

  mecefo_status_t power_round(const void* W, int64_t ldw, int left) {
    const int m = pl.m, n = pl.n, r = pl.r;
    const Operand x = opX();
    // right vectors: Y = W X [m x r] (K = n), X' = W^T Y [n x r] (K = m, W read as [K x M]);
    // left vectors:  Y = W^T X [n x r] (K = m), X' = W Y [m x r] (K = n)
    GemmLaunch g1 = left ? product(pl, false, false, W, nullptr, ldw, x.hi, x.lo, pl.ldx, Y32(), n, r, m, 0)
                         : product(pl, true, false, W, nullptr, ldw, x.hi, x.lo, pl.ldx, Y32(), m, r, n, 0);
    HIP_TRY(run_product(pl, base, g1, s));
    HIP_TRY(split_y());
    const Operand y = opY();
    GemmLaunch g2 = left ? product(pl, true, false, W, nullptr, ldw, y.hi, y.lo, pl.ldx, X32(cur ^ 1), m, r, n, 0)
                         : product(pl, false, false, W, nullptr, ldw, y.hi, y.lo, pl.ldx, X32(cur ^ 1), n, r, m, 0);
    HIP_TRY(run_product(pl, base, g2, s));
    cur ^= 1;
    return MECEFO_OK;
  }
};

mecefo_status_t check(int m, int n, int64_t ldw, int r, mecefo_dtype_t dtype, int power_iters, int cond_steps,
                      int polish_steps, bool* bf16) {
  if (dtype != MECEFO_F32 && dtype != MECEFO_BF16) return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "dtype must be MECEFO_F32 or MECEFO_BF16");
  *bf16 = dtype == MECEFO_BF16;
  if (m < 1 || n < 1) return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "m >= 1 and n >= 1 required");
  if (r < 1 || r > (m < n ? m : n)) return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "rank %d outside [1, min(m, n) = %d]", r, m < n ? m : n);
  if (ldw < n) return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "ldw %lld < n %d", (long long)ldw, n);
  if (*bf16 && ldw % 8) return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "bf16 path needs ldw to be a multiple of 8");
  if ((int64_t)m * ldw * 4 >= ((int64_t)1 << 31) || (int64_t)(m > n ? m : n) * up(r, 8) * 4 >= ((int64_t)1 << 31))
    return (mecefo_status_t)fail(MECEFO_ERR_UNSUPPORTED, "the matrix or the basis reaches 2 GiB");
  if (power_iters < 0 || cond_steps < 0 || polish_steps < 0 || power_iters > 1000 || cond_steps > 100 || polish_steps > 100)
    return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "iteration counts must be non-negative (and sane)");
  return MECEFO_OK;
}

}  // namespace
}  // namespace mecefo

using namespace mecefo;

extern "C" {

mecefo_status_t mecefo_projection_workspace_bytes(mecefo_dtype_t dtype, int m, int n, int r, int left,
                                                  size_t* out_bytes) {
  bool bf16;
  mecefo_status_t st = check(m, n, (n + 7) / 8 * 8, r, dtype, 0, 0, 0, &bf16);
  if (st != MECEFO_OK) return st;
  if (!out_bytes) return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "out_bytes is NULL");
  *out_bytes = make_plan(bf16, m, n, r, left).total;
  return MECEFO_OK;
}

mecefo_status_t mecefo_projection_refresh(mecefo_dtype_t dtype, const void* W, int m, int n, int64_t ldw, int left,
                                          const void* V0, int64_t ldv, int r, int power_iters, int cond_steps,
                                          int polish_steps, void* P, int64_t ldp, void* ws, size_t ws_bytes,
                                          void* hip_stream) {
  bool bf16;
  mecefo_status_t st = check(m, n, ldw, r, dtype, power_iters, cond_steps, polish_steps, &bf16);
  if (st != MECEFO_OK) return st;
  if (!W || !V0 || !P) return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "W, V0 and P are required");
  if (ldv < r || ldp < r) return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "ldv and ldp must be >= r");
  const int al = bf16 ? 16 : 4;
  if (((uintptr_t)W | (uintptr_t)V0 | (uintptr_t)P) % al) return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "W, V0 and P must be %d-byte aligned", al);
  Refresh R;
  R.pl = make_plan(bf16, m, n, r, left);
  if (R.pl.total > ws_bytes) return (mecefo_status_t)fail(MECEFO_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", ws_bytes, R.pl.total);
  if (!ws) return (mecefo_status_t)fail(MECEFO_ERR_INVALID_ARG, "workspace is NULL");
  R.base = (char*)up((int64_t)(uintptr_t)ws, 256);
  R.s = (hipStream_t)hip_stream;
  const Plan& pl = R.pl;
  const int dim = pl.dim;
  const int64_t ldx = pl.ldx;
  const unsigned gx = grid_for((int64_t)dim * ldx);

  // start basis -> fp32 master copy (padding columns zeroed: they are contracted as K padding)
  if (bf16) hipLaunchKernelGGL((convert2d_kernel<float, __bf16>), dim3(gx), dim3(256), 0, R.s, R.X32(0), ldx, (const __bf16*)V0, ldv, (int64_t)dim, r, (int)ldx);
  else hipLaunchKernelGGL((convert2d_kernel<float, float>), dim3(gx), dim3(256), 0, R.s, R.X32(0), ldx, (const float*)V0, ldv, (int64_t)dim, r, (int)ldx);
  HIP_TRY(hipGetLastError());
  // The start basis is only normalised: a previous projection is orthonormal already and Gaussian
  // noise is well conditioned; without power rounds it is conditioned for the polishing steps.
  st = R.condition(power_iters == 0 ? cond_steps : 0);
  if (st != MECEFO_OK) return st;
  for (int it = 0; it < power_iters; ++it) {
    st = R.power_round(W, ldw, left);
    if (st != MECEFO_OK) return st;
    st = R.condition(cond_steps);
    if (st != MECEFO_OK) return st;
  }
  for (int i = 0; i < polish_steps; ++i) {  // cubic steps X <- X + X (I - X^T X) / 2
    st = R.ns_step(1.5f, -0.5f, 0.f, true);
    if (st != MECEFO_OK) return st;
  }
  const unsigned gp = grid_for((int64_t)dim * r);
  if (bf16) hipLaunchKernelGGL((convert2d_kernel<__bf16, float>), dim3(gp), dim3(256), 0, R.s, (__bf16*)P, ldp, R.X32(R.cur), ldx, (int64_t)dim, r, r);
  else hipLaunchKernelGGL((convert2d_kernel<float, float>), dim3(gp), dim3(256), 0, R.s, (float*)P, ldp, R.X32(R.cur), ldx, (int64_t)dim, r, r);
  HIP_TRY(hipGetLastError());
  return MECEFO_OK;
}

}  // extern "C"

// Internal host-side interfaces between the C ABI (api.hip) and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace mecefo {

enum Epilogue : int {
  EPI_STORE = 0,       // C0[row, col] = acc                          (activation dtype)
  EPI_SPLIT_F32 = 1,   // partial[split][row, col] = acc   (fp32 split-K partial, row stride ldc)
  EPI_GRAD = 2,        // C0[row, col] (+)= acc                       (gradient dtype, optional accumulate)
  EPI_SWIGLU_FWD = 3,  // dual: G=C0, Z=C1, A=C2 = silu(g)*z
  EPI_SWIGLU_BWD = 4,  // dual: dA read from C0; C0=dG, C1=dZ, C2=A
  EPI_ATTN_P = 5,      // C0[row, col] = col <= row ? exp(scale * acc - rowvec[row]) : 0   (softmax from saved logsumexp)
  EPI_ATTN_DS = 6,     // C0[row, col] = C0[row, col] * (acc - rowvec[row]) * scale         (softmax backward, in place on P)
};

enum CausalK : int {
  CAUSAL_NONE = 0,
  CAUSAL_K_FROM_M = 1,   // terms with k < first row of the tile are zero: start the K loop there
  CAUSAL_K_UPTO_M = 2,   // terms with k > last row of the tile are zero: stop the K loop there
  CAUSAL_TILE = 3,       // output tiles entirely above the diagonal need no K loop; whole 256-blocks above it are not written
};

// One matrix product C[M x N] = sum over K-segments of opA(A_s) * opB(B_s).
//   a_kcontig: A_s is [M x K] row-major (K contiguous), else [K x M] (M contiguous).
//   b_kcontig: B_s is [N x K] row-major (K contiguous), else [K x N] (N contiguous).
// Dual products (SwiGLU epilogues) use one segment and B[0], B[1] as the gate and up
// matrices; both products share A and every size.
struct GemmProblem {
  const void* A[3];
  const void* B[3];
  void* C[3];
  int64_t lda, ldb, ldc;
  int M, N, K;
  int nseg;        // 1 to 3 K segments (ignored for dual products)
  int pad_cols;    // SwiGLU epilogues: columns [N, pad_cols) of the outputs are set to zero
  int kpad_ok;     // K-contiguous operands: bytes between K and the next multiple of 8 are known to be zero
  int tile_begin;  // filled by the launcher
  int tiles_m, tiles_n;
  // Batched products (attention: one product per (sequence, head)): `batch` independent products of
  // identical size; product z = zo * batch_inner + zi reads A + zo*a_bo + zi*a_bi, etc.; all six
  // offsets are counted in operand elements (an fp32 output behind bf16 operands counts two per element).
  int batch, batch_inner;
  int64_t a_bo, a_bi, b_bo, b_bi, c_bo, c_bi;
  const float* rowvec;   // attention epilogues: fp32 per output row, product z starts at z * M
  float scale;           // attention epilogues
  int causal;            // CausalK
};

struct GemmLaunch {
  GemmProblem p[3];
  int nprob;
  bool a_kcontig, b_kcontig;
  int epi;          // Epilogue
  bool bf16;        // operand dtype (bf16 MFMA path) or fp32
  bool out_f32;     // EPI_GRAD: gradient buffer dtype is fp32 (else same as operands)
  int accumulate;   // EPI_GRAD
  int splits;       // EPI_SPLIT_F32: number of K splits (partials laid out [split][M x ldc] per problem)
  float* partial;   // EPI_SPLIT_F32: base of the partial buffer; problem i starts at partial_off[i]
  int64_t partial_off[3];
  bool force_large; // bf16: use the 256 x 256 direct-to-LDS configuration even for few tiles (split launches)
  uint32_t* clk;    // measurement: 64 (cycles, wall ticks) pairs written by the direct-to-LDS kernel, or NULL
};

// Records the thread-local error text returned by mecefo_last_error() and returns `status`.
int fail(int status, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

// Kernels that need more than 64 KiB of dynamic LDS must have the limit raised once per device (the
// attribute belongs to the kernel's code object on that device).  One instance per kernel; ensure()
// is cheap after the first call on a device and safe from several host threads.
struct LdsLimitOnce {
  std::atomic<uint64_t> done{0};      // bit i: raised on device i (devices above 63 set it every time)
  hipError_t ensure(const void* kern, int bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint64_t bit = dev < 64 ? (uint64_t)1 << dev : 0;
    if (bit && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
    e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && bit) done.fetch_or(bit, std::memory_order_release);
    return e;
  }
};

// Process-wide switches behind mecefo_set_option (tests and measurements; 0 = the library decides).
struct Options {
  std::atomic<int> tile{0};        // bf16 GEMM configuration: 1 = 128x128, 2 = 256x256 / 4 waves, 3 = 256x256 / 8 waves
                                   // register-staged, 4 = 256x256 / 8 waves direct-to-LDS
  std::atomic<int> attn_gemm{0};   // 1: attention through batched GEMM launches instead of the fused kernels
};
Options& options();

// Raise the dynamic-LDS limit of every kernel that needs it on the current device (what the first
// launch of each kernel would otherwise do): mecefo_init.
hipError_t prepare_gemm_bf16_nt();
hipError_t prepare_gemm_bf16_nn();
hipError_t prepare_gemm_bf16_tn();
hipError_t prepare_attention_fwd();
hipError_t prepare_attention_bwd();

// Returns hipSuccess or the launch error.  Only enqueues.
hipError_t launch_gemm(GemmLaunch& g, hipStream_t stream);
hipError_t launch_gemm_bf16(GemmLaunch& g, hipStream_t stream);
hipError_t launch_gemm_f32(GemmLaunch& g, hipStream_t stream);

// Elementwise / reduction kernels (elementwise.hip).  `bf16` selects the storage type.
hipError_t launch_rmsnorm_fwd(bool bf16, const void* H, int64_t ldh, const void* gamma, float eps,
                              void* U, int64_t ldu, float* rstd, int64_t b, int d, hipStream_t s);
// dX = dOut + rmsnorm_backward(dU); per-block partial sums of dgamma go to dg_partial [nblk x d].
hipError_t launch_rmsnorm_bwd(bool bf16, const void* dU, int64_t lddu, const void* H, int64_t ldh,
                              const float* rstd, const void* gamma, const void* dOut, int64_t lddo,
                              void* dX, int64_t lddx, float* dg_partial, int nblk, int64_t b, int d,
                              hipStream_t s);
int rmsnorm_bwd_blocks(int64_t b);
hipError_t launch_dgamma_reduce(const float* dg_partial, int nblk, int d, void* dgamma, bool out_f32,
                                bool bf16, int accumulate, hipStream_t s);
// dX = dOut + dU  (no-norm variant)
hipError_t launch_add(bool bf16, const void* a, int64_t lda, const void* bsrc, int64_t ldb, void* out,
                      int64_t ldo, int64_t rows, int cols, hipStream_t s);
// C[M x N] (activation dtype) = sum over splits of partial[split][M*N]
hipError_t launch_splitk_reduce(bool bf16, const float* partial, int splits, int64_t mn, void* C,
                                hipStream_t s);
// Standalone SwiGLU backward from saved G, Z: reads dA (in DG), writes DG=dG, DZ=dZ, AA=A; pads zeroed.
hipError_t launch_swiglu_bwd(bool bf16, const void* G, const void* Z, int64_t ldgz, void* DG, void* DZ,
                             void* AA, int64_t ldf, int64_t b, int f, int pad_cols, hipStream_t s);


// Attention helpers (attention.hip).
hipError_t launch_rope_tables(float* cs, float* sn, int seq, int dh, double theta, hipStream_t s);
// In-place rotary rotation of a token-major [tokens x heads*dh] tensor (inverse: the transpose, for gradients).
hipError_t launch_rope(bool bf16, void* X, int64_t ldx, const float* cs, const float* sn, int64_t tokens,
                       int seq, int heads, int dh, bool inverse, hipStream_t s);
// Causal row softmax of `nprod` fp32 score matrices [seq x lds]: P (storage type) and the log-sum-exp L.
hipError_t launch_softmax_rows(bool bf16, const float* S, int64_t lds, void* P, int64_t ldp, float* L, int nprod,
                               int seq, float scale, hipStream_t s);
// D[(sequence*heads + head)*seq + s] = sum over the head's columns of dO * O.
hipError_t launch_attn_rowdot(bool bf16, const void* dO, int64_t lddo, const void* O, int64_t ldo, float* D,
                              int64_t tokens, int seq, int heads, int dh, hipStream_t s);


// Fused causal attention backward for dK, dV (attention_bwd.hip): also writes dS = P (dP - D) scale
// (bf16, [batch*heads][seq x ldp], zeros above the diagonal inside the diagonal 256-blocks) for the
// batched dQ = dS K product that follows.  bf16, head dimension 64 or 128.
bool attn_bwd_fused_supported(bool bf16, int dh, int seq, int64_t ldp);
hipError_t launch_attn_bwd_kv(const void* Q, const void* K, const void* V, int64_t ld_in, const void* dO,
                              void* dK, void* dV, int64_t ld_ws, const float* L, const float* D, void* dS,
                              int64_t ldp, int batch, int seq, int heads, int dh, float scale, hipStream_t s);


// Fused causal attention forward: O = softmax(scale Q K^T) V and the row log-sum-exp L [batch*heads][seq],
// no score or probability buffer.  Q, K, V, O token-major with row stride ld (elements), head h at
// columns h*dh.  bf16, head dimension 64 or 128, ld a multiple of 8.
bool attn_fwd_fused_supported(bool bf16, int dh, int seq, int64_t ld);
hipError_t launch_attn_fwd(const void* Q, const void* K, const void* V, void* O, int64_t ld, float* L, int batch,
                           int seq, int heads, int dh, float scale, hipStream_t s);

}  // namespace mecefo

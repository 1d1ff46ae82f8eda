// fp32 GEMM for the fp32 storage path (small reference-precision config): plain FMA,
// 64 x 64 output tile per 256-thread workgroup, 4 x 4 outputs per thread, K staged through
// LDS in slices of 16.  Layouts, K segments, dual products and epilogues mirror the bf16
// core so that the host orchestration is identical for both dtypes.
#include "gemm_common.hip.h"

namespace mecefo {

namespace {
constexpr int FT = 64;   // tile edge
constexpr int FK = 16;   // K slice

template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const KArgs args, int a_kc, int b_kc) {
  constexpr bool DUAL = epi_is_dual(EPI);
  __shared__ float As[FK][FT + 4];
  __shared__ float Bs[DUAL ? 2 : 1][FK][FT + 4];
  const int t = threadIdx.x;
  const int tx = t & 15, ty = t >> 4;
  const int nblocks = args.total_tiles * args.splits;
  const TileCoord tc = map_tile(args, xcd_remap(blockIdx.x, nblocks));
  const GemmProblem p = product_view<4>(args.p[tc.prob], tc.z);
  const int m0 = tc.tm * FT, n0 = tc.tn * FT;
  if (causal_tile_unused(p, m0, n0, FT)) return;
  const int nseg = DUAL ? 1 : p.nseg;
  const int kt_per_seg = (p.K + FK - 1) / FK;
  const int kt_total = kt_per_seg * nseg;
  const int kt_chunk = __builtin_amdgcn_readfirstlane((kt_total + args.splits - 1) / args.splits);
  int kt_begin = tc.split * kt_chunk;
  int kt_end = min(kt_total, kt_begin + kt_chunk);
  causal_clip(p, m0, n0, FT, FK, kt_begin, kt_end);

  float acc[4][4] = {}, acc2[4][4] = {};
  for (int kt = kt_begin; kt < kt_end; ++kt) {
    const int seg = (kt >= kt_per_seg ? 1 : 0) + (kt >= 2 * kt_per_seg ? 1 : 0);
    const int k0 = (kt - seg * kt_per_seg) * FK;
    const float* A = (const float*)p.A[DUAL ? 0 : seg];
    // stage A: 64 x 16 elements, 4 per thread
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = t + i * 256;
      int m, k;
      if (a_kc) { k = e & 15; m = e >> 4; } else { m = e & 63; k = e >> 6; }
      const int gm = m0 + m, gk = k0 + k;
      float v = 0.f;
      if (gm < p.M && gk < p.K) v = a_kc ? A[(int64_t)gm * p.lda + gk] : A[(int64_t)gk * p.lda + gm];
      As[k][m] = v;
    }
#pragma unroll
    for (int w = 0; w < (DUAL ? 2 : 1); ++w) {
      const float* B = (const float*)p.B[DUAL ? w : seg];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int e = t + i * 256;
        int n, k;
        if (b_kc) { k = e & 15; n = e >> 4; } else { n = e & 63; k = e >> 6; }
        const int gn = n0 + n, gk = k0 + k;
        float v = 0.f;
        if (gn < p.N && gk < p.K) v = b_kc ? B[(int64_t)gn * p.ldb + gk] : B[(int64_t)gk * p.ldb + gn];
        Bs[w][k][n] = v;
      }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < FK; ++k) {
      float a[4], b[4], b2[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[0][k][tx * 4 + j];
      if constexpr (DUAL) {
#pragma unroll
        for (int j = 0; j < 4; ++j) b2[j] = Bs[1][k][tx * 4 + j];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
          if constexpr (DUAL) acc2[i][j] = fmaf(a[i], b2[j], acc2[i][j]);
        }
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
      epilogue_elem<EPI, float>(p, args, tc.prob, tc.split, m0 + ty * 4 + i, n0 + tx * 4 + j,
                                acc[i][j], acc2[i][j]);
}

template <int EPI>
hipError_t run_f32(GemmLaunch& g, hipStream_t stream) {
  KArgs a;
  a.clk = nullptr;
  a.nprob = g.nprob;
  int tiles = 0;
  for (int i = 0; i < 3; ++i) {
    a.p[i] = g.p[i < g.nprob ? i : 0];
    a.partial_off[i] = g.partial_off[i];
    if (i >= g.nprob) continue;
    GemmProblem& p = a.p[i];
    p.tiles_m = (p.M + FT - 1) / FT;
    p.tiles_n = (p.N + FT - 1) / FT;
    p.tile_begin = tiles;
    tiles += p.tiles_m * p.tiles_n * (p.batch > 1 ? p.batch : 1);
    if (p.nseg < 2) { p.A[1] = p.A[0]; if (!epi_is_dual(EPI)) p.B[1] = p.B[0]; }
    if (p.nseg < 3) { p.A[2] = p.A[0]; p.B[2] = p.B[0]; }
  }
  a.total_tiles = tiles;
  fill_schedule(a);
  a.splits = (EPI == EPI_SPLIT_F32 && g.splits > 1) ? g.splits : 1;
  a.accumulate = g.accumulate;
  a.out_f32 = 1;
  a.partial = g.partial;
  if (tiles == 0) return hipSuccess;
  hipLaunchKernelGGL(gemm_f32_kernel<EPI>, dim3(tiles * a.splits), dim3(256), 0, stream, a,
                     (int)g.a_kcontig, (int)g.b_kcontig);
  return hipGetLastError();
}
}  // namespace

hipError_t launch_gemm_f32(GemmLaunch& g, hipStream_t s) {
  switch (g.epi) {
    case EPI_STORE: return run_f32<EPI_STORE>(g, s);
    case EPI_SPLIT_F32: return run_f32<EPI_SPLIT_F32>(g, s);
    case EPI_GRAD: return run_f32<EPI_GRAD>(g, s);
    case EPI_SWIGLU_FWD: return run_f32<EPI_SWIGLU_FWD>(g, s);
    case EPI_SWIGLU_BWD: return run_f32<EPI_SWIGLU_BWD>(g, s);
    case EPI_ATTN_P: return run_f32<EPI_ATTN_P>(g, s);
    case EPI_ATTN_DS: return run_f32<EPI_ATTN_DS>(g, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace mecefo

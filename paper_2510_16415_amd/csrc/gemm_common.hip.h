// Device-side pieces shared by the bf16 MFMA GEMM and the fp32 GEMM: kernel argument
// block, block-id -> tile mapping, and the per-element epilogues.
#pragma once
#include "mecefo_internal.h"

namespace mecefo {

struct KArgs {
  GemmProblem p[3];
  int nprob;
  int total_tiles;   // sum over problems of tiles_m * tiles_n
  int splits;        // >= 1; block count = total_tiles * splits
  int accumulate;
  int out_f32;
  float* partial;
  int64_t partial_off[3];
};

// The hardware hands consecutive workgroup ids to the 8 XCDs round-robin.  Renumber so
// that each XCD works on one contiguous range of logical ids: neighbouring tiles (which
// share operand panels) then hit the same XCD-private L2.
__device__ inline int xcd_remap(int bid, int nblocks) {
  const int xcd = bid & 7, local = bid >> 3;
  const int q = nblocks >> 3, rem = nblocks & 7;
  return xcd * q + (xcd < rem ? xcd : rem) + local;
}

struct TileCoord { int prob, tm, tn, split; };

// Grouped ordering inside one problem: walk GROUP tile-rows together so that concurrently
// running blocks reuse both A panels (same tile-row) and B panels (same tile-column).
__device__ inline TileCoord map_tile(const KArgs& a, int bid) {
  TileCoord tc;
  tc.split = bid / a.total_tiles;
  int t = bid - tc.split * a.total_tiles;
  int pi = 0;
  if (a.nprob > 1 && t >= a.p[1].tile_begin) pi = 1;
  if (a.nprob > 2 && t >= a.p[2].tile_begin) pi = 2;
  tc.prob = pi;
  t -= a.p[pi].tile_begin;
  const int tiles_m = a.p[pi].tiles_m, tiles_n = a.p[pi].tiles_n;
  constexpr int GROUP = 8;
  const int gsize = GROUP * tiles_n;
  const int g = t / gsize;
  const int first_m = g * GROUP;
  const int gm = min(tiles_m - first_m, GROUP);
  const int tt = t - g * gsize;
  // Integer division runs on the vector ALU; tell the compiler the results are wave-uniform so
  // that everything derived from them (buffer offsets, loop bounds) stays in scalar registers.
  tc.tm = __builtin_amdgcn_readfirstlane(first_m + tt % gm);
  tc.tn = __builtin_amdgcn_readfirstlane(tt / gm);
  tc.prob = __builtin_amdgcn_readfirstlane(tc.prob);
  tc.split = __builtin_amdgcn_readfirstlane(tc.split);
  return tc;
}

template <typename T> __device__ inline float to_f32(T x) { return (float)x; }
template <typename T> __device__ inline T from_f32(float x) { return (T)x; }

// silu(g) and its derivative.  PRECISE (fp32 storage path) uses expf and a true divide;
// the bf16 path uses the hardware exp2/rcp approximations, far below bf16 resolution.
template <bool PRECISE> __device__ inline float sigmoid_f(float g) {
  if constexpr (PRECISE) {
    return 1.0f / (1.0f + expf(-g));
  } else {
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896341f * g));
  }
}

// One output element (single products) or one (gate, up) pair (dual products).
template <int EPI, typename T>
__device__ inline void epilogue_elem(const GemmProblem& p, const KArgs& a, int prob, int split,
                                     int row, int col, float v, float v2) {
  if (row >= p.M) return;
  if constexpr (EPI == EPI_STORE) {
    if (col < p.N) ((T*)p.C[0])[(int64_t)row * p.ldc + col] = from_f32<T>(v);
  } else if constexpr (EPI == EPI_SPLIT_F32) {
    if (col < p.N) {
      float* base = a.partial + a.partial_off[prob] + (int64_t)split * p.M * p.ldc;
      base[(int64_t)row * p.ldc + col] = v;
    }
  } else if constexpr (EPI == EPI_GRAD) {
    if (col < p.N) {
      const int64_t idx = (int64_t)row * p.ldc + col;
      if (a.out_f32) {
        float* c = (float*)p.C[0];
        c[idx] = a.accumulate ? c[idx] + v : v;
      } else {
        T* c = (T*)p.C[0];
        c[idx] = from_f32<T>(a.accumulate ? to_f32<T>(c[idx]) + v : v);
      }
    }
  } else if constexpr (EPI == EPI_SWIGLU_FWD) {
    const int64_t idx = (int64_t)row * p.ldc + col;
    if (col < p.N) {
      constexpr bool PRECISE = sizeof(T) == 4;
      const float sg = sigmoid_f<PRECISE>(v);
      if (p.C[0]) ((T*)p.C[0])[idx] = from_f32<T>(v);
      if (p.C[1]) ((T*)p.C[1])[idx] = from_f32<T>(v2);
      ((T*)p.C[2])[idx] = from_f32<T>(v * sg * v2);
    } else if (col < p.pad_cols) {
      if (p.C[0]) ((T*)p.C[0])[idx] = from_f32<T>(0.f);
      if (p.C[1]) ((T*)p.C[1])[idx] = from_f32<T>(0.f);
      ((T*)p.C[2])[idx] = from_f32<T>(0.f);
    }
  } else if constexpr (EPI == EPI_SWIGLU_BWD) {
    const int64_t idx = (int64_t)row * p.ldc + col;
    T* dg = (T*)p.C[0];
    T* dz = (T*)p.C[1];
    T* aa = (T*)p.C[2];
    if (col < p.N) {
      constexpr bool PRECISE = sizeof(T) == 4;
      const float da = to_f32<T>(dg[idx]);
      const float sg = sigmoid_f<PRECISE>(v);
      const float s = v * sg;
      aa[idx] = from_f32<T>(s * v2);
      dz[idx] = from_f32<T>(da * s);
      dg[idx] = from_f32<T>(da * v2 * (sg * (1.0f + v * (1.0f - sg))));
    } else if (col < p.pad_cols) {
      aa[idx] = from_f32<T>(0.f);
      dz[idx] = from_f32<T>(0.f);
      dg[idx] = from_f32<T>(0.f);
    }
  }
}

constexpr bool epi_is_dual(int epi) { return epi == EPI_SWIGLU_FWD || epi == EPI_SWIGLU_BWD; }

}  // namespace mecefo

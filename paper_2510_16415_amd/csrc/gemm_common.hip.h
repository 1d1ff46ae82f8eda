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
  int krot;          // direct-to-LDS kernel: tile row tm starts its K loop at stage tm % krot (0: off)
  uint32_t* clk;     // measurement (NULL otherwise): every 64th workgroup stores its shader-clock cycles and
                     // its 100 MHz wall ticks, pair number (workgroup / 64) % 64
  // Schedule (filled by fill_schedule): the logical tile order is eight consecutive segments, one
  // per XCD; segment x lists, heaviest problem first, the x-th eighth of every problem's tiles.
  int order[3];         // problem indices, most work per tile first
  int lstart[8][3];     // logical index at which (segment x, slot s) starts
  int tstart[8][3];     // first tile (within its problem) of that chunk
};

// Host side: tile_begin / tiles_m / tiles_n must be set.  Longest-processing-time-first inside each
// XCD segment keeps the tail of a grouped launch short when the problems differ in K.
inline void fill_schedule(KArgs& a) {
  int idx[3] = {0, 1, 2};
  auto work = [&](int i) { return i < a.nprob ? (int64_t)a.p[i].K * (a.p[i].nseg > 1 ? a.p[i].nseg : 1) : (int64_t)-1; };
  for (int i = 0; i < 3; ++i)
    for (int j = i + 1; j < 3; ++j)
      if (work(idx[j]) > work(idx[i])) { int t = idx[i]; idx[i] = idx[j]; idx[j] = t; }
  int l = 0;
  for (int s = 0; s < 3; ++s) a.order[s] = idx[s];
  for (int x = 0; x < 8; ++x)
    for (int s = 0; s < 3; ++s) {
      const int pi = idx[s];
      const int T = pi < a.nprob ? a.p[pi].tiles_m * a.p[pi].tiles_n * (a.p[pi].batch > 1 ? a.p[pi].batch : 1) : 0;
      const int b0 = (int)((int64_t)x * T / 8), b1 = (int)((int64_t)(x + 1) * T / 8);
      a.lstart[x][s] = l;
      a.tstart[x][s] = b0;
      l += b1 - b0;
    }
}

// The hardware hands consecutive workgroup ids to the 8 XCDs round-robin.  Renumber so
// that each XCD works on one contiguous range of logical ids: neighbouring tiles (which
// share operand panels) then hit the same XCD-private L2.
__device__ inline int xcd_remap(int bid, int nblocks) {
  const int xcd = bid & 7, local = bid >> 3;
  const int q = nblocks >> 3, rem = nblocks & 7;
  return xcd * q + (xcd < rem ? xcd : rem) + local;
}

struct TileCoord { int prob, tm, tn, split, z; };

// Grouped ordering inside one problem: walk GROUP tile-rows together so that concurrently
// running blocks reuse both A panels (same tile-row) and B panels (same tile-column).
__device__ inline TileCoord map_tile(const KArgs& a, int bid) {
  TileCoord tc;
  tc.split = __builtin_amdgcn_readfirstlane(bid / a.total_tiles);
  const int l = __builtin_amdgcn_readfirstlane(bid - tc.split * a.total_tiles);
  // find the (segment, slot) chunk that holds logical index l: the last one starting at or before l
  int x = 0, sl = 0;
#pragma unroll
  for (int xi = 0; xi < 8; ++xi)
#pragma unroll
    for (int si = 0; si < 3; ++si)
      if (a.lstart[xi][si] <= l) { x = xi; sl = si; }
  const int pi = a.order[sl];
  tc.prob = pi;
  int t = l - a.lstart[x][sl] + a.tstart[x][sl];
  const int tiles_m = a.p[pi].tiles_m, tiles_n = a.p[pi].tiles_n;
  tc.z = 0;
  if (a.p[pi].batch > 1) {   // batched products: all tiles of one product are consecutive
    const int per = tiles_m * tiles_n;
    tc.z = __builtin_amdgcn_readfirstlane(t / per);
    t -= tc.z * per;
  }
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

// The problem as seen by one product of a batch: operand, output and row-vector pointers moved to
// product z.  ESZ = bytes per operand / output element.
template <int ESZ>
__device__ inline GemmProblem product_view(const GemmProblem& p, int z) {
  GemmProblem q = p;
  if (p.batch > 1) {
    const int zo = __builtin_amdgcn_readfirstlane(z / p.batch_inner), zi = z - zo * p.batch_inner;
    const int64_t ao = ((int64_t)zo * p.a_bo + (int64_t)zi * p.a_bi) * ESZ;
    const int64_t bo = ((int64_t)zo * p.b_bo + (int64_t)zi * p.b_bi) * ESZ;
    const int64_t co = ((int64_t)zo * p.c_bo + (int64_t)zi * p.c_bi) * ESZ;
    q.A[0] = (const char*)p.A[0] + ao;
    q.B[0] = (const char*)p.B[0] + bo;
    q.C[0] = (char*)p.C[0] + co;
    if (p.rowvec) q.rowvec = p.rowvec + (int64_t)z * p.M;
  }
  return q;
}

// Softmax products (CAUSAL_TILE): output blocks of 256 x 256 that lie entirely above the diagonal
// are never read by the products that consume the probabilities (their K loops are clipped to the
// same 256-aligned blocks whatever tile size they run with), so tiles inside such a block are
// neither computed nor written.  Tiles above the diagonal but inside a diagonal block still write
// their zeros.  Uniform over the workgroup.
__device__ inline bool causal_tile_unused(const GemmProblem& p, int m0, int n0, int bm) {
  return p.causal == CAUSAL_TILE && (n0 >> 8) > ((m0 + bm - 1) >> 8);
}

// Causal attention products only touch part of K (or nothing): clip the stage range [lo, hi).
__device__ inline void causal_clip(const GemmProblem& p, int m0, int n0, int bm, int bk, int& lo, int& hi) {
  if (p.causal == CAUSAL_K_FROM_M) lo = max(lo, m0 / bk);
  else if (p.causal == CAUSAL_K_UPTO_M) hi = min(hi, (m0 + bm + bk - 1) / bk);
  else if (p.causal == CAUSAL_TILE && n0 > m0 + bm - 1) hi = lo;
  lo = __builtin_amdgcn_readfirstlane(lo);
  hi = __builtin_amdgcn_readfirstlane(hi);
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
  } else if constexpr (EPI == EPI_ATTN_P) {
    if (col < p.N) {
      constexpr bool PRECISE = sizeof(T) == 4;
      float pr = 0.f;
      if (col <= row) {
        const float x = v * p.scale - p.rowvec[row];
        pr = PRECISE ? expf(x) : __builtin_amdgcn_exp2f(1.44269504088896341f * x);
      }
      ((T*)p.C[0])[(int64_t)row * p.ldc + col] = from_f32<T>(pr);
    }
  } else if constexpr (EPI == EPI_ATTN_DS) {
    if (col < p.N) {
      T* c = (T*)p.C[0] + (int64_t)row * p.ldc + col;
      *c = from_f32<T>(to_f32<T>(*c) * (v - p.rowvec[row]) * p.scale);
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

// Four consecutive output columns of one row (bf16 storage path): 8-byte stores of bf16 and
// 16-byte stores of fp32 when the group lies inside the matrix, else element by element.
// Row strides are multiples of 8 elements and col0 of 4, so the vector accesses are aligned.
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;

__device__ inline bf16x4_t pack_bf16x4(float a, float b, float c, float d) {
  bf16x4_t o;
  o[0] = (__bf16)a; o[1] = (__bf16)b; o[2] = (__bf16)c; o[3] = (__bf16)d;
  return o;
}

// Eight consecutive output columns of one row (bf16 outputs, 16-byte accesses), used by the
// LDS-staged epilogue; falls back to single elements at the ragged right edge.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8s_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

__device__ inline bf16x8s_t pack_bf16x8(const float (&v)[8]) {
  bf16x8s_t o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (__bf16)v[e];
  return o;
}

template <int EPI>
__device__ inline void epilogue_vec8(const GemmProblem& p, const KArgs& a, int prob, int split, int row,
                                     int col0, const float (&v)[8], const float (&v2)[8]) {
  if (row >= p.M) return;
  if (col0 + 8 > p.N) {
#pragma unroll
    for (int e = 0; e < 8; ++e) epilogue_elem<EPI, __bf16>(p, a, prob, split, row, col0 + e, v[e], v2[e]);
    return;
  }
  const int64_t idx = (int64_t)row * p.ldc + col0;
  if constexpr (EPI == EPI_STORE) {
    *(bf16x8s_t*)((__bf16*)p.C[0] + idx) = pack_bf16x8(v);
  } else if constexpr (EPI == EPI_ATTN_P) {
    const float lse = p.rowvec[row];
    float o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e)
      o[e] = (col0 + e <= row) ? __builtin_amdgcn_exp2f(1.44269504088896341f * (v[e] * p.scale - lse)) : 0.f;
    *(bf16x8s_t*)((__bf16*)p.C[0] + idx) = pack_bf16x8(o);
  } else if constexpr (EPI == EPI_ATTN_DS) {
    bf16x8s_t* c = (bf16x8s_t*)((__bf16*)p.C[0] + idx);
    const bf16x8s_t pr = *c;
    const float dsum = p.rowvec[row];
    float o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (float)pr[e] * (v[e] - dsum) * p.scale;
    *c = pack_bf16x8(o);
  } else if constexpr (EPI == EPI_SPLIT_F32) {
    float* base = a.partial + a.partial_off[prob] + (int64_t)split * p.M * p.ldc + idx;
    const f32x4_t o0 = {v[0], v[1], v[2], v[3]}, o1 = {v[4], v[5], v[6], v[7]};
    *(f32x4_t*)base = o0;
    *(f32x4_t*)(base + 4) = o1;
  } else if constexpr (EPI == EPI_GRAD) {
    if (a.out_f32) {
      float* c = (float*)p.C[0] + idx;
      f32x4_t o0 = {v[0], v[1], v[2], v[3]}, o1 = {v[4], v[5], v[6], v[7]};
      if (a.accumulate) { o0 += *(const f32x4_t*)c; o1 += *(const f32x4_t*)(c + 4); }
      *(f32x4_t*)c = o0;
      *(f32x4_t*)(c + 4) = o1;
    } else {
      bf16x8s_t* c = (bf16x8s_t*)((__bf16*)p.C[0] + idx);
      float o[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = v[e];
      if (a.accumulate) {
        const bf16x8s_t old = *c;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] += (float)old[e];
      }
      *c = pack_bf16x8(o);
    }
  } else if constexpr (EPI == EPI_SWIGLU_FWD) {
    float av[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) av[e] = v[e] * sigmoid_f<false>(v[e]) * v2[e];
    if (p.C[0]) *(bf16x8s_t*)((__bf16*)p.C[0] + idx) = pack_bf16x8(v);
    if (p.C[1]) *(bf16x8s_t*)((__bf16*)p.C[1] + idx) = pack_bf16x8(v2);
    *(bf16x8s_t*)((__bf16*)p.C[2] + idx) = pack_bf16x8(av);
  } else if constexpr (EPI == EPI_SWIGLU_BWD) {
    bf16x8s_t* dg = (bf16x8s_t*)((__bf16*)p.C[0] + idx);
    const bf16x8s_t da8 = *dg;
    float oa[8], oz[8], og[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float da = (float)da8[e];
      const float sg = sigmoid_f<false>(v[e]);
      const float s = v[e] * sg;
      oa[e] = s * v2[e];
      oz[e] = da * s;
      og[e] = da * v2[e] * (sg * (1.0f + v[e] * (1.0f - sg)));
    }
    *(bf16x8s_t*)((__bf16*)p.C[2] + idx) = pack_bf16x8(oa);
    *(bf16x8s_t*)((__bf16*)p.C[1] + idx) = pack_bf16x8(oz);
    *dg = pack_bf16x8(og);
  }
}

template <int EPI>
__device__ inline void epilogue_vec4(const GemmProblem& p, const KArgs& a, int prob, int split, int row,
                                     int col0, const float (&v)[4], const float (&v2)[4]) {
  if (row >= p.M) return;
  if (col0 + 4 > p.N) {
#pragma unroll
    for (int e = 0; e < 4; ++e) epilogue_elem<EPI, __bf16>(p, a, prob, split, row, col0 + e, v[e], v2[e]);
    return;
  }
  const int64_t idx = (int64_t)row * p.ldc + col0;
  if constexpr (EPI == EPI_STORE) {
    *(bf16x4_t*)((__bf16*)p.C[0] + idx) = pack_bf16x4(v[0], v[1], v[2], v[3]);
  } else if constexpr (EPI == EPI_SPLIT_F32) {
    float* base = a.partial + a.partial_off[prob] + (int64_t)split * p.M * p.ldc;
    f32x4_t o = {v[0], v[1], v[2], v[3]};
    *(f32x4_t*)(base + idx) = o;
  } else if constexpr (EPI == EPI_GRAD) {
    if (a.out_f32) {
      f32x4_t* c = (f32x4_t*)((float*)p.C[0] + idx);
      f32x4_t o = {v[0], v[1], v[2], v[3]};
      if (a.accumulate) o += *c;
      *c = o;
    } else {
      bf16x4_t* c = (bf16x4_t*)((__bf16*)p.C[0] + idx);
      if (a.accumulate) {
        const bf16x4_t old = *c;
        *c = pack_bf16x4(v[0] + (float)old[0], v[1] + (float)old[1], v[2] + (float)old[2], v[3] + (float)old[3]);
      } else {
        *c = pack_bf16x4(v[0], v[1], v[2], v[3]);
      }
    }
  } else if constexpr (EPI == EPI_SWIGLU_FWD) {
    float av[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) av[e] = v[e] * sigmoid_f<false>(v[e]) * v2[e];
    if (p.C[0]) *(bf16x4_t*)((__bf16*)p.C[0] + idx) = pack_bf16x4(v[0], v[1], v[2], v[3]);
    if (p.C[1]) *(bf16x4_t*)((__bf16*)p.C[1] + idx) = pack_bf16x4(v2[0], v2[1], v2[2], v2[3]);
    *(bf16x4_t*)((__bf16*)p.C[2] + idx) = pack_bf16x4(av[0], av[1], av[2], av[3]);
  } else if constexpr (EPI == EPI_SWIGLU_BWD) {
    bf16x4_t* dg = (bf16x4_t*)((__bf16*)p.C[0] + idx);
    const bf16x4_t da4 = *dg;
    float oa[4], oz[4], og[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float da = (float)da4[e];
      const float sg = sigmoid_f<false>(v[e]);
      const float s = v[e] * sg;
      oa[e] = s * v2[e];
      oz[e] = da * s;
      og[e] = da * v2[e] * (sg * (1.0f + v[e] * (1.0f - sg)));
    }
    *(bf16x4_t*)((__bf16*)p.C[2] + idx) = pack_bf16x4(oa[0], oa[1], oa[2], oa[3]);
    *(bf16x4_t*)((__bf16*)p.C[1] + idx) = pack_bf16x4(oz[0], oz[1], oz[2], oz[3]);
    *dg = pack_bf16x4(og[0], og[1], og[2], og[3]);
  }
}

}  // namespace mecefo

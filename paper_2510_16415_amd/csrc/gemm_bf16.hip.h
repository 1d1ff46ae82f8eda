// bf16 MFMA GEMM core for gfx950 (CDNA4): C = opA(A) * opB(B) with fp32 accumulation.
//
// One workgroup of 256 threads (four 64-wide wavefronts, 2 x 2) computes a BM x BN tile
// with v_mfma_f32_32x32x16_bf16.  Operand tiles of BK = 64 are staged through LDS in a
// K-contiguous layout [rows][64] (128 bytes per row) whose 16-byte chunks are XOR-swizzled
// by row so that the ds_read_b128 of an MFMA operand (32 rows, one chunk) is free of bank
// conflicts.  Operands that are K-strided in memory (the token-contraction of the weight
// gradient, and weights used as [K x N]) are transposed in registers (v_perm_b32) on the
// way from global memory to LDS, so the inner loop is the same for every layout.
// Global loads are buffer loads: out-of-range rows / K-tail chunks are turned into zeros
// by pointing the lane outside the buffer, which costs no branch.
#pragma once
#include "gemm_common.hip.h"

namespace mecefo {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

constexpr uint32_t kOOB = 0x80000000u;   // byte offset beyond every buffer: load returns 0
constexpr int kBK = 64;                   // K elements per LDS stage
constexpr int kRowBytes = kBK * 2;        // 128

__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void* p) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, 0x7FFFFFFF, 0x00020000);
}

// Swizzle: physical 16-byte chunk = logical chunk ^ swz(row).  Distinct for 8 consecutive
// rows, and rows r, r+8 differ in the low bit, so 16 consecutive rows also spread over
// 256 bytes of banks.  It depends on row % 16 only, so adding a multiple of 32 rows (the
// next MFMA block of a wave) leaves it unchanged.
__device__ inline int swz(int row) { return (row ^ ((row >> 3) & 1)) & 7; }

template <int BM_, int BN_>
struct TileCfg {
  static constexpr int BM = BM_, BN = BN_;
  static constexpr int WM = BM / 2, WN = BN / 2;     // per-wave tile (2 x 2 waves)
  static constexpr int TM = WM / 32, TN = WN / 32;   // 32x32 MFMA blocks per wave
  static constexpr int A_BYTES = BM * kRowBytes, B_BYTES = BN * kRowBytes;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
};

// ---- global -> register -> LDS staging of one operand tile (R rows x 64 K) ------------
// K-contiguous source: thread t owns chunk c = t%8 of rows r0 + 32*i.
template <int R, bool DUAL>
struct LoaderKC {
  static constexpr int NV = R / 32;
  u32x4_t v[NV];
  uint32_t voff[NV];
  int c, r0;
  __device__ inline void init(int t, int row_base, int rows_total, int64_t ld) {
    c = t & 7;
    r0 = t >> 3;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int ii = DUAL ? (i % (NV / 2)) : i;
      const int row = row_base + ii * 32 + r0;
      voff[i] = row < rows_total ? (uint32_t)(((int64_t)row * ld + c * 8) * 2) : kOOB;
    }
  }
  // k0: first K index of this stage inside the segment; kend: segment length.
  __device__ inline void load(__amdgpu_buffer_rsrc_t r0s, __amdgpu_buffer_rsrc_t r1s, int k0, int kend) {
    const int kk = k0 + c * 8;
    const bool kvalid = kk < kend;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const uint32_t off = kvalid ? voff[i] : kOOB;
      v[i] = __builtin_amdgcn_raw_buffer_load_b128((DUAL && i >= NV / 2) ? r1s : r0s, off, k0 * 2, 0);
    }
    if (kvalid && kk + 8 > kend) {   // ragged K tail inside a 16-byte chunk: zero it
      const int nvalid = kend - kk;  // 1..7
#pragma unroll
      for (int i = 0; i < NV; ++i) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          uint32_t w = v[i][e];
          if (2 * e >= nvalid) w = 0;
          else if (2 * e + 1 >= nvalid) w &= 0xFFFFu;
          v[i][e] = w;
        }
      }
    }
  }
  __device__ inline void store(uint8_t* lds) const {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int row = i * 32 + r0;
      *(u32x4_t*)(lds + row * kRowBytes + ((c ^ swz(row)) << 4)) = v[i];
    }
  }
};

// K-strided source ([K x R], R contiguous): thread t owns an (KB k) x (8 rows) block,
// loads KB 16-byte vectors along R, transposes to 8 K-contiguous pieces of KB elements.
template <int R>
struct LoaderKS {
  static constexpr int KB = R / 32;          // 8 (R=256) or 4 (R=128)
  static constexpr int MG = R / 8;
  u32x4_t v[KB];
  uint32_t voff;
  uint32_t ldb2;                             // row stride in bytes
  int mg, kg;
  __device__ inline void init(int t, int row_base, int rows_total, int64_t ld) {
    mg = t % MG;
    kg = t / MG;
    const int m = row_base + mg * 8;
    ldb2 = (uint32_t)(ld * 2);
    voff = m < rows_total ? (uint32_t)(((int64_t)(kg * KB) * ld + m) * 2) : kOOB;
  }
  __device__ inline void load(__amdgpu_buffer_rsrc_t rs, __amdgpu_buffer_rsrc_t, int k0, int kend) {
    const uint32_t soff = (uint32_t)k0 * ldb2;
#pragma unroll
    for (int kk = 0; kk < KB; ++kk) {
      const bool kvalid = (k0 + kg * KB + kk) < kend;
      const uint32_t off = (kvalid && voff != kOOB) ? voff + kk * ldb2 : kOOB;
      v[kk] = __builtin_amdgcn_raw_buffer_load_b128(rs, off, soff, 0);
    }
  }
  __device__ inline void store(uint8_t* lds) const {
    // in: v[k][j] = (row 2j | row 2j+1 << 16) at K index k.  out for row i: K-contiguous.
#pragma unroll
    for (int j = 0; j < 4; ++j) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int row = mg * 8 + 2 * j + h;
        const uint32_t sel = h ? 0x07060302u : 0x05040100u;
        uint8_t* dst = lds + row * kRowBytes;
        if constexpr (KB == 8) {
          u32x4_t o;
#pragma unroll
          for (int q = 0; q < 4; ++q) o[q] = __builtin_amdgcn_perm(v[2 * q + 1][j], v[2 * q][j], sel);
          *(u32x4_t*)(dst + ((kg ^ swz(row)) << 4)) = o;
        } else {
          u32x2_t o;
#pragma unroll
          for (int q = 0; q < 2; ++q) o[q] = __builtin_amdgcn_perm(v[2 * q + 1][j], v[2 * q][j], sel);
          *(u32x2_t*)(dst + (((kg >> 1) ^ swz(row)) << 4) + ((kg & 1) << 3)) = o;
        }
      }
    }
  }
};

template <int R, bool KC, bool DUAL> struct LoaderSel { using type = LoaderKC<R, DUAL>; };
template <int R, bool DUAL> struct LoaderSel<R, false, DUAL> {
  static_assert(!DUAL, "dual products need K-contiguous B");
  using type = LoaderKS<R>;
};

template <class Cfg, bool AKC, bool BKC, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const KArgs args) {
  constexpr bool DUAL = epi_is_dual(EPI);
  constexpr int BM = Cfg::BM, BN = Cfg::BN, TM = Cfg::TM, TN = Cfg::TN;
  constexpr int BN_OUT = DUAL ? BN / 2 : BN;       // output columns covered per tile
  static_assert(!DUAL || (TN % 2 == 0), "dual tiles pair MFMA blocks");
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  const int nblocks = args.total_tiles * args.splits;
  const TileCoord tc = map_tile(args, xcd_remap(blockIdx.x, nblocks));
  const GemmProblem& p = args.p[tc.prob];
  const int m0 = tc.tm * BM, n0 = tc.tn * BN_OUT;

  // K range of this block, in stages of 64, over nseg segments each padded to a stage.
  const int nseg = DUAL ? 1 : p.nseg;
  const int kt_per_seg = (p.K + kBK - 1) / kBK;
  const int kt_total = kt_per_seg * nseg;
  const int kt_chunk = (kt_total + args.splits - 1) / args.splits;
  const int kt_begin = tc.split * kt_chunk;
  const int kt_end = min(kt_total, kt_begin + kt_chunk);

  typename LoaderSel<BM, AKC, false>::type la;
  typename LoaderSel<BN, BKC, DUAL>::type lb;
  la.init(t, m0, p.M, p.lda);
  lb.init(t, n0, p.N, p.ldb);
  const __amdgpu_buffer_rsrc_t ra0 = make_rsrc(p.A[0]);
  const __amdgpu_buffer_rsrc_t ra1 = make_rsrc(p.A[1]);
  const __amdgpu_buffer_rsrc_t rb0 = make_rsrc(p.B[0]);
  const __amdgpu_buffer_rsrc_t rb1 = make_rsrc(p.B[1]);

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // per-lane LDS read addresses: row = lane%32 (+ block offsets), chunk = 2*ks + lane/32
  const int lrow = lane & 31;
  const int a_row = wm * Cfg::WM + lrow;
  const int a_base = a_row * kRowBytes + ((((lane >> 5) ^ swz(a_row)) & 7) << 4);
  int b_rowbase[TN];
  int b_base[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    int row;
    if constexpr (DUAL) {
      const int jj = j % (TN / 2);
      row = (j >= TN / 2 ? BN / 2 : 0) + wn * (Cfg::WN / 2) + jj * 32 + lrow;
    } else {
      row = wn * Cfg::WN + j * 32 + lrow;
    }
    b_rowbase[j] = row;
    b_base[j] = row * kRowBytes + ((((lane >> 5) ^ swz(row)) & 7) << 4);
  }

  auto issue_loads = [&](int kt) {
    const int seg = kt / kt_per_seg;
    const int k0 = (kt - seg * kt_per_seg) * kBK;
    if (DUAL) {
      la.load(ra0, ra0, k0, p.K);
      lb.load(rb0, rb1, k0, p.K);
    } else {
      la.load(seg ? ra1 : ra0, ra0, k0, p.K);
      lb.load(seg ? rb1 : rb0, rb0, k0, p.K);
    }
  };

  if (kt_begin < kt_end) {
    issue_loads(kt_begin);
    la.store(smem);
    lb.store(smem + Cfg::A_BYTES);
    __syncthreads();
    for (int kt = kt_begin; kt < kt_end; ++kt) {
      const int cur = (kt - kt_begin) & 1;
      const uint8_t* sa = smem + cur * Cfg::STAGE_BYTES;
      const uint8_t* sb = sa + Cfg::A_BYTES;
      const bool more = kt + 1 < kt_end;
      if (more) issue_loads(kt + 1);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        bf16x8_t af[TM], bfr[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
          af[i] = *(const bf16x8_t*)(sa + (a_base ^ (ks << 5)) + i * 32 * kRowBytes);
#pragma unroll
        for (int j = 0; j < TN; ++j)
          bfr[j] = *(const bf16x8_t*)(sb + (b_base[j] ^ (ks << 5)));
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
      }
      if (more) {
        uint8_t* na = smem + (cur ^ 1) * Cfg::STAGE_BYTES;
        la.store(na);
        lb.store(na + Cfg::A_BYTES);
      }
      __syncthreads();
    }
  }

  // Epilogue.  Accumulator element e of a 32x32 block: row 8*(e/4) + 4*(lane/32) + e%4, col lane%32.
  (void)b_rowbase;
  const int row_w = m0 + wm * Cfg::WM + 4 * (lane >> 5);
  constexpr int TNO = DUAL ? TN / 2 : TN;
  const int col_w = n0 + wn * (DUAL ? Cfg::WN / 2 : Cfg::WN) + lrow;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TNO; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = row_w + i * 32 + 8 * (e >> 2) + (e & 3);
        const int col = col_w + j * 32;
        const float v = acc[i][j][e];
        const float v2 = DUAL ? acc[i][DUAL ? j + TN / 2 : j][e] : 0.f;
        epilogue_elem<EPI, __bf16>(p, args, tc.prob, tc.split, row, col, v, v2);
      }
}

}  // namespace mecefo

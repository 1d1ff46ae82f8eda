// bf16 MFMA GEMM core for gfx950 (CDNA4): C = opA(A) * opB(B) with fp32 accumulation.
//
// One workgroup (WAVES_M x WAVES_N 64-wide wavefronts) computes a BM x BN tile with
// v_mfma_f32_32x32x16_bf16.  Operand tiles of BK = 64 are staged through LDS in a
// K-contiguous layout [rows][64] (128 bytes per row) whose 16-byte chunks are XOR-swizzled
// by row so that the ds_read_b128 of an MFMA operand (32 rows, one chunk) is free of bank
// conflicts.  Operands that are K-strided in memory (the token-contraction of the weight
// gradient, and weights used as [K x N]) are transposed in registers (v_perm_b32) on the
// way from global memory to LDS, so the inner loop is the same for every layout.
// Global loads are buffer loads: out-of-range rows / K-tail chunks are turned into zeros
// by pointing the lane outside the buffer, which costs no branch.
//
// Pipeline per K stage: global loads of stage k+1 are issued first; the four K=16 sub-steps
// run MFMAs on register fragments while the fragments of the next sub-step are fetched from
// LDS; stage k+1 is written to the other LDS buffer before the last sub-step, whose MFMAs
// then cover the barrier and the first fragment fetch of the next stage.
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

// Wave-uniform choice between the base pointers of up to three K segments, pinned to scalar
// registers half by half (a select on descriptors is otherwise lowered to per-lane moves and
// every load that uses the result to a loop over lanes).
__device__ inline const void* select_base(int seg, const void* p0, const void* p1, const void* p2) {
  const uint64_t a = (uint64_t)(seg == 0 ? p0 : (seg == 1 ? p1 : p2));
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
  return (const void*)(((uint64_t)hi << 32) | lo);
}

// Swizzle: physical 16-byte chunk = logical chunk ^ swz(row).  Distinct for 8 consecutive
// rows, and rows r, r+8 differ in the low bit, so 16 consecutive rows also spread over
// 256 bytes of banks.  It depends on row % 16 only, so adding a multiple of 32 rows (the
// next MFMA block of a wave) leaves it unchanged.
__device__ inline int swz(int row) { return (row ^ ((row >> 3) & 1)) & 7; }

template <int BM_, int BN_, int WAVES_M_, int WAVES_N_>
struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, WAVES_M = WAVES_M_, WAVES_N = WAVES_N_;
  static constexpr int NT = 64 * WAVES_M * WAVES_N;   // threads per workgroup
  static constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;   // per-wave tile
  static constexpr int TM = WM / 32, TN = WN / 32;             // 32x32 MFMA blocks per wave
  static constexpr int A_BYTES = BM * kRowBytes, B_BYTES = BN * kRowBytes;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
};

// ---- global -> register -> LDS staging of one operand tile (R rows x 64 K) ------------
// K-contiguous source: thread t owns chunk c = t%8 of rows r0 + RP*i (RP = NT/8 rows per pass).
template <int R, int NT, bool DUAL>
struct LoaderKC {
  static constexpr int RP = NT / 8;
  static constexpr int NV = R / RP;
  static_assert(NV >= 1 && (!DUAL || NV % 2 == 0), "tile too small for this workgroup");
  u32x4_t v[NV];
  uint32_t voff[NV];
  int c, r0;
  __device__ inline void init(int t, int row_base, int rows_total, int64_t ld) {
    c = t & 7;
    r0 = t >> 3;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int ii = DUAL ? (i % (NV / 2)) : i;
      const int row = row_base + ii * RP + r0;
      voff[i] = row < rows_total ? (uint32_t)(((int64_t)row * ld + c * 8) * 2) : kOOB;
    }
  }
  // k0: first K index of this stage inside the segment; kend: segment length.
  // `tail` (wave-uniform) says that this stage holds the ragged end of K.
  __device__ inline void load(__amdgpu_buffer_rsrc_t r0s, __amdgpu_buffer_rsrc_t r1s, int k0, int kend,
                              bool tail) {
    const int kk = k0 + c * 8;
    if (!tail) {
#pragma unroll
      for (int i = 0; i < NV; ++i)
        v[i] = __builtin_amdgcn_raw_buffer_load_b128((DUAL && i >= NV / 2) ? r1s : r0s, voff[i], k0 * 2, 0);
      return;
    }
    const bool kvalid = kk < kend;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const uint32_t off = kvalid ? voff[i] : kOOB;
      v[i] = __builtin_amdgcn_raw_buffer_load_b128((DUAL && i >= NV / 2) ? r1s : r0s, off, k0 * 2, 0);
    }
    if (kvalid && kk + 8 > kend) {   // ragged K end inside a 16-byte chunk: zero the excess
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
      const int row = i * RP + r0;
      *(u32x4_t*)(lds + row * kRowBytes + ((c ^ swz(row)) << 4)) = v[i];
    }
  }
};

// K-strided source ([K x R], R contiguous): thread t owns a (KB k) x (8 rows) block,
// loads KB 16-byte vectors along R, transposes to 8 K-contiguous pieces of KB elements.
template <int R, int NT>
struct LoaderKS {
  static constexpr int MG = R / 8;             // 8-row groups
  static constexpr int KG = NT / MG;           // K groups
  static constexpr int KB = kBK / KG;          // K rows per thread: 8, 4 or 2
  static_assert(KB == 8 || KB == 4 || KB == 2, "unsupported tile / workgroup combination");
  u32x4_t v[KB];
  uint32_t voff;
  uint32_t ldb2;                               // row stride in bytes
  int mg, kg;
  __device__ inline void init(int t, int row_base, int rows_total, int64_t ld) {
    mg = t % MG;
    kg = t / MG;
    const int m = row_base + mg * 8;
    ldb2 = (uint32_t)(ld * 2);
    voff = m < rows_total ? (uint32_t)(((int64_t)(kg * KB) * ld + m) * 2) : kOOB;
  }
  __device__ inline void load(__amdgpu_buffer_rsrc_t rs, __amdgpu_buffer_rsrc_t, int k0, int kend, bool tail) {
    const uint32_t soff = (uint32_t)k0 * ldb2;
    if (!tail) {
#pragma unroll
      for (int kk = 0; kk < KB; ++kk)
        v[kk] = __builtin_amdgcn_raw_buffer_load_b128(rs, voff == kOOB ? kOOB : voff + kk * ldb2, soff, 0);
      return;
    }
#pragma unroll
    for (int kk = 0; kk < KB; ++kk) {
      const bool kvalid = (k0 + kg * KB + kk) < kend;
      const uint32_t off = (kvalid && voff != kOOB) ? voff + kk * ldb2 : kOOB;
      v[kk] = __builtin_amdgcn_raw_buffer_load_b128(rs, off, soff, 0);
    }
  }
  __device__ inline void store(uint8_t* lds) const {
    // in: v[k][j] = (row 2j | row 2j+1 << 16) at K index k.  out for each row: K-contiguous.
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
        } else if constexpr (KB == 4) {
          u32x2_t o;
#pragma unroll
          for (int q = 0; q < 2; ++q) o[q] = __builtin_amdgcn_perm(v[2 * q + 1][j], v[2 * q][j], sel);
          *(u32x2_t*)(dst + (((kg >> 1) ^ swz(row)) << 4) + ((kg & 1) << 3)) = o;
        } else {
          const uint32_t o = __builtin_amdgcn_perm(v[1][j], v[0][j], sel);
          *(uint32_t*)(dst + (((kg >> 2) ^ swz(row)) << 4) + ((kg & 3) << 2)) = o;
        }
      }
    }
  }
};

template <int R, int NT, bool KC, bool DUAL> struct LoaderSel { using type = LoaderKC<R, NT, DUAL>; };
template <int R, int NT, bool DUAL> struct LoaderSel<R, NT, false, DUAL> {
  static_assert(!DUAL, "dual products need K-contiguous B");
  using type = LoaderKS<R, NT>;
};

template <class Cfg, bool AKC, bool BKC, int EPI>
__global__ __launch_bounds__(Cfg::NT) void gemm_bf16_kernel(const KArgs args) {
  constexpr bool DUAL = epi_is_dual(EPI);
  // fp32 outputs (gradients, split-K partials): issue the MFMA with swapped operands so that a
  // lane holds four consecutive columns and stores 16 bytes; bf16 outputs keep the layout in
  // which a half-wave writes 32 consecutive columns of one row.
  constexpr bool SWAP = EPI == EPI_GRAD || EPI == EPI_SPLIT_F32;
  constexpr int BM = Cfg::BM, BN = Cfg::BN, TM = Cfg::TM, TN = Cfg::TN, NT = Cfg::NT;
  constexpr int BN_OUT = DUAL ? BN / 2 : BN;       // output columns covered per tile
  static_assert(!DUAL || (TN % 2 == 0), "dual tiles pair MFMA blocks");
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;

  const int nblocks = args.total_tiles * args.splits;
  const TileCoord tc = map_tile(args, xcd_remap(blockIdx.x, nblocks));
  const GemmProblem p = product_view<2>(args.p[tc.prob], tc.z);
  const int m0 = tc.tm * BM, n0 = tc.tn * BN_OUT;
  if (causal_tile_unused(p, m0, n0, BM)) return;

  // K range of this block, in stages of 64, over nseg segments each padded to a stage.
  const int nseg = DUAL ? 1 : p.nseg;
  const int K = p.K;
  const int kt_per_seg = (K + kBK - 1) / kBK;
  const int kt_total = kt_per_seg * nseg;
  const int kt_chunk = __builtin_amdgcn_readfirstlane((kt_total + args.splits - 1) / args.splits);
  int kt_begin = tc.split * kt_chunk;
  int kt_end = min(kt_total, kt_begin + kt_chunk);
  causal_clip(p, m0, n0, BM, kBK, kt_begin, kt_end);

  typename LoaderSel<BM, NT, AKC, false>::type la;
  typename LoaderSel<BN, NT, BKC, DUAL>::type lb;
  la.init(t, m0, p.M, p.lda);
  lb.init(t, n0, p.N, p.ldb);
  const __amdgpu_buffer_rsrc_t ra0 = make_rsrc(p.A[0]);
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
    b_base[j] = row * kRowBytes + ((((lane >> 5) ^ swz(row)) & 7) << 4);
  }

  auto issue_loads = [&](int kt) {
    const int seg = (kt >= kt_per_seg ? 1 : 0) + (kt >= 2 * kt_per_seg ? 1 : 0);
    const int k0 = (kt - seg * kt_per_seg) * kBK;
    const bool tail = k0 + kBK > K;
    if (DUAL) {
      la.load(ra0, ra0, k0, K, tail);
      lb.load(rb0, rb1, k0, K, tail);
    } else {
      la.load(make_rsrc(select_base(seg, p.A[0], p.A[1], p.A[2])), ra0, k0, K, tail);
      lb.load(make_rsrc(select_base(seg, p.B[0], p.B[1], p.B[2])), rb0, k0, K, tail);
    }
  };

  bf16x8_t af[2][TM], bfr[2][TN];
  auto fetch = [&](int slot, const uint8_t* sa, const uint8_t* sb, int ks) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
      af[slot][i] = *(const bf16x8_t*)(sa + (a_base ^ (ks << 5)) + i * 32 * kRowBytes);
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[slot][j] = *(const bf16x8_t*)(sb + (b_base[j] ^ (ks << 5)));
  };
  auto mma = [&](int slot) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = SWAP ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[slot][j], af[slot][i], acc[i][j], 0, 0, 0)
                          : __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[slot][i], bfr[slot][j], acc[i][j], 0, 0, 0);
  };

  if (kt_begin < kt_end) {
    issue_loads(kt_begin);
    la.store(smem);
    lb.store(smem + Cfg::A_BYTES);
    __syncthreads();
    fetch(0, smem, smem + Cfg::A_BYTES, 0);
    for (int kt = kt_begin; kt < kt_end; ++kt) {
      const int cur = (kt - kt_begin) & 1;
      const uint8_t* sa = smem + cur * Cfg::STAGE_BYTES;
      const uint8_t* sb = sa + Cfg::A_BYTES;
      uint8_t* na = smem + (cur ^ 1) * Cfg::STAGE_BYTES;
      const bool more = kt + 1 < kt_end;
      if (more) issue_loads(kt + 1);
      fetch(1, sa, sb, 1);
      mma(0);
      fetch(0, sa, sb, 2);
      mma(1);
      fetch(1, sa, sb, 3);
      mma(0);
      if (more) {
        la.store(na);
        lb.store(na + Cfg::A_BYTES);
      }
      __syncthreads();
      if (more) fetch(0, na, na + Cfg::A_BYTES, 0);
      mma(1);
    }
  }

  // Epilogue.  Accumulator element e of a 32x32 block: row 8*(e/4) + 4*(lane/32) + e%4, col lane%32.
  if constexpr (!SWAP) {
    const int row_w = m0 + wm * Cfg::WM + 4 * (lane >> 5);
    constexpr int TNO = DUAL ? TN / 2 : TN;
    const int col_w = n0 + wn * (DUAL ? Cfg::WN / 2 : Cfg::WN) + (lane & 31);
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
    return;
  }
  // Swapped operands: the B fragment was the MFMA's row operand, so a lane holds, for
  // block (i, j), output row lane%32 and the four consecutive columns 8*g + 4*(lane/32) + 0..3
  // in accumulator elements 4g..4g+3 (g = 0..3): stores are 8 or 16 bytes wide.
  const int row_w = m0 + wm * Cfg::WM + lrow;
  constexpr int TNO = DUAL ? TN / 2 : TN;
  const int col_w = n0 + wn * (DUAL ? Cfg::WN / 2 : Cfg::WN) + 4 * (lane >> 5);
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TNO; ++j)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        float v[4], v2[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          v[e] = acc[i][j][4 * g4 + e];
          v2[e] = DUAL ? acc[i][DUAL ? j + TN / 2 : j][4 * g4 + e] : 0.f;
        }
        epilogue_vec4<EPI>(p, args, tc.prob, tc.split, row_w + i * 32, col_w + j * 32 + 8 * g4, v, v2);
      }
}

}  // namespace mecefo

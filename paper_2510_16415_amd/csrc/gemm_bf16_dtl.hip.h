// bf16 MFMA GEMM for gfx950 with direct-to-LDS operand staging.
//
// Same tiling and inner loop as gemm_bf16.hip.h (256 x 256 x 64 stages, eight wavefronts of
// 64 x 128, v_mfma_f32_32x32x16_bf16), but the operand tiles never pass through registers:
// `buffer_load_dwordx4 ... lds` writes 1 KiB per wavefront instruction straight into LDS
// (lane i lands at base + 16 i), and a stage is refilled as soon as the barrier that ends
// its last use has passed, one full stage ahead of its first use.
//   * K-contiguous operands keep the XOR-swizzled [rows][64] layout: the swizzle is applied by
//     choosing which 16-byte chunk of the row each lane fetches.
//   * K-strided operands ([K x rows] in memory: weights used as [K x N], activations in the
//     token contraction) stay in their memory order [64 k][256 rows] in LDS and are transposed
//     on the way to the MFMA registers by ds_read_b64_tr_b16 (each 16-lane group turns four
//     k-rows of 16 elements into four K-consecutive values per lane); their 16-byte chunks are
//     XOR-swizzled by k so that the four k-rows of a group fall into different banks.
// Rows and K positions outside the matrices are fetched from outside the buffer (zeros).
// A ragged K inside a 16-byte chunk cannot be masked on this path: the host only selects it
// when K is a multiple of 8 or the bytes behind K are known to be zero.
#pragma once
#include "gemm_bf16.hip.h"

namespace mecefo {

typedef __attribute__((ext_vector_type(4))) short s16x4_t;

// Buffer resource as four scalar words: base address, stride 0, 2 GiB range, raw dword format.
__device__ inline u32x4_t make_rsrc_words(const void* p) {
  const uint64_t a = (uint64_t)p;
  u32x4_t r;
  r[0] = (uint32_t)a;
  r[1] = (uint32_t)(a >> 32) & 0xFFFFu;
  r[2] = 0x7FFFFFFFu;
  r[3] = 0x00020000u;
  return r;
}

__device__ inline uint32_t lds_address(const void* p) {
  return (uint32_t)(size_t)(__attribute__((address_space(3))) const uint8_t*)p;
}

// One wavefront-wide fill: lane i fetches 16 bytes at voff + soff and they land at lds_addr + 16 i.
// Written as inline assembly so that the compiler does not serialise later LDS reads of the other
// stage behind it; the kernel waits for these loads itself (wait_fills) before the stage barrier.
__device__ inline void fill_lds_16B(u32x4_t rsrc, uint32_t lds_addr, uint32_t voff, uint32_t soff) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :: "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}
__device__ inline void wait_fills() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// ---- direct-to-LDS fill of one operand tile (256 rows x 64 K = 32 KiB, 32 wave instructions) ----
template <int NT, bool DUAL>
struct DmaKC {   // K-contiguous source; wave instruction g covers rows 8g..8g+7 (128 bytes each)
  static constexpr int NW = NT / 64, NI = 32 / NW;
  uint32_t voff[NI];
  int c;       // logical 16-byte chunk this lane fetches (same for all its instructions)
  int w;
  __device__ inline void init(int lane, int wave, int row_base, int rows_total, int64_t ld) {
    w = wave;
    const int rsub = lane >> 3;
    // swz(row) for row = 8g + rsub, g = q*NW + w: depends on rsub and the parity of w only
    c = (lane & 7) ^ ((rsub ^ (w & 1)) & 7);
#pragma unroll
    for (int q = 0; q < NI; ++q) {
      const int row = (q * NW + w) * 8 + rsub;
      const int gr = row_base + (DUAL ? (row & 127) : row);
      voff[q] = gr < rows_total ? (uint32_t)(((int64_t)gr * ld + c * 8) * 2) : kOOB;
    }
  }
  __device__ inline void issue(u32x4_t r0, u32x4_t r1, uint32_t tile, int k0, int K, bool tail) const {
    const bool kvalid = !tail || (k0 + c * 8 < K);
#pragma unroll
    for (int q = 0; q < NI; ++q) {
      const uint32_t off = kvalid ? voff[q] : kOOB;
      fill_lds_16B((DUAL && q >= NI / 2) ? r1 : r0, tile + (q * NW + w) * 1024, off, (uint32_t)k0 * 2);
    }
  }
};

__device__ inline int ks_swz(int k) { return (k & 7) << 1; }   // XOR on the 16-byte chunk index

template <int NT>
struct DmaKS {   // K-strided source; wave instruction g covers k rows 2g, 2g+1 (512 bytes each)
  static constexpr int NW = NT / 64, NI = 32 / NW;
  uint32_t voff;      // lane offset for q = 0; instruction q adds 2*NW*q rows
  uint32_t ld2;
  int krow0;          // k row of this lane for q = 0
  int w;
  __device__ inline void init(int lane, int wave, int row_base, int rows_total, int64_t ld) {
    w = wave;
    krow0 = 2 * w + (lane >> 5);
    const int cm = (lane & 31) ^ ks_swz(krow0);     // rows 2*NW*q apart share k & 7 (NW = 8)
    const int m = row_base + cm * 8;
    ld2 = (uint32_t)(ld * 2);
    voff = m < rows_total ? (uint32_t)(((int64_t)krow0 * ld + m) * 2) : kOOB;
  }
  __device__ inline void issue(u32x4_t r0, u32x4_t, uint32_t tile, int k0, int K, bool tail) const {
    const uint32_t soff = (uint32_t)k0 * ld2;
#pragma unroll
    for (int q = 0; q < NI; ++q) {
      const bool kvalid = !tail || (k0 + krow0 + 2 * NW * q < K);
      const uint32_t off = (kvalid && voff != kOOB) ? voff + (uint32_t)(2 * NW * q) * ld2 : kOOB;
      fill_lds_16B(r0, tile + (q * NW + w) * 1024, off, soff);
    }
  }
};

template <int NT, bool KC, bool DUAL> struct DmaSel { using type = DmaKC<NT, DUAL>; };
template <int NT, bool DUAL> struct DmaSel<NT, false, DUAL> {
  static_assert(!DUAL, "dual products need K-contiguous B");
  using type = DmaKS<NT>;
};

// ---- MFMA operand fetch from LDS ------------------------------------------------------
// NB blocks of 32 rows.  K-contiguous tiles: one ds_read_b128 per block and K sub-step.
template <int NB>
struct FragKC {
  int base[NB];
  // rows[i]: first tile row of block i for this wave
  __device__ inline void init(int lane, const int (&rows)[NB]) {
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int row = rows[i] + (lane & 31);
      base[i] = row * kRowBytes + ((((lane >> 5) ^ swz(row)) & 7) << 4);
    }
  }
  __device__ inline void fetch(bf16x8_t (&f)[NB], const uint8_t* tile, int ks) const {
#pragma unroll
    for (int i = 0; i < NB; ++i) f[i] = *(const bf16x8_t*)(tile + (base[i] ^ (ks << 5)));
  }
};

// K-strided tiles ([64 k][256 rows], 512 bytes per k): two transposing 8-byte reads per block.
template <int NB>
struct FragKS {
  int base[NB][2];
  __device__ inline void init(int lane, const int (&rows)[NB]) {
    const int kq = (lane & 15) >> 2, hi = lane >> 5, b = (lane >> 4) & 1, q4 = lane & 3;
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int m = rows[i] + 16 * b + 4 * q4;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int k = 8 * hi + 4 * h + kq;
        base[i][h] = k * 512 + ((((m >> 3) ^ ks_swz(k)) & 31) << 4) + ((m & 7) << 1);
      }
    }
  }
  __device__ inline void fetch(bf16x8_t (&f)[NB], const uint8_t* tile, int ks) const {
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;
      const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(tile + base[i][0] + ks * 16 * 512));
      const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(tile + base[i][1] + ks * 16 * 512));
      typedef __attribute__((ext_vector_type(8))) short s16x8_t;
      const s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      f[i] = __builtin_bit_cast(bf16x8_t, v);
    }
  }
};

template <int NB, bool KC> struct FragSel { using type = FragKC<NB>; };
template <int NB> struct FragSel<NB, false> { using type = FragKS<NB>; };

template <class Cfg, bool AKC, bool BKC, int EPI>
__global__ __launch_bounds__(Cfg::NT) void gemm_bf16_dtl_kernel(const KArgs args) {
  constexpr bool DUAL = epi_is_dual(EPI);
  // fp32 outputs (gradients, split-K partials): issue the MFMA with swapped operands so that a
  // lane holds four consecutive columns and stores 16 bytes; bf16 outputs keep the layout in
  // which a half-wave writes 32 consecutive columns of one row.
  constexpr bool SWAP = EPI == EPI_GRAD || EPI == EPI_SPLIT_F32;
  constexpr int BM = Cfg::BM, BN = Cfg::BN, TM = Cfg::TM, TN = Cfg::TN, NT = Cfg::NT;
  static_assert(BM == 256 && BN == 256 && NT == 512, "direct-to-LDS path is built for 256x256 tiles, 8 waves");
  constexpr int BN_OUT = DUAL ? BN / 2 : BN;
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;

  const int nblocks = args.total_tiles * args.splits;
  const TileCoord tc = map_tile(args, xcd_remap(blockIdx.x, nblocks));
  const GemmProblem& p = args.p[tc.prob];
  const int m0 = tc.tm * BM, n0 = tc.tn * BN_OUT;

  const int nseg = DUAL ? 1 : p.nseg;
  const int K = p.K;
  const int kt_per_seg = (K + kBK - 1) / kBK;
  const int kt_total = kt_per_seg * nseg;
  const int kt_chunk = __builtin_amdgcn_readfirstlane((kt_total + args.splits - 1) / args.splits);
  const int kt_begin = tc.split * kt_chunk;
  const int kt_end = min(kt_total, kt_begin + kt_chunk);

  typename DmaSel<NT, AKC, false>::type da;
  typename DmaSel<NT, BKC, DUAL>::type db;
  da.init(lane, wave, m0, p.M, p.lda);
  db.init(lane, wave, n0, p.N, p.ldb);
  const u32x4_t ra0 = make_rsrc_words(p.A[0]);
  const u32x4_t ra1 = make_rsrc_words(p.A[1]);
  const u32x4_t rb0 = make_rsrc_words(p.B[0]);
  const u32x4_t rb1 = make_rsrc_words(p.B[1]);
  const uint32_t smem_addr = lds_address(smem);

  int a_rows[TM], b_rows[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) a_rows[i] = wm * Cfg::WM + i * 32;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    if constexpr (DUAL) b_rows[j] = (j >= TN / 2 ? BN / 2 : 0) + wn * (Cfg::WN / 2) + (j % (TN / 2)) * 32;
    else b_rows[j] = wn * Cfg::WN + j * 32;
  }
  typename FragSel<TM, AKC>::type fa;
  typename FragSel<TN, BKC>::type fb;
  fa.init(lane, a_rows);
  fb.init(lane, b_rows);

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  auto issue = [&](int kt, uint32_t stage) {
    const int seg = kt >= kt_per_seg ? 1 : 0;
    const int k0 = (kt - seg * kt_per_seg) * kBK;
    const bool tail = k0 + kBK > K;
    if (DUAL) {
      da.issue(ra0, ra0, stage, k0, K, tail);
      db.issue(rb0, rb1, stage + Cfg::A_BYTES, k0, K, tail);
    } else {
      da.issue(seg ? ra1 : ra0, ra0, stage, k0, K, tail);
      db.issue(seg ? rb1 : rb0, rb0, stage + Cfg::A_BYTES, k0, K, tail);
    }
  };

  bf16x8_t af[2][TM], bfr[2][TN];
  auto mma = [&](int slot) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = SWAP ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[slot][j], af[slot][i], acc[i][j], 0, 0, 0)
                          : __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[slot][i], bfr[slot][j], acc[i][j], 0, 0, 0);
  };

  if (kt_begin < kt_end) {
    issue(kt_begin, smem_addr);
    wait_fills();
    __syncthreads();
    if (kt_begin + 1 < kt_end) issue(kt_begin + 1, smem_addr + Cfg::STAGE_BYTES);
    fa.fetch(af[0], smem, 0);
    fb.fetch(bfr[0], smem + Cfg::A_BYTES, 0);
    for (int kt = kt_begin; kt < kt_end; ++kt) {
      const int cur = (kt - kt_begin) & 1;
      uint8_t* sc = smem + cur * Cfg::STAGE_BYTES;
      uint8_t* sn = smem + (cur ^ 1) * Cfg::STAGE_BYTES;
      fa.fetch(af[1], sc, 1);
      fb.fetch(bfr[1], sc + Cfg::A_BYTES, 1);
      mma(0);
      fa.fetch(af[0], sc, 2);
      fb.fetch(bfr[0], sc + Cfg::A_BYTES, 2);
      mma(1);
      fa.fetch(af[1], sc, 3);
      fb.fetch(bfr[1], sc + Cfg::A_BYTES, 3);
      mma(0);
      // Every fragment of stage `cur` is in registers and stage `cur^1` has been filling for a
      // whole stage: wait for both, then refill `cur` with the stage after next.
      wait_fills();
      __syncthreads();
      if (kt + 2 < kt_end) issue(kt + 2, smem_addr + cur * Cfg::STAGE_BYTES);
      if (kt + 1 < kt_end) {
        fa.fetch(af[0], sn, 0);
        fb.fetch(bfr[0], sn + Cfg::A_BYTES, 0);
      }
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
  const int lrow = lane & 31;
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

// bf16 MFMA GEMM for gfx950 with direct-to-LDS operand staging.
//
// Same tiling as gemm_bf16.hip.h (256 x 256 output tile, eight wavefronts of 64 x 128), with two
// differences.  The products run on v_mfma_f32_16x16x32_bf16: on Gaussian operands the matrix cores
// are power-limited, and this shape moves half the accumulator bytes per multiply-add of the 32x32x16
// one -- a bare MFMA loop on random operands sustains 2100 TFLOP/s at 2.1 GHz with it against 1860 at
// 1.83 GHz.  And the operand tiles never pass through registers:
// `buffer_load_dwordx4 ... lds` writes 1 KiB per wavefront instruction straight into LDS
// (lane i lands at base + 16 i).  K is cut into stages of BK (32 or 64) held in a ring of NS
// LDS buffers; a buffer is refilled as soon as the barrier that ends its last use has passed,
// NS - 1 stages ahead of its next use, and the kernel waits (vmcnt) only for the stage it is
// about to read, leaving the younger fills in flight.
//   * K-contiguous operands keep the XOR-swizzled [rows][64] layout: the swizzle is applied by
//     choosing which 16-byte chunk of the row each lane fetches.
//   * K-strided operands ([K x rows] in memory: weights used as [K x N], activations in the
//     token contraction) stay in their memory order [64 k][256 rows] in LDS and are transposed
//     on the way to the MFMA registers by ds_read_b64_tr_b16 (each 16-lane group turns four
//     k-rows of 16 elements into four K-consecutive values per lane); their 16-byte chunks are
//     XOR-swizzled by k so that the eight k-rows of a 32-lane pass fall into different banks.
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

// Wave-uniform choice between the descriptors of up to three K segments.  Only the base words
// differ; they are selected word by word and pinned to scalar registers (a vector-typed select is
// otherwise lowered to vector moves, which the fill instruction cannot take).
__device__ inline u32x4_t select_rsrc(int seg, const u32x4_t& r0, const u32x4_t& r1, const u32x4_t& r2) {
  u32x4_t r = r0;
  r[0] = __builtin_amdgcn_readfirstlane(seg == 0 ? r0[0] : (seg == 1 ? r1[0] : r2[0]));
  r[1] = __builtin_amdgcn_readfirstlane(seg == 0 ? r0[1] : (seg == 1 ? r1[1] : r2[1]));
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
// Wait until at most `stages_left` younger stages (FPS fill instructions each, per wave) are in flight.
template <int FPS>
__device__ inline void wait_fills_leave(int stages_left) {
  if (stages_left <= 0) asm volatile("s_waitcnt vmcnt(%0)" :: "n"(0) : "memory");
  else if (stages_left == 1) asm volatile("s_waitcnt vmcnt(%0)" :: "n"(FPS) : "memory");
  else if (stages_left == 2) asm volatile("s_waitcnt vmcnt(%0)" :: "n"(2 * FPS) : "memory");
  else asm volatile("s_waitcnt vmcnt(%0)" :: "n"(3 * FPS) : "memory");
}

// ---- direct-to-LDS fill of one operand tile (256 rows x BK) --------------------------------
// Swizzle of the K-contiguous layout [rows][BK]: physical 16-byte chunk = logical ^ kc_swz(row).
// A 16-byte read of the 16x16x32 operand (lane l: row l % 16, chunk l / 16 of the step) is served 16
// lanes per clock, and the lanes of a clock are eight rows at one chunk plus the other eight rows of
// the block at the neighbouring chunk (lanes 0-7 with 24-31, 8-15 with 16-23, and the same in the
// upper half-wave; found by measurement: SQ_LDS_BANK_CONFLICT).  Rows of equal parity share their half
// of the 64 banks; XORing row bits 1-2 into chunk bits 1-2 spreads the four rows of a parity over the
// even (or odd) chunks and leaves the other chunks to the neighbouring-chunk rows.
template <int BK> __device__ inline int kc_swz(int row) {
  if constexpr (BK == 64) return row & 6;                  // 8 chunks per 128-byte row
  else return ((row >> 1) ^ (row >> 3)) & 3;               // 4 chunks per 64-byte row
}

template <int BK, int NT, bool DUAL>
struct DmaKC {   // K-contiguous source; one wave instruction covers RPI consecutive rows
  static constexpr int ROWB = BK * 2, CH = ROWB / 16, RPI = 1024 / ROWB;
  static constexpr int NW = NT / 64, NI = (256 / RPI) / NW;
  static_assert(NI >= 1 && (!DUAL || NI % 2 == 0), "unsupported stage size");
  uint32_t voff[NI];
  int c;       // logical 16-byte chunk this lane fetches (the same for all its instructions)
  int w;
  __device__ inline void init(int lane, int wave, int row_base, int rows_total, int64_t ld) {
    w = wave;
    const int rsub = lane / CH;
    c = (lane % CH) ^ kc_swz<BK>(w * RPI + rsub);   // instructions q*NW + w differ by multiples of 64 rows
#pragma unroll
    for (int q = 0; q < NI; ++q) {
      const int row = (q * NW + w) * RPI + rsub;
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

__device__ inline int ks_swz(int k) { return ((k & 7) << 1) ^ (k & 8); }   // XOR on the 16-byte chunk index
// Physical 16-byte chunk of logical chunk c (0..31, eight columns each) in k row k, and back.  A
// transposing read takes, per pass of 32 lanes, 32 bytes (two chunks) of each of eight k rows: four
// consecutive ones and the four that lie eight further on (the two 16-lane groups of a pass hold
// neighbouring K groups of the 16x16x32 operand).  LDS serves 256 bytes per clock from 64 banks, so
// the 16 chunks of a pass must differ in their low four bits: bit 0 is the chunk of the pair, the k
// row fills bits 1-2 (XOR with its low bits) and bit 3 (XOR with k bits 2 and 3); the second chunk
// pair of a row (bit 1 of c) also goes to the other half of the banks.  The map is its own inverse.
__device__ inline int ks_fold(int c) { return c ^ ((c & 2) << 2); }
__device__ inline int ks_phys(int c, int k) { return (ks_fold(c) ^ ks_swz(k)) & 31; }
__device__ inline int ks_logical(int pos, int k) { return ks_fold((pos ^ ks_swz(k)) & 31); }

template <int BK, int NT>
struct DmaKS {   // K-strided source; wave instruction g covers k rows 2g, 2g+1 (512 bytes each)
  static constexpr int NW = NT / 64, NI = (BK / 2) / NW;
  static_assert(NI >= 1 && NW == 8, "unsupported stage size");
  uint32_t voff;      // lane offset for q = 0; instruction q adds 2*NW*q rows
  uint32_t ld2;
  int krow0;          // k row of this lane for q = 0
  int w;
  __device__ inline void init(int lane, int wave, int row_base, int rows_total, int64_t ld) {
    w = wave;
    krow0 = 2 * w + (lane >> 5);
    const int cm = ks_logical(lane & 31, krow0);     // rows 16 q apart share k & 7
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

template <int BK, int NT, bool KC, bool DUAL> struct DmaSel { using type = DmaKC<BK, NT, DUAL>; };
template <int BK, int NT, bool DUAL> struct DmaSel<BK, NT, false, DUAL> {
  static_assert(!DUAL, "dual products need K-contiguous B");
  using type = DmaKS<BK, NT>;
};

// ---- MFMA operand fetch from LDS ------------------------------------------------------
// Operands of v_mfma_f32_16x16x32_bf16: NB blocks of 16 rows; lane l holds row l % 16 and the eight
// K values 8 (l / 16) .. + 7 of a 32-K step.  K-contiguous tiles: one ds_read_b128 per block and step.
template <int BK, int NB>
struct FragKC {
  int base[NB];
  // rows[i]: first tile row of block i for this wave
  __device__ inline void init(int lane, const int (&rows)[NB]) {
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int row = rows[i] + (lane & 15);
      base[i] = row * (BK * 2) + (((lane >> 4) ^ kc_swz<BK>(row)) << 4);
    }
  }
  __device__ inline bf16x8_t fetch_one(int i, const uint8_t* tile, int step) const {
    return *(const bf16x8_t*)(tile + (base[i] ^ (step << 6)));
  }
};

// K-strided tiles ([BK k][256 rows], 512 bytes per k): two transposing 8-byte reads per block.  Within
// a 16-lane group source lane 4 kq + q4 supplies rows 4 q4 .. + 3 at k row kq; the read hands result
// lane i the four K-consecutive values of row i.
template <int BK, int NB>
struct FragKS {
  int base[NB][2];
  __device__ inline void init(int lane, const int (&rows)[NB]) {
    const int kq = (lane & 15) >> 2, g = lane >> 4, q4 = lane & 3;
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      const int m = rows[i] + 4 * q4;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int k = 8 * g + 4 * h + kq;
        base[i][h] = k * 512 + (ks_phys(m >> 3, k) << 4) + ((m & 7) << 1);
      }
    }
  }
  __device__ inline bf16x8_t fetch_one(int i, const uint8_t* tile, int step) const {
    typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(tile + base[i][0] + step * 32 * 512));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(tile + base[i][1] + step * 32 * 512));
    typedef __attribute__((ext_vector_type(8))) short s16x8_t;
    const s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, v);
  }
};

template <int BK, int NB, bool KC> struct FragSel { using type = FragKC<BK, NB>; };
template <int BK, int NB> struct FragSel<BK, NB, false> { using type = FragKS<BK, NB>; };

// Pipeline shape of the direct-to-LDS kernel: K elements per stage and number of LDS buffers.
template <int BK_, int NS_> struct DtlPipe {
  static constexpr int BK = BK_, NS = NS_;
  static constexpr int A_BYTES = 256 * BK * 2, STAGE_BYTES = 2 * A_BYTES;
  // per-wave LDS slice of the staged epilogue: 32 rows x (128 + 8) floats, or 2 x 32 x (64 + 8)
  static constexpr int EP_WAVE_BYTES = 2 * 32 * 72 * 4;
  static constexpr int LDS_BYTES = NS * STAGE_BYTES > 8 * EP_WAVE_BYTES ? NS * STAGE_BYTES : 8 * EP_WAVE_BYTES;
  static_assert(NS >= 2 && NS <= 4 && (BK == 32 || BK == 64) && LDS_BYTES <= 160 * 1024, "bad pipeline");
  static_assert(32 * 136 * 4 <= EP_WAVE_BYTES, "epilogue slice too small");
};

template <class Cfg, class Pipe, bool AKC, bool BKC, int EPI>
__global__ __launch_bounds__(Cfg::NT) void gemm_bf16_dtl_kernel(const KArgs args) {
  constexpr bool DUAL = epi_is_dual(EPI);
  constexpr int BM = Cfg::BM, BN = Cfg::BN, NT = Cfg::NT;
  constexpr int TM = Cfg::WM / 16, TN = Cfg::WN / 16;     // 16x16 MFMA blocks per wave
  constexpr int BK = Pipe::BK, NS = Pipe::NS, KS = BK / 32, FPS = BK / 8;
  constexpr int A_BYTES = Pipe::A_BYTES, STAGE = Pipe::STAGE_BYTES;
  static_assert(BM == 256 && BN == 256 && NT == 512, "direct-to-LDS path is built for 256x256 tiles, 8 waves");
  constexpr int BN_OUT = DUAL ? BN / 2 : BN;
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wave / Cfg::WAVES_N, wn = wave % Cfg::WAVES_N;

  const int nblocks = args.total_tiles * args.splits;
  // Measurement only: shader-clock cycles and constant-rate (100 MHz) ticks this workgroup takes.
  uint64_t clk_c0 = 0, clk_w0 = 0;
  if (args.clk) { clk_c0 = clock64(); clk_w0 = wall_clock64(); }
  const TileCoord tc = map_tile(args, xcd_remap(blockIdx.x, nblocks));
  const GemmProblem p = product_view<2>(args.p[tc.prob], tc.z);
  const int m0 = tc.tm * BM, n0 = tc.tn * BN_OUT;
  if (causal_tile_unused(p, m0, n0, BM)) return;

  const int nseg = DUAL ? 1 : p.nseg;
  const int K = p.K;
  const int kt_per_seg = (K + BK - 1) / BK;
  const int kt_total = kt_per_seg * nseg;
  const int kt_chunk = __builtin_amdgcn_readfirstlane((kt_total + args.splits - 1) / args.splits);
  int kt_begin = tc.split * kt_chunk;
  int kt_end = min(kt_total, kt_begin + kt_chunk);
  causal_clip(p, m0, n0, BM, BK, kt_begin, kt_end);

  typename DmaSel<BK, NT, AKC, false>::type da;
  typename DmaSel<BK, NT, BKC, DUAL>::type db;
  da.init(lane, wave, m0, p.M, p.lda);
  db.init(lane, wave, n0, p.N, p.ldb);
  const u32x4_t ra0 = make_rsrc_words(p.A[0]);
  const u32x4_t ra1 = make_rsrc_words(p.A[1]);
  const u32x4_t rb0 = make_rsrc_words(p.B[0]);
  const u32x4_t rb1 = make_rsrc_words(p.B[1]);
  const u32x4_t ra2 = make_rsrc_words(p.A[2]);
  const u32x4_t rb2 = make_rsrc_words(p.B[2]);
  const uint32_t smem_addr = lds_address(smem);

  int a_rows[TM], b_rows[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) a_rows[i] = wm * Cfg::WM + i * 16;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    if constexpr (DUAL) b_rows[j] = (j >= TN / 2 ? BN / 2 : 0) + wn * (Cfg::WN / 2) + (j % (TN / 2)) * 16;
    else b_rows[j] = wn * Cfg::WN + j * 16;
  }
  typename FragSel<BK, TM, AKC>::type fa;
  typename FragSel<BK, TN, BKC>::type fb;
  fa.init(lane, a_rows);
  fb.init(lane, b_rows);

  f32x4_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;

  auto issue = [&](int kt, uint32_t stage) {
    const int seg = (kt >= kt_per_seg ? 1 : 0) + (kt >= 2 * kt_per_seg ? 1 : 0);
    const int k0 = (kt - seg * kt_per_seg) * BK;
    const bool tail = k0 + BK > K;
    if (DUAL) {
      da.issue(ra0, ra0, stage, k0, K, tail);
      db.issue(rb0, rb1, stage + A_BYTES, k0, K, tail);
    } else {
      da.issue(select_rsrc(seg, ra0, ra1, ra2), ra0, stage, k0, K, tail);
      db.issue(select_rsrc(seg, rb0, rb1, rb2), rb0, stage + A_BYTES, k0, K, tail);
    }
  };

  // Fragments: A double-buffered by K step, B single-buffered -- a B block is reloaded for the next
  // step right behind the MFMAs of its column, the last use of its present contents.
  bf16x8_t af[2][TM], bfr[TN];
  static_assert(TM <= TN, "the A reloads ride on the first columns of the step");
  // One 32-K step: MFMAs column by column; behind column j the loads of the next step's B block j and
  // (for j < TM) A block j from `next`, step `ns`.  (Behind the very last step of the K loop these
  // loads fetch fragments nobody uses: cheaper than a branch per column.)
  auto step = [&](int cur, const uint8_t* next, int ns) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[cur][i], bfr[j], acc[i][j], 0, 0, 0);
      bfr[j] = fb.fetch_one(j, next + A_BYTES, ns);
      if (j < TM) af[cur ^ 1][j] = fa.fetch_one(j, next, ns);
    }
    // The scheduler's built-in pattern that alternates single MFMAs with single LDS reads.  Measured
    // against its other pattern, none, and an order pinned column by column (same box, alternating
    // runs): the large launches +4 to +9 %.
    __builtin_amdgcn_iglp_opt(1);
  };
  // The two waves that share a SIMD (w and w + 4) run the same instruction stream; a raised issue
  // priority for one of them keeps the pair slightly out of step, so that one tends to issue MFMAs
  // while the other waits on LDS.
  if (NT == 512 && wave >= 4) __builtin_amdgcn_s_setprio(1);
  const int nst = kt_end - kt_begin;
  // The (up to eight) tiles of a tile column run at the same time on one XCD and share their B panel.
  // Each starts its K loop at a different stage (rotation by the tile row, wrapping around), so that
  // they do not all ask L2 for the same lines at the same moment: the first request of a line then
  // misses and the others hit, instead of queueing behind the miss.  A rotation of one stage per tile
  // row keeps every shared line in use for at most eight stages, well inside the 4 MB L2 (larger
  // strides measured slower).  Measured on the 7B-shaped layer: recompute launch -3.5 %, the others
  // -1 % to 0.  The summation order over K depends on the tile row only, so reruns stay bit-equal.
  const int rot = args.krot > 0 && nst > 0 ? __builtin_amdgcn_readfirstlane((tc.tm % args.krot) % nst) : 0;
  auto kmap = [&](int i) {
    int k = kt_begin + i + rot;
    return k >= kt_end ? k - nst : k;
  };
  if (nst > 0) {
    // Fill every buffer of the ring, wait for the first stage only.
#pragma unroll
    for (int s = 0; s < NS; ++s)
      if (s < nst) issue(kmap(s), smem_addr + s * STAGE);
    wait_fills_leave<FPS>(min(NS, nst) - 1);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < TM; ++i) af[0][i] = fa.fetch_one(i, smem, 0);
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[j] = fb.fetch_one(j, smem + A_BYTES, 0);
    int buf = 0;
    static_assert(KS == 2, "two 32-K steps per stage");
    for (int kt = kt_begin; kt < kt_end; ++kt) {
      const uint8_t* sc = smem + buf * STAGE;
      const int nbuf = buf + 1 == NS ? 0 : buf + 1;
      step(0, sc, 1);
      // Every fragment of this stage is in registers or on its way.  Wait for the next stage only
      // (younger fills stay in flight), meet the other waves, then refill this buffer NS stages ahead.
      wait_fills_leave<FPS>(min(NS - 2, kt_end - kt - 2));
      __syncthreads();
      if (kt + NS < kt_end) issue(kmap(kt - kt_begin + NS), smem_addr + buf * STAGE);
      step(1, smem + nbuf * STAGE, 0);
      buf = nbuf;
    }
  }

  // Epilogue, staged through LDS so that global accesses are 16 bytes per lane and cover whole
  // rows (bf16: eight columns per access, fp32: two accesses of four).  Accumulator element e of a 16x16 block sits at row
  // 4*(lane/16) + e, column lane%16; each wave writes 32 rows of its sub-tile as fp32
  // into its own LDS slice (row stride RS floats, chosen so that the 16-lane groups hit
  // different banks), then reads rows back eight columns per lane.  The operand stages are
  // free at this point: the loop's last barrier followed every fragment fetch and every fill.
  {
    constexpr int TNO = DUAL ? TN / 2 : TN;
    constexpr int W = TNO * 16;                 // columns per matrix in this wave's sub-tile
    constexpr int RS = W + 4;                   // 4*RS % 64 == 16: the four row groups of a store, and neighbouring rows of a read, fall on different banks
    constexpr int MAT = 32 * RS;                // floats per staged matrix
    float* ep = (float*)(smem + wave * Pipe::EP_WAVE_BYTES);
    const int wr_off = (4 * (lane >> 4)) * RS + (lane & 15);
    constexpr int LPR = W / 8;                  // lanes per row when reading back
    constexpr int RPI = 64 / LPR;               // rows per read instruction
    const int rd_row = lane / LPR, rd_c8 = (lane % LPR) * 8;
    const int row_w = m0 + wm * Cfg::WM;
    const int col_w = n0 + wn * (DUAL ? Cfg::WN / 2 : Cfg::WN) + rd_c8;
#pragma unroll
    for (int i = 0; i < TM / 2; ++i) {        // 32 rows = two block rows at a time
#pragma unroll
      for (int ih = 0; ih < 2; ++ih)
#pragma unroll
        for (int j = 0; j < TNO; ++j)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int o = wr_off + (16 * ih + e) * RS + j * 16;
            ep[o] = acc[2 * i + ih][j][e];
            if constexpr (DUAL) ep[MAT + o] = acc[2 * i + ih][j + TN / 2][e];
          }
      // fp32 outputs: four columns per lane, so that one store instruction covers whole 512-byte row
      // pieces (with eight columns per lane each of the two 16-byte stores would fill every other
      // 16 bytes of its lines)
      if ((EPI == EPI_GRAD && args.out_f32) || EPI == EPI_SPLIT_F32) {
        constexpr int LPR4 = W / 4, RPI4 = 64 / LPR4;
        const int r4 = lane / LPR4, c4 = (lane % LPR4) * 4;
#pragma unroll
        for (int it = 0; it < 32 / RPI4; ++it) {
          const int rl = it * RPI4 + r4;
          const f32x4_t g = *(const f32x4_t*)(ep + rl * RS + c4);
          const float v4[4] = {g[0], g[1], g[2], g[3]}, z4[4] = {0.f, 0.f, 0.f, 0.f};
          epilogue_vec4<EPI>(p, args, tc.prob, tc.split, row_w + i * 32 + rl, col_w - rd_c8 + c4, v4, z4);
        }
        continue;
      }
#pragma unroll
      for (int it = 0; it < 32 / RPI; ++it) {
        const int rl = it * RPI + rd_row;
        const float* src = ep + rl * RS + rd_c8;
        float v[8], v2[8];
        const f32x4_t g0 = *(const f32x4_t*)src, g1 = *(const f32x4_t*)(src + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) { v[e] = g0[e]; v[4 + e] = g1[e]; v2[e] = 0.f; v2[4 + e] = 0.f; }
        if constexpr (DUAL) {
          const f32x4_t z0 = *(const f32x4_t*)(src + MAT), z1 = *(const f32x4_t*)(src + MAT + 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) { v2[e] = z0[e]; v2[4 + e] = z1[e]; }
        }
        epilogue_vec8<EPI>(p, args, tc.prob, tc.split, row_w + i * 32 + rl, col_w, v, v2);
      }
    }
  }
  if (args.clk && (blockIdx.x & 63) == 0 && t == 0) {
    uint32_t* o = args.clk + 2 * ((blockIdx.x >> 6) & 63);
    o[0] = (uint32_t)(clock64() - clk_c0);
    o[1] = (uint32_t)(wall_clock64() - clk_w0);
  }
}

}  // namespace mecefo

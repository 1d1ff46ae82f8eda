// Host-side launch helpers for the bf16 MFMA GEMM instantiations.
#pragma once
#include "gemm_bf16_dtl.hip.h"

namespace mecefo {

using CfgL4 = TileCfg<256, 256, 2, 2>;   // 4 waves x (128 x 128): fewest LDS reads per MFMA
using CfgL8 = TileCfg<256, 256, 4, 2>;   // 8 waves x (64 x 128): two waves per SIMD hide latency
using CfgS = TileCfg<128, 128, 2, 2>;    // small problems: 4 waves x (64 x 64), more blocks

inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// Total 256x256 tiles of a launch; below this many the 128x128 configuration is used.
inline int bf16_tiles(const GemmLaunch& g, int bm, int bn) {
  const bool dual = epi_is_dual(g.epi);
  int t = 0;
  for (int i = 0; i < g.nprob; ++i)
    t += cdiv(g.p[i].M, bm) * cdiv(g.p[i].N, dual ? bn / 2 : bn) * (g.p[i].batch > 1 ? g.p[i].batch : 1);
  return t;
}
// 256 x 256 tiles (direct-to-LDS kernel) when they give at least half of the 256 CUs a tile; a
// split-K launch counts its parts, provided each keeps eight or more K stages.  Below that the
// 128 x 128 configuration fills the chip better.
inline bool bf16_use_large(const GemmLaunch& g) {
  const int tl = bf16_tiles(g, 256, 256);
  if (tl >= 128) return true;
  if (g.epi == EPI_SPLIT_F32 && g.splits > 1) {
    int stages = 1 << 30;
    for (int i = 0; i < g.nprob; ++i) {
      const int st = cdiv(g.p[i].K, 64) * (g.p[i].nseg > 1 ? g.p[i].nseg : 1);
      if (st < stages) stages = st;
    }
    return tl * g.splits >= 128 && stages / g.splits >= 8;
  }
  return false;
}

// The direct-to-LDS kernel cannot mask a ragged K inside a 16-byte chunk.
inline bool bf16_dtl_ok(const GemmLaunch& g) {
  for (int i = 0; i < g.nprob; ++i)
    if ((g.a_kcontig || g.b_kcontig) && (g.p[i].K % 8) && !g.p[i].kpad_ok) return false;
  return true;
}

// 0: 128x128 / 4 waves, 1: 256x256 / 4 waves, 2: 256x256 / 8 waves (register staging),
// 3: 256x256 / 8 waves, direct-to-LDS, 2 x 64-K stages.  mecefo_set_option("tile", ...) forces one.
inline int bf16_tile_choice(const GemmLaunch& g) {
  int c = (bf16_use_large(g) || g.force_large) ? 3 : 0;
  const int forced = options().tile.load(std::memory_order_relaxed);
  if (forced >= 1 && forced <= 4) c = forced - 1;
  if (c >= 3 && !bf16_dtl_ok(g)) c = 2;
  return c;
}

// Two 64 KiB stages, refilled one stage ahead.  Measured alternatives that lost: four 32-K stages
// (64-byte row pieces double the L2 request count); rings of three buffers, symmetric or A2+B3 /
// A3+B2; a second barrier that lets two fills overlap; one operand staged through registers two
// stages ahead; line-touch prefetch of later stages (+8 %).  Fill latency is not what bounds the
// loop (a fills-only loop runs a stage in 0.9-1.3 us, the full loop gives it 1.4): LDS traffic of
// fills plus fragment reads and MFMA issue are both near a stage's length, and on Gaussian operands
// the matrix cores are power-limited.
using PipeA = DtlPipe<64, 2>;

struct NoPipe { static constexpr int LDS_BYTES = 0; };

// One kernel instantiation: its entry point, its dynamic LDS size and the once-per-device limit raise.
template <class Cfg, bool AKC, bool BKC, int EPI, class Pipe>
struct Bf16Kernel {
  static constexpr bool DTL = Pipe::LDS_BYTES > 0;
  static constexpr int LDS = DTL ? Pipe::LDS_BYTES : Cfg::LDS_BYTES;
  static auto entry() -> void (*)(const KArgs) {
    if constexpr (DTL) return gemm_bf16_dtl_kernel<Cfg, Pipe, AKC, BKC, EPI>;
    else return gemm_bf16_kernel<Cfg, AKC, BKC, EPI>;
  }
  static hipError_t prepare() {
    static LdsLimitOnce limit;
    return limit.ensure((const void*)entry(), LDS);
  }
};

template <class Cfg, bool AKC, bool BKC, int EPI, class Pipe = NoPipe>
hipError_t run_bf16(GemmLaunch& g, hipStream_t stream) {
  using Kern = Bf16Kernel<Cfg, AKC, BKC, EPI, Pipe>;
  constexpr int LDS = Kern::LDS;
  constexpr bool DUAL = epi_is_dual(EPI);
  KArgs a;
  a.nprob = g.nprob;
  int tiles = 0;
  for (int i = 0; i < 3; ++i) {
    a.p[i] = g.p[i < g.nprob ? i : 0];
    a.partial_off[i] = g.partial_off[i];
    if (i >= g.nprob) continue;
    GemmProblem& p = a.p[i];
    p.tiles_m = cdiv(p.M, Cfg::BM);
    p.tiles_n = cdiv(p.N, DUAL ? Cfg::BN / 2 : Cfg::BN);
    p.tile_begin = tiles;
    tiles += p.tiles_m * p.tiles_n * (p.batch > 1 ? p.batch : 1);
    if (p.nseg < 2) { p.A[1] = p.A[0]; if (!DUAL) p.B[1] = p.B[0]; }
    if (p.nseg < 3) { p.A[2] = p.A[0]; p.B[2] = p.B[0]; }
  }
  a.total_tiles = tiles;
  fill_schedule(a);
  a.splits = (EPI == EPI_SPLIT_F32 && g.splits > 1) ? g.splits : 1;
  a.accumulate = g.accumulate;
  a.out_f32 = g.out_f32;
  a.partial = g.partial;
  a.krot = 8;
  a.clk = g.clk;
  if (tiles == 0) return hipSuccess;
  const hipError_t e = Kern::prepare();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(Kern::entry(), dim3(tiles * a.splits), dim3(Cfg::NT), LDS, stream, a);
  return hipGetLastError();
}

// Limit raise for the four configurations of one (layout, epilogue) pair.
template <bool AKC, bool BKC, int EPI>
hipError_t prepare_bf16() {
  hipError_t e = Bf16Kernel<CfgS, AKC, BKC, EPI, NoPipe>::prepare();
  if (e == hipSuccess) e = Bf16Kernel<CfgL4, AKC, BKC, EPI, NoPipe>::prepare();
  if (e == hipSuccess) e = Bf16Kernel<CfgL8, AKC, BKC, EPI, NoPipe>::prepare();
  if (e == hipSuccess) e = Bf16Kernel<CfgL8, AKC, BKC, EPI, PipeA>::prepare();
  return e;
}

template <bool AKC, bool BKC, int EPI>
hipError_t run_bf16_auto(GemmLaunch& g, hipStream_t stream) {
  switch (bf16_tile_choice(g)) {
    case 1: return run_bf16<CfgL4, AKC, BKC, EPI>(g, stream);
    case 2: return run_bf16<CfgL8, AKC, BKC, EPI>(g, stream);
    case 3: return run_bf16<CfgL8, AKC, BKC, EPI, PipeA>(g, stream);
    default: return run_bf16<CfgS, AKC, BKC, EPI>(g, stream);
  }
}

hipError_t launch_gemm_bf16_nt(GemmLaunch& g, hipStream_t s);
hipError_t launch_gemm_bf16_nn(GemmLaunch& g, hipStream_t s);
hipError_t launch_gemm_bf16_tn(GemmLaunch& g, hipStream_t s);

}  // namespace mecefo

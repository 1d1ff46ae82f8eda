// Fused causal attention backward for the key/value side (standard-mode block backward, Alg. 3
// first branch): for one (sequence, head) and one block of 128 keys, a workgroup walks the query
// blocks at and below the diagonal and keeps everything between the two softmax products and the
// dK / dV accumulations in registers:
//     S  = Q_i K_j^T          P  = exp(scale S - L_i)       (causal mask)
//     dP = dO_i V_j^T         dS = P (dP - D_i) scale
//     dV_j += P^T dO_i        dK_j += dS^T Q_i
// Only dS goes to memory (bf16, [query x key] per product): dQ = dS K is then one batched GEMM on
// the GEMM core.  The probabilities are never materialised.
//
// Mapping to v_mfma_f32_32x32x16_bf16 (wave64): each of the four waves owns 32 keys.  Its K_j and
// V_j rows sit in registers as B operands for the whole walk.  S and dP come out with query rows
// along the accumulator elements and the wave's keys along the lanes, which is exactly the A
// operand of the two accumulations (keys along lanes, queries along K) once the K order of those
// MFMAs is taken as the accumulator's own row order: a lane of the lower half-wave holds rows
// 0-3 and 8-11 of every 16, the upper half rows 4-7 and 12-15, and the B operands (dO_i, Q_i, read
// from LDS with transposing reads) are fetched in that same order.  No LDS round trip for P or dS.
#include <math.h>

#include <type_traits>

#include "attention_tiles.hip.h"
#include "mecefo_internal.h"

namespace mecefo {
namespace {

constexpr int kBr = 64;     // queries per step
constexpr int kBc = 128;    // keys per workgroup (4 waves x 32)

struct AttnBwdArgs {
  const __bf16 *Q, *K, *V, *dO;     // token-major [tokens x ld*], head h at columns h*dh
  int64_t ldq, ldk, ldv, lddo;
  const float *L, *D;               // [nz][seq]
  __bf16* dS;                       // [nz][seq x ldp]
  int64_t ldp;
  __bf16 *dK, *dV;                  // token-major, row stride ldg
  int64_t ldg;
  int seq, heads, nz, nkb;
  float scale;
};

template <int DH>
__global__ __launch_bounds__(256) void attn_bwd_kv_kernel(const AttnBwdArgs a) {
  constexpr int RB = DH * 2;            // bytes per tile row
  constexpr int CH = RB / 16;           // 16-byte chunks per row
  constexpr int RPI = 64 / CH;          // tile rows per wave-wide fill instruction
  constexpr int TILE = kBr * RB;        // one [64 x DH] tile
  constexpr int FILLS = (kBr / RPI) / 4;   // fill instructions per wave and tile
  constexpr int KT = DH / 16;           // MFMA K steps over the head dimension
  constexpr int NB = DH / 32;           // 32-column blocks of dK / dV
  constexpr float kLog2e = 1.44269504088896341f;
  // LDS: two stages of (Q tile, dO tile), then L and D of the two stages
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];   // 4 * TILE + 4 * kBr * 4 bytes
  float* ld_stage = (float*)(smem + 4 * TILE);     // [stage][0: L, 1: D][64]

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int hi = lane >> 5, l32 = lane & 31;
  // heavy key blocks (small j: most query blocks below them) first
  const int j = __builtin_amdgcn_readfirstlane((int)blockIdx.x / a.nz);
  const int z = __builtin_amdgcn_readfirstlane((int)blockIdx.x - j * a.nz);
  const int bi = z / a.heads, h = z - bi * a.heads;
  const int seq = a.seq;
  const int k0 = j * kBc;                              // first key of the workgroup
  const int kw = k0 + 32 * wave;                       // first key of this wave
  const int64_t tok0 = (int64_t)bi * seq;              // first token of the sequence
  const __bf16* Qz = a.Q + tok0 * a.ldq + (int64_t)h * DH;
  const __bf16* dOz = a.dO + tok0 * a.lddo + (int64_t)h * DH;
  const float* Lz = a.L + (int64_t)z * seq;
  const float* Dz = a.D + (int64_t)z * seq;
  __bf16* dSz = a.dS + (int64_t)z * seq * a.ldp;

  // K and V rows of this wave as B operands: lane holds key kw + l32, head-dim 16 t + 8 hi .. + 7
  bf16x8_t kf[KT], vf[KT];
  {
    const int key = kw + l32;
    const bool ok = key < seq;
    const __bf16* kp = a.K + (tok0 + key) * a.ldk + (int64_t)h * DH + 8 * hi;
    const __bf16* vp = a.V + (tok0 + key) * a.ldv + (int64_t)h * DH + 8 * hi;
#pragma unroll
    for (int s = 0; s < KT; ++s) {
      bf16x8_t zero = {};
      kf[s] = ok ? *(const bf16x8_t*)(kp + 16 * s) : zero;
      vf[s] = ok ? *(const bf16x8_t*)(vp + 16 * s) : zero;
    }
  }

  f32x16_t dk[NB], dv[NB];
#pragma unroll
  for (int n = 0; n < NB; ++n)
#pragma unroll
    for (int e = 0; e < 16; ++e) { dk[n][e] = 0.f; dv[n][e] = 0.f; }

  // Query blocks: the consumer of dS reads whole 256 x 256 blocks on the diagonal, so rows from the
  // start of that block get zeros even where every query lies before the keys of this workgroup.
  const int q_zero_from = (k0 >> 8) << 8;
  const int qb_first = k0 / kBr;                       // first query block with a query >= k0
  const int qb_end = (seq + kBr - 1) / kBr;

  // zeros above the diagonal inside the diagonal block: rows [q_zero_from, k0), this wave's 32 keys
  for (int q = q_zero_from + hi; q < k0 && q < seq; q += 2) {
    const int key = kw + l32;
    if (key < seq) dSz[(int64_t)q * a.ldp + key] = (__bf16)0.f;
  }
  const u32x4_t rq = make_rsrc_words(Qz);
  const u32x4_t rdo = make_rsrc_words(dOz);
  const uint32_t smem_addr = lds_address(smem);
  // fill addressing: instruction f of this wave covers tile rows (4 f + wave) * RPI .. + RPI - 1
  const int frow = lane / CH, fpc = lane % CH;
  // L (times log2 e) and D of a query block: threads 0-63 carry L, 64-127 carry D.  The values of the
  // block after next are loaded into a register a whole step before they are written to LDS, so
  // that no wave ever waits on these loads.
  const int ld_which = t >> 6, ld_r = t & 63;
  auto load_ld = [&](int qb) -> float {
    float v = ld_which ? 0.f : INFINITY;      // rows behind the sequence: P = exp2(x - inf) = 0
    const int q = qb * kBr + ld_r;
    if (t < 2 * kBr && q < seq) v = ld_which ? Dz[q] : Lz[q] * kLog2e;
    return v;
  };
  auto put_ld = [&](int stage, float v) {
    if (t < 2 * kBr) ld_stage[(stage * 2 + ld_which) * kBr + ld_r] = v;
  };
  // per-lane parts of the fill offsets; the query block contributes a wave-uniform offset
  uint32_t fq_off[FILLS], fd_off[FILLS];
  int f_row[FILLS];
#pragma unroll
  for (int f = 0; f < FILLS; ++f) {
    const int row = (f * 4 + wave) * RPI + frow;
    const int c = fpc ^ tile_swz<DH>(row);
    f_row[f] = row;
    fq_off[f] = (uint32_t)(((int64_t)row * a.ldq + c * 8) * 2);
    fd_off[f] = (uint32_t)(((int64_t)row * a.lddo + c * 8) * 2);
  }
  auto issue = [&](int qb, int stage) {
    const int q0 = qb * kBr;
    const uint32_t sq = (uint32_t)((int64_t)q0 * a.ldq * 2), sd = (uint32_t)((int64_t)q0 * a.lddo * 2);
#pragma unroll
    for (int f = 0; f < FILLS; ++f) {
      const bool ok = q0 + f_row[f] < seq;
      const uint32_t lds_off = (uint32_t)(stage * 2 * TILE + (f * 4 + wave) * 1024);
      fill_lds_16B(rq, smem_addr + lds_off, ok ? fq_off[f] : kOOB, sq);
      fill_lds_16B(rdo, smem_addr + lds_off + TILE, ok ? fd_off[f] : kOOB, sd);
    }
  };

  // LDS read offsets, fixed for the whole walk.  A operands (rows = queries, K = head dim): row
  // 32 mb + l32, chunk 2 s + hi; the K step only flips chunk bits, so it is an XOR with s << 5.
  int a_off[2];
#pragma unroll
  for (int mb = 0; mb < 2; ++mb) {
    const int row = 32 * mb + l32;
    a_off[mb] = row * RB + ((hi ^ tile_swz<DH>(row)) << 4);
  }
  auto read_a = [&](const uint8_t* tile, int mb, int s) {
    return *(const bf16x8_t*)(tile + (a_off[mb] ^ (s << 5)));
  };
  // B operands of the accumulations (K = queries in accumulator order, N = head dim): 16 queries
  // 16 u .., columns 32 n ..; two transposing reads of four query rows each.  The column block n
  // flips chunk bits 2-3 (XOR with n << 6), the query group u is a constant row offset.
  const int kq = (lane & 15) >> 2, b16 = (lane >> 4) & 1, q4 = lane & 3;
  int bt_off[2][NB];
#pragma unroll
  for (int hh = 0; hh < 2; ++hh) {
    const int row = 4 * hi + 8 * hh + kq;
    const int base = row * RB + (((2 * b16 + (q4 >> 1)) ^ tile_swz<DH>(row)) << 4) + (q4 & 1) * 8;
#pragma unroll
    for (int n = 0; n < NB; ++n) bt_off[hh][n] = base ^ (n << 6);
  }
  auto read_bt = [&](const uint8_t* tile, int u, int n) {
    typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(tile + bt_off[0][n] + u * 16 * RB));
    const s16x4_t up = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(tile + bt_off[1][n] + u * 16 * RB));
    typedef __attribute__((ext_vector_type(8))) short s16x8_t;
    const s16x8_t v = __builtin_shufflevector(lo, up, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, v);
  };

  const float c1 = a.scale * kLog2e;
  const int key = kw + l32;
  // dS fragments double as the values to store: fragment u holds, for this lane's key, the query rows
  // 16 u + 4 hi + {0..3} and 16 u + 8 + 4 hi + {0..3}.  Stores are issued one step late, behind the next
  // step's fills, so that the wait at the top of a step finds them long complete.
  // One 2-byte buffer store per element: the row part of the offset is wave-uniform, and rows behind
  // the sequence (or lanes whose key is) fall outside the descriptor's range and are dropped.
  const __amdgpu_buffer_rsrc_t rds = __builtin_amdgcn_make_buffer_rsrc(dSz, 0, (int)((int64_t)seq * a.ldp * 2), 0x00020000);
  const uint32_t ldp2 = (uint32_t)(a.ldp * 2);
  const uint32_t ds_lane = key < seq ? (uint32_t)(key * 2) + (uint32_t)(4 * hi) * ldp2 : kOOB;
  auto store_ds = [&](int q0, const bf16x8_t (&f)[4]) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const u32x4_t w = __builtin_bit_cast(u32x4_t, f[u]);       // two bf16 values per word
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t row = (uint32_t)(q0 + 16 * u + 8 * (e >> 2) + (e & 3));    // + 4 hi, in ds_lane
        const uint32_t v = (e & 1) ? w[e >> 1] >> 16 : w[e >> 1];
        __builtin_amdgcn_raw_buffer_store_b16((short)v, rds, ds_lane + row * ldp2, 0, 0);
      }
    }
  };
  bf16x8_t pf[4], dsf[4];        // A operands of the accumulations: 16 queries each
  // One query block.  MASK: the block touches the diagonal or the end of the sequence (the only
  // blocks that need the causal / length comparison per element).
  auto step = [&](auto mask_tag, const uint8_t* tq, const uint8_t* tdo, const float* Ls, const float* Ds, int q0) {
    constexpr bool MASK = decltype(mask_tag)::value;
    f32x16_t s_acc[2], dp_acc[2];
    auto sdp = [&](int mb) {
#pragma unroll
      for (int e = 0; e < 16; ++e) { s_acc[mb][e] = 0.f; dp_acc[mb][e] = 0.f; }
      bf16x8_t qa[2], da[2];
      qa[0] = read_a(tq, mb, 0); da[0] = read_a(tdo, mb, 0);
#pragma unroll
      for (int s = 0; s < KT; ++s) {
        if (s + 1 < KT) { qa[(s + 1) & 1] = read_a(tq, mb, s + 1); da[(s + 1) & 1] = read_a(tdo, mb, s + 1); }
        s_acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[s & 1], kf[s], s_acc[mb], 0, 0, 0);
        dp_acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(da[s & 1], vf[s], dp_acc[mb], 0, 0, 0);
      }
    };
    auto softmax = [&](int mb) {
      float p[16], ds[16];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int rbase = 32 * mb + 8 * g + 4 * hi;            // four consecutive query rows
        const f32x4_t l4 = *(const f32x4_t*)(Ls + rbase);
        const f32x4_t d4 = *(const f32x4_t*)(Ds + rbase);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int e = 4 * g + r;
          float pe = __builtin_amdgcn_exp2f(s_acc[mb][e] * c1 - l4[r]);
          if constexpr (MASK) {
            const int q = q0 + rbase + r;
            pe = (key <= q && key < seq) ? pe : 0.f;
          }
          p[e] = pe;
          ds[e] = pe * (dp_acc[mb][e] - d4[r]) * a.scale;
        }
      }
#pragma unroll
      for (int u2 = 0; u2 < 2; ++u2) {
        bf16x8_t pv, dsv;
#pragma unroll
        for (int e = 0; e < 8; ++e) { pv[e] = (__bf16)p[8 * u2 + e]; dsv[e] = (__bf16)ds[8 * u2 + e]; }
        pf[2 * mb + u2] = pv;
        dsf[2 * mb + u2] = dsv;
      }
    };
    bf16x8_t bo[2][NB], bq[2][NB];    // [slot][n]: dO^T and Q^T fragments
    auto fetch_bt = [&](int slot, int u) {
#pragma unroll
      for (int n = 0; n < NB; ++n) { bo[slot][n] = read_bt(tdo, u, n); bq[slot][n] = read_bt(tq, u, n); }
    };
    auto acc = [&](int u) {
#pragma unroll
      for (int n = 0; n < NB; ++n) {
        dv[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf[u], bo[u & 1][n], dv[n], 0, 0, 0);
        dk[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dsf[u], bq[u & 1][n], dk[n], 0, 0, 0);
      }
    };
    sdp(0);
    sdp(1);
    fetch_bt(0, 0);       // in flight while the softmax arithmetic runs
    softmax(0);
    softmax(1);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (u + 1 < 4) fetch_bt((u + 1) & 1, u + 1);
      acc(u);
    }
  };
  if (qb_first < qb_end) {
    put_ld(0, load_ld(qb_first));
    float ld_next = load_ld(qb_first + 1);
    issue(qb_first, 0);
    for (int qb = qb_first; qb < qb_end; ++qb) {
      const int stage = (qb - qb_first) & 1;
      // wait for this stage's fills (issued one step ago), meet the other waves, prefetch the next
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      if (qb + 1 < qb_end) {
        put_ld(stage ^ 1, ld_next);
        issue(qb + 1, stage ^ 1);
        ld_next = load_ld(qb + 2);
      }
      if (qb > qb_first) store_ds((qb - 1) * kBr, dsf);
      const uint8_t* tq = smem + stage * 2 * TILE;
      const uint8_t* tdo = tq + TILE;
      const float* Ls = ld_stage + (stage * 2) * kBr;
      const float* Ds = Ls + kBr;
      const int q0 = qb * kBr;
      const bool need_mask = q0 < k0 + kBc || k0 + kBc > seq;
      if (need_mask) step(std::true_type{}, tq, tdo, Ls, Ds, q0);
      else step(std::false_type{}, tq, tdo, Ls, Ds, q0);
    }
    store_ds((qb_end - 1) * kBr, dsf);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  // dK, dV of this wave: accumulator rows are keys, lanes are head-dim columns
#pragma unroll
  for (int n = 0; n < NB; ++n)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int key = kw + 8 * (e >> 2) + 4 * hi + (e & 3);
      if (key < seq) {
        const int64_t off = (tok0 + key) * a.ldg + (int64_t)h * DH + 32 * n + l32;
        a.dK[off] = (__bf16)dk[n][e];
        a.dV[off] = (__bf16)dv[n][e];
      }
    }
}

}  // namespace

bool attn_bwd_fused_supported(bool bf16, int dh, int seq, int64_t ldp) {
  return bf16 && (dh == 64 || dh == 128) && seq >= 1 && ldp % 8 == 0;
}

// Q, K, V: caller tensors (row stride ld_in); dO, dK, dV: workspace tensors (row stride ld_ws).
static hipError_t attn_bwd_limit(int dh) {
  static LdsLimitOnce limit[2];
  void (*kern)(const AttnBwdArgs) = dh == 128 ? attn_bwd_kv_kernel<128> : attn_bwd_kv_kernel<64>;
  return limit[dh == 128].ensure((const void*)kern, 4 * kBr * dh * 2 + 4 * kBr * 4);
}
hipError_t prepare_attention_bwd() {
  const hipError_t e = attn_bwd_limit(64);
  return e != hipSuccess ? e : attn_bwd_limit(128);
}

hipError_t launch_attn_bwd_kv(const void* Q, const void* K, const void* V, int64_t ld_in, const void* dO,
                              void* dK, void* dV, int64_t ld_ws, const float* L, const float* D, void* dS,
                              int64_t ldp, int batch, int seq, int heads, int dh, float scale, hipStream_t s) {
  AttnBwdArgs a;
  a.Q = (const __bf16*)Q; a.K = (const __bf16*)K; a.V = (const __bf16*)V; a.dO = (const __bf16*)dO;
  a.ldq = a.ldk = a.ldv = ld_in; a.lddo = ld_ws;
  a.L = L; a.D = D; a.dS = (__bf16*)dS; a.ldp = ldp;
  a.dK = (__bf16*)dK; a.dV = (__bf16*)dV; a.ldg = ld_ws;
  a.seq = seq; a.heads = heads; a.nz = batch * heads; a.nkb = (seq + kBc - 1) / kBc;
  a.scale = scale;
  if (a.nz == 0 || seq == 0) return hipSuccess;
  const dim3 grid((unsigned)(a.nz * a.nkb));
  const int lds = 4 * kBr * dh * 2 + 4 * kBr * 4;
  void (*kern)(const AttnBwdArgs) = dh == 128 ? attn_bwd_kv_kernel<128> : attn_bwd_kv_kernel<64>;
  const hipError_t e = attn_bwd_limit(dh);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, grid, dim3(256), lds, s, a);
  return hipGetLastError();
}

}  // namespace mecefo

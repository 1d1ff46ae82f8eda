// Fused causal attention forward (block forward, Alg. 2): O = softmax(scale Q K^T) V and the row
// log-sum-exp L, without materialising scores or probabilities.  One workgroup per (sequence, head,
// block of 128 queries); each of its four waves owns 32 queries and walks the key blocks (64 keys) up
// to the diagonal with a running maximum and sum per query.
//
// MFMA mapping (v_mfma_f32_32x32x16_bf16, wave64): the scores are computed transposed,
// S^T = K_blk Q_w^T, with the wave's rotated Q rows register-resident as the B operand.  The
// accumulator then has keys along its elements and the wave's queries along the lanes, so that
//   * the softmax statistics of a query live in one lane (plus its partner 32 lanes away), and
//   * P^T in the accumulator is already the B operand of O^T += V^T P^T, with the K order of that MFMA
//     taken as the accumulator's row order (lower half-wave: rows 0-3, 8-11 of every 16; upper:
//     4-7, 12-15); V^T is fetched from the row-major LDS tile with transposing reads in that order.
// The output accumulator O^T has the head dimension along its elements and queries along lanes:
// rescaling by the running-maximum correction is one multiply per element with a per-lane factor.
#include <math.h>

#include "attention_tiles.hip.h"
#include "mecefo_internal.h"

namespace mecefo {
namespace {

constexpr int kFq = 128;    // queries per workgroup (4 waves x 32)
constexpr int kFk = 64;     // keys per step

struct AttnFwdArgs {
  const __bf16 *Q, *K, *V;     // token-major, row stride ld, head h at columns h*dh
  __bf16* O;
  int64_t ld;
  float* L;                    // [nz][seq]
  int seq, heads, nz, nqb;
  float scale;
};

template <int DH>
__global__ __launch_bounds__(256, 2) void attn_fwd_kernel(const AttnFwdArgs a) {
  constexpr int RB = DH * 2, CH = RB / 16, RPI = 64 / CH, TILE = kFk * RB;
  constexpr int FILLS = (kFk / RPI) / 4;
  constexpr int KT = DH / 16, NB = DH / 32;
  constexpr float kLog2e = 1.44269504088896341f, kLn2 = 0.69314718055994531f;
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];   // two stages of (K tile, V tile)

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int hi = lane >> 5, l32 = lane & 31;
  // late query blocks (most key blocks) first
  const int jq = __builtin_amdgcn_readfirstlane(a.nqb - 1 - (int)blockIdx.x / a.nz);
  const int z = __builtin_amdgcn_readfirstlane((int)blockIdx.x % a.nz);
  const int bi = z / a.heads, h = z - bi * a.heads;
  const int seq = a.seq;
  const int q0 = jq * kFq, qw = q0 + 32 * wave;
  const int64_t tok0 = (int64_t)bi * seq;
  const __bf16* Kz = a.K + tok0 * a.ld + (int64_t)h * DH;
  const __bf16* Vz = a.V + tok0 * a.ld + (int64_t)h * DH;

  // the wave's Q rows as B operands: lane holds query qw + l32, head-dim 16 s + 8 hi .. + 7
  const int q = qw + l32;
  bf16x8_t qf[KT];
  {
    const __bf16* qp = a.Q + (tok0 + q) * a.ld + (int64_t)h * DH + 8 * hi;
#pragma unroll
    for (int s = 0; s < KT; ++s) {
      bf16x8_t zero = {};
      qf[s] = q < seq ? *(const bf16x8_t*)(qp + 16 * s) : zero;
    }
  }
  f32x16_t ot[NB];
#pragma unroll
  for (int n = 0; n < NB; ++n)
#pragma unroll
    for (int e = 0; e < 16; ++e) ot[n][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;     // running maximum (log2 units) and sum of this lane's query

  const u32x4_t rk = make_rsrc_words(Kz);
  const u32x4_t rv = make_rsrc_words(Vz);
  const uint32_t smem_addr = lds_address(smem);
  const int frow = lane / CH, fpc = lane % CH;
  uint32_t f_off[FILLS];
  int f_row[FILLS];
#pragma unroll
  for (int f = 0; f < FILLS; ++f) {
    const int row = (f * 4 + wave) * RPI + frow;
    f_row[f] = row;
    f_off[f] = (uint32_t)(((int64_t)row * a.ld + (fpc ^ tile_swz<DH>(row)) * 8) * 2);
  }
  auto issue = [&](int kb, int stage) {
    const int k0 = kb * kFk;
    const uint32_t so = (uint32_t)((int64_t)k0 * a.ld * 2);
#pragma unroll
    for (int f = 0; f < FILLS; ++f) {
      const uint32_t off = k0 + f_row[f] < seq ? f_off[f] : kOOB;
      const uint32_t lds_off = (uint32_t)(stage * 2 * TILE + (f * 4 + wave) * 1024);
      fill_lds_16B(rk, smem_addr + lds_off, off, so);
      fill_lds_16B(rv, smem_addr + lds_off + TILE, off, so);
    }
  };
  // A operand of S^T (rows = keys, K = head dim): row 32 kb2 + l32, chunk 2 s + hi
  int a_off[2];
#pragma unroll
  for (int kb2 = 0; kb2 < 2; ++kb2) {
    const int row = 32 * kb2 + l32;
    a_off[kb2] = row * RB + ((hi ^ tile_swz<DH>(row)) << 4);
  }
  // A operand of O^T (rows = head dim, K = keys in accumulator order): transposing reads of V
  const int kq = (lane & 15) >> 2, b16 = (lane >> 4) & 1, q4 = lane & 3;
  int vt_off[2][NB];
#pragma unroll
  for (int hh = 0; hh < 2; ++hh) {
    const int row = 4 * hi + 8 * hh + kq;
    const int base = row * RB + (((2 * b16 + (q4 >> 1)) ^ tile_swz<DH>(row)) << 4) + (q4 & 1) * 8;
#pragma unroll
    for (int n = 0; n < NB; ++n) vt_off[hh][n] = base ^ (n << 6);
  }
  auto read_vt = [&](const uint8_t* tile, int u, int n) {
    typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(tile + vt_off[0][n] + u * 16 * RB));
    const s16x4_t up = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(tile + vt_off[1][n] + u * 16 * RB));
    typedef __attribute__((ext_vector_type(8))) short s16x8_t;
    const s16x8_t v = __builtin_shufflevector(lo, up, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, v);
  };

  const float c1 = a.scale * kLog2e;
  // key blocks 0 .. the one holding the last query of the workgroup
  const int last_q = min(q0 + kFq, seq) - 1;
  const int kb_end = last_q / kFk + 1;
  issue(0, 0);
  for (int kb = 0; kb < kb_end; ++kb) {
    const int stage = kb & 1;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (kb + 1 < kb_end) issue(kb + 1, stage ^ 1);
    const int k0 = kb * kFk;
    if (k0 > qw + 31) continue;            // every key of this block lies after the wave's queries
    const uint8_t* tk = smem + stage * 2 * TILE;
    const uint8_t* tv = tk + TILE;

    f32x16_t st[2];
#pragma unroll
    for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
      for (int e = 0; e < 16; ++e) st[kb2][e] = 0.f;
#pragma unroll
    for (int s = 0; s < KT; ++s)
#pragma unroll
      for (int kb2 = 0; kb2 < 2; ++kb2)
        st[kb2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8_t*)(tk + (a_off[kb2] ^ (s << 5))), qf[s], st[kb2], 0, 0, 0);

    // scores in log2 units with the causal / length mask; running maximum
    const bool need_mask = k0 + kFk - 1 > qw || k0 + kFk > seq;
    float x[2][16];
    float mloc = -INFINITY;
#pragma unroll
    for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        float v = st[kb2][e] * c1;
        if (need_mask) {
          const int key = k0 + 32 * kb2 + 8 * (e >> 2) + 4 * hi + (e & 3);
          if (key > q || key >= seq) v = -INFINITY;
        }
        x[kb2][e] = v;
        mloc = fmaxf(mloc, v);
      }
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64));
    const float m_new = fmaxf(m_run, mloc);
    // a query with no visible key so far (only rows behind the sequence) keeps everything at zero
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
    float lsum = 0.f;
    bf16x8_t pf[4];
#pragma unroll
    for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
      for (int u2 = 0; u2 < 2; ++u2) {
        bf16x8_t pv;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float pe = __builtin_amdgcn_exp2f(x[kb2][8 * u2 + e] - m_use);
          lsum += pe;
          pv[e] = (__bf16)pe;
        }
        pf[2 * kb2 + u2] = pv;
      }
    lsum += __shfl_xor(lsum, 32, 64);
    l_run = l_run * alpha + lsum;
    m_run = m_new;
#pragma unroll
    for (int n = 0; n < NB; ++n)
#pragma unroll
      for (int e = 0; e < 16; ++e) ot[n][e] *= alpha;
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int n = 0; n < NB; ++n)
        ot[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_vt(tv, u, n), pf[u], ot[n], 0, 0, 0);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  if (q < seq) {
    const float inv = l_run > 0.f ? 1.0f / l_run : 0.f;
    if (hi == 0) a.L[(int64_t)z * seq + q] = (m_run + log2f(l_run)) * kLn2;
    __bf16* op = a.O + (tok0 + q) * a.ld + (int64_t)h * DH;
#pragma unroll
    for (int n = 0; n < NB; ++n)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        // four consecutive head-dim values: rows 8 g + 4 hi + 0..3 of block n
        typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4v_t;
        bf16x4v_t o4;
#pragma unroll
        for (int r = 0; r < 4; ++r) o4[r] = (__bf16)(ot[n][4 * g + r] * inv);
        *(bf16x4v_t*)(op + 32 * n + 8 * g + 4 * hi) = o4;
      }
  }
}

}  // namespace

bool attn_fwd_fused_supported(bool bf16, int dh, int seq, int64_t ld) {
  return bf16 && (dh == 64 || dh == 128) && seq >= 1 && ld % 8 == 0;
}

// Q, K, V, O: token-major [batch*seq x ld], head h at columns h*dh; L [batch*heads*seq] fp32.
static hipError_t attn_fwd_limit(int dh) {
  static LdsLimitOnce limit[2];
  void (*kern)(const AttnFwdArgs) = dh == 128 ? attn_fwd_kernel<128> : attn_fwd_kernel<64>;
  return limit[dh == 128].ensure((const void*)kern, 4 * kFk * dh * 2);
}
hipError_t prepare_attention_fwd() {
  const hipError_t e = attn_fwd_limit(64);
  return e != hipSuccess ? e : attn_fwd_limit(128);
}

hipError_t launch_attn_fwd(const void* Q, const void* K, const void* V, void* O, int64_t ld, float* L, int batch,
                           int seq, int heads, int dh, float scale, hipStream_t s) {
  AttnFwdArgs a;
  a.Q = (const __bf16*)Q; a.K = (const __bf16*)K; a.V = (const __bf16*)V; a.O = (__bf16*)O;
  a.ld = ld; a.L = L;
  a.seq = seq; a.heads = heads; a.nz = batch * heads; a.nqb = (seq + kFq - 1) / kFq;
  a.scale = scale;
  if (a.nz == 0 || seq == 0) return hipSuccess;
  const int lds = 4 * kFk * dh * 2;
  void (*kern)(const AttnFwdArgs) = dh == 128 ? attn_fwd_kernel<128> : attn_fwd_kernel<64>;
  const hipError_t e = attn_fwd_limit(dh);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)(a.nz * a.nqb)), dim3(256), lds, s, a);
  return hipGetLastError();
}

}  // namespace mecefo

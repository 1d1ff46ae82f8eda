// C ABI of the degraded block backward: argument validation, workspace carving and the
// order in which the kernels are enqueued.  Every arithmetic step runs in the kernels.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "../../include/mecefo.h"
#include "gemm_bf16_launch.hip.h"
#include "mecefo_internal.h"

using namespace mecefo;

namespace mecefo {
hipError_t launch_gemm(GemmLaunch& g, hipStream_t s) {
  if (!g.bf16) return launch_gemm_f32(g, s);
  if (g.a_kcontig && g.b_kcontig) return launch_gemm_bf16_nt(g, s);
  if (g.a_kcontig && !g.b_kcontig) return launch_gemm_bf16_nn(g, s);
  if (!g.a_kcontig && !g.b_kcontig) return launch_gemm_bf16_tn(g, s);
  return hipErrorInvalidValue;
}
}  // namespace mecefo

namespace mecefo {
Options& options() {
  static Options o;
  return o;
}

thread_local char g_err[512] = "";

int fail(int st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}
}  // namespace mecefo

namespace {

// Status-typed front of mecefo::fail; a macro so that the compiler still checks the format string
// against the arguments at every call site.
#define fail(st, ...) ((mecefo_status_t)mecefo::fail((int)(st), __VA_ARGS__))

constexpr int64_t kMaxBytes = (int64_t)1 << 31;

inline int64_t up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

struct Ctx {
  const mecefo_ffn_desc_t* d;
  bool bf16;
  int esz;          // bytes per activation element
  int64_t b;
  int dm, ff;
  int64_t ldf;      // row stride of internal [b x f] buffers
  bool grad_f32;
};

mecefo_status_t check_desc(const mecefo_ffn_desc_t* d, Ctx* c) {
  if (!d) return fail(MECEFO_ERR_INVALID_ARG, "descriptor is NULL");
  if (d->dtype != MECEFO_F32 && d->dtype != MECEFO_BF16)
    return fail(MECEFO_ERR_INVALID_ARG, "dtype must be MECEFO_F32 or MECEFO_BF16");
  if (d->grad_dtype != MECEFO_F32 && d->grad_dtype != d->dtype)
    return fail(MECEFO_ERR_UNSUPPORTED, "grad_dtype must be MECEFO_F32 or equal to dtype");
  if (d->tokens < 0 || d->d_model < 1 || d->d_ff < 1)
    return fail(MECEFO_ERR_INVALID_ARG, "tokens >= 0, d_model >= 1, d_ff >= 1 required");
  if (d->ld_act_d < d->d_model || d->ld_act_f < d->d_ff || d->ld_w_fd < d->d_model || d->ld_w_df < d->d_ff)
    return fail(MECEFO_ERR_INVALID_ARG, "a row stride is smaller than the logical width");
  c->d = d;
  c->bf16 = d->dtype == MECEFO_BF16;
  c->esz = c->bf16 ? 2 : 4;
  c->b = d->tokens;
  c->dm = d->d_model;
  c->ff = d->d_ff;
  c->ldf = up(d->d_ff, 8);
  c->grad_f32 = d->grad_dtype == MECEFO_F32;
  if (c->bf16) {
    if (d->d_model % 8)
      return fail(MECEFO_ERR_UNSUPPORTED, "bf16 path needs d_model to be a multiple of 8 (got %d)", d->d_model);
    if (d->ld_act_d % 8 || d->ld_act_f % 8 || d->ld_w_fd % 8 || d->ld_w_df % 8)
      return fail(MECEFO_ERR_INVALID_ARG,
                  "bf16 path needs every row stride to be a multiple of 8 elements (pad d_ff=%d to %lld)",
                  d->d_ff, (long long)up(d->d_ff, 8));
  }
  const int64_t big = d->tokens * (d->ld_act_f > d->ld_act_d ? d->ld_act_f : d->ld_act_d);
  const int64_t wbig = (int64_t)d->d_ff * d->ld_w_fd > (int64_t)d->d_model * d->ld_w_df
                           ? (int64_t)d->d_ff * d->ld_w_fd : (int64_t)d->d_model * d->ld_w_df;
  if (big * c->esz >= kMaxBytes || wbig * 4 >= kMaxBytes)
    return fail(MECEFO_ERR_UNSUPPORTED, "a tensor reaches 2 GiB; split the token batch");
  return MECEFO_OK;
}

mecefo_status_t check_ptr(const Ctx& c, const void* p, const char* name, bool required = true) {
  if (!p) return required ? fail(MECEFO_ERR_INVALID_ARG, "%s is NULL", name) : MECEFO_OK;
  if (((uintptr_t)p) % (c.bf16 ? 16 : 4)) return fail(MECEFO_ERR_INVALID_ARG, "%s is not %d-byte aligned", name, c.bf16 ? 16 : 4);
  return MECEFO_OK;
}

// Bytes spanned by a [b x d_model] activation tensor with row stride ld.
size_t act_span(const Ctx& c, int64_t ld) { return c.b > 0 ? (size_t)(((c.b - 1) * ld + c.dm) * c.esz) : 0; }

// An output may coincide with an input it is allowed to overwrite (same pointer), or lie apart from it;
// a partial overlap would let the kernels read rows that are already overwritten.
mecefo_status_t check_alias(const void* out, const char* out_name, const void* in, const char* in_name, size_t bytes) {
  if (!out || !in || out == in || bytes == 0) return MECEFO_OK;
  const uintptr_t a = (uintptr_t)out, b = (uintptr_t)in;
  if (a < b + bytes && b < a + bytes)
    return fail(MECEFO_ERR_INVALID_ARG, "%s overlaps %s without being equal to it", out_name, in_name);
  return MECEFO_OK;
}

mecefo_status_t check_proj(const Ctx& c, const mecefo_proj_t& P, int dim, const char* name) {
  if (!P.P) return fail(MECEFO_ERR_INVALID_ARG, "projection %s is NULL", name);
  if (P.r < 1 || P.r > dim) return fail(MECEFO_ERR_INVALID_ARG, "projection %s: rank %d outside [1, %d]", name, P.r, dim);
  if (P.ld < P.r) return fail(MECEFO_ERR_INVALID_ARG, "projection %s: ld %lld < r %d", name, (long long)P.ld, P.r);
  if (c.bf16 && (P.ld % 8 || ((uintptr_t)P.P) % 16))
    return fail(MECEFO_ERR_INVALID_ARG, "projection %s: bf16 path needs ld %% 8 == 0 and a 16-byte aligned pointer", name);
  return MECEFO_OK;
}

#define TRY(x) do { mecefo_status_t st__ = (x); if (st__ != MECEFO_OK) return st__; } while (0)
#define HIP_TRY(x) do { hipError_t e__ = (x); if (e__ != hipSuccess) return fail(MECEFO_ERR_LAUNCH, "%s: %s", #x, hipGetErrorString(e__)); } while (0)

// ---- optional per-stage timing (measurement only) --------------------------------------
constexpr int kClkPairs = 64;      // (cycles, wall ticks) pairs per stage launch
struct Profiler {
  bool on = false;
  std::vector<hipEvent_t> ev;     // pairs (start, stop)
  std::vector<int> stage;
  size_t used = 0;                // events used
  uint32_t* clk = nullptr;        // device: [stage launches][kClkPairs][2], zero-filled by mecefo_profile_enable
  uint32_t* cur_clk = nullptr;    // slot of the stage that is being enqueued
  double mhz[MECEFO_STAGE_COUNT] = {};
} g_prof;

struct StageTimer {
  hipStream_t s;
  bool active;
  StageTimer(int stage, hipStream_t stream) : s(stream), active(false) {
    if (g_prof.on && g_prof.used + 2 <= g_prof.ev.size()) {
      active = true;
      g_prof.stage[g_prof.used / 2] = stage;
      g_prof.cur_clk = g_prof.clk ? g_prof.clk + (g_prof.used / 2) * kClkPairs * 2 : nullptr;
      (void)hipEventRecord(g_prof.ev[g_prof.used], s);
    }
  }
  ~StageTimer() {
    if (active) {
      (void)hipEventRecord(g_prof.ev[g_prof.used + 1], s);
      g_prof.used += 2;
      g_prof.cur_clk = nullptr;
    }
  }
};
#define STAGE(id, stream) StageTimer stage_timer__((id), (stream))

// ---- workspace ------------------------------------------------------------------------
struct Workspace {
  // offsets in bytes from the (256-byte aligned) workspace base
  size_t U, rstd, DG, DZ, AA, dU, T[3], C[3], partial, dgp, total;
  int splits;
  int64_t c_elems[3];
};

// Split count for the token contraction of Eq. (2): the outputs ([f x r], [d x r]) are small, so
// the long token dimension is cut to get enough workgroups for 256 CUs.
int choose_splits(const Ctx& c, const int64_t c_rows[3], const int r[3]) {
  int tiles_l = 0, tiles_s = 0, tiles_f = 0;
  for (int i = 0; i < 3; ++i) {
    if (r[i] <= 0) continue;
    tiles_l += cdiv((int)c_rows[i], 256) * cdiv(r[i], 256);
    tiles_s += cdiv((int)c_rows[i], 128) * cdiv(r[i], 128);
    tiles_f += cdiv((int)c_rows[i], 64) * cdiv(r[i], 64);
  }
  int tiles, ktiles, target;
  if (!c.bf16) { tiles = tiles_f; ktiles = cdiv((int)c.b, 16); target = 512; }
  else if (tiles_l >= 160) { tiles = tiles_l; ktiles = cdiv((int)c.b, 64); target = 256; }
  else {
    // Mid-size layers: 256 x 256 tiles on the direct-to-LDS kernel, cut along the tokens into just
    // enough parts for half the chip, beat 128 x 128 tiles as long as every part keeps eight K
    // stages (the launcher applies the same rule when it picks the tile configuration).
    ktiles = cdiv((int)c.b, 64);
    const int s_l = tiles_l > 0 ? cdiv(128, tiles_l) : 0;
    if (s_l >= 1 && s_l <= 16 && ktiles / s_l >= 8) return s_l;
    tiles = tiles_s; target = 512;
  }
  if (tiles == 0) return 1;
  int s = cdiv(target, tiles);
  const int smax = ktiles / 4 > 1 ? ktiles / 4 : 1;
  if (s > smax) s = smax;
  if (s > 16) s = 16;
  return s < 1 ? 1 : s;
}

// K splits for a launch that stores activation-dtype outputs but has too few 256 x 256 tiles to fill
// the chip (mid-size layers: dU = dG Wg + dZ Wu with a small d, the projections with a small r):
// the long contraction is cut so that about 256 workgroups exist, fp32 partials are summed in order.
constexpr int kMaxStoreSplits = 4;
int store_splits(bool bf16, int tiles_large, int min_stages) {
  if (!bf16 || tiles_large <= 0 || tiles_large >= 128 || min_stages < 32) return 1;
  int sp = cdiv(256, tiles_large);
  if (sp > min_stages / 8) sp = min_stages / 8;
  if (sp > kMaxStoreSplits) sp = kMaxStoreSplits;
  return sp < 1 ? 1 : sp;
}
int store_splits_du(const Ctx& c) {   // dU [b x d], two K segments of length f
  return store_splits(c.bf16, cdiv((int)c.b, 256) * cdiv(c.dm, 256), 2 * cdiv(c.ff, 64));
}
int store_splits_project(const Ctx& c, const int r[3], mecefo_side_t side) {   // T_i [b x r_i]
  int tiles = 0, stages = 0;
  for (int i = 0; i < 3; ++i) {
    if (r[i] <= 0) continue;
    tiles += cdiv((int)c.b, 256) * cdiv(r[i], 256);
    const int k = side == MECEFO_SIDE_INPUT ? (i < 2 ? c.dm : c.ff) : (i < 2 ? c.ff : c.dm);
    if (cdiv(k, 64) > stages) stages = cdiv(k, 64);      // the longest contraction sets the pace of the launch
  }
  if (tiles <= 0 || !c.bf16 || tiles >= 128 || stages < 16) return 1;
  // as many parts as fit the chip in one go, none shorter than four K stages of the longest problem
  int sp = 256 / tiles;
  if (sp > stages / 4) sp = stages / 4;
  if (sp > 8) sp = 8;
  return sp < 1 ? 1 : sp;
}

Workspace layout(const Ctx& c, const int r[3], mecefo_side_t side, int force_splits) {
  Workspace w;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += (size_t)up((int64_t)bytes, 256); return o; };
  const size_t act_d = (size_t)c.b * c.dm * c.esz, act_f = (size_t)c.b * c.ldf * c.esz;
  w.U = take(act_d);
  w.rstd = take((size_t)c.b * 4);
  w.DG = take(act_f);
  w.DZ = take(act_f);
  w.AA = take(act_f);
  w.dU = take(act_d);
  // C_i rows: SIDE_INPUT: gate/up -> f, down -> d (output dim); SIDE_OUTPUT: gate/up -> d, down -> f.
  int64_t c_rows[3];
  c_rows[0] = c_rows[1] = side == MECEFO_SIDE_INPUT ? c.ff : c.dm;
  c_rows[2] = side == MECEFO_SIDE_INPUT ? c.dm : c.ff;
  int64_t sum_c = 0;
  for (int i = 0; i < 3; ++i) {
    const int64_t rr = up(r[i] > 0 ? r[i] : 0, 8);
    w.T[i] = take((size_t)c.b * rr * c.esz);
    w.c_elems[i] = c_rows[i] * rr;
    w.C[i] = take((size_t)w.c_elems[i] * c.esz);
    sum_c += c_rows[i] * rr;
  }
  w.splits = force_splits > 0 ? force_splits : choose_splits(c, c_rows, r);
  // one partial buffer serves the launches that split K, one after the other on the stream
  size_t partial = w.splits > 1 ? (size_t)w.splits * sum_c * 4 : 0;
  const int sdu = store_splits_du(c), spr = store_splits_project(c, r, side);
  if (sdu > 1 && (size_t)sdu * c.b * c.dm * 4 > partial) partial = (size_t)sdu * c.b * c.dm * 4;
  if (spr > 1) {
    size_t t = 0;
    for (int i = 0; i < 3; ++i) t += (size_t)c.b * up(r[i] > 0 ? r[i] : 0, 8) * 4;
    if ((size_t)spr * t > partial) partial = (size_t)spr * t;
  }
  w.partial = take(partial);
  w.dgp = take((size_t)rmsnorm_bwd_blocks(c.b) * c.dm * 4);
  w.total = off + 256;   // slack for aligning the caller's base pointer
  return w;
}

struct Bufs { char* base; Workspace w; };

mecefo_status_t carve(const Ctx& c, const int r[3], mecefo_side_t side, void* ws, size_t ws_bytes, Bufs* out) {
  Workspace w = layout(c, r, side, 0);
  while (w.total > ws_bytes && w.splits > 1) w = layout(c, r, side, w.splits - 1);
  if (w.total > ws_bytes)
    return fail(MECEFO_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", ws_bytes, w.total);
  if (!ws) return fail(MECEFO_ERR_INVALID_ARG, "workspace is NULL");
  out->base = (char*)up((int64_t)(uintptr_t)ws, 256);
  out->w = w;
  return MECEFO_OK;
}

GemmLaunch new_launch(const Ctx& c, bool akc, bool bkc, int epi) {
  GemmLaunch g;
  memset(&g, 0, sizeof(g));
  g.a_kcontig = akc;
  g.b_kcontig = bkc;
  g.epi = epi;
  g.bf16 = c.bf16;
  g.out_f32 = c.grad_f32;
  g.splits = 1;
  g.clk = g_prof.cur_clk;
  return g;
}

GemmProblem prob(const void* A0, const void* A1, int64_t lda, const void* B0, const void* B1, int64_t ldb,
                 void* C0, void* C1, void* C2, int64_t ldc, int M, int N, int K, int nseg, int pad_cols = 0) {
  GemmProblem p;
  memset(&p, 0, sizeof(p));
  p.A[0] = A0; p.A[1] = A1 ? A1 : A0;
  p.B[0] = B0; p.B[1] = B1 ? B1 : B0;
  p.C[0] = C0; p.C[1] = C1; p.C[2] = C2;
  p.lda = lda; p.ldb = ldb; p.ldc = ldc;
  p.M = M; p.N = N; p.K = K; p.nseg = nseg; p.pad_cols = pad_cols;
  return p;
}

// A store launch into the library's own buffers (row stride == ldc of every problem), cut along K
// into `splits` parts when that fills the chip better.
mecefo_status_t launch_store_split(const Ctx& c, const Bufs& bf, GemmLaunch& g, int splits, hipStream_t s) {
  if (splits <= 1) {
    HIP_TRY(launch_gemm(g, s));
    return MECEFO_OK;
  }
  g.epi = EPI_SPLIT_F32;
  g.splits = splits;
  g.force_large = true;
  g.partial = (float*)(bf.base + bf.w.partial);
  void* C[3];
  int64_t poff = 0;
  for (int i = 0; i < g.nprob; ++i) {
    C[i] = g.p[i].C[0];
    g.partial_off[i] = poff;
    poff += (int64_t)splits * g.p[i].M * g.p[i].ldc;
  }
  HIP_TRY(launch_gemm(g, s));
  for (int i = 0; i < g.nprob; ++i)
    HIP_TRY(launch_splitk_reduce(c.bf16, g.partial + g.partial_off[i], splits, (int64_t)g.p[i].M * g.p[i].ldc, C[i], s));
  return MECEFO_OK;
}

// dA = dY Wd  ->  recompute G, Z from U and apply the SwiGLU backward in the epilogue
// (DG = dG, DZ = dZ, AA = A)  ->  dU = dG Wg + dZ Wu.   Sec. 3.3 (Rcomp) + exact Dgrad.
mecefo_status_t recompute_and_dgrad(const Ctx& c, const Bufs& bf, const void* U, int64_t ldu, const void* dY,
                                    int64_t lddy, const void* Wg, const void* Wu, const void* Wd,
                                    const void* Gsaved, const void* Zsaved, void* dU, int64_t lddu,
                                    hipStream_t s) {
  const mecefo_ffn_desc_t& d = *c.d;
  char* base = bf.base;
  void* DG = base + bf.w.DG; void* DZ = base + bf.w.DZ; void* AA = base + bf.w.AA;
  const int b = (int)c.b;
  if (b == 0) return MECEFO_OK;
  {  // dA = dY Wd   [b x f], K = d
    STAGE(MECEFO_STAGE_DGRAD_DOWN, s);
    GemmLaunch g = new_launch(c, true, false, EPI_STORE);
    g.nprob = 1;
    g.p[0] = prob(dY, nullptr, lddy, Wd, nullptr, d.ld_w_df, DG, nullptr, nullptr, c.ldf, b, c.ff, c.dm, 1);
    HIP_TRY(launch_gemm(g, s));
  }
  if (Gsaved) {
    STAGE(MECEFO_STAGE_SWIGLU_BWD, s);
    HIP_TRY(launch_swiglu_bwd(c.bf16, Gsaved, Zsaved, d.ld_act_f, DG, DZ, AA, c.ldf, c.b, c.ff, (int)c.ldf, s));
  } else {  // G = U Wg^T, Z = U Wu^T with the SwiGLU backward fused into the epilogue
    STAGE(MECEFO_STAGE_RECOMPUTE, s);
    GemmLaunch g = new_launch(c, true, true, EPI_SWIGLU_BWD);
    g.nprob = 1;
    g.p[0] = prob(U, nullptr, ldu, Wg, Wu, d.ld_w_fd, DG, DZ, AA, c.ldf, b, c.ff, c.dm, 1, (int)c.ldf);
    HIP_TRY(launch_gemm(g, s));
  }
  if (dU) {  // dU = dG Wg + dZ Wu   [b x d], two K segments of length f
    STAGE(MECEFO_STAGE_DGRAD_GATE_UP, s);
    GemmLaunch g = new_launch(c, true, false, EPI_STORE);
    g.nprob = 1;
    g.p[0] = prob(DG, DZ, c.ldf, Wg, Wu, d.ld_w_fd, dU, nullptr, nullptr, lddu, b, c.dm, c.ff, 2);
    g.p[0].kpad_ok = 1;   // DG / DZ padding columns were written as zeros; the weight rows are predicated exactly
    // K is only cut when dU is the workspace's own [b x d] buffer (the reduction writes whole rows)
    TRY(launch_store_split(c, bf, g, dU == base + bf.w.dU ? store_splits_du(c) : 1, s));
  }
  return MECEFO_OK;
}

// Eq. (2) for the three FFN matrices, each as project -> contract over tokens -> expand.
//   SIDE_INPUT : T = X P [b x r];  C = Gy^T T [m x r];  dW [m x n] = C P^T.
//   SIDE_OUTPUT: T = Gy P [b x r]; C = X^T T [n x r];   dW [m x n] = P C^T.
// gate: (Gy, X) = (dG, U); up: (dZ, U); down: (dY, A).
mecefo_status_t lowrank_wgrad(const Ctx& c, const Bufs& bf, const void* U, int64_t ldu, const void* dY,
                              int64_t lddy, const mecefo_proj_t P[3], mecefo_side_t side, void* dW[3],
                              int accumulate, hipStream_t s, int exact_mask = 0) {
  const mecefo_ffn_desc_t& d = *c.d;
  char* base = bf.base;
  const int b = (int)c.b;
  const void* Gy[3] = {base + bf.w.DG, base + bf.w.DZ, dY};
  const int64_t ldgy[3] = {c.ldf, c.ldf, lddy};
  const void* X[3] = {U, U, base + bf.w.AA};
  const int64_t ldx[3] = {ldu, ldu, c.ldf};
  const int m_out[3] = {c.ff, c.ff, c.dm};   // rows of dW
  const int n_in[3] = {c.dm, c.dm, c.ff};    // cols of dW
  const int64_t lddw[3] = {d.ld_w_fd, d.ld_w_fd, d.ld_w_df};
  const bool in = side == MECEFO_SIDE_INPUT;
  int64_t ldt[3];
  void* T[3];
  void* C[3];
  for (int i = 0; i < 3; ++i) { ldt[i] = up(P[i].r, 8); T[i] = base + bf.w.T[i]; C[i] = base + bf.w.C[i]; }
  // matrices that take Eq. (2) and matrices that take the exact weight gradient
  int lr[3], ex[3], n_lr = 0, n_ex = 0;
  for (int i = 0; i < 3; ++i) {
    if (exact_mask & (1 << i)) ex[n_ex++] = i;
    else lr[n_lr++] = i;
  }

  if (n_ex > 0) {  // exact Wgrad: dW = Gy^T X, contraction over tokens
    STAGE(MECEFO_STAGE_WGRAD_EXACT, s);
    GemmLaunch g = new_launch(c, false, false, EPI_GRAD);
    g.nprob = n_ex;
    g.accumulate = accumulate;
    for (int j = 0; j < n_ex; ++j) {
      const int i = ex[j];
      g.p[j] = prob(Gy[i], nullptr, ldgy[i], X[i], nullptr, ldx[i], dW[i], nullptr, nullptr, lddw[i], m_out[i], n_in[i], b, 1);
    }
    HIP_TRY(launch_gemm(g, s));
  }
  if (n_lr == 0) return MECEFO_OK;

  if (b > 0) {  // project: T = (X or Gy) P, contraction over the projected dimension
    STAGE(MECEFO_STAGE_PROJECT, s);
    GemmLaunch g = new_launch(c, true, false, EPI_STORE);
    g.nprob = n_lr;
    for (int j = 0; j < n_lr; ++j) {
      const int i = lr[j];
      g.p[j] = prob(in ? X[i] : Gy[i], nullptr, in ? ldx[i] : ldgy[i], P[i].P, nullptr, P[i].ld, T[i], nullptr,
                    nullptr, ldt[i], b, P[i].r, in ? n_in[i] : m_out[i], 1);
      // the K-contiguous operand is one of the library's own zero-padded [b x f] buffers (A, dG, dZ)
      const void* a_op = in ? X[i] : Gy[i];
      g.p[j].kpad_ok = (a_op == base + bf.w.AA || a_op == base + bf.w.DG || a_op == base + bf.w.DZ) ? 1 : 0;
    }
    int rr[3] = {0, 0, 0};
    for (int j = 0; j < n_lr; ++j) rr[lr[j]] = P[lr[j]].r;
    TRY(launch_store_split(c, bf, g, store_splits_project(c, rr, side), s));
  }
  {  // contract over tokens: C = (Gy or X)^T T   [rows x r], K = b
    const int splits = b > 0 ? bf.w.splits : 1;
    GemmLaunch g = new_launch(c, false, false, splits > 1 ? EPI_SPLIT_F32 : EPI_STORE);
    g.nprob = n_lr;
    g.splits = splits;
    g.partial = (float*)(base + bf.w.partial);
    int64_t poff = 0;
    for (int j = 0; j < n_lr; ++j) {
      const int i = lr[j];
      const int rows = in ? m_out[i] : n_in[i];
      g.p[j] = prob(in ? Gy[i] : X[i], nullptr, in ? ldgy[i] : ldx[i], T[i], nullptr, ldt[i], C[i], nullptr,
                    nullptr, ldt[i], rows, P[i].r, b, 1);
      g.partial_off[j] = poff;
      poff += (int64_t)splits * rows * ldt[i];
    }
    {
      STAGE(MECEFO_STAGE_CONTRACT, s);
      g.clk = g_prof.cur_clk;
      HIP_TRY(launch_gemm(g, s));
    }
    if (splits > 1) {
      STAGE(MECEFO_STAGE_SPLITK_REDUCE, s);
      // partial of problem j is [split][rows x ldt]; the reduction keeps that row stride
      for (int j = 0; j < n_lr; ++j) {
        const int i = lr[j];
        const int rows = in ? m_out[i] : n_in[i];
        HIP_TRY(launch_splitk_reduce(c.bf16, g.partial + g.partial_off[j], splits, (int64_t)rows * ldt[i], C[i], s));
      }
    }
  }
  {  // expand: dW = C P^T (SIDE_INPUT) or P C^T (SIDE_OUTPUT), K = r, into the gradient buffers
    STAGE(MECEFO_STAGE_EXPAND, s);
    GemmLaunch g = new_launch(c, true, true, EPI_GRAD);
    g.nprob = n_lr;
    g.accumulate = accumulate;
    for (int j = 0; j < n_lr; ++j) {
      const int i = lr[j];
      g.p[j] = in ? prob(C[i], nullptr, ldt[i], P[i].P, nullptr, P[i].ld, dW[i], nullptr, nullptr, lddw[i],
                         m_out[i], n_in[i], P[i].r, 1)
                  : prob(P[i].P, nullptr, P[i].ld, C[i], nullptr, ldt[i], dW[i], nullptr, nullptr, lddw[i],
                         m_out[i], n_in[i], P[i].r, 1);
    }
    HIP_TRY(launch_gemm(g, s));
  }
  return MECEFO_OK;
}


// ---- standard-mode backward (Alg. 3, first branch) ----------------------------------------
struct FullWs {
  size_t dH, dQ, dK, dV, D, P, cs, sn, total;
  int64_t ldp;     // row stride of one [seq x seq] probability matrix
};

FullWs full_layout(const Ctx& c, const mecefo_attn_desc_t& a, size_t ffn_total) {
  FullWs w;
  size_t off = (size_t)up((int64_t)ffn_total, 256);
  auto take = [&](size_t bytes) { size_t o = off; off += (size_t)up((int64_t)bytes, 256); return o; };
  const size_t act_d = (size_t)c.b * c.dm * c.esz;
  w.ldp = up(a.seq, 8);
  w.dH = take(act_d);
  w.dQ = take(act_d);
  w.dK = take(act_d);
  w.dV = take(act_d);
  w.D = take((size_t)c.b * a.heads * 4);
  w.P = take((size_t)a.batch * a.heads * a.seq * w.ldp * c.esz);
  const int dh = c.dm / (a.heads > 0 ? a.heads : 1);
  w.cs = take((size_t)a.seq * (dh / 2) * 4);
  w.sn = take((size_t)a.seq * (dh / 2) * 4);
  w.total = off + 256;
  return w;
}

mecefo_status_t check_attn(const Ctx& c, const mecefo_attn_desc_t* a) {
  if (!a) return fail(MECEFO_ERR_INVALID_ARG, "attention descriptor is NULL");
  if (a->batch < 0 || a->seq < 0 || a->heads < 1) return fail(MECEFO_ERR_INVALID_ARG, "batch >= 0, seq >= 0, heads >= 1 required");
  if ((int64_t)a->batch * a->seq != c.b) return fail(MECEFO_ERR_INVALID_ARG, "batch * seq = %lld differs from tokens = %lld", (long long)a->batch * a->seq, (long long)c.b);
  if (c.dm % a->heads) return fail(MECEFO_ERR_INVALID_ARG, "d_model %d is not a multiple of heads %d", c.dm, a->heads);
  const int dh = c.dm / a->heads;
  if (dh % 2) return fail(MECEFO_ERR_INVALID_ARG, "head dimension %d must be even (rotary pairs)", dh);
  if (c.bf16 && dh % 8) return fail(MECEFO_ERR_UNSUPPORTED, "bf16 path needs a head dimension that is a multiple of 8 (got %d)", dh);
  if (c.dm > 16384) return fail(MECEFO_ERR_UNSUPPORTED, "d_model above 16384 is not built for the attention backward");
  if (a->ld_w_dd < c.dm) return fail(MECEFO_ERR_INVALID_ARG, "ld_w_dd is smaller than d_model");
  if (c.bf16 && a->ld_w_dd % 8) return fail(MECEFO_ERR_INVALID_ARG, "bf16 path needs ld_w_dd to be a multiple of 8");
  if (!(a->rope_theta > 0.f)) return fail(MECEFO_ERR_INVALID_ARG, "rope_theta must be positive");
  if ((int64_t)a->seq * up(a->seq, 8) * c.esz >= kMaxBytes || (int64_t)c.dm * a->ld_w_dd * 4 >= kMaxBytes)
    return fail(MECEFO_ERR_UNSUPPORTED, "a [seq x seq] score matrix or a [d x d] weight reaches 2 GiB");
  return MECEFO_OK;
}

// One batched attention product per (sequence, head): operands are token-major [b x d] tensors
// (head h at columns h*dh) or the [batch*heads][seq x ldp] probability buffer.
void per_head_tokens(const mecefo_attn_desc_t& a, int dh, int64_t ld, int64_t* bo, int64_t* bi) {
  *bo = (int64_t)a.seq * ld;
  *bi = dh;
}
void per_head_scores(const mecefo_attn_desc_t& a, int64_t ldp, int64_t* bo, int64_t* bi) {
  *bi = (int64_t)a.seq * ldp;
  *bo = *bi * a.heads;
}

// ---- block forward ------------------------------------------------------------------------
struct FwdWs {
  size_t Xn, rstd, Q, K, V, O, L, A, S32, P, cs, sn, total;
  int64_t ldp;
  int hc;        // heads per attention chunk
};

// The block forward takes the fused attention kernel (no score or probability buffer) whenever it is
// built for the shape; mecefo_set_option("attention", "gemm") keeps the materialised-score form for testing.  The
// workspace query and the call consult the same predicate.
bool fwd_attention_fused(const Ctx& c, const mecefo_attn_desc_t& a) {
  if (options().attn_gemm.load(std::memory_order_relaxed)) return false;
  // bf16 descriptors have row strides that are multiples of 8 (checked with the descriptor)
  return attn_fwd_fused_supported(c.bf16, c.dm / (a.heads > 0 ? a.heads : 1), a.seq > 0 ? a.seq : 1, 8);
}

FwdWs fwd_layout(const Ctx& c, const mecefo_attn_desc_t& a) {
  FwdWs w;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += (size_t)up((int64_t)bytes, 256); return o; };
  const size_t act_d = (size_t)c.b * c.dm * c.esz;
  const int dh = c.dm / (a.heads > 0 ? a.heads : 1);
  w.ldp = up(a.seq, 8);
  w.Xn = take(act_d);
  w.rstd = take((size_t)c.b * 4);
  w.Q = take(act_d); w.K = take(act_d); w.V = take(act_d); w.O = take(act_d);
  w.L = take((size_t)c.b * a.heads * 4);
  w.A = take((size_t)c.b * c.ldf * c.esz);
  // fp32 scores of one chunk of heads of one sequence: at most 256 MiB
  const int64_t per_head = (int64_t)a.seq * w.ldp * 4;
  int64_t hc = per_head > 0 ? ((int64_t)256 << 20) / per_head : a.heads;
  if (hc < 1) hc = 1;
  if (hc > a.heads) hc = a.heads;
  w.hc = (int)hc;
  const bool fused = fwd_attention_fused(c, a);
  w.S32 = take(fused ? 0 : (size_t)hc * per_head);
  w.P = take(fused ? 0 : (size_t)hc * a.seq * w.ldp * c.esz);
  w.cs = take((size_t)a.seq * (dh / 2) * 4);
  w.sn = take((size_t)a.seq * (dh / 2) * 4);
  w.total = off + 256;
  return w;
}

mecefo_status_t check_lowrank_args(const Ctx& c, const mecefo_proj_t P[3], mecefo_side_t side, int exact_mask = 0) {
  if (side != MECEFO_SIDE_INPUT && side != MECEFO_SIDE_OUTPUT) return fail(MECEFO_ERR_INVALID_ARG, "side must be MECEFO_SIDE_INPUT or MECEFO_SIDE_OUTPUT");
  const bool in = side == MECEFO_SIDE_INPUT;
  if (!(exact_mask & 1)) TRY(check_proj(c, P[0], in ? c.dm : c.ff, "Pg"));
  if (!(exact_mask & 2)) TRY(check_proj(c, P[1], in ? c.dm : c.ff, "Pu"));
  if (!(exact_mask & 4)) TRY(check_proj(c, P[2], in ? c.ff : c.dm, "Pd"));
  return MECEFO_OK;
}

}  // namespace

// ---- scratch of the entry point that allocates nothing ------------------------------------
// Device memory that exists once per GPU from the moment the code object is loaded there.  In host code
// the name below stands for the symbol, not for an address: the address on the current device comes from
// hipGetSymbolAddress and is kept per device.
static __device__ __align__(256) unsigned char scratch[MECEFO_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

mecefo_status_t scratch_on_current_device(void** out) {
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(MECEFO_ERR_UNSUPPORTED, "device index %d is beyond the %d the scratch table holds", dev, kMaxDevices);
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {   // several threads may resolve at once: every one of them gets the same address
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(MECEFO_ERR_LAUNCH, "hipGetSymbolAddress returned a NULL scratch address");
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return MECEFO_OK;
}
}  // namespace

extern "C" {

const char* mecefo_last_error(void) { return g_err; }
const char* mecefo_version(void) { return "mecefo-gfx950 0.2"; }

mecefo_status_t mecefo_init(void) {
  HIP_TRY(prepare_gemm_bf16_nt());
  HIP_TRY(prepare_gemm_bf16_nn());
  HIP_TRY(prepare_gemm_bf16_tn());
  HIP_TRY(prepare_attention_fwd());
  HIP_TRY(prepare_attention_bwd());
  void* p = nullptr;
  TRY(scratch_on_current_device(&p));
  return MECEFO_OK;
}

mecefo_status_t mecefo_set_option(const char* name, const char* value) {
  if (!name || !value) return fail(MECEFO_ERR_INVALID_ARG, "option name and value are required");
  if (!strcmp(name, "tile")) {
    static const char* const names[5] = {"auto", "S", "L4", "L8R", "L8"};
    for (int i = 0; i < 5; ++i)
      if (!strcmp(value, names[i])) { options().tile.store(i, std::memory_order_relaxed); return MECEFO_OK; }
    return fail(MECEFO_ERR_INVALID_ARG, "option tile: value must be auto, S, L4, L8R or L8 (got %s)", value);
  }
  if (!strcmp(name, "attention")) {
    if (!strcmp(value, "auto")) { options().attn_gemm.store(0, std::memory_order_relaxed); return MECEFO_OK; }
    if (!strcmp(value, "gemm")) { options().attn_gemm.store(1, std::memory_order_relaxed); return MECEFO_OK; }
    return fail(MECEFO_ERR_INVALID_ARG, "option attention: value must be auto or gemm (got %s)", value);
  }
  return fail(MECEFO_ERR_INVALID_ARG, "unknown option %s", name);
}

mecefo_status_t mecefo_profile_enable(int max_launches) {
  if (max_launches < 1) return fail(MECEFO_ERR_INVALID_ARG, "max_launches must be >= 1");
  for (hipEvent_t e : g_prof.ev) (void)hipEventDestroy(e);
  g_prof.ev.assign((size_t)max_launches * 2, nullptr);
  g_prof.stage.assign((size_t)max_launches, 0);
  for (auto& e : g_prof.ev) HIP_TRY(hipEventCreate(&e));
  if (g_prof.clk) { (void)hipFree(g_prof.clk); g_prof.clk = nullptr; }
  const size_t clk_bytes = (size_t)max_launches * kClkPairs * 2 * sizeof(uint32_t);
  HIP_TRY(hipMalloc((void**)&g_prof.clk, clk_bytes));
  HIP_TRY(hipMemset(g_prof.clk, 0, clk_bytes));
  g_prof.used = 0;
  g_prof.on = true;
  return MECEFO_OK;
}

mecefo_status_t mecefo_profile_clock_mhz(double* mhz_by_stage) {
  if (!mhz_by_stage) return fail(MECEFO_ERR_INVALID_ARG, "output array is NULL");
  for (int i = 0; i < MECEFO_STAGE_COUNT; ++i) mhz_by_stage[i] = g_prof.mhz[i];
  return MECEFO_OK;
}

mecefo_status_t mecefo_profile_collect(double* ms_by_stage, int* launches_by_stage) {
  if (!ms_by_stage || !launches_by_stage) return fail(MECEFO_ERR_INVALID_ARG, "output arrays are NULL");
  for (int i = 0; i < MECEFO_STAGE_COUNT; ++i) { ms_by_stage[i] = 0.0; launches_by_stage[i] = 0; g_prof.mhz[i] = 0.0; }
  g_prof.on = false;
  g_prof.cur_clk = nullptr;
  for (size_t i = 0; i + 1 < g_prof.used; i += 2) {
    HIP_TRY(hipEventSynchronize(g_prof.ev[i + 1]));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, g_prof.ev[i], g_prof.ev[i + 1]));
    const int st = g_prof.stage[i / 2];
    ms_by_stage[st] += ms;
    launches_by_stage[st] += 1;
  }
  if (g_prof.clk && g_prof.used >= 2) {   // shader clock per stage: cycles / wall ticks (100 MHz) of the sampled workgroups
    const size_t launches = g_prof.used / 2;
    std::vector<uint32_t> h(launches * kClkPairs * 2);
    HIP_TRY(hipMemcpy(h.data(), g_prof.clk, h.size() * sizeof(uint32_t), hipMemcpyDeviceToHost));
    double cyc[MECEFO_STAGE_COUNT] = {}, ticks[MECEFO_STAGE_COUNT] = {};
    for (size_t l = 0; l < launches; ++l)
      for (int k = 0; k < kClkPairs; ++k) {
        const uint32_t c = h[(l * kClkPairs + k) * 2], w = h[(l * kClkPairs + k) * 2 + 1];
        if (c && w) { cyc[g_prof.stage[l]] += c; ticks[g_prof.stage[l]] += w; }
      }
    for (int i = 0; i < MECEFO_STAGE_COUNT; ++i) g_prof.mhz[i] = ticks[i] > 0 ? 100.0 * cyc[i] / ticks[i] : 0.0;
  }
  if (g_prof.clk) { (void)hipFree(g_prof.clk); g_prof.clk = nullptr; }
  for (hipEvent_t e : g_prof.ev) (void)hipEventDestroy(e);
  g_prof.ev.clear();
  g_prof.stage.clear();
  g_prof.used = 0;
  return MECEFO_OK;
}

mecefo_status_t mecefo_workspace_bytes(const mecefo_ffn_desc_t* desc, int r_gate, int r_up, int r_down,
                                       size_t* out_bytes) {
  Ctx c;
  TRY(check_desc(desc, &c));
  if (!out_bytes) return fail(MECEFO_ERR_INVALID_ARG, "out_bytes is NULL");
  if (r_gate < 0 || r_up < 0 || r_down < 0) return fail(MECEFO_ERR_INVALID_ARG, "ranks must be >= 0");
  const int r[3] = {r_gate, r_up, r_down};
  const size_t a = layout(c, r, MECEFO_SIDE_INPUT, 0).total;
  const size_t b2 = layout(c, r, MECEFO_SIDE_OUTPUT, 0).total;
  *out_bytes = a > b2 ? a : b2;
  return MECEFO_OK;
}

mecefo_status_t mecefo_ffn_fwd_recompute(const mecefo_ffn_desc_t* desc, const void* U, const void* Wg,
                                         const void* Wu, const void* Wd, void* G, void* Z, void* A, void* Y,
                                         void* ws, size_t ws_bytes, void* hip_stream) {
  (void)ws; (void)ws_bytes;
  Ctx c;
  TRY(check_desc(desc, &c));
  TRY(check_ptr(c, U, "U")); TRY(check_ptr(c, Wg, "Wg")); TRY(check_ptr(c, Wu, "Wu"));
  TRY(check_ptr(c, G, "G", false)); TRY(check_ptr(c, Z, "Z", false)); TRY(check_ptr(c, A, "A"));
  TRY(check_ptr(c, Y, "Y", false));
  if (Y) TRY(check_ptr(c, Wd, "Wd (needed for Y)"));
  hipStream_t s = (hipStream_t)hip_stream;
  const int b = (int)c.b;
  if (b == 0) return MECEFO_OK;
  const int pad = (int)(up(c.ff, 8) <= desc->ld_act_f ? up(c.ff, 8) : c.ff);
  {
    GemmLaunch g = new_launch(c, true, true, EPI_SWIGLU_FWD);
    g.nprob = 1;
    g.p[0] = prob(U, nullptr, desc->ld_act_d, Wg, Wu, desc->ld_w_fd, G, Z, A, desc->ld_act_f, b, c.ff, c.dm, 1, pad);
    HIP_TRY(launch_gemm(g, s));
  }
  if (Y) {  // Y = A Wd^T   [b x d], K = f
    GemmLaunch g = new_launch(c, true, true, EPI_STORE);
    g.nprob = 1;
    g.p[0] = prob(A, nullptr, desc->ld_act_f, Wd, nullptr, desc->ld_w_df, Y, nullptr, nullptr, desc->ld_act_d, b, c.dm, c.ff, 1);
    HIP_TRY(launch_gemm(g, s));
  }
  return MECEFO_OK;
}

mecefo_status_t mecefo_ffn_bwd_exact(const mecefo_ffn_desc_t* desc, const void* U, const void* dY,
                                     const void* Wg, const void* Wu, const void* Wd, const void* G,
                                     const void* Z, void* dU, void* dWg, void* dWu, void* dWd, int accumulate,
                                     void* ws, size_t ws_bytes, void* hip_stream) {
  Ctx c;
  TRY(check_desc(desc, &c));
  TRY(check_ptr(c, U, "U", c.b > 0)); TRY(check_ptr(c, dY, "dY", c.b > 0));
  TRY(check_ptr(c, Wg, "Wg")); TRY(check_ptr(c, Wu, "Wu")); TRY(check_ptr(c, Wd, "Wd"));
  if ((G == nullptr) != (Z == nullptr)) return fail(MECEFO_ERR_INVALID_ARG, "G and Z must both be given or both be NULL");
  TRY(check_ptr(c, G, "G", false)); TRY(check_ptr(c, Z, "Z", false)); TRY(check_ptr(c, dU, "dU", false));
  if (!dWg || !dWu || !dWd) return fail(MECEFO_ERR_INVALID_ARG, "dWg, dWu, dWd are required");
  if (c.bf16 && (((uintptr_t)dWg | (uintptr_t)dWu | (uintptr_t)dWd) % 16)) return fail(MECEFO_ERR_INVALID_ARG, "gradient buffers must be 16-byte aligned");
  const int r0[3] = {0, 0, 0};
  Bufs bf;
  TRY(carve(c, r0, MECEFO_SIDE_INPUT, ws, ws_bytes, &bf));
  hipStream_t s = (hipStream_t)hip_stream;
  TRY(recompute_and_dgrad(c, bf, U, desc->ld_act_d, dY, desc->ld_act_d, Wg, Wu, Wd, G, Z, dU, desc->ld_act_d, s));
  // exact Wgrad: dWg = dG^T U, dWu = dZ^T U [f x d]; dWd = dY^T A [d x f]; contraction over tokens
  STAGE(MECEFO_STAGE_WGRAD_EXACT, s);
  GemmLaunch g = new_launch(c, false, false, EPI_GRAD);
  g.nprob = 3;
  g.accumulate = accumulate;
  const int b = (int)c.b;
  char* base = bf.base;
  g.p[0] = prob(base + bf.w.DG, nullptr, c.ldf, U, nullptr, desc->ld_act_d, dWg, nullptr, nullptr, desc->ld_w_fd, c.ff, c.dm, b, 1);
  g.p[1] = prob(base + bf.w.DZ, nullptr, c.ldf, U, nullptr, desc->ld_act_d, dWu, nullptr, nullptr, desc->ld_w_fd, c.ff, c.dm, b, 1);
  g.p[2] = prob(dY, nullptr, desc->ld_act_d, base + bf.w.AA, nullptr, c.ldf, dWd, nullptr, nullptr, desc->ld_w_df, c.dm, c.ff, b, 1);
  HIP_TRY(launch_gemm(g, s));
  return MECEFO_OK;
}

mecefo_status_t mecefo_ffn_bwd_lowrank(const mecefo_ffn_desc_t* desc, const void* U, const void* dY,
                                       const void* Wg, const void* Wu, const void* Wd, mecefo_proj_t Pg,
                                       mecefo_proj_t Pu, mecefo_proj_t Pd, mecefo_side_t side, void* dU,
                                       void* dWg, void* dWu, void* dWd, int accumulate, void* ws,
                                       size_t ws_bytes, void* hip_stream) {
  Ctx c;
  TRY(check_desc(desc, &c));
  TRY(check_ptr(c, U, "U", c.b > 0)); TRY(check_ptr(c, dY, "dY", c.b > 0));
  TRY(check_ptr(c, Wg, "Wg")); TRY(check_ptr(c, Wu, "Wu")); TRY(check_ptr(c, Wd, "Wd"));
  TRY(check_ptr(c, dU, "dU", false));
  if (!dWg || !dWu || !dWd) return fail(MECEFO_ERR_INVALID_ARG, "dWg, dWu, dWd are required");
  if (c.bf16 && (((uintptr_t)dWg | (uintptr_t)dWu | (uintptr_t)dWd) % 16)) return fail(MECEFO_ERR_INVALID_ARG, "gradient buffers must be 16-byte aligned");
  const mecefo_proj_t P[3] = {Pg, Pu, Pd};
  TRY(check_lowrank_args(c, P, side));
  const int r[3] = {Pg.r, Pu.r, Pd.r};
  Bufs bf;
  TRY(carve(c, r, side, ws, ws_bytes, &bf));
  hipStream_t s = (hipStream_t)hip_stream;
  TRY(recompute_and_dgrad(c, bf, U, desc->ld_act_d, dY, desc->ld_act_d, Wg, Wu, Wd, nullptr, nullptr, dU, desc->ld_act_d, s));
  void* dW[3] = {dWg, dWu, dWd};
  return lowrank_wgrad(c, bf, U, desc->ld_act_d, dY, desc->ld_act_d, P, side, dW, accumulate, s);
}

mecefo_status_t mecefo_block_bwd_skip_ex(const mecefo_ffn_desc_t* desc, const void* H, const void* dOut,
                                         const void* gamma, const void* Wg, const void* Wu, const void* Wd,
                                         mecefo_proj_t Pg, mecefo_proj_t Pu, mecefo_proj_t Pd, mecefo_side_t side,
                                         const mecefo_skip_options_t* opt, void* dX, void* dgamma, void* dWg,
                                         void* dWu, void* dWd, int accumulate, void* ws, size_t ws_bytes,
                                         void* hip_stream) {
  Ctx c;
  TRY(check_desc(desc, &c));
  const void* Gs = opt ? opt->G : nullptr;
  const void* Zs = opt ? opt->Z : nullptr;
  const int exact_mask = opt ? opt->exact_wgrad_mask : 0;
  if (exact_mask & ~7) return fail(MECEFO_ERR_INVALID_ARG, "exact_wgrad_mask has bits beyond gate (1), up (2), down (4)");
  if ((Gs == nullptr) != (Zs == nullptr)) return fail(MECEFO_ERR_INVALID_ARG, "G and Z must both be given or both be NULL");
  TRY(check_ptr(c, Gs, "G", false)); TRY(check_ptr(c, Zs, "Z", false));
  TRY(check_ptr(c, H, "H", c.b > 0)); TRY(check_ptr(c, dOut, "dOut", c.b > 0)); TRY(check_ptr(c, gamma, "gamma", false));
  TRY(check_ptr(c, Wg, "Wg")); TRY(check_ptr(c, Wu, "Wu")); TRY(check_ptr(c, Wd, "Wd"));
  TRY(check_ptr(c, dX, "dX", c.b > 0));
  if (!dWg || !dWu || !dWd) return fail(MECEFO_ERR_INVALID_ARG, "dWg, dWu, dWd are required");
  if (c.bf16 && (((uintptr_t)dWg | (uintptr_t)dWu | (uintptr_t)dWd) % 16)) return fail(MECEFO_ERR_INVALID_ARG, "gradient buffers must be 16-byte aligned");
  if (dgamma && !gamma) return fail(MECEFO_ERR_INVALID_ARG, "dgamma requested but gamma is NULL");
  TRY(check_alias(dX, "dX", dOut, "dOut", act_span(c, desc->ld_act_d)));
  TRY(check_alias(dX, "dX", H, "H", act_span(c, desc->ld_act_d)));
  const mecefo_proj_t P[3] = {Pg, Pu, Pd};
  TRY(check_lowrank_args(c, P, side, exact_mask));
  const int r[3] = {(exact_mask & 1) ? 0 : Pg.r, (exact_mask & 2) ? 0 : Pu.r, (exact_mask & 4) ? 0 : Pd.r};
  Bufs bf;
  TRY(carve(c, r, side, ws, ws_bytes, &bf));
  hipStream_t s = (hipStream_t)hip_stream;
  char* base = bf.base;
  const void* U = H;
  int64_t ldu = desc->ld_act_d;
  float* rstd = (float*)(base + bf.w.rstd);
  if (gamma && c.b > 0) {  // recompute the norm output from the stored tensor
    STAGE(MECEFO_STAGE_NORM_FWD, s);
    HIP_TRY(launch_rmsnorm_fwd(c.bf16, H, desc->ld_act_d, gamma, desc->rms_eps, base + bf.w.U, c.dm, rstd, c.b, c.dm, s));
    U = base + bf.w.U;
    ldu = c.dm;
  }
  void* dUb = base + bf.w.dU;
  TRY(recompute_and_dgrad(c, bf, U, ldu, dOut, desc->ld_act_d, Wg, Wu, Wd, Gs, Zs, dUb, c.dm, s));
  // Skip the MHA connection: the gradient handed to the previous layer is dH = dOut + normbwd(dU).
  auto norm_backward = [&]() -> mecefo_status_t {
    STAGE(MECEFO_STAGE_NORM_BWD, s);
    if (gamma) {
      const int nblk = rmsnorm_bwd_blocks(c.b);
      float* dgp = dgamma ? (float*)(base + bf.w.dgp) : nullptr;
      if (c.b > 0)
        HIP_TRY(launch_rmsnorm_bwd(c.bf16, dUb, c.dm, H, desc->ld_act_d, rstd, gamma, dOut, desc->ld_act_d, dX,
                                   desc->ld_act_d, dgp, nblk, c.b, c.dm, s));
      if (dgamma) HIP_TRY(launch_dgamma_reduce(dgp, c.b > 0 ? nblk : 0, c.dm, dgamma, c.grad_f32, c.bf16, accumulate, s));
    } else if (c.b > 0) {
      HIP_TRY(launch_add(c.bf16, dOut, desc->ld_act_d, dUb, c.dm, dX, desc->ld_act_d, c.b, c.dm, s));
    }
    return MECEFO_OK;
  };
  // Eq. (2) reads dOut (the down projection's output gradient) and, without a norm, H itself: when dX
  // is a buffer of its own the norm backward goes first, while dU is still in the caches and before
  // the weight gradients flood them; when dX overwrites dOut (or H) it has to wait for Eq. (2).
  const bool dx_first = dX != dOut && dX != H;
  if (dx_first) TRY(norm_backward());
  void* dW[3] = {dWg, dWu, dWd};
  TRY(lowrank_wgrad(c, bf, U, ldu, dOut, desc->ld_act_d, P, side, dW, accumulate, s, exact_mask));
  if (!dx_first) TRY(norm_backward());
  return MECEFO_OK;
}

mecefo_status_t mecefo_block_bwd_skip(const mecefo_ffn_desc_t* desc, const void* H, const void* dOut,
                                      const void* gamma, const void* Wg, const void* Wu, const void* Wd,
                                      mecefo_proj_t Pg, mecefo_proj_t Pu, mecefo_proj_t Pd, mecefo_side_t side,
                                      void* dX, void* dgamma, void* dWg, void* dWu, void* dWd, int accumulate,
                                      void* ws, size_t ws_bytes, void* hip_stream) {
  return mecefo_block_bwd_skip_ex(desc, H, dOut, gamma, Wg, Wu, Wd, Pg, Pu, Pd, side, nullptr, dX, dgamma, dWg, dWu,
                                  dWd, accumulate, ws, ws_bytes, hip_stream);
}

mecefo_status_t mecefo_block_full_workspace_bytes(const mecefo_ffn_desc_t* desc, const mecefo_attn_desc_t* attn,
                                                  size_t* out_bytes) {
  Ctx c;
  TRY(check_desc(desc, &c));
  TRY(check_attn(c, attn));
  if (!out_bytes) return fail(MECEFO_ERR_INVALID_ARG, "out_bytes is NULL");
  const int r0[3] = {0, 0, 0};
  *out_bytes = full_layout(c, *attn, layout(c, r0, MECEFO_SIDE_INPUT, 0).total).total;
  return MECEFO_OK;
}

mecefo_status_t mecefo_block_bwd_full(const mecefo_ffn_desc_t* desc, const mecefo_attn_desc_t* attn,
                                      const mecefo_block_inputs_t* in, const mecefo_block_grads_t* out,
                                      int accumulate, void* ws, size_t ws_bytes, void* hip_stream) {
  Ctx c;
  TRY(check_desc(desc, &c));
  TRY(check_attn(c, attn));
  if (!in || !out) return fail(MECEFO_ERR_INVALID_ARG, "input or output table is NULL");
  const bool any = c.b > 0;
  TRY(check_ptr(c, in->X, "X", any)); TRY(check_ptr(c, in->H, "H", any)); TRY(check_ptr(c, in->dOut, "dOut", any));
  TRY(check_ptr(c, in->g_attn, "g_attn")); TRY(check_ptr(c, in->g_ffn, "g_ffn"));
  TRY(check_ptr(c, in->Wq, "Wq")); TRY(check_ptr(c, in->Wk, "Wk")); TRY(check_ptr(c, in->Wv, "Wv")); TRY(check_ptr(c, in->Wo, "Wo"));
  TRY(check_ptr(c, in->Wg, "Wg")); TRY(check_ptr(c, in->Wu, "Wu")); TRY(check_ptr(c, in->Wd, "Wd"));
  TRY(check_ptr(c, in->Q, "Q", any)); TRY(check_ptr(c, in->K, "K", any)); TRY(check_ptr(c, in->V, "V", any)); TRY(check_ptr(c, in->O, "O", any));
  if (any && !in->L) return fail(MECEFO_ERR_INVALID_ARG, "L is NULL");
  TRY(check_ptr(c, out->dX, "dX", any));
  void* grads[9] = {out->dg_attn, out->dg_ffn, out->dWq, out->dWk, out->dWv, out->dWo, out->dWg, out->dWu, out->dWd};
  for (void* g : grads) {
    if (!g) return fail(MECEFO_ERR_INVALID_ARG, "every gradient buffer is required");
    if (c.bf16 && ((uintptr_t)g % 16)) return fail(MECEFO_ERR_INVALID_ARG, "gradient buffers must be 16-byte aligned");
  }
  const int r0[3] = {0, 0, 0};
  const Workspace fw = layout(c, r0, MECEFO_SIDE_INPUT, 0);
  const FullWs w = full_layout(c, *attn, fw.total);
  if (w.total > ws_bytes) return fail(MECEFO_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", ws_bytes, w.total);
  if (!ws) return fail(MECEFO_ERR_INVALID_ARG, "workspace is NULL");
  Bufs bf;
  bf.base = (char*)up((int64_t)(uintptr_t)ws, 256);
  bf.w = fw;
  char* base = bf.base;
  hipStream_t s = (hipStream_t)hip_stream;
  const mecefo_ffn_desc_t& d = *desc;
  const mecefo_attn_desc_t& a = *attn;
  const int b = (int)c.b, dm = c.dm, dh = dm / a.heads, S = a.seq;
  const int nblk = rmsnorm_bwd_blocks(c.b);
  float* rstd = (float*)(base + fw.rstd);
  float* dgp = (float*)(base + fw.dgp);
  void* Ub = base + fw.U;       // norm(H), later norm(X)
  void* dUb = base + fw.dU;     // dU, later dO, later dXn
  void* dH = base + w.dH;
  void* dQ = base + w.dQ; void* dK = base + w.dK; void* dV = base + w.dV;
  float* D = (float*)(base + w.D);
  void* P = base + w.P;
  float* cs = (float*)(base + w.cs); float* sn = (float*)(base + w.sn);

  // ---- FFN module, exact: dH = dOut + normbwd(dU), dWg, dWu, dWd, dg_ffn
  if (any) {
    STAGE(MECEFO_STAGE_NORM_FWD, s);
    HIP_TRY(launch_rmsnorm_fwd(c.bf16, in->H, d.ld_act_d, in->g_ffn, d.rms_eps, Ub, dm, rstd, c.b, dm, s));
  }
  TRY(recompute_and_dgrad(c, bf, Ub, dm, in->dOut, d.ld_act_d, in->Wg, in->Wu, in->Wd, nullptr, nullptr, dUb, dm, s));
  {
    STAGE(MECEFO_STAGE_WGRAD_EXACT, s);
    GemmLaunch g = new_launch(c, false, false, EPI_GRAD);
    g.nprob = 3;
    g.accumulate = accumulate;
    g.p[0] = prob(base + fw.DG, nullptr, c.ldf, Ub, nullptr, dm, out->dWg, nullptr, nullptr, d.ld_w_fd, c.ff, dm, b, 1);
    g.p[1] = prob(base + fw.DZ, nullptr, c.ldf, Ub, nullptr, dm, out->dWu, nullptr, nullptr, d.ld_w_fd, c.ff, dm, b, 1);
    g.p[2] = prob(in->dOut, nullptr, d.ld_act_d, base + fw.AA, nullptr, c.ldf, out->dWd, nullptr, nullptr, d.ld_w_df, dm, c.ff, b, 1);
    HIP_TRY(launch_gemm(g, s));
  }
  {
    STAGE(MECEFO_STAGE_NORM_BWD, s);
    if (any)
      HIP_TRY(launch_rmsnorm_bwd(c.bf16, dUb, dm, in->H, d.ld_act_d, rstd, in->g_ffn, in->dOut, d.ld_act_d, dH, dm,
                                 dgp, nblk, c.b, dm, s));
    HIP_TRY(launch_dgamma_reduce(dgp, any ? nblk : 0, dm, out->dg_ffn, c.grad_f32, c.bf16, accumulate, s));
  }

  // ---- attention module
  if (any) {
    STAGE(MECEFO_STAGE_NORM_FWD, s);
    HIP_TRY(launch_rmsnorm_fwd(c.bf16, in->X, d.ld_act_d, in->g_attn, d.rms_eps, Ub, dm, rstd, c.b, dm, s));
  }
  {  // dWo = dH^T O  [d x d], K = tokens;  dO = dH Wo  [b x d], K = d
    STAGE(MECEFO_STAGE_ATTN_OUT_BWD, s);
    GemmLaunch g = new_launch(c, false, false, EPI_GRAD);
    g.nprob = 1;
    g.accumulate = accumulate;
    g.p[0] = prob(dH, nullptr, dm, in->O, nullptr, d.ld_act_d, out->dWo, nullptr, nullptr, a.ld_w_dd, dm, dm, b, 1);
    HIP_TRY(launch_gemm(g, s));
    if (any) {
      GemmLaunch h = new_launch(c, true, false, EPI_STORE);
      h.nprob = 1;
      h.p[0] = prob(dH, nullptr, dm, in->Wo, nullptr, a.ld_w_dd, dUb, nullptr, nullptr, dm, b, dm, dm, 1);
      HIP_TRY(launch_gemm(h, s));
    }
  }
  if (any) {
    const void* dO = dUb;
    const float scale = 1.0f / sqrtf((float)dh);
    int64_t tok_bo, tok_bi, ws_bo, ws_bi, sc_bo, sc_bi;
    per_head_tokens(a, dh, d.ld_act_d, &tok_bo, &tok_bi);   // caller tensors Q, K, V
    per_head_tokens(a, dh, dm, &ws_bo, &ws_bi);             // workspace tensors dO, dQ, dK, dV
    per_head_scores(a, w.ldp, &sc_bo, &sc_bi);
    auto batched = [&](GemmProblem& p, int64_t abo, int64_t abi, int64_t bbo, int64_t bbi, int64_t cbo, int64_t cbi) {
      p.batch = a.batch * a.heads;
      p.batch_inner = a.heads;
      p.a_bo = abo; p.a_bi = abi; p.b_bo = bbo; p.b_bi = bbi; p.c_bo = cbo; p.c_bi = cbi;
    };
    {
      STAGE(MECEFO_STAGE_ATTN_ROWDOT, s);
      HIP_TRY(launch_attn_rowdot(c.bf16, dO, dm, in->O, d.ld_act_d, D, c.b, S, a.heads, dh, s));
    }
    // mecefo_set_option("attention", "gemm") forces the five-product form
    const bool fused = attn_bwd_fused_supported(c.bf16, dh, S, w.ldp) && !options().attn_gemm.load(std::memory_order_relaxed);
    if (fused) {  // dK, dV and dS in one kernel; P stays in registers
      STAGE(MECEFO_STAGE_ATTN_FUSED_KV, s);
      HIP_TRY(launch_attn_bwd_kv(in->Q, in->K, in->V, d.ld_act_d, dO, dK, dV, dm, in->L, D, P, w.ldp, a.batch, S,
                                 a.heads, dh, scale, s));
    }
    if (!fused) {
      {  // P = exp(scale Q K^T - L) below the diagonal, 0 above
        STAGE(MECEFO_STAGE_ATTN_PROBS, s);
        GemmLaunch g = new_launch(c, true, true, EPI_ATTN_P);
        g.nprob = 1;
        g.p[0] = prob(in->Q, nullptr, d.ld_act_d, in->K, nullptr, d.ld_act_d, P, nullptr, nullptr, w.ldp, S, S, dh, 1);
        batched(g.p[0], tok_bo, tok_bi, tok_bo, tok_bi, sc_bo, sc_bi);
        g.p[0].rowvec = in->L; g.p[0].scale = scale; g.p[0].causal = CAUSAL_TILE;
        HIP_TRY(launch_gemm(g, s));
      }
      {  // dV = P^T dO   [seq x dh], contraction over the query index
        STAGE(MECEFO_STAGE_ATTN_DV, s);
        GemmLaunch g = new_launch(c, false, false, EPI_STORE);
        g.nprob = 1;
        g.p[0] = prob(P, nullptr, w.ldp, dO, nullptr, dm, dV, nullptr, nullptr, dm, S, dh, S, 1);
        batched(g.p[0], sc_bo, sc_bi, ws_bo, ws_bi, ws_bo, ws_bi);
        g.p[0].causal = CAUSAL_K_FROM_M;
        HIP_TRY(launch_gemm(g, s));
      }
      {  // dS = P * (dO V^T - D) * scale, in place on P
        STAGE(MECEFO_STAGE_ATTN_DS, s);
        GemmLaunch g = new_launch(c, true, true, EPI_ATTN_DS);
        g.nprob = 1;
        g.p[0] = prob(dO, nullptr, dm, in->V, nullptr, d.ld_act_d, P, nullptr, nullptr, w.ldp, S, S, dh, 1);
        batched(g.p[0], ws_bo, ws_bi, tok_bo, tok_bi, sc_bo, sc_bi);
        g.p[0].rowvec = D; g.p[0].scale = scale; g.p[0].causal = CAUSAL_TILE;
        HIP_TRY(launch_gemm(g, s));
      }
    }
    {  // dQ = dS K   [seq x dh], contraction over the key index
      STAGE(MECEFO_STAGE_ATTN_DQ, s);
      GemmLaunch g = new_launch(c, true, false, EPI_STORE);
      g.nprob = 1;
      g.p[0] = prob(P, nullptr, w.ldp, in->K, nullptr, d.ld_act_d, dQ, nullptr, nullptr, dm, S, dh, S, 1);
      batched(g.p[0], sc_bo, sc_bi, tok_bo, tok_bi, ws_bo, ws_bi);
      g.p[0].causal = CAUSAL_K_UPTO_M;
      HIP_TRY(launch_gemm(g, s));
    }
    if (!fused) {  // dK = dS^T Q   [seq x dh], contraction over the query index
      STAGE(MECEFO_STAGE_ATTN_DK, s);
      GemmLaunch g = new_launch(c, false, false, EPI_STORE);
      g.nprob = 1;
      g.p[0] = prob(P, nullptr, w.ldp, in->Q, nullptr, d.ld_act_d, dK, nullptr, nullptr, dm, S, dh, S, 1);
      batched(g.p[0], sc_bo, sc_bi, tok_bo, tok_bi, ws_bo, ws_bi);
      g.p[0].causal = CAUSAL_K_FROM_M;
      HIP_TRY(launch_gemm(g, s));
    }
    {
      STAGE(MECEFO_STAGE_ROPE_BWD, s);
      HIP_TRY(launch_rope_tables(cs, sn, S, dh, (double)a.rope_theta, s));
      HIP_TRY(launch_rope(c.bf16, dQ, dm, cs, sn, c.b, S, a.heads, dh, true, s));
      HIP_TRY(launch_rope(c.bf16, dK, dm, cs, sn, c.b, S, a.heads, dh, true, s));
    }
  }
  {  // dWq, dWk, dWv = (dQ, dK, dV)^T Xn   [d x d], K = tokens
    STAGE(MECEFO_STAGE_QKV_WGRAD, s);
    GemmLaunch g = new_launch(c, false, false, EPI_GRAD);
    g.nprob = 3;
    g.accumulate = accumulate;
    void* dst[3] = {out->dWq, out->dWk, out->dWv};
    const void* src[3] = {dQ, dK, dV};
    for (int i = 0; i < 3; ++i)
      g.p[i] = prob(src[i], nullptr, dm, Ub, nullptr, dm, dst[i], nullptr, nullptr, a.ld_w_dd, dm, dm, b, 1);
    HIP_TRY(launch_gemm(g, s));
  }
  if (any) {  // dXn = dQ Wq + dK Wk + dV Wv   [b x d], three K segments of length d
    STAGE(MECEFO_STAGE_QKV_DGRAD, s);
    GemmLaunch g = new_launch(c, true, false, EPI_STORE);
    g.nprob = 1;
    g.p[0] = prob(dQ, dK, dm, in->Wq, in->Wk, a.ld_w_dd, dUb, nullptr, nullptr, dm, b, dm, dm, 3);
    g.p[0].A[2] = dV; g.p[0].B[2] = in->Wv;
    HIP_TRY(launch_gemm(g, s));
  }
  {  // dX = dH + normbwd(dXn), dg_attn
    STAGE(MECEFO_STAGE_NORM_BWD, s);
    if (any)
      HIP_TRY(launch_rmsnorm_bwd(c.bf16, dUb, dm, in->X, d.ld_act_d, rstd, in->g_attn, dH, dm, out->dX, d.ld_act_d,
                                 dgp, nblk, c.b, dm, s));
    HIP_TRY(launch_dgamma_reduce(dgp, any ? nblk : 0, dm, out->dg_attn, c.grad_f32, c.bf16, accumulate, s));
  }
  return MECEFO_OK;
}

mecefo_status_t mecefo_block_fwd_workspace_bytes(const mecefo_ffn_desc_t* desc, const mecefo_attn_desc_t* attn,
                                                 size_t* out_bytes) {
  Ctx c;
  TRY(check_desc(desc, &c));
  TRY(check_attn(c, attn));
  if (!out_bytes) return fail(MECEFO_ERR_INVALID_ARG, "out_bytes is NULL");
  *out_bytes = fwd_layout(c, *attn).total;
  return MECEFO_OK;
}

mecefo_status_t mecefo_block_fwd(const mecefo_ffn_desc_t* desc, const mecefo_attn_desc_t* attn,
                                 const mecefo_block_fwd_inputs_t* in, const mecefo_block_fwd_outputs_t* out,
                                 void* ws, size_t ws_bytes, void* hip_stream) {
  Ctx c;
  TRY(check_desc(desc, &c));
  TRY(check_attn(c, attn));
  if (!in || !out) return fail(MECEFO_ERR_INVALID_ARG, "input or output table is NULL");
  const bool any = c.b > 0;
  TRY(check_ptr(c, in->X, "X", any));
  TRY(check_ptr(c, in->g_attn, "g_attn")); TRY(check_ptr(c, in->g_ffn, "g_ffn"));
  TRY(check_ptr(c, in->Wq, "Wq")); TRY(check_ptr(c, in->Wk, "Wk")); TRY(check_ptr(c, in->Wv, "Wv")); TRY(check_ptr(c, in->Wo, "Wo"));
  TRY(check_ptr(c, in->Wg, "Wg")); TRY(check_ptr(c, in->Wu, "Wu")); TRY(check_ptr(c, in->Wd, "Wd"));
  TRY(check_ptr(c, out->Out, "Out", any)); TRY(check_ptr(c, out->H, "H", any));
  const int given = (out->Q != nullptr) + (out->K != nullptr) + (out->V != nullptr) + (out->O != nullptr) + (out->L != nullptr);
  if (given != 0 && given != 5) return fail(MECEFO_ERR_INVALID_ARG, "Q, K, V, O, L must all be given (standard mode) or all be NULL (neighbor mode)");
  TRY(check_ptr(c, out->Q, "Q", false)); TRY(check_ptr(c, out->K, "K", false)); TRY(check_ptr(c, out->V, "V", false)); TRY(check_ptr(c, out->O, "O", false));
  if (any && out->Out == in->X) return fail(MECEFO_ERR_INVALID_ARG, "Out must not alias X");
  const FwdWs w = fwd_layout(c, *attn);
  if (w.total > ws_bytes) return fail(MECEFO_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", ws_bytes, w.total);
  if (!ws) return fail(MECEFO_ERR_INVALID_ARG, "workspace is NULL");
  if (!any) return MECEFO_OK;
  char* base = (char*)up((int64_t)(uintptr_t)ws, 256);
  hipStream_t s = (hipStream_t)hip_stream;
  const mecefo_ffn_desc_t& d = *desc;
  const mecefo_attn_desc_t& a = *attn;
  const int b = (int)c.b, dm = c.dm, dh = dm / a.heads, S = a.seq;
  const bool keep = given == 5;
  void* Xn = base + w.Xn;
  float* rstd = (float*)(base + w.rstd);
  void* Q = keep ? out->Q : base + w.Q; void* K = keep ? out->K : base + w.K;
  void* V = keep ? out->V : base + w.V; void* O = keep ? out->O : base + w.O;
  float* L = keep ? out->L : (float*)(base + w.L);
  const int64_t ldq = keep ? d.ld_act_d : dm;   // row stride of Q, K, V, O
  float* cs = (float*)(base + w.cs); float* sn = (float*)(base + w.sn);
  float* S32 = (float*)(base + w.S32);
  void* P = base + w.P;
  const size_t rowbytes = (size_t)dm * c.esz;

  HIP_TRY(launch_rmsnorm_fwd(c.bf16, in->X, d.ld_act_d, in->g_attn, d.rms_eps, Xn, dm, rstd, c.b, dm, s));
  {  // Q, K, V = Xn Wq^T, Xn Wk^T, Xn Wv^T  [b x d], K = d
    GemmLaunch g = new_launch(c, true, true, EPI_STORE);
    g.nprob = 3;
    void* dst[3] = {Q, K, V};
    const void* wt[3] = {in->Wq, in->Wk, in->Wv};
    for (int i = 0; i < 3; ++i) g.p[i] = prob(Xn, nullptr, dm, wt[i], nullptr, a.ld_w_dd, dst[i], nullptr, nullptr, ldq, b, dm, dm, 1);
    HIP_TRY(launch_gemm(g, s));
  }
  HIP_TRY(launch_rope_tables(cs, sn, S, dh, (double)a.rope_theta, s));
  HIP_TRY(launch_rope(c.bf16, Q, ldq, cs, sn, c.b, S, a.heads, dh, false, s));
  HIP_TRY(launch_rope(c.bf16, K, ldq, cs, sn, c.b, S, a.heads, dh, false, s));
  const float scale = 1.0f / sqrtf((float)dh);
  const bool fused = fwd_attention_fused(c, a);
  if (fused) HIP_TRY(launch_attn_fwd(Q, K, V, O, ldq, L, a.batch, S, a.heads, dh, scale, s));
  for (int bi = 0; bi < (fused ? 0 : a.batch); ++bi)
    for (int h0 = 0; h0 < a.heads; h0 += w.hc) {
      const int hc = a.heads - h0 < w.hc ? a.heads - h0 : w.hc;
      const int64_t tok = ((int64_t)bi * S * ldq + (int64_t)h0 * dh) * c.esz;
      const char* Qc = (const char*)Q + tok; const char* Kc = (const char*)K + tok; const char* Vc = (const char*)V + tok;
      char* Oc = (char*)O + tok;
      auto batched = [&](GemmProblem& p, int64_t abi, int64_t bbi, int64_t cbi) {
        p.batch = hc; p.batch_inner = hc;
        p.a_bo = 0; p.b_bo = 0; p.c_bo = 0; p.a_bi = abi; p.b_bi = bbi; p.c_bi = cbi;
      };
      {  // raw scores q.k in fp32, blocks above the diagonal skipped
        GemmLaunch g = new_launch(c, true, true, EPI_GRAD);
        g.out_f32 = true;
        g.nprob = 1;
        g.p[0] = prob(Qc, nullptr, ldq, Kc, nullptr, ldq, S32, nullptr, nullptr, w.ldp, S, S, dh, 1);
        // output offsets are counted in operand elements: fp32 scores behind bf16 operands take two each
        batched(g.p[0], dh, dh, (int64_t)S * w.ldp * (c.bf16 ? 2 : 1));
        g.p[0].causal = CAUSAL_TILE;
        HIP_TRY(launch_gemm(g, s));
      }
      HIP_TRY(launch_softmax_rows(c.bf16, S32, w.ldp, P, w.ldp, L + ((int64_t)bi * a.heads + h0) * S, hc, S, scale, s));
      {  // O = P V  [seq x dh], contraction over the keys up to the diagonal block
        GemmLaunch g = new_launch(c, true, false, EPI_STORE);
        g.nprob = 1;
        g.p[0] = prob(P, nullptr, w.ldp, Vc, nullptr, ldq, Oc, nullptr, nullptr, ldq, S, dh, S, 1);
        batched(g.p[0], (int64_t)S * w.ldp, dh, dh);
        g.p[0].causal = CAUSAL_K_UPTO_M;
        HIP_TRY(launch_gemm(g, s));
      }
    }
  // H = X + O Wo^T: the product accumulates onto a copy of X
  HIP_TRY(hipMemcpy2DAsync(out->H, (size_t)d.ld_act_d * c.esz, in->X, (size_t)d.ld_act_d * c.esz, rowbytes, (size_t)b, hipMemcpyDeviceToDevice, s));
  {
    GemmLaunch g = new_launch(c, true, true, EPI_GRAD);
    g.out_f32 = false;
    g.accumulate = 1;
    g.nprob = 1;
    g.p[0] = prob(O, nullptr, ldq, in->Wo, nullptr, a.ld_w_dd, out->H, nullptr, nullptr, d.ld_act_d, b, dm, dm, 1);
    HIP_TRY(launch_gemm(g, s));
  }
  // FFN: U = norm(H), A = silu(U Wg^T) * (U Wu^T), Out = H + A Wd^T
  HIP_TRY(launch_rmsnorm_fwd(c.bf16, out->H, d.ld_act_d, in->g_ffn, d.rms_eps, Xn, dm, rstd, c.b, dm, s));
  void* AA = base + w.A;
  {
    GemmLaunch g = new_launch(c, true, true, EPI_SWIGLU_FWD);
    g.nprob = 1;
    g.p[0] = prob(Xn, nullptr, dm, in->Wg, in->Wu, d.ld_w_fd, nullptr, nullptr, AA, c.ldf, b, c.ff, dm, 1, (int)c.ldf);
    HIP_TRY(launch_gemm(g, s));
  }
  HIP_TRY(hipMemcpy2DAsync(out->Out, (size_t)d.ld_act_d * c.esz, out->H, (size_t)d.ld_act_d * c.esz, rowbytes, (size_t)b, hipMemcpyDeviceToDevice, s));
  {
    GemmLaunch g = new_launch(c, true, true, EPI_GRAD);
    g.out_f32 = false;
    g.accumulate = 1;
    g.nprob = 1;
    g.p[0] = prob(AA, nullptr, c.ldf, in->Wd, nullptr, d.ld_w_df, out->Out, nullptr, nullptr, d.ld_act_d, b, dm, c.ff, 1);
    HIP_TRY(launch_gemm(g, s));
  }
  return MECEFO_OK;
}

mecefo_status_t mecefo_stack_workspace_bytes(const mecefo_ffn_desc_t* desc, const mecefo_attn_desc_t* attn,
                                             int r_gate, int r_up, int r_down, size_t* out_bytes) {
  size_t fwd = 0, bwd = 0;
  TRY(mecefo_block_fwd_workspace_bytes(desc, attn, &fwd));
  TRY(mecefo_workspace_bytes(desc, r_gate, r_up, r_down, &bwd));
  if (!out_bytes) return fail(MECEFO_ERR_INVALID_ARG, "out_bytes is NULL");
  // two [b x ld] activation buffers for the forward ping-pong behind the larger of the two workspaces
  const size_t act = (size_t)up((int64_t)desc->tokens * desc->ld_act_d * (desc->dtype == MECEFO_BF16 ? 2 : 4), 256);
  *out_bytes = (fwd > bwd ? fwd : bwd) + 2 * act + 512;
  return MECEFO_OK;
}

mecefo_status_t mecefo_stack_fwd_neighbor(const mecefo_ffn_desc_t* desc, const mecefo_attn_desc_t* attn,
                                          int n_layers, const mecefo_layer_weights_t* layers, const void* X0,
                                          void* const* H, void* X_out, void* ws, size_t ws_bytes,
                                          void* hip_stream) {
  Ctx c;
  TRY(check_desc(desc, &c));
  TRY(check_attn(c, attn));
  if (n_layers < 1) return fail(MECEFO_ERR_INVALID_ARG, "n_layers must be >= 1");
  if (!layers || !H) return fail(MECEFO_ERR_INVALID_ARG, "layers and H are required");
  if (c.b > 0 && X_out == X0) return fail(MECEFO_ERR_INVALID_ARG, "X_out must not alias X0");
  size_t inner = 0;
  TRY(mecefo_block_fwd_workspace_bytes(desc, attn, &inner));
  const size_t act = (size_t)up(c.b * desc->ld_act_d * c.esz, 256);
  if (!ws) return fail(MECEFO_ERR_INVALID_ARG, "workspace is NULL");
  char* base = (char*)up((int64_t)(uintptr_t)ws, 256);
  const size_t lead = (size_t)(base - (char*)ws);
  if (lead + 2 * act + inner > ws_bytes) return fail(MECEFO_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", ws_bytes, lead + 2 * act + inner);
  void* pp[2] = {base, base + act};
  void* inner_ws = base + 2 * act;
  const void* x = X0;
  for (int l = 0; l < n_layers; ++l) {
    const mecefo_layer_weights_t& w = layers[l];
    mecefo_block_fwd_inputs_t in = {x, w.g_attn, w.g_ffn, w.Wq, w.Wk, w.Wv, w.Wo, w.Wg, w.Wu, w.Wd};
    void* y = l == n_layers - 1 ? X_out : pp[l & 1];
    mecefo_block_fwd_outputs_t out = {y, H[l], nullptr, nullptr, nullptr, nullptr, nullptr};
    mecefo_status_t st = mecefo_block_fwd(desc, attn, &in, &out, inner_ws, ws_bytes - lead - 2 * act, hip_stream);
    if (st != MECEFO_OK) return st;
    x = y;
  }
  return MECEFO_OK;
}

mecefo_status_t mecefo_stack_bwd_skip(const mecefo_ffn_desc_t* desc, int n_layers, const mecefo_layer_weights_t* layers,
                                      const void* const* H, const mecefo_layer_lowrank_t* lowrank, mecefo_side_t side,
                                      const void* dOut_top, void* dX_bottom, int accumulate, void* ws,
                                      size_t ws_bytes, void* hip_stream) {
  if (n_layers < 1) return fail(MECEFO_ERR_INVALID_ARG, "n_layers must be >= 1");
  if (!layers || !H || !lowrank) return fail(MECEFO_ERR_INVALID_ARG, "layers, H and lowrank are required");
  // the gradient travels down in dX_bottom's buffer: every layer overwrites its dOut with its dX
  const void* g = dOut_top;
  for (int l = n_layers - 1; l >= 0; --l) {
    const mecefo_layer_weights_t& w = layers[l];
    const mecefo_layer_lowrank_t& q = lowrank[l];
    mecefo_status_t st = mecefo_block_bwd_skip(desc, H[l], g, w.g_ffn, w.Wg, w.Wu, w.Wd, q.Pg, q.Pu, q.Pd, side,
                                               dX_bottom, q.dg_ffn, q.dWg, q.dWu, q.dWd, accumulate, ws, ws_bytes,
                                               hip_stream);
    if (st != MECEFO_OK) return st;
    g = dX_bottom;
  }
  return MECEFO_OK;
}


mecefo_status_t mecefo_block_bwd_skip_noalloc(const mecefo_ffn_desc_t* desc, const void* H, const void* dOut,
                                              const void* gamma, const void* Wg, const void* Wu, const void* Wd,
                                              mecefo_proj_t Pg, mecefo_proj_t Pu, mecefo_proj_t Pd, mecefo_side_t side,
                                              void* dX, void* dgamma, void* dWg, void* dWu, void* dWd, int accumulate,
                                              void* hip_stream) {
  size_t need = 0;
  TRY(mecefo_workspace_bytes(desc, Pg.r > 0 ? Pg.r : 0, Pu.r > 0 ? Pu.r : 0, Pd.r > 0 ? Pd.r : 0, &need));
  if (need > (size_t)MECEFO_NOALLOC_SCRATCH_BYTES)
    return fail(MECEFO_ERR_WORKSPACE_TOO_SMALL,
                "this shape needs %zu bytes of scratch; the static buffer of mecefo_block_bwd_skip_noalloc holds %zu "
                "(use mecefo_block_bwd_skip with a workspace of the caller's)", need, (size_t)MECEFO_NOALLOC_SCRATCH_BYTES);
  void* ws = nullptr;
  TRY(scratch_on_current_device(&ws));
  // Nothing in the scratch has to start at zero: every region of the workspace layout is written by a
  // kernel of this call before a later kernel of the same call reads it.
  return mecefo_block_bwd_skip(desc, H, dOut, gamma, Wg, Wu, Wd, Pg, Pu, Pd, side, dX, dgamma, dWg, dWu, dWd, accumulate,
                               ws, (size_t)MECEFO_NOALLOC_SCRATCH_BYTES, hip_stream);
}

// ---- Alg. 1 / Alg. 3 bookkeeping and the stack backward with a mode per layer ----------------
int mecefo_refresh_due(int64_t t, int64_t tau) { return tau >= 1 && t >= 0 && t % tau == 0; }

void mecefo_counters_reset(int64_t* t, int n_layers) {
  if (!t) return;
  for (int l = 0; l < n_layers; ++l) t[l] = 0;
}

mecefo_status_t mecefo_stack_mixed_workspace_bytes(const mecefo_ffn_desc_t* desc, const mecefo_attn_desc_t* attn,
                                                   int r_gate, int r_up, int r_down, size_t* out_bytes) {
  size_t full = 0, skip = 0;
  TRY(mecefo_block_full_workspace_bytes(desc, attn, &full));
  TRY(mecefo_workspace_bytes(desc, r_gate, r_up, r_down, &skip));
  if (!out_bytes) return fail(MECEFO_ERR_INVALID_ARG, "out_bytes is NULL");
  size_t best = full > skip ? full : skip;
  // projection refresh of the three FFN matrices, one after the other in the same workspace (either side)
  const int rr[3] = {r_gate, r_up, r_down};
  for (int i = 0; i < 3; ++i) {
    if (rr[i] <= 0) continue;
    const int m = i < 2 ? desc->d_ff : desc->d_model, n = i < 2 ? desc->d_model : desc->d_ff;
    for (int left = 0; left < 2; ++left) {
      size_t pw = 0;
      TRY(mecefo_projection_workspace_bytes(desc->dtype, m, n, rr[i], left, &pw));
      if (pw > best) best = pw;
    }
  }
  *out_bytes = best;
  return MECEFO_OK;
}

mecefo_status_t mecefo_stack_bwd_mixed(const mecefo_ffn_desc_t* desc, const mecefo_attn_desc_t* attn, int n_layers,
                                       const mecefo_mode_t* modes, const mecefo_block_inputs_t* in,
                                       const mecefo_block_grads_t* grads, const mecefo_layer_lowrank_t* lowrank,
                                       mecefo_side_t side, const mecefo_refresh_policy_t* policy, int64_t* t,
                                       const void* dOut_top, void* dX_bottom, int accumulate, void* ws,
                                       size_t ws_bytes, void* hip_stream) {
  if (n_layers < 1) return fail(MECEFO_ERR_INVALID_ARG, "n_layers must be >= 1");
  if (!modes || !in || !grads) return fail(MECEFO_ERR_INVALID_ARG, "modes, in and grads are required");
  if (!desc) return fail(MECEFO_ERR_INVALID_ARG, "descriptor is NULL");
  bool any_neighbor = false;
  for (int l = 0; l < n_layers; ++l) {
    if (modes[l] != MECEFO_MODE_STANDARD && modes[l] != MECEFO_MODE_NEIGHBOR)
      return fail(MECEFO_ERR_INVALID_ARG, "layer %d: mode must be MECEFO_MODE_STANDARD or MECEFO_MODE_NEIGHBOR", l);
    any_neighbor |= modes[l] == MECEFO_MODE_NEIGHBOR;
  }
  if (any_neighbor && !lowrank) return fail(MECEFO_ERR_INVALID_ARG, "lowrank is required when a layer runs in neighbor mode");
  if ((policy == nullptr) != (t == nullptr)) return fail(MECEFO_ERR_INVALID_ARG, "policy and t must both be given or both be NULL");
  if (policy && (policy->tau < 1 || policy->power_iters < 1 || policy->cond_steps < 0 || policy->polish_steps < 0))
    return fail(MECEFO_ERR_INVALID_ARG, "refresh policy: tau >= 1, power_iters >= 1, cond_steps >= 0, polish_steps >= 0 required");
  const bool left = side == MECEFO_SIDE_OUTPUT;
  // the gradient travels down in dX_bottom's buffer: every layer overwrites its dOut with its dX
  const void* g = dOut_top;
  for (int l = n_layers - 1; l >= 0; --l) {
    const mecefo_block_inputs_t& x = in[l];
    const mecefo_block_grads_t& o = grads[l];
    mecefo_status_t st;
    if (modes[l] == MECEFO_MODE_STANDARD) {           // Alg. 3, first branch: exact gradients, MHA included
      mecefo_block_inputs_t xi = x;
      xi.dOut = g;
      mecefo_block_grads_t oi = o;
      oi.dX = dX_bottom;
      st = mecefo_block_bwd_full(desc, attn, &xi, &oi, accumulate, ws, ws_bytes, hip_stream);
    } else {                                          // neighbor branch
      const mecefo_layer_lowrank_t& q = lowrank[l];
      if (policy && mecefo_refresh_due(t[l], policy->tau)) {
        // V1 of the current weights (Alg. 3: every tau neighbor steps of this layer), warm-started from and
        // written over the layer's present projection
        const void* W[3] = {x.Wg, x.Wu, x.Wd};
        const mecefo_proj_t P[3] = {q.Pg, q.Pu, q.Pd};
        for (int i = 0; i < 3; ++i) {
          const int m = i < 2 ? desc->d_ff : desc->d_model, n = i < 2 ? desc->d_model : desc->d_ff;
          const int64_t ldw = i < 2 ? desc->ld_w_fd : desc->ld_w_df;
          st = mecefo_projection_refresh(desc->dtype, W[i], m, n, ldw, left ? 1 : 0, P[i].P, P[i].ld, P[i].r,
                                         policy->power_iters, policy->cond_steps, policy->polish_steps,
                                         const_cast<void*>(P[i].P), P[i].ld, ws, ws_bytes, hip_stream);
          if (st != MECEFO_OK) return st;
        }
      }
      st = mecefo_block_bwd_skip(desc, x.H, g, x.g_ffn, x.Wg, x.Wu, x.Wd, q.Pg, q.Pu, q.Pd, side, dX_bottom,
                                 q.dg_ffn, q.dWg, q.dWu, q.dWd, accumulate, ws, ws_bytes, hip_stream);
      if (st == MECEFO_OK && t) t[l] += 1;            // Alg. 3: the local step counter of this layer
    }
    if (st != MECEFO_OK) return st;
    g = dX_bottom;
  }
  return MECEFO_OK;
}

}  // extern "C"

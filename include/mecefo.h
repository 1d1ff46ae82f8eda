/*
 * mecefo.h -- C ABI of the MI355X (gfx950) degraded transformer-block backward of
 * MeCeFO (arxiv 2510.16415).
 *
 * What the calls compute (paper passages they follow):
 *   - Alg. 3, neighbor branch: recompute the FFN activations from the one stored
 *     tensor, form the three FFN weight gradients with Eq. (2), skip the MHA
 *     connection and hand the activation gradient to the previous layer.
 *   - Sec. 3.2 (skip-connection): the MHA branch is cut in the backward pass only;
 *     no MHA parameter gets a gradient on this rank.
 *   - Sec. 3.3 (selective recomputation): only the input of the FFN module is kept.
 *   - Sec. 3.4 Eq. (2): G_W = G_y x^T ~= G_y (x^T V1) V1^T, V1 in R^{n x r}.
 *   - Sec. 2: LLaMA block, FFN = W_down( silu(W_gate u) * (W_up u) ), RMSNorm, residual.
 * Around that hot path, further below: the standard-mode backward (Alg. 3, first branch), the
 * block forward of both modes (Alg. 2), a stack of blocks in neighbor mode, tunable variants,
 * the projection refresh (Alg. 3, every tau steps), Eq. (1) gradient averaging and AdamW (Alg. 1).
 *
 * Notation (row-major, token index along rows, weights in [out x in] layout):
 *   b tokens, d = d_model, f = d_ff, r = rank.
 *   H  [b x d]  stored FFN-module input (residual stream before the FFN norm)
 *   U  [b x d]  = RMSNorm(H) * gamma          Wg, Wu [f x d]   Wd [d x f]
 *   G = U Wg^T, Z = U Wu^T [b x f];  S = silu(G);  A = S*Z;  Y = A Wd^T;  Out = H + Y.
 *
 * Memory and ownership: EVERY data pointer is a DEVICE pointer owned by the caller
 * (descriptors and size outputs are host memory).  The library allocates and frees
 * nothing; scratch comes from the caller's workspace, sized by
 * mecefo_workspace_bytes().  Calls only enqueue work on the given HIP stream
 * (a hipStream_t passed as void*, NULL = default stream) and return without
 * synchronising.  Workspace contents are undefined after a call; two calls that
 * share a workspace must be ordered on the same stream.
 * Stream capture: the calls are capturable into a HIP graph.  The first launch of a kernel on a
 * device also raises that kernel's dynamic-LDS limit (hipFuncSetAttribute, host side, once per kernel
 * and device); mecefo_init() does that for every kernel of the library up front, so a caller that
 * captures calls it once per device before the capture (no eager warm-up run is needed).
 *
 * Layout rules: every matrix is row-major with an explicit row stride in elements.
 * dtype MECEFO_BF16: storage bf16, fp32 accumulation in MFMA; all data pointers must
 * be 16-byte aligned and all row strides multiples of 8 elements (so an odd d_ff such
 * as 5461 needs ld >= 5464); columns between the logical width and the stride are
 * never read as data.  dtype MECEFO_F32: no alignment rule beyond 4 bytes.
 * Every tensor must be smaller than 2 GiB.  With tokens == 0 the [b x *] pointers may be NULL.
 *
 * Errors: argument checks happen on the host before anything is enqueued; on a
 * non-OK status nothing was launched by that call (MECEFO_ERR_LAUNCH excepted) and
 * mecefo_last_error() returns a thread-local description.  No C++ exception
 * crosses this boundary.
 */
#ifndef MECEFO_H_
#define MECEFO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MECEFO_OK = 0,
  MECEFO_ERR_INVALID_ARG = 1,          /* NULL required pointer, bad size/stride/alignment/rank */
  MECEFO_ERR_UNSUPPORTED = 2,          /* dtype combination or size not built */
  MECEFO_ERR_WORKSPACE_TOO_SMALL = 3,
  MECEFO_ERR_LAUNCH = 4                /* HIP reported an error while enqueuing */
} mecefo_status_t;

typedef enum { MECEFO_F32 = 0, MECEFO_BF16 = 1 } mecefo_dtype_t;

/* Which side of y = W x Eq. (2) projects.
 * MECEFO_SIDE_INPUT  (the paper's form): P = V1 in R^{n_in x r};  dW = (Gy^T (X P)) P^T.
 * MECEFO_SIDE_OUTPUT (mirror form):      P in R^{m_out x r};      dW = P ((X^T (Gy P)))^T. */
typedef enum { MECEFO_SIDE_INPUT = 0, MECEFO_SIDE_OUTPUT = 1 } mecefo_side_t;

typedef struct {
  int64_t tokens;               /* b */
  int32_t d_model, d_ff;        /* d, f */
  int64_t ld_act_d, ld_act_f;   /* row strides of caller [b x d] and [b x f] tensors (>= d, >= f) */
  int64_t ld_w_fd, ld_w_df;     /* row strides of Wg/Wu/dWg/dWu [f x d] and Wd/dWd [d x f] */
  mecefo_dtype_t dtype;         /* activations, weights, projections */
  mecefo_dtype_t grad_dtype;    /* dWg/dWu/dWd/dgamma buffers: MECEFO_F32, or equal to dtype */
  float rms_eps;                /* RMSNorm epsilon; used only when gamma != NULL */
} mecefo_ffn_desc_t;

/* Projection matrix, row-major [dim x r] with row stride ld (>= r).  dim is the
 * projected dimension: SIDE_INPUT: d for gate/up, f for down; SIDE_OUTPUT: f for
 * gate/up, d for down.  1 <= r <= dim.  P is opaque data: it need not be orthonormal
 * nor related to the current weights (Alg. 3 reuses it for tau steps). */
typedef struct { const void* P; int32_t r; int64_t ld; } mecefo_proj_t;

/* Bytes of workspace that any of the calls below needs for this descriptor and these
 * ranks (pass the largest ranks you will use; 0 if only the non-low-rank calls are used). */
mecefo_status_t mecefo_workspace_bytes(const mecefo_ffn_desc_t* desc, int r_gate, int r_up,
                                       int r_down, size_t* out_bytes);

/* Sec. 3.3 Rcomp.  In: U [b x d] (ld_act_d), Wg, Wu [f x d], Wd [d x f] or NULL.
 * Out: G, Z, A [b x f] (ld_act_f); Y [b x d] (ld_act_d) = A Wd^T, or NULL to skip the
 * down projection (the backward never needs it).  Any of G, Z may be NULL (not stored). */
mecefo_status_t mecefo_ffn_fwd_recompute(const mecefo_ffn_desc_t* desc, const void* U,
    const void* Wg, const void* Wu, const void* Wd,
    void* G, void* Z, void* A, void* Y, void* ws, size_t ws_bytes, void* hip_stream);

/* Exact FFN backward (the comparator Eq. (2) approximates).  In: U, dY [b x d];
 * weights; G, Z [b x f] saved activations, or both NULL to recompute them from U.
 * Out: dU [b x d] (may be NULL), dWg, dWu [f x d], dWd [d x f] in grad_dtype.
 * accumulate = 0 overwrites the dW buffers, 1 adds to them. */
mecefo_status_t mecefo_ffn_bwd_exact(const mecefo_ffn_desc_t* desc, const void* U, const void* dY,
    const void* Wg, const void* Wu, const void* Wd, const void* G, const void* Z,
    void* dU, void* dWg, void* dWu, void* dWd, int accumulate,
    void* ws, size_t ws_bytes, void* hip_stream);

/* Alg. 3 neighbor branch, FFN part: recompute from U, exact dU, Eq. (2) weight gradients. */
mecefo_status_t mecefo_ffn_bwd_lowrank(const mecefo_ffn_desc_t* desc, const void* U, const void* dY,
    const void* Wg, const void* Wu, const void* Wd,
    mecefo_proj_t Pg, mecefo_proj_t Pu, mecefo_proj_t Pd, mecefo_side_t side,
    void* dU, void* dWg, void* dWu, void* dWd, int accumulate,
    void* ws, size_t ws_bytes, void* hip_stream);

/* Whole neighbor-mode backward of one block (Alg. 3: recompute, Eq. (2), skip MHA).
 * In: H [b x d] stored FFN-module input; dOut [b x d] gradient of the block output;
 * gamma [d] FFN-norm gain (dtype), or NULL meaning the stored tensor feeds the FFN
 * directly (U = H).  Out: dX [b x d] = dOut + normbwd(dU): the gradient handed to the
 * previous layer (the MHA branch contributes nothing); dX may alias dOut.  dgamma [d]
 * in grad_dtype or NULL.  dWg, dWu, dWd as above.  No MHA weight or gradient buffer is
 * an argument: this rank produces none (Sec. 3.2). */
mecefo_status_t mecefo_block_bwd_skip(const mecefo_ffn_desc_t* desc, const void* H,
    const void* dOut, const void* gamma,
    const void* Wg, const void* Wu, const void* Wd,
    mecefo_proj_t Pg, mecefo_proj_t Pu, mecefo_proj_t Pd, mecefo_side_t side,
    void* dX, void* dgamma, void* dWg, void* dWu, void* dWd, int accumulate,
    void* ws, size_t ws_bytes, void* hip_stream);

/* mecefo_block_bwd_skip for callers that can neither allocate nor bring a workspace: code under HIP graph
 * capture, tight serving or training loops and harnesses that forbid hipMalloc.  Same arguments and results
 * as mecefo_block_bwd_skip without ws / ws_bytes: the scratch is a buffer of MECEFO_NOALLOC_SCRATCH_BYTES
 * that the library holds in static device memory on every GPU it is loaded on (until the process ends), so
 * the call itself allocates and frees nothing.  Shapes whose workspace (mecefo_workspace_bytes) exceeds that
 * size are rejected with MECEFO_ERR_WORKSPACE_TOO_SMALL before anything is enqueued (64 MiB covers e.g.
 * 2048 tokens at d = 512, f = 1376, r = 128; the 7B-shaped layer needs 0.75 GiB and the caller's own
 * workspace).  All calls on one GPU share that GPU's buffer and it keeps the last call's contents: calls
 * that overlap in time on one GPU (different streams or host threads) race; order them on one stream. */
#define MECEFO_NOALLOC_SCRATCH_BYTES (64u << 20)
mecefo_status_t mecefo_block_bwd_skip_noalloc(const mecefo_ffn_desc_t* desc, const void* H,
    const void* dOut, const void* gamma,
    const void* Wg, const void* Wu, const void* Wd,
    mecefo_proj_t Pg, mecefo_proj_t Pu, mecefo_proj_t Pd, mecefo_side_t side,
    void* dX, void* dgamma, void* dWg, void* dWu, void* dWd, int accumulate,
    void* hip_stream);

/* ---- Standard-mode backward of one block (Alg. 3, first branch: the rank runs its own layer
 * without approximation).  Block: H = X + MHA(norm(X; g_attn)); Out = H + FFN(norm(H; g_ffn));
 * MHA = causal multi-head attention with rotary position embedding (pairs (j, j + dh/2) of a
 * head rotated by position * theta^(-2j/dh)), softmax scale 1/sqrt(dh), no biases (Sec. 2).
 * This is the comparator that the neighbor-mode call is measured against (Sec. 3.5 overhead,
 * Table 6): every gradient is exact.  The FFN activations are recomputed from H as in the
 * neighbor branch; the attention tensors below are the ones a forward pass keeps. */
typedef struct {
  int32_t batch, seq;     /* sequences and tokens per sequence; batch * seq == desc->tokens     */
  int32_t heads;          /* d_model % heads == 0 and dh = d_model / heads even                   */
  float rope_theta;       /* rotary base (10000 for LLaMA)                                        */
  int64_t ld_w_dd;        /* row stride of Wq, Wk, Wv, Wo and their gradients [d x d]             */
} mecefo_attn_desc_t;

/* Inputs: all [b x d] tensors are token-major with row stride ld_act_d; head h owns columns
 * [h*dh, (h+1)*dh).  Q and K are stored after the rotation.  L [batch*heads*seq] fp32 is the
 * row-wise log-sum-exp of the scaled, causally masked scores, index (sequence*heads + head)*seq + s. */
typedef struct {
  const void *X, *H, *dOut;                 /* block input, FFN-module input, output gradient  */
  const void *g_attn, *g_ffn;               /* [d] gains of the two RMSNorms                    */
  const void *Wq, *Wk, *Wv, *Wo;            /* [d x d], y = W x                                  */
  const void *Wg, *Wu, *Wd;                 /* FFN weights                                       */
  const void *Q, *K, *V, *O;                /* saved by the forward pass, [b x d]                */
  const float* L;                           /* saved log-sum-exp                                  */
} mecefo_block_inputs_t;

/* Outputs: dX [b x d] (activation dtype; may alias dOut); the rest in grad_dtype, overwritten or
 * accumulated into as `accumulate` says.  All are required. */
typedef struct {
  void* dX;
  void *dg_attn, *dg_ffn;
  void *dWq, *dWk, *dWv, *dWo;
  void *dWg, *dWu, *dWd;
} mecefo_block_grads_t;

/* Workspace of mecefo_block_bwd_full: dominated by the materialised attention probabilities,
 * batch*heads*seq*seq elements of the activation dtype. */
mecefo_status_t mecefo_block_full_workspace_bytes(const mecefo_ffn_desc_t* desc,
    const mecefo_attn_desc_t* attn, size_t* out_bytes);

mecefo_status_t mecefo_block_bwd_full(const mecefo_ffn_desc_t* desc, const mecefo_attn_desc_t* attn,
    const mecefo_block_inputs_t* in, const mecefo_block_grads_t* out, int accumulate,
    void* ws, size_t ws_bytes, void* hip_stream);

/* ---- Forward of one block in either mode (Alg. 2: the forward pass is the same computation in
 * both modes; what differs is what is kept for the backward).  Computes
 *   H = X + MHA(norm(X; g_attn)),  Out = H + FFN(norm(H; g_ffn)).
 * Standard mode: pass buffers for H, Q, K, V, O [b x d] and L [batch*heads*seq] (fp32); they are
 * exactly what mecefo_block_bwd_full takes.  Neighbor mode (Sec. 3.3: only the input of the FFN
 * module is kept): pass H only and NULL for Q, K, V, O, L; the attention tensors then live in the
 * workspace and are dropped.  Out [b x d] is required and must not alias X; H is required. */
typedef struct {
  const void* X;
  const void *g_attn, *g_ffn;
  const void *Wq, *Wk, *Wv, *Wo;
  const void *Wg, *Wu, *Wd;
} mecefo_block_fwd_inputs_t;

typedef struct {
  void* Out;
  void* H;
  void *Q, *K, *V, *O;   /* all four given, or all four NULL */
  float* L;              /* given iff Q is given */
} mecefo_block_fwd_outputs_t;

/* Workspace: a few [b x d] activations and one [b x ld_act_f] activation.  bf16 with head dimension
 * 64 or 128 runs the attention as one fused kernel (running maximum and sum per query, no score
 * buffer); other shapes add fp32 scores and probabilities of a chunk of heads (at most 256 MiB of
 * scores).  mecefo_set_option("attention", "gemm") selects the second form everywhere (testing); the
 * query and the call consult the same switch, so set it before both. */
mecefo_status_t mecefo_block_fwd_workspace_bytes(const mecefo_ffn_desc_t* desc,
    const mecefo_attn_desc_t* attn, size_t* out_bytes);
mecefo_status_t mecefo_block_fwd(const mecefo_ffn_desc_t* desc, const mecefo_attn_desc_t* attn,
    const mecefo_block_fwd_inputs_t* in, const mecefo_block_fwd_outputs_t* out,
    void* ws, size_t ws_bytes, void* hip_stream);

/* ---- A stack of n_layers identical blocks in neighbor mode (Alg. 2 and Alg. 3 per layer, chained):
 * the forward keeps H_l of every layer and nothing else; the backward walks the layers from the top,
 * handing each layer's dX to the layer below as its dOut.  Both only enqueue (HIP-graph capturable:
 * a whole pass is one launch sequence without host decisions). */
typedef struct {
  const void *g_attn, *g_ffn;
  const void *Wq, *Wk, *Wv, *Wo;     /* unused by the backward: no MHA gradient in neighbor mode */
  const void *Wg, *Wu, *Wd;
} mecefo_layer_weights_t;

typedef struct {
  mecefo_proj_t Pg, Pu, Pd;
  void *dg_ffn, *dWg, *dWu, *dWd;     /* grad_dtype; dg_ffn may be NULL */
} mecefo_layer_lowrank_t;

/* X0 [b x d] -> X_out [b x d] (must not alias X0); H[l] [b x d] receives layer l's FFN-module input. */
mecefo_status_t mecefo_stack_workspace_bytes(const mecefo_ffn_desc_t* desc, const mecefo_attn_desc_t* attn,
    int r_gate, int r_up, int r_down, size_t* out_bytes);
mecefo_status_t mecefo_stack_fwd_neighbor(const mecefo_ffn_desc_t* desc, const mecefo_attn_desc_t* attn,
    int n_layers, const mecefo_layer_weights_t* layers, const void* X0, void* const* H, void* X_out,
    void* ws, size_t ws_bytes, void* hip_stream);
/* dOut_top [b x d]: gradient of the last layer's output; dX_bottom [b x d]: gradient of the first
 * layer's input (may alias dOut_top). */
mecefo_status_t mecefo_stack_bwd_skip(const mecefo_ffn_desc_t* desc, int n_layers,
    const mecefo_layer_weights_t* layers, const void* const* H, const mecefo_layer_lowrank_t* lowrank,
    mecefo_side_t side, const void* dOut_top, void* dX_bottom, int accumulate,
    void* ws, size_t ws_bytes, void* hip_stream);

/* ---- Mode per layer and the local step counters (Alg. 1: a node that takes over a failed peer's layers
 * runs those layers in neighbor mode and sets their counters t_{i,l} to zero; Alg. 3: in neighbor mode
 * the projection of layer l is recomputed from the current weights whenever t_{i,l} mod tau == 0, then
 * recompute, Eq. (2) and the skip run, and t_{i,l} grows by one; Sec. 5, extension paragraph: the skip may
 * be applied to a subset of the layers).  Counters are host integers owned by the caller. */
typedef enum { MECEFO_MODE_STANDARD = 0, MECEFO_MODE_NEIGHBOR = 1 } mecefo_mode_t;

typedef struct {
  int64_t tau;                                     /* refresh period, >= 1 (the paper's runs: 100)          */
  int32_t power_iters, cond_steps, polish_steps;   /* arguments of mecefo_projection_refresh (warm start)    */
} mecefo_refresh_policy_t;

/* 1 when a layer whose counter reads t must recompute its projection before this backward (t mod tau == 0). */
int mecefo_refresh_due(int64_t t, int64_t tau);
/* Alg. 1, on a failure: the counters of the layers taken over start again at zero (host memory). */
void mecefo_counters_reset(int64_t* t, int n_layers);

/* Backward of a stack whose layers run in the mode given per layer (host array modes[n_layers]), from the
 * top layer down, each layer's dX handed to the layer below in dX_bottom's buffer (may alias dOut_top).
 * in[l] / grads[l]: a standard-mode layer needs every field as mecefo_block_bwd_full does (dOut and dX are
 * ignored: the chain supplies them); a neighbor-mode layer reads in[l].H, g_ffn, Wg, Wu, Wd only, takes
 * its projections and FFN gradient buffers from lowrank[l], and leaves every MHA gradient buffer untouched.
 * policy and t [n_layers] (both or neither): when given, a neighbor-mode layer with
 * mecefo_refresh_due(t[l], policy->tau) first overwrites its three projections (device memory behind
 * lowrank[l].Pg/Pu/Pd) with mecefo_projection_refresh of its weights, warm-started from their present
 * contents, and t[l] is incremented after the layer's backward has been enqueued; standard-mode layers
 * leave t[l] alone.  The refresh decision is taken on the host while enqueuing: a captured graph replays
 * the decisions of the capture.  Workspace: mecefo_stack_mixed_workspace_bytes.
 * Errors: modes, policy and the pointer arrays are checked before anything is enqueued; the per-layer
 * argument checks run as each layer is reached, so when layer l is rejected the layers above it have
 * already been enqueued and their counters advanced (the returned message names the failing check). */
mecefo_status_t mecefo_stack_mixed_workspace_bytes(const mecefo_ffn_desc_t* desc, const mecefo_attn_desc_t* attn,
    int r_gate, int r_up, int r_down, size_t* out_bytes);
mecefo_status_t mecefo_stack_bwd_mixed(const mecefo_ffn_desc_t* desc, const mecefo_attn_desc_t* attn,
    int n_layers, const mecefo_mode_t* modes, const mecefo_block_inputs_t* in,
    const mecefo_block_grads_t* grads, const mecefo_layer_lowrank_t* lowrank, mecefo_side_t side,
    const mecefo_refresh_policy_t* policy, int64_t* t, const void* dOut_top, void* dX_bottom,
    int accumulate, void* ws, size_t ws_bytes, void* hip_stream);

/* ---- After the backward pass of a layer (Alg. 1): gradient average and optimizer step.
 * mecefo_grad_average is Eq. (1) on gradient buffers that live on this GPU (the exchange between
 * ranks is not part of the library): out = mean over the ranks r with contributes[r] != 0 of
 * grads[r], summed in rank order.  For q, k, v, o those are the ranks that are neither failed nor
 * neighbors; for gate, up, down every rank.  A rank that does not contribute may pass NULL.
 * If no rank contributes the result is zero (the paper leaves this case open).
 * grads: host array of n_ranks (<= 16) device pointers to n_elems elements of grad_dtype each
 * (padding elements of strided matrices are averaged along); out may alias one of them. */
mecefo_status_t mecefo_grad_average(mecefo_dtype_t grad_dtype, const void* const* grads,
    const int32_t* contributes, int n_ranks, void* out, int64_t n_elems, void* hip_stream);

/* AdamW with decoupled weight decay (the paper's training configuration: beta1 0.9, beta2 0.999,
 * eps 1e-8, weight decay 0.01), step >= 1:
 *   m = b1 m + (1-b1) g;  v = b2 v + (1-b2) g^2;
 *   w = w (1 - lr wd) - lr (m / (1 - b1^step)) / (sqrt(v / (1 - b2^step)) + eps).
 * W [n_elems] in w_dtype (updated in place), G in grad_dtype (F32 or w_dtype), M and V fp32. */
mecefo_status_t mecefo_adamw_step(mecefo_dtype_t w_dtype, mecefo_dtype_t grad_dtype, void* W,
    const void* G, float* M, float* V, int64_t n_elems, int64_t step, float lr, float beta1,
    float beta2, float eps, float weight_decay, void* hip_stream);

/* ---- Projection refresh (Alg. 3: every tau neighbor steps the projection of a layer is recomputed
 * from its current weights, W = U S V^T, V1 = the first r columns of V; Sec. 3.4).
 * The call approximates span(V1) on the GEMM core without an SVD or a QR factorisation:
 * `power_iters` rounds of subspace iteration X <- W^T (W X), each followed by a Frobenius
 * normalisation and `cond_steps` quintic Newton-Schulz steps (each multiplies a small singular
 * value of X by 3.44: about log(k^2)/log(3.44) + 3 steps for k = s_1/s_r; 5 to 8 in practice) X <- X (aI + bA + cA^2), A = X^T X,
 * which re-condition the basis without changing its span; `polish_steps` cubic steps
 * X <- X + X (I - X^T X)/2 then drive X^T X to the identity (3 reach the bf16 floor, 5 the fp32 one).  The error of the subspace after q
 * rounds is of order (s_{r+1}/s_r)^(2q) times the error of the start basis (plus the rounding of
 * the storage type), so a warm start (the previous projection) needs few rounds.
 * In: W [m x n] row-major (row stride ldw); left = 0: right singular vectors (the paper's V1,
 * basis [n x r]); left = 1: left singular vectors (basis [m x r], for MECEFO_SIDE_OUTPUT);
 * V0 [dim x r] (row stride ldv) start basis of full column rank: the previous projection or
 * Gaussian noise.  Out: P [dim x r] (row stride ldp), the same layout mecefo_proj_t takes; P may
 * alias V0.  1 <= r <= min(m, n).  bf16: 16-byte aligned pointers, ldw % 8 == 0.  Only enqueues. */
mecefo_status_t mecefo_projection_workspace_bytes(mecefo_dtype_t dtype, int m, int n, int r, int left,
    size_t* out_bytes);
mecefo_status_t mecefo_projection_refresh(mecefo_dtype_t dtype, const void* W, int m, int n, int64_t ldw,
    int left, const void* V0, int64_t ldv, int r, int power_iters, int cond_steps, int polish_steps,
    void* P, int64_t ldp, void* ws, size_t ws_bytes, void* hip_stream);

/* ---- Tunable variants of the neighbor branch (Sec. 5, extension paragraph: the skip, the
 * recomputation depth and the rank are knobs).  mecefo_block_bwd_skip_ex is mecefo_block_bwd_skip
 * with two options; opt == NULL or all-zero options give exactly mecefo_block_bwd_skip.
 *   G, Z [b x f] (ld_act_f): extra checkpoints.  When given, the gate and up projections kept by
 *     the forward pass are used and the recompute GEMM is not run (b*f*2 more elements kept per
 *     layer, 4bdf fewer FLOPs).
 *   exact_wgrad_mask: bit 0 gate, bit 1 up, bit 2 down: those matrices get the exact weight
 *     gradient G_y^T x instead of Eq. (2) (their mecefo_proj_t argument is ignored).  Mask 7 is the
 *     skip-connection and recomputation without the low-rank approximation.
 * The rank itself is per matrix in the mecefo_proj_t arguments. */
typedef struct {
  const void *G, *Z;
  int32_t exact_wgrad_mask;
} mecefo_skip_options_t;

mecefo_status_t mecefo_block_bwd_skip_ex(const mecefo_ffn_desc_t* desc, const void* H,
    const void* dOut, const void* gamma,
    const void* Wg, const void* Wu, const void* Wd,
    mecefo_proj_t Pg, mecefo_proj_t Pu, mecefo_proj_t Pd, mecefo_side_t side,
    const mecefo_skip_options_t* opt,
    void* dX, void* dgamma, void* dWg, void* dWu, void* dWd, int accumulate,
    void* ws, size_t ws_bytes, void* hip_stream);

/* Measurement aid (not part of the hot path; the only calls that create HIP objects).
 * After mecefo_profile_enable(n) every kernel stage enqueued by the calls above is bracketed
 * by a pair of HIP events on the call's own stream, for at most n stage launches.
 * mecefo_profile_collect() waits for them, adds elapsed milliseconds and launch counts per
 * stage into two arrays of MECEFO_STAGE_COUNT entries, and switches timing off again.
 * While timing is on, the bf16 direct-to-LDS GEMM launches also sample the shader clock (every 64th
 * workgroup stores the core-clock cycles and the constant-rate 100 MHz ticks it ran for);
 * mecefo_profile_clock_mhz() returns, after a collect, the average clock in MHz per stage (0 where no
 * such launch ran).  These calls allocate and free a small device buffer and HIP events, are not
 * thread-safe and keep process-wide state: they are meant for benchmarks, one host thread at a time. */
typedef enum {
  MECEFO_STAGE_NORM_FWD = 0,       /* RMSNorm recompute from the stored tensor               */
  MECEFO_STAGE_DGRAD_DOWN = 1,     /* dA = dY Wd                                             */
  MECEFO_STAGE_RECOMPUTE = 2,      /* G, Z = U Wg^T, U Wu^T with fused SwiGLU backward       */
  MECEFO_STAGE_SWIGLU_BWD = 3,     /* standalone SwiGLU backward (saved activations given)   */
  MECEFO_STAGE_DGRAD_GATE_UP = 4,  /* dU = dG Wg + dZ Wu                                     */
  MECEFO_STAGE_PROJECT = 5,        /* Eq. (2): T = X P (three matrices, one launch)          */
  MECEFO_STAGE_CONTRACT = 6,       /* Eq. (2): C = Gy^T T over tokens                        */
  MECEFO_STAGE_SPLITK_REDUCE = 7,  /* sum of the split partials of C                         */
  MECEFO_STAGE_EXPAND = 8,         /* Eq. (2): dW = C P^T                                    */
  MECEFO_STAGE_NORM_BWD = 9,       /* dX = dOut + normbwd(dU), dgamma                        */
  MECEFO_STAGE_WGRAD_EXACT = 10,   /* exact dW = Gy^T X (comparator)                         */
  MECEFO_STAGE_ATTN_OUT_BWD = 11,  /* dWo = dH^T O and dO = dH Wo                             */
  MECEFO_STAGE_ATTN_ROWDOT = 12,   /* D = rowsum(dO * O)                                     */
  MECEFO_STAGE_ATTN_PROBS = 13,    /* P = exp(scale Q K^T - L), causal                       */
  MECEFO_STAGE_ATTN_DV = 14,       /* dV = P^T dO                                            */
  MECEFO_STAGE_ATTN_DS = 15,       /* dS = P * (dO V^T - D) * scale                          */
  MECEFO_STAGE_ATTN_DQ = 16,       /* dQ = dS K                                              */
  MECEFO_STAGE_ATTN_DK = 17,       /* dK = dS^T Q                                            */
  MECEFO_STAGE_ROPE_BWD = 18,      /* inverse rotation of dQ, dK (and the angle tables)      */
  MECEFO_STAGE_QKV_WGRAD = 19,     /* dWq, dWk, dWv = (dQ, dK, dV)^T Xn                      */
  MECEFO_STAGE_QKV_DGRAD = 20,     /* dXn = dQ Wq + dK Wk + dV Wv                            */
  MECEFO_STAGE_ATTN_FUSED_KV = 21, /* dK, dV and dS in one kernel (P kept in registers)      */
  MECEFO_STAGE_COUNT = 22
} mecefo_stage_t;
mecefo_status_t mecefo_profile_enable(int max_stage_launches);
mecefo_status_t mecefo_profile_collect(double* ms_by_stage, int* launches_by_stage);
mecefo_status_t mecefo_profile_clock_mhz(double* mhz_by_stage);

/* Prepares the current device: raises the dynamic-LDS limit of every kernel that needs more than the
 * default (what the first launch of each kernel would otherwise do on the host).  Optional; for callers
 * that capture the calls into a HIP graph without running them eagerly first.  Idempotent, cheap after
 * the first call on a device, safe from several host threads. */
mecefo_status_t mecefo_init(void);

/* Process-wide switches for tests and measurements (not needed for normal use; the library chooses
 * by shape).  name "tile": bf16 GEMM configuration, value "auto" | "S" (128x128) | "L4" | "L8R" (256x256,
 * register-staged) | "L8" (256x256, direct-to-LDS).  name "attention": "auto" | "gemm" (batched GEMM
 * launches instead of the fused attention kernels).  Affects calls made after it returns. */
mecefo_status_t mecefo_set_option(const char* name, const char* value);

/* Description of the last non-OK status returned on this thread ("" if none). */
const char* mecefo_last_error(void);

/* Library version string (static storage). */
const char* mecefo_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MECEFO_H_ */

/*
 * librom - Routing Mamba (RoM) layer forward pass and recurrent step for AMD MI355X (gfx950).
 *
 * C ABI.  Every pointer in rom_weights and every tensor / workspace argument is a
 * DEVICE pointer to caller-owned memory unless a comment says "host".  The library
 * allocates no device memory, launches everything asynchronously on the caller's HIP
 * stream and never synchronises (the rom_profile_* helpers excepted).  Buffers must stay
 * valid until the stream has passed the end of the call.
 * Because of that a call with profiling off may be recorded into a HIP graph (stream capture)
 * and replayed.  (The first use on a device of a kernel that needs more than 64 KiB of LDS sets
 * a function attribute - once per device and kernel, thread-safe; it is not a stream operation.)
 *
 * The layer (paper Sec. 4.2, Eq. (9)-(13), on top of the Mamba layer of Sec. 3.1,
 * Eq. (1)-(6)):
 *
 *   router      l[n,e] = x[n,:] . w_router[e,:] + b_router[e]; the top-K experts per token
 *               are picked on the logits (descending, lowest index on ties); P = softmax(l);
 *               gate[n,k] = P[n, idx[n,k]]   (gate_mode 0, Eq. (9) as printed) or that value
 *               divided by the sum over the K selected (gate_mode 1, text before Eq. (9)).
 *   in/gate     xz[n,:] = sum_k w_in[idx[n,k]] x[n,:]            (Eq. (10)/(11), unweighted sum)
 *   conv        u = SiLU(conv_b + causal depthwise conv_k(xz[:, :d_inner]))        (Eq. (2))
 *   x / dt      [dt_low | B | C][n,:] = sum_k w_x[e_k] u[n,:];
 *               dt[n,:] = softplus(sum_k w_dt[e_k] dt_low[n,:] + dt_bias)
 *               (e_k = idx[n,k] when n_experts_xdt == n_experts - the "Conv, Gate, dt, x, Out"
 *               variant of Table 1 - or the single shared module when n_experts_xdt == 1,
 *               the paper's default of Sec. 4.3, in which case there is no sum over k)
 *   scan        h <- exp(dt*A) h + dt*B*u ;  y = C.h + D*u ;  A = -exp(A_log)          (Eq. (5))
 *   gate        g = y * SiLU(xz[:, d_inner:])                                (Eq. (6)/(10)/(13))
 *   out         out[n,:] = sum_k gate[n,k] * (w_out[idx[n,k]] g[n,:])           (Eq. (12)/(13))
 *
 * Token order: n = b*L + t.  Slot order: s = n*K + k, k in descending-logit order.
 * All matrices are row-major; projection weights are stored "out-features major"
 * ([expert][out][in], the layout of a linear layer's weight).
 */
#ifndef ROM_H_
#define ROM_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ROM_API __attribute__((visibility("default")))

#define ROM_OK             0
#define ROM_E_INVAL       (-1)  /* NULL pointer, bad enum, bad size, misaligned pointer      */
#define ROM_E_WORKSPACE   (-2)  /* workspace smaller than rom_workspace_bytes()               */
#define ROM_E_UNSUPPORTED (-3)  /* shape outside what this build implements (see rom_dims)    */
#define ROM_E_HIP         (-4)  /* a HIP launch reported an error                             */
#define ROM_E_STATIC_LIMIT (-5) /* rom_step_static: the call does not fit the static scratch  */

#define ROM_DTYPE_F32  0        /* fp32 weights, activations, arithmetic                      */
#define ROM_DTYPE_BF16 1        /* bf16 weights/activations, fp32 accumulation and scan state */

/* Shape of one layer.  Supported: d_state == 16, d_conv == 4, 1 <= top_k <= n_experts <= 64,
 * top_k <= 8, d_inner % 16 == 0, d_model % 8 == 0, n_experts_xdt in {1, n_experts}.  Anything else
 * returns ROM_E_UNSUPPORTED / ROM_E_INVAL.  (bf16 projections whose inner dimension is not a
 * multiple of 8 run on the plain FMA kernel instead of the MFMA one.) */
typedef struct rom_dims {
  int32_t d_model;        /* D_m                                             */
  int32_t d_inner;        /* D_e (paper: 2 D_m)                              */
  int32_t d_state;        /* D_s (paper: 16)                                 */
  int32_t d_conv;         /* k   (paper: 4)                                  */
  int32_t dt_rank;        /* R   (paper: D_m / 16)                           */
  int32_t n_experts;      /* E                                               */
  int32_t top_k;          /* K                                               */
  int32_t n_experts_xdt;  /* E (routed x/dt projections) or 1 (shared)       */
  int32_t dtype;          /* ROM_DTYPE_*                                     */
  int32_t gate_mode;      /* 0: masked softmax (Eq. (9)); 1: renormalised over the K selected */
} rom_dims;

/* Layer parameters.  "T" is float for ROM_DTYPE_F32 and bf16 (16-bit) for ROM_DTYPE_BF16.
 * All pointers must be 16-byte aligned. */
typedef struct rom_weights {
  const void  *w_router;  /* T   [E, d_model]                                                  */
  const float *b_router;  /* f32 [E] or NULL                                                   */
  const void  *w_in;      /* T   [E, 2*d_inner, d_model]; rows [0,d_inner) conv branch (Eq. (11)),
                                 rows [d_inner, 2*d_inner) gate branch (Eq. (10))              */
  const float *conv_w;    /* f32 [d_inner, d_conv]; tap j multiplies the input at t-(d_conv-1)+j */
  const float *conv_b;    /* f32 [d_inner] or NULL                                             */
  const void  *w_x;       /* T   [E_xdt, dt_rank + 2*d_state, d_inner]; rows = dt_low | B | C  */
  const void  *w_dt;      /* T   [E_xdt, d_inner, dt_rank]                                     */
  const float *dt_bias;   /* f32 [d_inner]                                                     */
  const float *A_log;     /* f32 [d_inner, d_state]; A = -exp(A_log)                           */
  const float *D;         /* f32 [d_inner]                                                     */
  const void  *w_out;     /* T   [E, d_model, d_inner]                                         */
} rom_weights;

/* Byte offsets, inside the workspace of rom_layer_forward / rom_step, of the intermediate
 * tensors a caller may want to inspect after the call (tests compare them stage by stage).
 * An offset of (size_t)-1 means "not materialised for these dims". */
typedef struct rom_ws_layout {
  size_t total_bytes;
  size_t expert_idx;   /* i32 [N*K]                                        */
  size_t gate;         /* f32 [N*K]                                        */
  size_t counts;       /* i32 [E]                                          */
  size_t offsets;      /* i32 [E+1]                                        */
  size_t perm;         /* i32 [N*K] sorted position -> slot                */
  size_t inv_perm;     /* i32 [N*K] slot -> sorted position                */
  size_t logits;       /* f32 [N, E]                                       */
  size_t xz;           /* T   [N, 2*d_inner]  (sum over k already applied) */
  size_t u;            /* T   [N, d_inner]                                 */
  size_t dt_low;       /* T   [N, dt_rank]                                 */
  size_t bc;           /* f32 [N, 2*d_state]  B then C                     */
  size_t dt;           /* T   [N, d_inner]    after softplus               */
  size_t g;            /* T   [N, d_inner]    gated scan output            */
} rom_ws_layout;

/* Workspace size in bytes for a call with B sequences of L tokens (rom_step: L = 1;
 * rom_route: the same formula with B*L = N).  Returns 0 if dims are invalid or unsupported.
 * host-only; dims is a host pointer. */
ROM_API size_t rom_workspace_bytes(const rom_dims *dims, int64_t B, int64_t L);

/* Workspace of rom_route alone for N tokens (a few MiB at most: the row map and per-block
 * histograms of the counting sort); rom_workspace_bytes(dims, N, 1) is an accepted upper bound. */
ROM_API size_t rom_route_workspace_bytes(const rom_dims *dims, int64_t N);

/* Fills *layout (host) for the same arguments; returns ROM_OK or an error. */
ROM_API int rom_workspace_layout(const rom_dims *dims, int64_t B, int64_t L, rom_ws_layout *layout);

/* Router and expert grouping only (Eq. (9) and the permutation the grouped projections use).
 *   x          T   [N, d_model]
 *   expert_idx i32 [N, K]   out  experts per token, k-th column = (k+1)-th largest logit
 *   gate       f32 [N, K]   out  gating weights R of Eq. (9) for those experts
 *   counts     i32 [E]      out  slots per expert (sum = N*K: no capacity limit, nothing dropped)
 *   offsets    i32 [E+1]    out  exclusive prefix sum of counts
 *   perm       i32 [N*K]    out  perm[p] = slot at sorted position p (grouped by expert,
 *                                ascending slot inside an expert)
 *   inv_perm   i32 [N*K]    out  inverse of perm
 *   logits     f32 [N, E]   out, may be NULL
 *   ws/ws_bytes             workspace of at least rom_route_workspace_bytes(dims, N)
 * N == 0 is a successful no-op.  Errors are reported before anything is launched. */
ROM_API int rom_route(const rom_dims *dims, const rom_weights *w, const void *x, int64_t N,
              int32_t *expert_idx, float *gate, int32_t *counts, int32_t *offsets,
              int32_t *perm, int32_t *inv_perm, float *logits,
              void *ws, size_t ws_bytes, void *hip_stream);

/* Load-balance statistics of one layer's routing decision, Eq. (16) (appendix on the auxiliary
 * load-balance loss; the layer itself never uses them):
 *   frac[i]      = counts[i] / (N * K)              share of the (token, k) slots sent to expert i
 *   mean_prob[i] = (1/N) sum_n softmax(logits[n, :])[i]   full softmax over all E experts
 *   loss[0]      = alpha * E * sum_i frac[i] * mean_prob[i]
 * The model-level loss of Eq. (16) is the sum of loss[0] over the layers.
 *   logits     f32 [N, E]  as written by rom_route, or by rom_layer_forward / rom_step into the
 *                          workspace region rom_ws_layout.logits (N = B * L)
 *   counts     i32 [E]     as written by rom_route, or the workspace region rom_ws_layout.counts
 *   frac, mean_prob  f32 [E]  out;  loss  f32 [1]  out   (all device pointers)
 *   ws/ws_bytes  a workspace that is large enough for a forward call over these N tokens
 *                (rom_workspace_bytes(dims, B, L) for any B * L = N; only its first part, up to
 *                rom_ws_layout.xz, is needed).  It may be the workspace the logits and counts
 *                live in: the scratch this call uses lies at the same offset for every such
 *                (B, L) and overlaps no region named in rom_ws_layout.
 * The sums are taken in a fixed order: repeated calls give identical bits.
 * N <= 0 is ROM_E_INVAL (the mean over no tokens is undefined). */
ROM_API int rom_balance_stats(const rom_dims *dims, const float *logits, const int32_t *counts,
                      int64_t N, float alpha, float *frac, float *mean_prob, float *loss,
                      void *ws, size_t ws_bytes, void *hip_stream);

/* The whole layer, Eq. (9)-(13).
 *   x              T   [B, L, d_model]
 *   conv_state_in  f32 [B, d_inner, d_conv-1] oldest first, or NULL (zeros): the conv-branch
 *                  inputs (xz[:, :d_inner]) of the d_conv-1 tokens before this call
 *   ssm_state_in   f32 [B, d_inner, d_state] or NULL (zeros)
 *   out            T   [B, L, d_model]; must not alias x
 *   conv_state_out / ssm_state_out: same shapes, written if not NULL (may alias the *_in)
 * B == 0 or L == 0 is a successful no-op. */
ROM_API int rom_layer_forward(const rom_dims *dims, const rom_weights *w, const void *x,
                      int64_t B, int64_t L,
                      const float *conv_state_in, const float *ssm_state_in,
                      void *out, float *conv_state_out, float *ssm_state_out,
                      void *ws, size_t ws_bytes, void *hip_stream);

/* One new token per sequence (constant-time recurrent inference, Eq. (5) advanced one step):
 *   x [B, d_model] -> out [B, d_model]; conv_state / ssm_state are updated in place. */
ROM_API int rom_step(const rom_dims *dims, const rom_weights *w, const void *x, int64_t B,
             float *conv_state, float *ssm_state, void *out,
             void *ws, size_t ws_bytes, void *hip_stream);

/* rom_step for callers that cannot allocate device memory or hold a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and the
 * same result, bit for bit, as rom_step, minus the workspace: the intermediates live in a
 * 32 MiB array that is part of the library's device image (one copy per GPU, held until the
 * process ends).  The call allocates and frees nothing.
 * Limit: rom_workspace_bytes(dims, B, 1) <= 32 MiB (256 sequences at d_model 2048 with 8 experts
 * need 11.4 MiB); beyond it the call returns ROM_E_STATIC_LIMIT before anything is launched.
 * All calls on one GPU share that GPU's array: calls that overlap on one GPU (different streams
 * or host threads) race on it; calls queued on one stream do not.  The array keeps the last
 * call's contents; the step reads no region before writing it, so nothing needs clearing. */
ROM_API int rom_step_static(const rom_dims *dims, const rom_weights *w, const void *x, int64_t B,
                    float *conv_state, float *ssm_state, void *out, void *hip_stream);

/* ---- Backward pass of the layer (training, Sec. 5.1): the gradient of a scalar loss with respect to
 * the layer input and every parameter, given d loss / d out.  Reverse-mode differentiation of
 * Eq. (9)-(13) over Eq. (1)-(6); the TopK indicator of Eq. (9) is piecewise constant and gets no
 * gradient, the router is trained through the gate weights R_i of Eq. (12) (no jitter, no SparseMixer
 * estimator: the paper names those as options of its training runs only).  Zero initial conv / scan
 * states, no state gradient.
 * Any top_k the forward pass takes: with top_k > 1 every selected expert's projection receives the
 * token's gradient (Eq. (10)/(11) are indicator sums), the out projection's is weighted by the
 * slot's gate, and the gate's own gradient is d_out against that expert's output.
 * At most 2^24 (token, k) slots per call.
 * All gradient buffers are f32 device memory of the parameter's shape, written (not accumulated):
 * d_A_log is with respect to A_log.  d_b_router and d_conv_b may be NULL. */
typedef struct rom_grads {
  float *d_w_router;  /* [E, d_model]                          */
  float *d_b_router;  /* [E] or NULL                           */
  float *d_w_in;      /* [E, 2*d_inner, d_model]               */
  float *d_conv_w;    /* [d_inner, d_conv]                     */
  float *d_conv_b;    /* [d_inner] or NULL                     */
  float *d_w_x;       /* [E_xdt, dt_rank + 2*d_state, d_inner] */
  float *d_w_dt;      /* [E_xdt, d_inner, dt_rank]             */
  float *d_dt_bias;   /* [d_inner]                             */
  float *d_A_log;     /* [d_inner, d_state]                    */
  float *d_D;         /* [d_inner]                             */
  float *d_w_out;     /* [E, d_model, d_inner]                 */
} rom_grads;

/* Workspace bytes of rom_layer_backward (0 if dims are invalid or unsupported). */
ROM_API size_t rom_backward_workspace_bytes(const rom_dims *dims, int64_t B, int64_t L);

/*   x      T [B, L, d_model]   the layer input of the forward call
 *   d_out  T [B, L, d_model]   d loss / d out
 *   d_x    T [B, L, d_model]   out: d loss / d x (must alias neither x nor d_out)
 *   grads  host struct of device pointers, see above
 *   ws     rom_backward_workspace_bytes(dims, B, L) bytes, 256-byte aligned
 * The call runs the forward pass into its workspace first (activations are recomputed, nothing has
 * to be kept from an earlier rom_layer_forward call), then the backward pass; asynchronous on
 * hip_stream like every other call.  Results are deterministic (fixed summation orders, no atomics).
 * B == 0 or L == 0 is a successful no-op. */
ROM_API int rom_layer_backward(const rom_dims *dims, const rom_weights *w, const void *x, int64_t B, int64_t L,
                       const void *d_out, void *d_x, const rom_grads *grads, void *ws, size_t ws_bytes,
                       void *hip_stream);

/* The same without the forward recomputation, for a training step that has just run the forward pass
 * itself: the caller's rom_layer_forward(dims, w, x, B, L, NULL, NULL, out, NULL, NULL, ws, ws_bytes,
 * stream) - zero initial states, the SAME ws of rom_backward_workspace_bytes(dims, B, L) bytes (a
 * workspace of that size is also a valid forward workspace), the same x and weights, nothing else
 * writing to ws in between - leaves the activations where this call reads them.  Identical results to
 * rom_layer_backward, bit for bit; everything else as documented there. */
ROM_API int rom_layer_backward_saved(const rom_dims *dims, const rom_weights *w, const void *x, int64_t B, int64_t L,
                             const void *d_out, void *d_x, const rom_grads *grads, void *ws, size_t ws_bytes,
                             void *hip_stream);

/* ---- Pre-norm residual block (appendix, architectures overview: every layer sits behind a
 * pre-norm and a skip connection):   out = x + RoM(RMSNorm(x)),
 *   RMSNorm(x)[n, :] = x[n, :] / sqrt(mean_d(x[n, d]^2) + eps) * norm_weight[:].
 * The norm is never materialised.  The router kernel accumulates each token's sum of squares
 * while it reads x for the logits and applies norm_weight itself; the in projection runs on the
 * raw x with a weight whose columns were pre-multiplied by norm_weight (rom_fold_norm, once per
 * weight load) and scales every output row by the token's 1/rms in its epilogue; the skip is
 * added where the out projection (K == 1) or the combine (K > 1) writes out.
 * The block calls below therefore expect w->w_in to be the FOLDED weight; all other members of
 * rom_weights are the plain ones. */

/* w_in_folded[e, o, d] = w_in[e, o, d] * norm_weight[d], rounded once to T.
 *   w_in, w_in_folded  T [E, 2*d_inner, d_model] (device); may be the same buffer
 *   norm_weight        f32 [d_model] (device) */
ROM_API int rom_fold_norm(const rom_dims *dims, const void *w_in, const float *norm_weight,
                  void *w_in_folded, void *hip_stream);

/* The same for any projection weight stored [n_rows][d_model] (the input projections of the Mamba2
 * and Gated DeltaNet layers below): w_folded[r, d] = w[r, d] * norm_weight[d], rounded once to the
 * type.  w, w_folded T [n_rows, d_model] (device; may be the same buffer); dtype ROM_DTYPE_*. */
ROM_API int rom_fold_norm_rows(int dtype, const void *w, const float *norm_weight, void *w_folded,
                               int64_t n_rows, int32_t d_model, void *hip_stream);

/* One block: arguments as rom_layer_forward plus
 *   norm_weight  f32 [d_model] (device, 16-byte aligned), eps >= 0
 * out must not alias x (x is read again for the skip).  Workspace: rom_workspace_bytes(dims, B, L).
 * The intermediates named in rom_ws_layout are those of the inner layer (xz is the projection
 * of the normalised input). */
ROM_API int rom_block_forward(const rom_dims *dims, const rom_weights *w, const float *norm_weight,
                      float eps, const void *x, int64_t B, int64_t L,
                      const float *conv_state_in, const float *ssm_state_in,
                      void *out, float *conv_state_out, float *ssm_state_out,
                      void *ws, size_t ws_bytes, void *hip_stream);

/* Backward pass of one block (zero initial states): d_x and the gradients of every parameter of
 * out = x + RoM(RMSNorm(x)).  Arguments as rom_layer_backward, with
 *   w              the PLAIN weights (w->w_in not folded)
 *   norm_weight    f32 [d_model] (device), eps >= 0
 *   d_norm_weight  f32 [d_model] (device), written
 *   d_gate_ffn     f32 [B*L, K] (device) or NULL: d loss / d gate from an FFN-MoE layer that ran on this
 *                  block's routing decision (rom_ffn_moe_backward's d_gate); added to the layer's own
 *                  gate gradient before the router's backward
 *   ws             rom_block_backward_workspace_bytes(dims, B, L) bytes, 256-byte aligned
 * The call materialises RMSNorm(x) in the activation type, runs the layer's forward and backward on
 * it (rom_layer_backward) and takes the result through the norm's adjoint, adding d_out for the skip.
 * Deterministic. */
ROM_API size_t rom_block_backward_workspace_bytes(const rom_dims *dims, int64_t B, int64_t L);
ROM_API int rom_block_backward(const rom_dims *dims, const rom_weights *w, const float *norm_weight, float eps,
                               const void *x, int64_t B, int64_t L, const void *d_out, const float *d_gate_ffn,
                               void *d_x, const rom_grads *grads, float *d_norm_weight, void *ws,
                               size_t ws_bytes, void *hip_stream);

/* The two halves of that call for a training step that needs the block's output before it has d_out:
 * rom_block_forward_train computes out = x + RoM(RMSNorm(x)) with the arithmetic the backward
 * recomputes (materialised norm in the activation type, PLAIN weights) and leaves every activation
 * in ws; rom_block_backward_saved then runs the backward pass alone.  Same ws
 * (rom_block_backward_workspace_bytes), same x, weights, norm_weight and eps, nothing else writing
 * to ws in between; the routing decision is in ws at the offsets of rom_workspace_layout.  Results
 * identical to rom_block_backward, bit for bit.  out must not alias x. */
ROM_API int rom_block_forward_train(const rom_dims *dims, const rom_weights *w, const float *norm_weight,
                                    float eps, const void *x, int64_t B, int64_t L, void *out, void *ws,
                                    size_t ws_bytes, void *hip_stream);
ROM_API int rom_block_backward_saved(const rom_dims *dims, const rom_weights *w, const float *norm_weight,
                                     float eps, const void *x, int64_t B, int64_t L, const void *d_out,
                                     const float *d_gate_ffn, void *d_x, const rom_grads *grads,
                                     float *d_norm_weight, void *ws, size_t ws_bytes, void *hip_stream);

/* One new token per sequence through one block; states updated in place (see rom_step). */
ROM_API int rom_block_step(const rom_dims *dims, const rom_weights *w, const float *norm_weight,
                   float eps, const void *x, int64_t B, float *conv_state, float *ssm_state,
                   void *out, void *ws, size_t ws_bytes, void *hip_stream);

/* One block's parameters inside a stack (host struct; the pointers are device pointers). */
typedef struct rom_block {
  rom_weights  w;            /* w.w_in folded with norm_weight (rom_fold_norm) */
  const float *norm_weight;  /* f32 [d_model] */
} rom_block;

/* n_layers blocks of the same shape, one after another: layer j reads layer j-1's output.
 *   blocks        host array [n_layers]
 *   x             T [B, L, d_model];  out  T [B, L, d_model], must not alias x
 *   tmp           T [B, L, d_model] scratch (the layers write tmp and out in turn); may be
 *                 NULL when n_layers == 1; must alias neither x nor out
 *   conv_state_in / ssm_state_in    f32 [n_layers, B, d_inner, d_conv-1] / [n_layers, B, d_inner,
 *                 d_state], or NULL (zeros); *_out likewise, written if not NULL (may alias *_in)
 *   ws            one layer's workspace, rom_workspace_bytes(dims, B, L), reused by every layer
 * Every block's pointers are checked before the first layer is launched. */
ROM_API int rom_stack_forward(const rom_dims *dims, const rom_block *blocks, int n_layers, float eps,
                      const void *x, int64_t B, int64_t L,
                      const float *conv_state_in, const float *ssm_state_in,
                      void *out, float *conv_state_out, float *ssm_state_out,
                      void *tmp, void *ws, size_t ws_bytes, void *hip_stream);

/* One new token per sequence through the whole stack: x, out, tmp T [B, d_model]; the
 * [n_layers, B, ...] states are updated in place. */
ROM_API int rom_stack_step(const rom_dims *dims, const rom_block *blocks, int n_layers, float eps,
                   const void *x, int64_t B, float *conv_state, float *ssm_state,
                   void *out, void *tmp, void *ws, size_t ws_bytes, void *hip_stream);

/* ---- FFN-MoE layer that shares the routing decision of the RoM layer in front of it (appendix,
 * the two equations after the architectures overview):
 *   y[n, :] = sum_k gate[n, k] * f_{e(n,k)}(x[n, :]),   f_i(v) = W_down,i (SiLU(W_gate,i v) * (W_up,i v))
 * It has no router: the expert of every (token, k) slot and its weight come from the preceding
 * rom_route / rom_layer_forward / rom_block_forward call over the same N tokens, as the grouping
 * that call produced.  Optionally the experts see RMSNorm(x) (pre_norm; the norm's scale is
 * folded into the packed weight) and x is added to the result (add_skip). */
typedef struct rom_ffn_weights {
  const void *w_gate_up;  /* T [E, 2*d_ff, d_model] in the PACKED row order of rom_ffn_pack_gate_up */
  const void *w_down;     /* T [E, d_model, d_ff]                                              */
} rom_ffn_weights;

/* Workspace bytes of rom_ffn_moe_forward for N tokens (0 if dims / d_ff are unsupported:
 * d_ff must be a positive multiple of 16).  Only d_model, n_experts, top_k and dtype of dims
 * matter, but dims must be a valid layer shape. */
ROM_API size_t rom_ffn_workspace_bytes(const rom_dims *dims, int32_t d_ff, int64_t N);

/* Weight preparation, once per weight load.  w_gate_up is the plain layout, T [E, 2*d_ff, d_model]
 * with rows [0, d_ff) the gate projection and rows [d_ff, 2*d_ff) the up projection.  The packed
 * layout interleaves them in blocks of eight features,
 *   w_packed[e, 16*b + t, :]     = w_gate_up[e, 8*b + t, :]         (gate feature 8b+t, t < 8)
 *   w_packed[e, 16*b + 8 + t, :] = w_gate_up[e, d_ff + 8*b + t, :]  (up feature 8b+t),
 * so that the projection kernel finds a feature's gate and up pre-activations in one lane's
 * accumulators and can apply SiLU(gate) * up before it writes anything.  norm_weight (f32
 * [d_model], device) != NULL multiplies every row's columns by the pre-norm's scale (use that
 * weight with pre_norm != 0 only); NULL packs without scaling.  Not in place. */
ROM_API int rom_ffn_pack_gate_up(const rom_dims *dims, int32_t d_ff, const void *w_gate_up,
                         const float *norm_weight, void *w_packed, void *hip_stream);

/*   x        T   [N, d_model];  out  T [N, d_model], must not alias x
 *   offsets  i32 [E+1], perm i32 [N*K], inv_perm i32 [N*K], gate f32 [N, K]: as written by
 *            rom_route, or the workspace regions of the same names after a layer / block call
 *            (that workspace must stay untouched until this call has run)
 *   pre_norm != 0: experts see x / sqrt(mean(x^2) + eps) * norm_weight (scale packed into the weight)
 *   add_skip != 0: out = x + y
 *   ws       rom_ffn_workspace_bytes(dims, d_ff, N) bytes, 256-byte aligned, distinct from the
 *            workspace that holds offsets / perm / inv_perm / gate
 * N == 0 is a successful no-op. */
ROM_API int rom_ffn_moe_forward(const rom_dims *dims, int32_t d_ff, const rom_ffn_weights *w,
                        int pre_norm, float eps, int add_skip, const void *x, int64_t N,
                        const int32_t *offsets, const int32_t *perm, const int32_t *inv_perm,
                        const float *gate, void *out, void *ws, size_t ws_bytes, void *hip_stream);

/* Backward pass of the FFN-MoE layer: gradients of y = (x +) sum_k gate_k f_{e_k}(x~), x~ = RMSNorm(x) or x.
 *   w             the packed weights of rom_ffn_pack_gate_up WITHOUT the norm's scale folded in
 *   norm_weight   f32 [d_model] (device): the experts see RMSNorm(x); NULL: they see x
 *   x, d_out      T [N, d_model];  offsets, perm, inv_perm, gate: the routing decision, as for the forward
 *   d_x           T [N, d_model], written (aliases neither x nor d_out)
 *   d_gate        f32 [N, K], written: d loss / d gate of every slot - the caller adds it to the gate
 *                 gradient of the RoM layer whose router made the decision
 *   grads         d_w_gate_up f32 [E, 2*d_ff, d_model] in the PACKED row order, d_w_down f32
 *                 [E, d_model, d_ff], d_norm_weight f32 [d_model] (required iff norm_weight != NULL)
 *   ws            rom_ffn_backward_workspace_bytes(dims, d_ff, N) bytes, 256-byte aligned
 * The call recomputes the forward pass with the pre-activations kept.  Deterministic. */
typedef struct rom_ffn_grads {
  float *d_w_gate_up;
  float *d_w_down;
  float *d_norm_weight;
} rom_ffn_grads;
ROM_API size_t rom_ffn_backward_workspace_bytes(const rom_dims *dims, int32_t d_ff, int64_t N);
ROM_API int rom_ffn_moe_backward(const rom_dims *dims, int32_t d_ff, const rom_ffn_weights *w,
                                 const float *norm_weight, float eps, int add_skip, const void *x, int64_t N,
                                 const int32_t *offsets, const int32_t *perm, const int32_t *inv_perm,
                                 const float *gate, const void *d_out, void *d_x, float *d_gate,
                                 const rom_ffn_grads *grads, void *ws, size_t ws_bytes, void *hip_stream);

/* The two halves of that call for a training step: rom_ffn_moe_forward_train computes the layer's output
 * (out T [N, d_model], must not alias x) with the pre-activations, the experts' inputs and outputs
 * kept in ws; rom_ffn_moe_backward_saved then runs the backward pass alone on the same ws
 * (rom_ffn_backward_workspace_bytes), same arguments, nothing else writing to ws in between.
 * Gradients identical to rom_ffn_moe_backward, bit for bit. */
ROM_API int rom_ffn_moe_forward_train(const rom_dims *dims, int32_t d_ff, const rom_ffn_weights *w,
                                      const float *norm_weight, float eps, int add_skip, const void *x,
                                      int64_t N, const int32_t *offsets, const int32_t *perm,
                                      const int32_t *inv_perm, const float *gate, void *out, void *ws,
                                      size_t ws_bytes, void *hip_stream);
ROM_API int rom_ffn_moe_backward_saved(const rom_dims *dims, int32_t d_ff, const rom_ffn_weights *w,
                                       const float *norm_weight, float eps, int add_skip, const void *x,
                                       int64_t N, const int32_t *offsets, const int32_t *perm,
                                       const int32_t *inv_perm, const float *gate, const void *d_out,
                                       void *d_x, float *d_gate, const rom_ffn_grads *grads, void *ws,
                                       size_t ws_bytes, void *hip_stream);

/* The hybrid of the appendix (RoM + FFN-MoE with shared routing), as a stack: layer j is the RoM
 * block blocks[j]; if ffns[j].w_gate_up is not NULL an FFN-MoE block (pre-norm if ffn_pre_norm,
 * always with its skip) follows it and runs on the routing decision that RoM block has just made
 * - the grouping is picked up from the RoM workspace on the device, nothing visits the host.
 *   blocks, ffns   host arrays [n_layers]; every FFN has the same d_ff
 *   tmp            T [B, L, d_model] scratch (needed as soon as the stack has more than one block
 *                  of either kind); x, out, tmp pairwise distinct
 *   ws             rom_workspace_bytes(dims, B, L);  ffn_ws  rom_ffn_workspace_bytes(dims, d_ff, B*L),
 *                  distinct from ws (may be NULL if no layer has an FFN)
 * States as in rom_stack_forward. */
ROM_API int rom_hybrid_stack_forward(const rom_dims *dims, int32_t d_ff, const rom_block *blocks,
                             const rom_ffn_weights *ffns, int ffn_pre_norm, int n_layers, float eps,
                             const void *x, int64_t B, int64_t L,
                             const float *conv_state_in, const float *ssm_state_in,
                             void *out, float *conv_state_out, float *ssm_state_out,
                             void *tmp, void *ws, size_t ws_bytes, void *ffn_ws, size_t ffn_ws_bytes,
                             void *hip_stream);

/* ---------------------------------------------------------------------------------------------
 * RoM on a Mamba2 layer (Sec. 5.2, Table 3; the paragraph on streamlined SSMs: every major projection
 * of the block becomes a mixture of experts under the one shared router).  The paper prints no
 * equations for this variant; what is computed (readings: the published Mamba2 layer, routed the
 * way Eq. (9)-(13) route the Mamba layer):
 *
 *   router      as in rom_layer_forward (Eq. (9))
 *   in          zxbcdt[n,:] = sum_k w_in[idx[n,k]] x[n,:]        (unweighted sum, as Eq. (10)/(11));
 *               columns z [d_inner] | x [d_inner] | B [d_state] | C [d_state] | dt [n_heads]
 *   conv        x | B | C <- SiLU(conv_b + causal depthwise conv_4(x | B | C))
 *   scan        per head h (headdim channels), dt = softplus(dt + dt_bias[h]), A = -exp(A_log[h]):
 *               H <- exp(dt A) H + dt x B^T ;  y = H C + D[h] x          (H: headdim x d_state)
 *   gate, norm  g = RMSNorm(y * SiLU(z)) * norm_w       (over all d_inner channels, eps inside the root)
 *   out         out[n,:] = sum_k gate[n,k] * (w_out[idx[n,k]] g[n,:])              (as Eq. (12)/(13))
 *
 * Supported: ROM_DTYPE_BF16, headdim == 64, d_state in {64, 128}, d_conv == 4, d_inner a multiple of
 * 512 (n_heads = d_inner / 64 a multiple of 8), d_model % 8 == 0, 1 <= top_k <= n_experts <= 64,
 * top_k <= 8.  Anything else: ROM_E_UNSUPPORTED / ROM_E_INVAL. */
typedef struct rom_mamba2_dims {
  int32_t d_model;
  int32_t d_inner;
  int32_t d_state;        /* N                                               */
  int32_t d_conv;         /* 4                                               */
  int32_t headdim;        /* P; n_heads = d_inner / headdim                  */
  int32_t n_experts;
  int32_t top_k;
  int32_t dtype;          /* ROM_DTYPE_BF16                                  */
  int32_t gate_mode;      /* as rom_dims                                     */
} rom_mamba2_dims;

/* All pointers 16-byte aligned device pointers; "T" is bf16. */
typedef struct rom_mamba2_weights {
  const void  *w_router;  /* T   [E, d_model]                                                   */
  const float *b_router;  /* f32 [E] or NULL                                                    */
  const void  *w_in;      /* T   [E, 2*d_inner + 2*d_state + n_heads, d_model]; rows z | x | B | C | dt */
  const float *conv_w;    /* f32 [d_inner + 2*d_state, 4] over the channels x | B | C           */
  const float *conv_b;    /* f32 [d_inner + 2*d_state] or NULL                                  */
  const float *dt_bias;   /* f32 [n_heads]                                                      */
  const float *A_log;     /* f32 [n_heads]; A = -exp(A_log)                                     */
  const float *D;         /* f32 [n_heads]                                                      */
  const float *norm_w;    /* f32 [d_inner]                                                      */
  const void  *w_out;     /* T   [E, d_model, d_inner]                                          */
} rom_mamba2_weights;

/* Byte offsets of the intermediates inside the workspace after rom_mamba2_forward. */
typedef struct rom_mamba2_ws_layout {
  size_t total_bytes;
  size_t expert_idx;   /* i32 [N*K]                                        */
  size_t gate;         /* f32 [N*K]                                        */
  size_t counts;       /* i32 [E]                                          */
  size_t offsets;      /* i32 [E+1]                                        */
  size_t perm;         /* i32 [N*K]                                        */
  size_t inv_perm;     /* i32 [N*K]                                        */
  size_t logits;       /* f32 [N, E]                                       */
  size_t zxbcdt;       /* T   [N, 2*d_inner + 2*d_state + n_heads]  (sum over k applied) */
  size_t xbc;          /* T   [N, d_inner + 2*d_state]  after conv + SiLU  */
  size_t yz;           /* T   [N, d_inner]  (y + D x) * SiLU(z)            */
  size_t g;            /* T   [N, d_inner]  after the RMS norm             */
} rom_mamba2_ws_layout;

/* host-only; 0 / an error for invalid or unsupported dims */
ROM_API size_t rom_mamba2_workspace_bytes(const rom_mamba2_dims *dims, int64_t B, int64_t L);
ROM_API int rom_mamba2_workspace_layout(const rom_mamba2_dims *dims, int64_t B, int64_t L,
                                        rom_mamba2_ws_layout *layout);

/* The layer above on B sequences of L tokens.
 *   x, out          T [B, L, d_model] (distinct);  eps: the norm's epsilon (>= 0)
 *   conv_state_in   f32 [B, d_inner + 2*d_state, 3] or NULL (zeros): the conv's inputs (x | B | C
 *                   channels) at the three steps before the first, oldest first
 *   ssm_state_in    f32 [B, n_heads, d_state, headdim] or NULL (zeros): H before the first step
 *   conv_state_out, ssm_state_out   the same after the last step, or NULL (not wanted).  An output
 *                   state may be the same buffer as its input only for L <= 32.
 *   ws              rom_mamba2_workspace_bytes(dims, B, L), 256-byte aligned
 * Asynchronous on hip_stream, allocates nothing; B * L == 0 is a successful no-op; errors are
 * reported before anything is launched.  At most 2^30 (token, k) slots and 65535 sequences.
 * With profiling on, the stages are recorded under ROM_STAGE_ROUTE, _PERMUTE, _IN_PROJ, _CONV,
 * _SCAN (recurrence + gate), _DT_PROJ (the RMS norm: this layer has no dt projection), _OUT_PROJ,
 * _COMBINE. */
ROM_API int rom_mamba2_forward(const rom_mamba2_dims *dims, const rom_mamba2_weights *w, const void *x,
                               int64_t B, int64_t L, float eps, const float *conv_state_in,
                               const float *ssm_state_in, void *out, float *conv_state_out,
                               float *ssm_state_out, void *ws, size_t ws_bytes, void *hip_stream);

/* The pre-norm residual block around the layer above (appendix: every layer sits behind a pre-norm
 * and a skip connection): out = x + layer(RMSNorm(x)), RMSNorm with scale norm_weight (f32 [d_model],
 * device) and norm_eps.  As in rom_block_forward the norm is never materialised: the router applies it
 * itself, the input projection runs on the raw x with w->w_in FOLDED (rom_fold_norm_rows over its
 * E * (2*d_inner + 2*d_state + n_heads) rows) and scales its rows by 1/rms, the skip is added where the
 * output projection or the combine writes out.  out must not alias x (ROM_E_INVAL).  Everything else
 * as rom_mamba2_forward; with L == 1 and the states passed as both input and output (allowed up to
 * L == 32) the call is the block's recurrent step. */
ROM_API int rom_mamba2_block_forward(const rom_mamba2_dims *dims, const rom_mamba2_weights *w,
                                     const float *norm_weight, float norm_eps, const void *x, int64_t B,
                                     int64_t L, float eps, const float *conv_state_in,
                                     const float *ssm_state_in, void *out, float *conv_state_out,
                                     float *ssm_state_out, void *ws, size_t ws_bytes, void *hip_stream);

/* One new token for each of B sequences (the recurrent form of the layer above): x, out T [B, d_model];
 * conv_state and ssm_state (layouts above, both required) are read and updated in place.
 *   ws   rom_mamba2_workspace_bytes(dims, B, 1)
 * The state is 8 * d_state / 16 times the Mamba layer's (d_state 128: 2 MiB per sequence at d_inner
 * 4096); one call reads and writes it once. */
ROM_API int rom_mamba2_step(const rom_mamba2_dims *dims, const rom_mamba2_weights *w, const void *x,
                            int64_t B, float eps, float *conv_state, float *ssm_state, void *out,
                            void *ws, size_t ws_bytes, void *hip_stream);

/* ---------------------------------------------------------------------------------------------
 * RoM on a Gated DeltaNet layer (Sec. 5.2, Table 3: every major projection of the block under the one
 * shared router).  The paper prints no equations for this variant; what is computed (readings: the
 * published Gated DeltaNet layer, routed the way Eq. (9)-(13) route the Mamba layer):
 *
 *   router      as in rom_layer_forward (Eq. (9))
 *   in          p[n,:] = sum_k w_in[idx[n,k]] x[n,:]            (unweighted sum, as Eq. (10)/(11));
 *               columns z [D_v] | q [D_k] | k [D_k] | v [D_v] | b [H] | a [H]   (D_k = H d_k, D_v = H d_v)
 *   conv        q | k | v <- SiLU(conv_b + causal depthwise conv_4(q | k | v))
 *   per head    q <- q / sqrt(sum q^2 + 1e-6) / sqrt(d_k),  k <- k / sqrt(sum k^2 + 1e-6),
 *               beta = sigmoid(b),  g = -exp(A_log[h]) softplus(a + dt_bias[h]);
 *               S <- exp(g) S;  u = beta (v - S k);  S <- S + u k^T;  o = S q       (S: d_v x d_k)
 *   norm, gate  y = RMSNorm_head(o) * norm_w * SiLU(z)      (norm over each head's d_v channels)
 *   out         out[n,:] = sum_k gate[n,k] * (w_out[idx[n,k]] y[n,:])              (as Eq. (12)/(13))
 *
 * Supported: ROM_DTYPE_BF16, d_v == 64, d_k in {64, 128}, d_conv == 4, n_heads % 4 == 0, d_model % 8
 * == 0, 1 <= top_k <= n_experts <= 64, top_k <= 8.  Anything else: ROM_E_UNSUPPORTED / ROM_E_INVAL. */
typedef struct rom_gdn_dims {
  int32_t d_model;
  int32_t n_heads;        /* H                                               */
  int32_t d_k;            /* key / query channels per head                   */
  int32_t d_v;            /* value channels per head                         */
  int32_t d_conv;         /* 4                                               */
  int32_t n_experts;
  int32_t top_k;
  int32_t dtype;          /* ROM_DTYPE_BF16                                  */
  int32_t gate_mode;      /* as rom_dims                                     */
} rom_gdn_dims;

/* All pointers 16-byte aligned device pointers; "T" is bf16. */
typedef struct rom_gdn_weights {
  const void  *w_router;  /* T   [E, d_model]                                                   */
  const float *b_router;  /* f32 [E] or NULL                                                    */
  const void  *w_in;      /* T   [E, 2*D_v + 2*D_k + 2*H, d_model]; rows z | q | k | v | b | a  */
  const float *conv_w;    /* f32 [2*D_k + D_v, 4] over the channels q | k | v                   */
  const float *conv_b;    /* f32 [2*D_k + D_v] or NULL                                          */
  const float *dt_bias;   /* f32 [H]                                                            */
  const float *A_log;     /* f32 [H]                                                            */
  const float *norm_w;    /* f32 [d_v]                                                          */
  const void  *w_out;     /* T   [E, d_model, D_v]                                              */
} rom_gdn_weights;

/* Byte offsets of the intermediates inside the workspace after rom_gdn_forward. */
typedef struct rom_gdn_ws_layout {
  size_t total_bytes;
  size_t expert_idx;   /* i32 [N*K]                                        */
  size_t gate;         /* f32 [N*K]                                        */
  size_t counts;       /* i32 [E]                                          */
  size_t offsets;      /* i32 [E+1]                                        */
  size_t perm;         /* i32 [N*K]                                        */
  size_t inv_perm;     /* i32 [N*K]                                        */
  size_t logits;       /* f32 [N, E]                                       */
  size_t proj;         /* T   [N, 2*D_v + 2*D_k + 2*H]  (sum over k applied) */
  size_t qkv;          /* T   [N, 2*D_k + D_v]  after conv + SiLU (not normalised) */
  size_t y;            /* T   [N, D_v]  after norm and gate                */
} rom_gdn_ws_layout;

/* host-only; 0 / an error for invalid or unsupported dims */
ROM_API size_t rom_gdn_workspace_bytes(const rom_gdn_dims *dims, int64_t B, int64_t L);
ROM_API int rom_gdn_workspace_layout(const rom_gdn_dims *dims, int64_t B, int64_t L, rom_gdn_ws_layout *layout);

/* The layer above on B sequences of L tokens.
 *   x, out          T [B, L, d_model] (distinct);  eps: the head norm's epsilon (>= 0)
 *   conv_state_in   f32 [B, 2*D_k + D_v, 3] or NULL (zeros): the conv's inputs at the three steps
 *                   before the first, oldest first
 *   ssm_state_in    f32 [B, H, d_k, d_v] or NULL (zeros): S^T before the first step
 *   conv_state_out, ssm_state_out   the same after the last step, or NULL.  An output state may be the
 *                   same buffer as its input only for L <= 32.
 *   ws              rom_gdn_workspace_bytes(dims, B, L), 256-byte aligned
 * One workgroup walks a (sequence, head) from its first step to its last: the call is parallel over
 * B * H only.  Asynchronous on hip_stream, allocates nothing; B * L == 0 is a successful no-op; errors
 * are reported before anything is launched.  With profiling on, the stages are recorded under
 * ROM_STAGE_ROUTE, _PERMUTE, _IN_PROJ, _CONV, _SCAN (delta rule + norm + gate), _OUT_PROJ, _COMBINE. */
ROM_API int rom_gdn_forward(const rom_gdn_dims *dims, const rom_gdn_weights *w, const void *x, int64_t B,
                            int64_t L, float eps, const float *conv_state_in, const float *ssm_state_in,
                            void *out, float *conv_state_out, float *ssm_state_out, void *ws,
                            size_t ws_bytes, void *hip_stream);

/* The pre-norm residual block around it: out = x + layer(RMSNorm(x)); w->w_in FOLDED with norm_weight
 * (rom_fold_norm_rows over its E * (2*D_v + 2*D_k + 2*H) rows); see rom_mamba2_block_forward. */
ROM_API int rom_gdn_block_forward(const rom_gdn_dims *dims, const rom_gdn_weights *w, const float *norm_weight,
                                  float norm_eps, const void *x, int64_t B, int64_t L, float eps,
                                  const float *conv_state_in, const float *ssm_state_in, void *out,
                                  float *conv_state_out, float *ssm_state_out, void *ws, size_t ws_bytes,
                                  void *hip_stream);

/* One new token for each of B sequences (the recurrent form of rom_gdn_forward): x, out T [B, d_model];
 * conv_state and ssm_state (layouts above, both required) are read and updated in place.
 *   ws   rom_gdn_workspace_bytes(dims, B, 1) */
ROM_API int rom_gdn_step(const rom_gdn_dims *dims, const rom_gdn_weights *w, const void *x, int64_t B, float eps,
                         float *conv_state, float *ssm_state, void *out, void *ws, size_t ws_bytes,
                         void *hip_stream);

/* Static description of an error code. */
ROM_API const char *rom_strerror(int code);

/* Per-stage timing for benchmarks.  While enabled, rom_layer_forward and rom_step record a HIP
 * event at every stage boundary (a stage = a kernel or small kernel group) on the caller's
 * stream.  rom_profile_collect synchronises on those events, adds the elapsed milliseconds of
 * every recorded stage into stage_ms (host, ROM_STAGE_COUNT doubles), stores the number of calls
 * in *n_calls (host) and resets the recorder.  max_calls == 0 disables recording and frees the
 * events.  Process-wide and not thread-safe: a benchmark's tool, not part of the serving path. */
#define ROM_STAGE_ROUTE     0  /* router logits, top-K, gates                         */
#define ROM_STAGE_PERMUTE   1  /* histogram, offsets, stable permutation              */
#define ROM_STAGE_IN_PROJ   2  /* grouped GEMM, Eq. (10)/(11) (+ sum over k if K > 1)  */
#define ROM_STAGE_CONV      3  /* causal depthwise conv + SiLU, Eq. (2)                */
#define ROM_STAGE_X_PROJ    4  /* grouped GEMM dt_low | B | C                          */
#define ROM_STAGE_DT_PROJ   5  /* grouped GEMM + bias + softplus                       */
#define ROM_STAGE_SCAN      6  /* selective scan + D skip + SiLU(z) gating, Eq. (5)/(6) */
#define ROM_STAGE_OUT_PROJ  7  /* grouped GEMM Eq. (13) (+ gate scaling if K == 1)     */
#define ROM_STAGE_COMBINE   8  /* un-permute + gate-weighted sum, Eq. (12) (K > 1)     */
#define ROM_STAGE_COUNT     9
ROM_API int rom_profile_enable(int max_calls);
/* Restricts the timing to the stages whose bit (1u << ROM_STAGE_*) is set; the default is all.  An
 * event between two kernels costs several microseconds of launch overlap, so a benchmark that
 * wants one kernel's duration inside an otherwise undisturbed call selects that stage alone. */
ROM_API int rom_profile_select(unsigned stage_mask);
ROM_API int rom_profile_collect(double *stage_ms, int *n_calls);
/* The same per call: stage_ms (host) [max_calls][ROM_STAGE_COUNT] receives the milliseconds of
 * every stage of each of the first max_calls recorded calls (0 for a stage that did not run). */
ROM_API int rom_profile_collect_calls(double *stage_ms, int max_calls, int *n_calls);
/* A kernel of known HBM traffic for scaling hardware counter readings: copies n_bytes (a multiple
 * of 16; src, dst device pointers, 16-byte aligned, distinct) with one plain kernel
 * (calib_copy_kernel): n_bytes read, n_bytes written. */
ROM_API int rom_profile_copy(const void *src, void *dst, size_t n_bytes, void *hip_stream);
ROM_API const char *rom_stage_name(int stage);
/* Issue-rate probes behind `bench.py --probe` (what a wavefront of this chip issues per clock is
 * measured, not assumed).  One asynchronous launch of n_blocks workgroups of 256 threads:
 *   kind 0: p1 (1 or 8) independent chains of one instruction, p0 = 0 v_fma_f32, 1 v_exp_f32,
 *           2 v_mov_b32_dpp; 64 * iters instructions per wavefront;
 *   kind 1: the pipelined scan's tile on registers only; p0 = parts (bit 0 decay / input, bit 1 the
 *           FMA chain, bit 2 reduction and gate: 3, 6 or 7), p1 = 0 registers only, 1 with the
 *           tile's LDS reads, 2 also a barrier per tile; 64 * iters steps per wavefront.
 * scratch: device, n_blocks * 1024 bytes.  Unknown combinations return ROM_E_INVAL. */
ROM_API int rom_probe(int kind, int p0, int p1, int n_blocks, int iters, void *scratch, size_t scratch_bytes,
              void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ROM_H_ */

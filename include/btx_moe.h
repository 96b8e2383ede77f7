/*
 * btx_moe.h - C ABI of the MI355X (gfx950) Mixture-of-Experts feed-forward layer
 * of Branch-Train-MiX (arXiv 2403.07816).
 *
 * The layer (Sec. 3.2):   FF_MoE(x) = sum_i g_i(W_l x) * FF_i(x)
 * with a linear router W_l, a sparse routing function g, and per-expert SwiGLU
 * feed-forward sublayers FF_i(x) = (silu(x W1_i) * (x W3_i)) W2_i taken from the
 * branched expert models.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers unless the comment says "host".
 *   - Tensors are row-major and contiguous.  T = tokens, d = model width,
 *     f = feed-forward width per expert, E = experts, k = experts per token,
 *     R = T*k routed rows.
 *   - The caller owns every buffer, including the workspace; the library
 *     allocates nothing.  No result depends on an earlier call.  The only
 *     process-wide state is set-up and tooling: per device, the kernels'
 *     raised dynamic-LDS limit (btx_init) and the optional stage-event table
 *     (btx_profile_stages).
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call returns without synchronising.  Group sizes
 *     never travel to the host.
 *   - The return value is a btx_status.  Nothing throws, aborts or prints.
 *     Arguments are validated before anything is launched; on an error status
 *     no kernel has been enqueued.
 *   - T == 0 is a valid no-op (BTX_OK).
 *   - Rows move as 16-byte pieces: every tensor of rows (x, the expert weights and their
 *     gradients, saved activations, outputs, workspaces) starts on a 16-byte boundary, and
 *     the expert strides are multiples of 8 elements; BTX_ERR_INVALID_ARG otherwise.
 *   - Every kernel is free of atomics: results are bit-identical run to run.  The order
 *     of every sum is fixed by the shapes, the routing counts and the number of compute
 *     units of the device (the bf16 up-projection, down-projection and input-gradient
 *     products cut the tiles of a partly filled last round of workgroups into up to eight K
 *     ranges, added in ascending order by a second kernel).
 *   - Outputs must not alias inputs unless stated.  NaN/Inf inputs give
 *     unspecified results.
 */
#ifndef BTX_MOE_H
#define BTX_MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  BTX_OK = 0,
  BTX_ERR_INVALID_ARG = 1, /* null pointer, bad size, bad enum, k > E, ...            */
  BTX_ERR_UNSUPPORTED = 2, /* valid by the paper but outside what the kernels accept  */
  BTX_ERR_WORKSPACE = 3,   /* workspace smaller than the matching *_workspace_bytes() */
  BTX_ERR_HIP = 4          /* a HIP launch reported an error                          */
} btx_status;

typedef enum {
  BTX_F32 = 0, /* float                                    */
  BTX_BF16 = 1 /* bfloat16 storage, fp32 accumulation      */
} btx_dtype;

/* Routing function g (Sec. 3.2 and Sec. 3.3 "Routing method"). */
typedef enum {
  /* Top-k: keep the k largest logits, softmax over the kept ones (equal to the
   * full softmax renormalised over the chosen k).  Gates sum to 1 per token. */
  BTX_ROUTE_TOPK_RENORM = 0,
  /* Switch: k = 1, expert = argmax, gate = that expert's full-softmax probability. */
  BTX_ROUTE_SWITCH_TOP1 = 1,
  /* Sample top-1: k = 1, expert = first e with cumsum_{j<=e} softmax_j > U[t]
   * (E-1 if none), gate = that expert's full-softmax probability. */
  BTX_ROUTE_SAMPLE_TOP1 = 2,
  /* Sec. 3.3 "Sample Top-1" as printed, training time: soft sample y = softmax((logits + G) / tau)
   * with Gumbel noise G supplied by the caller, all but its largest entry zeroed: that expert
   * is run with gate y_max.  The load-balancing probabilities stay softmax(logits). */
  BTX_ROUTE_GUMBEL_TOP1 = 3
} btx_route_mode;

/* u_i of the load-balancing loss L_LB = alpha * E * sum_i u_i p_i (Sec. 3.3),
 * p_i = batch mean of softmax_i. */
typedef enum {
  BTX_LB_TOKEN_FRAC = 0, /* u_i = counts_i / (T*k): share of routed (token,slot) pairs */
  BTX_LB_GATE_MEAN = 1   /* u_i = (sum_t g_i) / T: the formula as printed              */
} btx_lb_mode;

/* btx_moe_ff_backward flags */
#define BTX_FLAG_LB_GRAD_THROUGH_U 1u /* BTX_LB_GATE_MEAN only: also differentiate u_i */

const char* btx_status_string(int status);
int btx_version(void);

/* One-time set-up on the CURRENT device: raises the dynamic-LDS limit of every expert-GEMM
 * kernel (they use all 160 KB of a compute unit's LDS).  Optional: the first bf16 call of
 * btx_moe_ff_forward / btx_moe_ff_backward on a device does the same by itself, but that
 * set-up cannot be recorded into a HIP graph, so a caller that captures its very first step
 * calls btx_init() before beginning the capture (once per device that it uses).  It also
 * looks up the device address of btx_moe_route_noalloc's fixed workspace.
 * Idempotent.  Errors: BTX_ERR_HIP. */
int btx_init(void);

/* Profiling aid (the one piece of process-wide state; not thread-safe; off by default).
 * events: HOST array of 2*n_pairs hipEvent_t handles owned by the caller.  While set,
 * stage s of any later call records events[2s] before and events[2s+1] after its
 * kernels on the caller's stream, so that single kernels can be timed inside the real
 * sequence.  n_pairs = 0 switches it off.  Stage ids: */
enum {
  BTX_STAGE_ROUTE = 0,        /* btx_moe_route: all three kernels                  */
  BTX_STAGE_GATHER_X = 1,     /* forward: x -> expert-grouped rows                 */
  BTX_STAGE_UP = 2,           /* forward: xs W1, xs W3, SwiGLU                     */
  BTX_STAGE_DOWN = 3,         /* forward: act W2                                   */
  BTX_STAGE_COMBINE = 4,      /* forward: gate-weighted un-permute                 */
  BTX_STAGE_GATHER_DY = 5,    /* backward: dY -> grouped rows                      */
  BTX_STAGE_BWD_ACT = 6,      /* backward: dys W2^T + SwiGLU backward              */
  BTX_STAGE_BWD_DX = 7,       /* backward: dh1 W1^T + dh3 W3^T                     */
  BTX_STAGE_GATHER_X_BWD = 8, /* backward: x -> grouped rows (for dW1, dW3)        */
  BTX_STAGE_DW13 = 9,         /* backward: dW1, dW3                                */
  BTX_STAGE_DW2 = 10,         /* backward: dW2                                     */
  BTX_STAGE_ROUTER_BWD = 11,  /* backward: router gradients and final dX           */
  BTX_STAGE_NORM_BWD = 12,    /* btx_rmsnorm_backward: both kernels                */
  BTX_STAGE_COUNT = 13
};
int btx_profile_stages(void** events, int n_pairs);

/* ---------------------------------------------------------------------------
 * btx_moe_route - router linear, softmax, selection, gates, load-balancing
 * statistics and the token -> expert grouping (Sec. 3.2: W_l x and
 * g = SoftMax(TopK(.)); Sec. 3.3: load balancing, Switch, sample top-1; the
 * grouping is what "skip FF_i where the gate is zero" needs).
 *
 *   x          [T,d]   x_dtype (BTX_F32 or BTX_BF16)
 *   W_router   [d,E]   fp32
 *   b_router   [E]     fp32, may be NULL (the paper's router has no bias)
 *   U          [T]     fp32 in [0,1); required iff route_mode == SAMPLE_TOP1;
 *              [T,E]   fp32 Gumbel noise (-log(-log(uniform))) iff route_mode == GUMBEL_TOP1
 *   tau                temperature of GUMBEL_TOP1 (> 0); ignored by the other modes
 *   capacity_factor    0 = dropless.  > 0: every expert keeps its first
 *                      ceil(capacity_factor * T*k / E) pairs in (t,j) order (Sec. 4.3: "a hard
 *                      limit after which routed tokens will be dropped"; the product is taken in
 *                      double precision on the float passed, so 0.8f, which lies above 0.8,
 *                      gives 209 and not 208 at T*k/E = 260); a dropped pair gets
 *                      inv_pos = -1, no grouped row and contributes nothing to the layer's output
 *                      or to dg; counts, gate_sum and lb_loss describe the routing before drops,
 *                      offsets the kept rows; perm[r] = 0 for r >= offsets[E]
 * Selection: logits are accumulated in fp32; ties go to the lower expert index;
 * topk_idx lists the chosen experts by descending logit.
 * Outputs
 *   topk_idx   [T,k]   int32 expert ids
 *   gates      [T,k]   fp32
 *   probs      [T,E]   fp32 full softmax (kept for the backward pass)
 *   counts     [E]     int32 routed pairs per expert (before any capacity drop)
 *   offsets    [E+1]   int32 exclusive prefix of counts
 *   perm       [R]     int32: perm[r] = t*k+j of the pair stored at grouped row r;
 *                      rows of expert e are offsets[e]..offsets[e+1]-1, in (t,j) order
 *   inv_pos    [T,k]   int32: inverse of perm (-1: pair dropped)
 *   gate_sum   [E]     fp32 sum_t g_{t,e}
 *   prob_sum   [E]     fp32 sum_t softmax_{t,e}
 *   lb_loss    [1]     fp32 lb_alpha * E * sum_e u_e * prob_sum_e / T
 * Requirements: 1 <= k <= E <= 64; d % 8 == 0; SWITCH/SAMPLE/GUMBEL need k == 1;
 * T*k < 2^31.  workspace >= btx_moe_route_workspace_bytes(T,d,E,k).
 */
size_t btx_moe_route_workspace_bytes(int T, int d, int E, int k);
int btx_moe_route(const void* x, int x_dtype, const float* W_router, const float* b_router, const float* U,
                  int T, int d, int E, int k, int route_mode, int lb_mode, float lb_alpha, float tau,
                  float capacity_factor, int32_t* topk_idx, float* gates, float* probs, int32_t* counts, int32_t* offsets,
                  int32_t* perm, int32_t* inv_pos, float* gate_sum, float* prob_sum, float* lb_loss,
                  void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * btx_moe_route_noalloc - btx_moe_route for callers that cannot allocate device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and bit-identical results, but without the workspace pair: the
 * workspace is a fixed array of btx_moe_route_noalloc_max_workspace_bytes() (4 MiB) inside the
 * library's device image, which every GPU the library runs on holds until the process ends.
 * The call allocates and frees nothing.
 *   - A problem whose btx_moe_route_workspace_bytes(T,d,E,k) exceeds that size is refused with
 *     BTX_ERR_WORKSPACE before anything else is checked or launched (T = 16384, d = 4096,
 *     E = 64 needs 2 MiB).
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 *     streams, two threads) race and give unspecified results; calls on one stream are safe.
 *     Nothing in the array has to start at zero, every call overwrites what it reads.
 *   - The array's device address is looked up on the first call on a device (or by btx_init);
 *     that look-up is not a stream operation and may precede a capture.
 */
size_t btx_moe_route_noalloc_max_workspace_bytes(void);
int btx_moe_route_noalloc(const void* x, int x_dtype, const float* W_router, const float* b_router, const float* U,
                          int T, int d, int E, int k, int route_mode, int lb_mode, float lb_alpha, float tau,
                          float capacity_factor, int32_t* topk_idx, float* gates, float* probs, int32_t* counts,
                          int32_t* offsets, int32_t* perm, int32_t* inv_pos, float* gate_sum, float* prob_sum,
                          float* lb_loss, void* stream);

/* ---------------------------------------------------------------------------
 * btx_moe_norm_route - btx_moe_route with the block's pre-normalisation folded into the
 * router's read of the rows.  The seed model (Sec. 4.1: Llama-2 7B) normalises the residual
 * stream h before its feed-forward sublayer,
 *     xn[t,c] = gain[c] * h[t,c] * rstd[t],   rstd[t] = 1 / sqrt(mean_c h[t,c]^2 + eps),
 * and the block's output is h + FF_MoE(xn): xn is the x of Sec. 3.2, h goes to
 * btx_moe_ff_forward as `residual`.  One kernel reads h, writes xn (for the expert
 * GEMMs) and rstd (for the backward pass) and routes on xn.
 *
 *   h      [T,d]  x_dtype   raw rows
 *   gain   [d]    fp32
 *   eps           >= 0
 *   xn     [T,d]  x_dtype   out; must not alias h
 *   rstd   [T]    fp32      out
 * Mean square, rstd and the product are evaluated in fp64 and xn is rounded once to x_dtype;
 * the logits are computed from those rounded values, exactly as btx_moe_route would from xn.
 * Everything else as btx_moe_route (same workspace size).
 */
int btx_moe_norm_route(const void* h, int x_dtype, const float* gain, float eps, void* xn, float* rstd,
                       const float* W_router, const float* b_router, const float* U, int T, int d, int E, int k,
                       int route_mode, int lb_mode, float lb_alpha, float tau, float capacity_factor,
                       int32_t* topk_idx, float* gates, float* probs, int32_t* counts, int32_t* offsets, int32_t* perm,
                       int32_t* inv_pos, float* gate_sum, float* prob_sum, float* lb_loss, void* workspace,
                       size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * btx_rmsnorm_backward - backward of that normalisation (chain rule; the paper prints no
 * backward pass).  dXn is the dX that btx_moe_ff_backward returns when it is given xn as x:
 *     dH[t]    = rstd[t] * gain * dXn[t] - h[t] * rstd[t]^3 * (sum_c gain_c dXn[t,c] h[t,c]) / d  (+ dres[t])
 *     dgain[c] = sum_t dXn[t,c] * h[t,c] * rstd[t]
 *
 *   dXn, h  [T,d]  dtype
 *   gain    [d]    fp32;  rstd [T] fp32 as written by btx_moe_norm_route
 *   dres    [T,d]  dtype, may be NULL: added to dH (the gradient that reaches h through the
 *                  residual connection, i.e. the dY given to btx_moe_ff_backward)
 *   dH      [T,d]  dtype  out; may alias dXn or dres
 *   dgain   [d]    fp32   out (overwritten)
 * fp32 arithmetic, sums in a fixed order (bit-reproducible).
 * Requirements: d % 8 == 0, d <= 16384; workspace >= btx_rmsnorm_backward_workspace_bytes(T,d).
 */
size_t btx_rmsnorm_backward_workspace_bytes(int T, int d);
int btx_rmsnorm_backward(const void* dXn, const void* h, const float* gain, const float* rstd, const void* dres,
                         int dtype, int T, int d, void* dH, float* dgain, void* workspace, size_t workspace_bytes,
                         void* stream);

/* ---------------------------------------------------------------------------
 * btx_moe_ff_forward - gather tokens into expert groups, the expert SwiGLU
 * FFNs as grouped GEMMs, and the gate-weighted combine (layer equation of
 * Sec. 3.2; FF_i is the seed model's 3-matrix feed-forward, Sec. 4.1).
 *
 *   x   [T,d]            dtype
 *   W1, W3  expert e at  W + e*w13_expert_stride elements, [d,f] row-major
 *   W2      expert e at  W2 + e*w2_expert_stride elements, [f,d] row-major
 *   gates, offsets, perm, inv_pos: as written by btx_moe_route
 *   residual [T,d]       dtype, may be NULL: the transformer block's input, added to the sum
 *                        (h + FF_MoE(norm(h)) in one pass; with a capacity limit a token whose
 *                        pairs were all dropped passes through as the residual alone).  May be x
 *                        itself or out (elementwise in t).
 *   out [T,d]            dtype:  out[t] = residual[t] + sum_j gates[t,j] * FF_{idx[t,j]}(x[t]),
 *                        summed in fp32 (residual first, then j ascending), rounded once
 *   save_h1, save_h3 [R,f] dtype, grouped-row order: x W1_e and x W3_e, kept for
 *                        the backward pass.  Both NULL = forward only.
 * dtype BTX_BF16: bf16 storage, bf16 MFMA products, fp32 accumulation; the
 * activation silu(h1)*h3 and the expert output are rounded to bf16 once each.
 * dtype BTX_F32: plain fp32 FMA kernels (parity path, not the fast path).
 * Requirements: d % 8 == 0, f % 8 == 0, strides >= d*f and multiples of 8.
 * Limits (BTX_ERR_UNSUPPORTED beyond them; also for btx_moe_ff_backward): the bf16 kernels (d and f
 * multiples of 32, both >= 64) address the padded grouped rows with 32-bit byte offsets,
 * ceil(R/64)*64 + 64*E < 2^23 (about 8.3 M routed rows); the plain kernels (fp32, or bf16 with other
 * d, f) take R/64 + E <= 65535 row tiles (about 4.1 M routed rows).
 */
size_t btx_moe_ff_forward_workspace_bytes(int T, int d, int f, int E, int k, int dtype);
int btx_moe_ff_forward(const void* x, const void* W1, const void* W3, const void* W2, int dtype,
                       int64_t w13_expert_stride, int64_t w2_expert_stride, int T, int d, int f, int E, int k,
                       const float* gates, const int32_t* offsets, const int32_t* perm, const int32_t* inv_pos,
                       const void* residual, void* out, void* save_h1, void* save_h3,
                       void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * btx_moe_ff_backward - gradients of  <dY, out> + lb_grad_scale * lb_loss  with
 * the discrete expert selection held fixed (chain rule on Sec. 3.2's layer
 * equation and Sec. 3.3's load-balancing loss; the paper trains the layer by
 * gradient descent but prints no backward).
 *
 *   dY [T,d] dtype; x, W*, strides, routing outputs, save_h1/save_h3 as in forward
 *   lb_grad_scale: upstream gradient of lb_loss (1 when it is added to the
 *                  training loss as in Sec. 3.3; 0 = no load-balancing gradient)
 *   noise [T,E], tau: the Gumbel noise and temperature given to btx_moe_route when
 *                  route_mode == GUMBEL_TOP1 (the soft sample is recomputed from probs,
 *                  noise and tau); noise must be NULL for the other modes
 * Outputs (overwritten, never accumulated into)
 *   dX        [T,d]  dtype
 *   dW_router [d,E]  fp32
 *   db_router [E]    fp32, may be NULL
 *   dW1, dW3, dW2    stacked like W1/W3/W2 (same strides), dW_dtype; all three
 *                    NULL = frozen experts (router and input gradients only).
 *                    Experts with no routed rows get zeros.
 * Requirements as forward; dW_dtype must equal dtype or be BTX_F32.
 */
size_t btx_moe_ff_backward_workspace_bytes(int T, int d, int f, int E, int k, int dtype);
int btx_moe_ff_backward(const void* dY, const void* x, const float* W_router, const void* W1, const void* W3,
                        const void* W2, int dtype, int64_t w13_expert_stride, int64_t w2_expert_stride,
                        int T, int d, int f, int E, int k, int route_mode, int lb_mode, float lb_alpha,
                        float lb_grad_scale, unsigned flags, const float* noise, float tau,
                        const int32_t* topk_idx, const float* gates, const float* probs,
                        const int32_t* offsets, const int32_t* perm, const int32_t* inv_pos,
                        const float* gate_sum, const float* prob_sum, const int32_t* counts,
                        const void* save_h1, const void* save_h3,
                        void* dX, float* dW_router, float* db_router, void* dW1, void* dW3, void* dW2,
                        int dW_dtype, void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * btx_merge_average - elementwise mean of N same-shape tensors: how the
 * non-feed-forward parameters (attention, embeddings, ...) of the branched
 * models are merged (Sec. 3.2).
 *
 *   inputs  HOST array of N device pointers, each [numel] of dtype
 *   out     [numel] dtype; may alias any inputs[i]
 * BTX_BF16: the sum is taken in fp32 in input order and its quotient by N is
 * rounded to bf16 once (no double rounding through fp32).  BTX_F32: sum and
 * division in fp64, rounded once to fp32.  The mean of N equal tensors is
 * that tensor, bit for bit.
 * Requirements: 1 <= N <= 16, numel >= 0, pointers aligned to 16 bytes.
 */
int btx_merge_average(const void* const* inputs, int N, void* out, int64_t numel, int dtype, void* stream);

/* ---------------------------------------------------------------------------
 * btx_merge_weighted - the merge of Sec. 3.2 with caller-chosen coefficients:
 * out = sum_n weights[n] * inputs[n], elementwise.  (The paper only averages;
 * this is the same pass with the 1/N replaced by a weight per model, e.g. to
 * favour the seed model or a domain.  The weights are used as given, they are
 * not normalised.)
 *
 *   inputs   HOST array of N device pointers, each [numel] of dtype
 *   weights  HOST array of N finite floats
 *   out      [numel] dtype; may alias any inputs[i]
 * The sum is accumulated in fp64 in input order (every product is exact there)
 * and rounded once to the storage type, for bf16 without a detour through fp32.
 * Requirements: 1 <= N <= 16, numel >= 0, pointers aligned to 16 bytes.
 */
int btx_merge_weighted(const void* const* inputs, const float* weights, int N, void* out, int64_t numel, int dtype,
                       void* stream);

/* ---------------------------------------------------------------------------
 * btx_mix_experts - MiX construction utilities of Sec. 3.3: "Splitting Experts"
 * (each of the N FFs is cut along d_ff into C chunks, giving N*C experts of width
 * f/C: expert i*C+c owns columns [c*f/C, (c+1)*f/C) of W1_i and W3_i and the same
 * rows of W2_i) and "Blending Experts" (each FF is cut into N chunks and expert n is
 * built from the n-th chunk of FF 0, FF 1, ... in that order; width stays f).  A
 * one-off copy made when the MoE is built; every element is moved unchanged.
 *   W1, W3: DEVICE [N,d,f]; W2: DEVICE [N,f,d]; contiguous, element type `dtype`.
 *   mode: BTX_MIX_SPLIT (C >= 1, f % C == 0, N*C <= 64) or BTX_MIX_BLEND (C ignored,
 *         f % N == 0).
 *   oW1, oW3: DEVICE [N*C,d,f/C] (split) or [N,d,f] (blend); oW2: [N*C,f/C,d] or
 *         [N,f,d].  Caller-owned, must not be the input buffers.
 * Errors: BTX_ERR_INVALID_ARG (NULL or aliased pointers, bad mode or chunk count),
 * BTX_ERR_HIP. */
typedef enum { BTX_MIX_SPLIT = 0, BTX_MIX_BLEND = 1 } btx_mix_mode;
int btx_mix_experts(const void* W1, const void* W3, const void* W2, int dtype, int N, int d, int f, int mode, int C,
                    void* oW1, void* oW3, void* oW2, void* stream);

/* ---------------------------------------------------------------------------
 * btx_adamw_step - fused AdamW update (Sec. 4.1: "AdamW optimizer with weight decay
 * 0.1"; the moment decay rates and eps are not stated and are arguments), for the
 * weight gradients btx_moe_ff_backward returns:
 *   m <- beta1 m + (1-beta1) g;  v <- beta2 v + (1-beta2) g^2
 *   p <- p - lr * ( (m/(1-beta1^step)) / (sqrt(v/(1-beta2^step)) + eps) + weight_decay * p )
 * in fp32, elementwise, in place.
 *   master, m, v  DEVICE [numel] fp32, 16-byte aligned: master weights and moments
 *   grad          DEVICE [numel] grad_dtype (BTX_BF16 or BTX_F32), 16-byte aligned
 *   lowp          DEVICE [numel] bf16, 8-byte aligned, may be NULL: receives the updated
 *                 weights rounded once to bf16 (the copy the layer's GEMMs read)
 *   step          1-based count of updates, for the bias corrections
 *   lr, beta1, beta2, eps, weight_decay: floats; the arithmetic runs on the float values as
 *                 passed (1 - 0.999f is 1.3e-5 relative away from 0.001)
 * Errors: BTX_ERR_INVALID_ARG (NULL / misaligned pointers, step < 1, beta outside [0,1),
 * negative eps), BTX_ERR_HIP. */
int btx_adamw_step(float* master, float* m, float* v, const void* grad, int grad_dtype, void* lowp, int64_t numel,
                   int step, float lr, float beta1, float beta2, float eps, float weight_decay, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BTX_MOE_H */

/*
 * revffn.h - C ABI of the RevFFN reversible block for AMD MI355X (gfx950).
 *
 * The block (paper section 3.1, Eq. 1-2, with the projection adapters of
 * section 3.2) splits the hidden state H[B,S,d] into two streams of width
 * h = d/2 and updates them as
 *
 *     Y1 = X1 + P_dn_a( Attn_pt(P_up_a Norm X1, P_up_a Norm X2, P_up_a Norm X2) )
 *     Y2 = X2 + P_dn_m( MoE_pt(P_up_m Norm Y1) )
 *
 * where Attn_pt is multi-head softmax attention (queries from stream 1, keys and
 * values from stream 2) and MoE_pt is a top-k routed mixture of SwiGLU experts
 * plus an optional sigmoid-gated shared SwiGLU expert.  The inverse rebuilds
 * (X1, X2) from (Y1, Y2); the backward pass recomputes all activations from a
 * supplied (rebuilt) input instead of reading cached ones.
 *
 * Conventions common to every call
 *  - All tensor pointers are DEVICE pointers owned by the caller.  The library
 *    never frees or reallocates them.  Host pointers are marked "host".
 *  - Element type of streams, weights and gradients is given by config.dtype:
 *    0 = float32, 1 = bfloat16 (fp32 accumulation).  b_router and the routing
 *    outputs are always float32 / int32.  With config.fp32_streams the four
 *    residual streams x1, x2, y1, y2 of every call are float32 arrays instead
 *    (the gradient streams dy1, dy2, dx1, dx2 keep config.dtype).
 *  - Linear weights are row-major [out, in] and are applied as x @ W^T.
 *  - A stream is token-major [T, h], T = B*S, token t = b*S + s, with row
 *    stride `ld` elements (ld >= h).  ld = d lets the two halves of one [T, d]
 *    hidden tensor be passed without a copy (section 3.1, the split display).
 *  - Every compute call only enqueues work and returns; it never synchronises the host (the setters and getters of
 *    the tolerance-driven inverse and revffn_profile_read say where they wait).
 *    Work is ordered after what `hip_stream` (a hipStream_t; NULL = the default
 *    stream) already holds, and `hip_stream` is ordered after all of it when the call
 *    returns; independent branches inside a call run on four helper streams owned by
 *    the context (default priority; revffn_set_helper_streams(ctx, 0) or the environment
 *    variable REVFFN_NO_STREAMS=1 at creation keep everything on `hip_stream`).  Calls on one context must be issued on one stream at a time
 *    (they share the context workspace).
 *  - Return value: 0 on success, a negative REVFFN_E* code otherwise.  No call
 *    throws or aborts.  Arguments are validated before the first launch, so REVFFN_EINVAL / ESHAPE / ENULL mean
 *    that nothing has been enqueued; REVFFN_EHIP / EUNSUPPORTED can come from the middle of a call, after part
 *    of its work has been enqueued (outputs are then undefined).
 *  - Results are deterministic: no floating-point atomics anywhere, so the same
 *    inputs give bit-identical outputs, and the routing recomputed by the
 *    inverse/backward from Y1 is bit-identical to the forward routing.
 */
#ifndef REVFFN_H
#define REVFFN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  REVFFN_OK = 0,
  REVFFN_EINVAL = -1,      /* bad config value                                  */
  REVFFN_ESHAPE = -2,      /* B, S or ld out of range for this context          */
  REVFFN_ENULL = -3,       /* a required pointer is NULL                        */
  REVFFN_EWORKSPACE = -4,  /* device allocation of the workspace failed         */
  REVFFN_EHIP = -5,        /* a HIP runtime call failed                         */
  REVFFN_EUNSUPPORTED = -6 /* valid request this build does not implement       */
};

enum { REVFFN_F32 = 0, REVFFN_BF16 = 1 };

/* Geometry and the readings the paper leaves open (all switchable). */
typedef struct revffn_config {
  int32_t d_model;         /* d; even                                             */
  int32_t n_heads;         /* n_heads * head_dim == d_model                       */
  int32_t head_dim;        /* even (rotary pairs)                                 */
  int32_t n_experts;       /* E, 1..256                                           */
  int32_t top_k;           /* 1..min(E, 16)                                       */
  int32_t d_expert;        /* I, routed expert intermediate width                 */
  int32_t d_shared;        /* Is, shared expert intermediate width; 0 = none      */
  int32_t dtype;           /* REVFFN_F32 or REVFFN_BF16                           */
  int32_t causal;          /* 1 = causal mask                                     */
  int32_t use_rope;        /* 1 = rotary encoding on Q and K (half-split pairs)   */
  int32_t norm_topk_prob;  /* 1 = renormalise routing weights over the top-k set  */
  int32_t n_inv_iters;     /* fixed-point iterations of the inverse (>= 0);
                              the paper uses 1 (end of section 3.1)               */
  float rope_theta;        /* e.g. 1e6                                            */
  float rms_eps;           /* e.g. 1e-6                                           */
  int32_t fp32_streams;    /* 1 = the residual streams x1, x2, y1, y2 (and the
                              rebuilt ones) are float32 arrays whatever dtype is;
                              weights, activations inside the block and the gradient
                              streams dy*, dx* keep dtype.  The coupling adds of
                              Eq. 1-2 and the subtractions of the inverse then round
                              to float32 instead of dtype, which removes the storage
                              rounding from the reconstruction.  0 = streams have
                              dtype.  No effect with dtype REVFFN_F32.             */
  int32_t symmetric;       /* 1 = the symmetric comparison block section 3.1
                              contrasts the layout with: queries come from stream 2
                              as well, Y1 = X1 + Attn(Norm X2, Norm X2, Norm X2),
                              Y2 as in Eq. 2.  The branch of Eq. 1 then ignores X1,
                              so revffn_inverse is closed-form and exact (no
                              iteration: n_inv_iters and the tolerance are ignored,
                              residual = 0), dX1 is the gradient at Y1 and the
                              gradient of norm_a1 is zero.  0 = the paper's
                              asymmetric block (Eq. 1).                            */
  int32_t fp32_grads;      /* 1 = every weight-gradient buffer of revffn_grads is a
                              float32 array whatever dtype is (the GEMMs accumulate
                              in float32 anyway; this skips the rounding of the
                              result to dtype).  0 = gradients have dtype.  The
                              input gradients dx1, dx2 keep dtype either way.      */
} revffn_config;

/* Weights of one block.  Device pointers, dtype = config.dtype unless noted. */
typedef struct revffn_weights {
  const void *norm_a1, *norm_a2, *norm_m; /* [h] RMSNorm gains for X1, X2, Y1        */
  const void *pup_a, *pdn_a;              /* [d,h], [h,d] attention adapters (3.2)   */
  const void *pup_m, *pdn_m;              /* [d,h], [h,d] MoE adapters (3.2)         */
  const void *wq, *wk, *wv, *wo;          /* [d,d]                                   */
  const void *bq, *bk, *bv;               /* [d] or NULL                             */
  const void *w_router;                   /* [E,d]                                   */
  const float *b_router;                  /* [E] float32 or NULL (added to logits)   */
  const void *w_gate_up;                  /* [E,2I,d]: I gate rows then I up rows    */
  const void *w_down;                     /* [E,d,I]                                 */
  const void *ws_gate_up;                 /* [2Is,d]; NULL iff d_shared == 0         */
  const void *ws_down;                    /* [d,Is]                                  */
  const void *ws_gate;                    /* [d] shared-expert sigmoid gate          */
} revffn_weights;

/* Where weight gradients go: same shapes and dtype as the weights (b_router:
 * float32).  A NULL field means "this gradient is not wanted" and its GEMM is
 * skipped (section 3.3: stage 1 trains only the adapters; stage 2 keeps the
 * routers frozen).  Non-NULL fields are OVERWRITTEN, not accumulated.  With
 * config.fp32_grads every buffer holds float32. */
typedef struct revffn_grads {
  void *norm_a1, *norm_a2, *norm_m;
  void *pup_a, *pdn_a, *pup_m, *pdn_m;
  void *wq, *wk, *wv, *wo;
  void *bq, *bk, *bv;
  void *w_router;
  float *b_router;
  void *w_gate_up, *w_down;
  void *ws_gate_up, *ws_down, *ws_gate;
} revffn_grads;

/* Pre-merged adapter weights (section 3.2: each pre-trained module is wrapped as P_dn(module(P_up .)), so with static
 * weights the products can be formed once).  Device buffers owned by the caller, dtype = config.dtype except
 * w_router (float32); filled by revffn_merge_adapters, read by revffn_forward_merged / revffn_inverse_merged. */
typedef struct revffn_merged {
  void *wq, *wk, *wv;     /* [d,h]   = Wq P_up_a, Wk P_up_a, Wv P_up_a                               */
  void *wo;               /* [h,d]   = P_dn_a Wo                                                      */
  void *w_gate_up;        /* [E,2I,h] = W_gate_up[e] P_up_m                                           */
  void *w_down;           /* [E,h,I] = P_dn_m W_down[e]                                               */
  void *ws_gate_up;       /* [2Is,h] = Ws_gate_up P_up_m;  NULL iff d_shared == 0                     */
  void *ws_down;          /* [h,Is]  = P_dn_m Ws_down                                                 */
  float *w_router;        /* [E (+1 with a shared expert), h] float32 = [W_r ; ws_gate] P_up_m diag(norm_m) */
} revffn_merged;

typedef struct revffn_ctx revffn_ctx; /* opaque: owns the device workspace only */

/* Device bytes a context for up to max_B x max_S tokens allocates; 0 if cfg is invalid. */
size_t revffn_workspace_bytes(const revffn_config *cfg, int32_t max_B, int32_t max_S);

/* Validate cfg (host) and allocate the workspace on the current device.
 * The only calls that allocate or free device memory are create and destroy. */
int revffn_create(revffn_ctx **out, const revffn_config *cfg, int32_t max_B, int32_t max_S);
void revffn_destroy(revffn_ctx *ctx);

/* Change the inverse's fixed-point iteration count of an existing context. */
int revffn_set_inv_iters(revffn_ctx *ctx, int32_t n_inv_iters);

/* Tolerance-driven inverse (the fixed-point iteration of section 3.1 run to a stopping rule instead of a fixed
 * count).  tol > 0: every inverse on this context (revffn_inverse, revffn_inverse_backward, each block of
 * revffn_stack_backward) iterates until max |x_n - x_(n-1)| <= tol (absolute, in the units of the streams) or
 * max_iters (1..1024) iterations have run, whichever comes first, and n_inv_iters is ignored.
 * The decision is taken on the device, per block of rows: a query row's iterate depends on that row alone (keys and
 * values come from the rebuilt stream 2, which the iteration does not change), so a block that has met the
 * tolerance keeps its iterate, bit for bit the one a fixed count of that many iterations gives, while other blocks
 * go on.  block_positions > 0: a block is a run of that many positions of one sequence (the error of the iteration
 * sits in the first causal positions, which see few keys: section 3.1, last paragraph); block_positions == 0 (and
 * revffn_set_inverse_tolerance): one block, the whole call stops together.  The call enqueues all max_iters
 * iterations and returns; workgroups whose rows are all finished exit at once (a finished iteration costs its
 * launches, a few microseconds each, so max_iters should be a small cap).  The calls stay asynchronous and can be
 * captured into a HIP graph.  In bf16 successive iterates stop changing at the rounding of the stored iterate (about
 * 2^-8 of its largest element); a tolerance below that floor runs to max_iters.  tol = 0 switches back to the fixed
 * count.  Both setters wait for the device and reset the statistics below (call them outside graph capture).
 * Return REVFFN_EINVAL for a negative or NaN tol, max_iters out of range or a negative block_positions. */
int revffn_set_inverse_tolerance(revffn_ctx *ctx, float tol, int32_t max_iters);
int revffn_set_inverse_tolerance_blocked(revffn_ctx *ctx, float tol, int32_t max_iters, int32_t block_positions);

/* Statistics of the tolerance-driven inverse since the tolerance was set, kept on the device and read back here
 * (the call waits for the device): inverses run, iterations summed over them (per inverse: the largest count over
 * its blocks), and the iteration count and residual (largest over the blocks, each at its last iteration) of the
 * most recent one.  Any pointer may be NULL.  All zero while the tolerance is off. */
int revffn_get_inverse_stats(revffn_ctx *ctx, int64_t *calls, int64_t *iters_total,
                             int32_t *last_iters, float *last_residual);

/* Per block of the most recent tolerance-driven inverse: iterations run and the residual at the last of them, in
 * block order (sequence-major, then position range).  iters / residuals: HOST arrays of cap entries (either may be
 * NULL); *n_blocks receives the number of blocks (B * ceil(S / block_positions), or 1).  Waits for the device. */
int revffn_get_inverse_blocks(revffn_ctx *ctx, int32_t *iters, float *residuals, int32_t cap, int32_t *n_blocks);

/* Eq. 1-2.  x1, x2: [T,h] inputs; y1, y2: [T,h] outputs, all with row stride ld.
 * y1 may alias x1 and y2 may alias x2 (in-place update). */
int revffn_forward(revffn_ctx *ctx, const revffn_weights *w,
                   const void *x1, const void *x2, void *y1, void *y2,
                   int32_t B, int32_t S, int64_t ld, void *hip_stream);

/* Inverse display of section 3.1: X2^ = Y2 - MoE branch at Y1 (exact up to the
 * rounding of one subtraction); X1^ by n_inv_iters fixed-point iterations
 * x <- Y1 - attention branch(x, X2^) started at x = Y1.  x1 may alias y1 and x2
 * may alias y2.  residual (device float[1], may be NULL) receives
 * max |x_n - x_(n-1)| of the last iteration, so a caller can detect a
 * non-contracting iteration. */
int revffn_inverse(revffn_ctx *ctx, const revffn_weights *w,
                   const void *y1, const void *y2, void *x1, void *x2,
                   int32_t B, int32_t S, int64_t ld, float *residual, void *hip_stream);

/* Gradient of Eq. 1-2 at block input (x1, x2) (normally the rebuilt one) for
 * upstream gradients (dy1, dy2).  Activations are recomputed, none is cached
 * between calls (section 3.1).  y1: the exact stream-1 block output held by the
 * sweep, used for the MoE half so that the recomputed routing equals the forward
 * routing; NULL = recompute it as x1 + attention branch.  dx1/dx2 may alias
 * dy1/dy2.  g may be NULL (input gradients only). */
int revffn_backward(revffn_ctx *ctx, const revffn_weights *w,
                    const void *x1, const void *x2, const void *y1,
                    const void *dy1, const void *dy2, void *dx1, void *dx2,
                    const revffn_grads *g, int32_t B, int32_t S, int64_t ld, void *hip_stream);

/* The non-reversible comparison route (the stored-activation baseline of the memory / speed comparison, section
 * 4): the same gradient as revffn_backward(x1, x2, y1, ...), taken from the activations that the immediately
 * preceding revffn_forward(x1, x2 -> y1, y2) on this context left in its workspace: no inverse, no recomputation,
 * at the price of one context (one block's activations) per layer held between the two calls.  Returns
 * REVFFN_EINVAL if the last call on this context was not an out-of-place revffn_forward with the same x1, x2, y1,
 * B, S, ld, or if dx1/dx2 alias x1, x2 or y1; the stored state serves one call.  Same bits as revffn_backward. */
int revffn_backward_stored(revffn_ctx *ctx, const revffn_weights *w,
                           const void *x1, const void *x2, const void *y1,
                           const void *dy1, const void *dy2, void *dx1, void *dx2,
                           const revffn_grads *g, int32_t B, int32_t S, int64_t ld, void *hip_stream);

/* One step of the reversible backward sweep (section 3.1): revffn_inverse followed by
 * revffn_backward at the rebuilt input, in one call.  The MoE half is evaluated once, at the
 * exact y1, and serves both the inverse (X2^ = Y2 - MoE branch) and the backward pass; the
 * results are bit-identical to the two separate calls.  x1/x2 (rebuilt input, out) may alias
 * y1/y2; dx1/dx2 may alias dy1/dy2. */
int revffn_inverse_backward(revffn_ctx *ctx, const revffn_weights *w,
                            const void *y1, const void *y2, void *x1, void *x2,
                            const void *dy1, const void *dy2, void *dx1, void *dx2,
                            const revffn_grads *g, int32_t B, int32_t S, int64_t ld,
                            float *residual, void *hip_stream);

/* Pre-merged adapters, for passes with static weights (inference-like forward passes; rebuilding inputs).
 * revffn_merge_adapters forms the products of revffn_merged from w (matrix-core GEMMs; about 1 Tflop at the
 * Qwen1.5-MoE shape, so it pays only when the weights stay fixed over many calls; the merged set is half the size
 * of the block's weights).  revffn_forward_merged / revffn_inverse_merged compute Eq. 1-2 / the inverse display from
 * it: no adapter GEMMs, projections and expert gate-up GEMMs contract over h instead of d, expert down GEMMs write
 * width h, and half the expert weight bytes are streamed.  w still supplies the norm gains, the q/k/v biases and
 * b_router (and must be the weights m was merged from).  Same conventions as revffn_forward / revffn_inverse (in
 * place allowed, residual optional); results agree with the unmerged calls to the rounding of the merged products
 * (they are stored in dtype), not bit for bit.  The inverse runs config.n_inv_iters iterations (the tolerance rule
 * applies to the unmerged calls only).  Gradients are taken with revffn_backward on the unmerged weights: it is
 * the same function.  REVFFN_EUNSUPPORTED with config.symmetric. */
int revffn_merge_adapters(revffn_ctx *ctx, const revffn_weights *w, const revffn_merged *m, void *hip_stream);
int revffn_forward_merged(revffn_ctx *ctx, const revffn_weights *w, const revffn_merged *m,
                          const void *x1, const void *x2, void *y1, void *y2,
                          int32_t B, int32_t S, int64_t ld, void *hip_stream);
int revffn_inverse_merged(revffn_ctx *ctx, const revffn_weights *w, const revffn_merged *m,
                          const void *y1, const void *y2, void *x1, void *x2,
                          int32_t B, int32_t S, int64_t ld, float *residual, void *hip_stream);

/* Stack of n_blocks blocks (section 3.1: only the last hidden state is kept).
 * Forward: (x1,x2) -> (y1,y2) through w[0..n_blocks-1], no stream swap between
 * blocks; y may alias x.  Backward sweep: starting from the stack output (y1,y2),
 * which is OVERWRITTEN in place by each block's rebuilt input, and (dy1,dy2),
 * overwritten in place by the gradient flowing down; on return they hold the
 * rebuilt stack input and its gradient.  g: host array of n_blocks grads structs
 * or NULL. */
int revffn_stack_forward(revffn_ctx *ctx, const revffn_weights *w /*host array*/, int32_t n_blocks,
                         const void *x1, const void *x2, void *y1, void *y2,
                         int32_t B, int32_t S, int64_t ld, void *hip_stream);
int revffn_stack_backward(revffn_ctx *ctx, const revffn_weights *w /*host array*/,
                          const revffn_grads *g /*host array or NULL*/, int32_t n_blocks,
                          void *y1, void *y2, void *dy1, void *dy2,
                          int32_t B, int32_t S, int64_t ld, void *hip_stream);

/* Parity taps (not on the hot path).  Copy the routing of the most recent
 * forward / inverse / backward call on ctx into caller DEVICE buffers (any may
 * be NULL): idx [T,k] expert per slot, slots by descending logit, equal logits
 * to the lower expert index; wts [T,k] routing weights; counts [E];
 * offsets [E+1] exclusive prefix sum; row_map [T*k]: permuted row -> t*k + slot,
 * grouped by expert, (token, slot) order kept inside an expert. */
int revffn_get_routing(revffn_ctx *ctx, int32_t *idx, float *wts, int32_t *counts,
                       int32_t *offsets, int32_t *row_map, void *hip_stream);

/* With taps enabled, forward/inverse also keep the two branch outputs (the terms
 * added to X1 and X2 in Eq. 1-2) in float32, before the residual add rounds them
 * away.  which: 0 = attention branch [T,h], 1 = MoE branch [T,h].  dst: device
 * float [T,h], dense. */
int revffn_enable_taps(revffn_ctx *ctx, int32_t on);
int revffn_get_branch(revffn_ctx *ctx, int32_t which, float *dst, void *hip_stream);

/* Select kernels: 0 = automatic (MFMA kernels where the shape allows),
 * 1 = force the generic kernels (any shape, slow).  For tests. */
int revffn_set_kernel_mode(revffn_ctx *ctx, int32_t mode);

/* Helper streams on (default) or off for the following calls.  Off: every kernel of a call runs on
 * `hip_stream` in program order (same results bit for bit; used to time kernels one at a time). */
int revffn_set_helper_streams(revffn_ctx *ctx, int32_t on);

/* Kernel-level entry points for unit tests and micro-benchmarks of the two dense kernels
 * (they need no context).  dtype as in revffn_config; kernel_mode as in
 * revffn_set_kernel_mode.  op_gemm: C[M,N] = A . B with A(m,k) = a[m*lda+k] (a_trans=0) or
 * a[k*lda+m] (a_trans=1), B(k,n) = b[n*ldb+k] (b_trans=0) or b[k*ldb+n] (b_trans=1); C has
 * dtype `dtype`, or float32 if out_f32.  op_attention_*: softmax(Q K^T / sqrt(dh) + causal
 * mask) V on q,k,v,o,d_o,dq,dk,dv laid out [B*S, H*dh] (head hh in columns hh*dh..), lse
 * and dvec float [B,H,S]; the backward needs o and lse from the forward and uses dvec as
 * scratch.  Return 0, REVFFN_EINVAL, or REVFFN_EUNSUPPORTED (kernel_mode 2 = MFMA kernels
 * only, refused when the shape does not fit them).  op_gemm only: kernel_mode + 256 * t with
 * t in 1..4 forces one tile shape of the MFMA kernel for this launch (1 = 128x64, 2 = 128x128, 3 = 256x128,
 * 4 = 256x256), so that a test can reach every shape at small sizes. */
int revffn_op_gemm(int32_t dtype, int32_t kernel_mode, const void *a, const void *b, void *c,
                   int32_t M, int32_t N, int32_t K, int64_t lda, int64_t ldb, int64_t ldc,
                   int32_t a_trans, int32_t b_trans, int32_t out_f32, void *hip_stream);
int revffn_op_attention_fwd(int32_t dtype, int32_t kernel_mode, const void *q, const void *k,
                            const void *v, void *o, float *lse, int32_t B, int32_t S, int32_t H,
                            int32_t dh, int32_t causal, void *hip_stream);
int revffn_op_attention_bwd(int32_t dtype, int32_t kernel_mode, const void *q, const void *k,
                            const void *v, const void *o, const void *d_o, const float *lse,
                            float *dvec, void *dq, void *dk, void *dv, int32_t B, int32_t S,
                            int32_t H, int32_t dh, int32_t causal, void *hip_stream);

/* For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): revffn_op_attention_bwd with its float scratch dvec[B,H,S] taken from a device array built into the
 * library (4 MiB, held by every GPU the library runs on until the process ends) instead of a caller buffer.  Same
 * kernels and the same bits as revffn_op_attention_bwd.  Limit: B * H * S <= 1048576 rows, else REVFFN_ESHAPE and
 * nothing is enqueued.  The call allocates and frees nothing (no hipMalloc / hipFree, no allocating library routine)
 * and only enqueues work on hip_stream.  Every call on one GPU shares that GPU's array: calls that may overlap on one
 * GPU (different streams, different threads) race on it and must be serialised by the caller.  Nothing in the array
 * needs to start at zero: each call's first kernel writes every element the later kernels of that call read. */
int revffn_op_attention_bwd_noalloc(int32_t dtype, int32_t kernel_mode, const void *q, const void *k,
                                    const void *v, const void *o, const void *d_o, const float *lse,
                                    void *dq, void *dk, void *dv, int32_t B, int32_t S,
                                    int32_t H, int32_t dh, int32_t causal, void *hip_stream);

/* Host-only check hook (no GPU work): where the MFMA GEMM's XCD-aware launch places its workgroups.
 * Workgroups reach the 8 XCDs round-robin by linear id; the kernel maps workgroup `i` back to a tile so that
 * each XCD works on tiles that share operands.  This call runs the same index function on the host for every
 * workgroup of the grid the launcher would use and writes (n-tile, m-tile, group) to out[3*i..3*i+2], or
 * (-1,-1,-1) for a workgroup that exits without a tile.  group_mode 0: dense problem of tiles_m x tiles_n tiles
 * of bm x bn elements; 1: expert tile list with room for tiles_m entries of which n_used are in use,
 * tile_first[t] (host pointer, n_used entries, may be NULL) = (first tile of t's expert) << 16 | tiles of that
 * expert; 2: per-expert weight gradients, n_groups experts of tiles_m x tiles_n tiles each, n_used != 0: the placement
 * taken while the routing is even (two XCDs share an expert), n_used == 0: the plain walk over all tiles.  Returns the
 * number of workgroups in the grid, or REVFFN_EINVAL (bad arguments, or more workgroups than max_wg). */
int revffn_op_tile_placement(int32_t group_mode, int32_t tiles_m, int32_t tiles_n, int32_t bm, int32_t bn,
                             int32_t n_groups, const int32_t *tile_first, int32_t n_used, int32_t *out,
                             int32_t max_wg);

/* Per-kernel timing for measurement (off by default).  While enabled, every GEMM and
 * attention launch of this context is bracketed by two HIP events recorded on the launch
 * stream, together with its algorithmic work: GEMM 2*M*N*K flops and each operand and the
 * result moved once; attention core 4*B*S*S*d flops forward, 10*B*S*S*d backward, halved
 * under the causal mask.  enable(on) also discards earlier records.  read() blocks the
 * host until the recorded events have completed and returns the sums over all launches of
 * kernel `kid` since enable: elapsed milliseconds, launch count, flops, bytes (any output
 * may be NULL).  kernel_name(kid) is the kernel family the id stands for, NULL past the
 * last id.  Families: the matrix-core GEMM by operand layout ("gemm_mfma_nt" / "_nn" / "_tn"),
 * the same three over per-expert weights ("..._experts": tile lists or per-expert row
 * ranges, each expert's weights moved once), the generic GEMM, and the attention kernels. */
int revffn_profile_enable(revffn_ctx *ctx, int32_t on);
int revffn_profile_read(revffn_ctx *ctx, int32_t kid, double *ms_total, int64_t *launches,
                        double *flops, double *bytes);
const char *revffn_profile_kernel_name(int32_t kid);

const char *revffn_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* REVFFN_H */

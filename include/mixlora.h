/*
 * mixlora.h - C ABI of the MI355X (gfx950) MixLoRA feed-forward block.
 *
 * The block replaces the dense FFN of a LLaMA-style layer (Eq. 5) by N LoRA experts that
 * all sit on one frozen SwiGLU FFN (Eq. 6, Section 3.3) behind a top-k softmax router
 * (Eq. 7, renormalised as in Algorithm 1) with the auxiliary load-balance loss of Eq. 8-9.
 * The frozen gate/up projections are computed once per token and shared by the experts
 * (Section 3.3, "Reducing the Computational Complexity (I)"; Algorithm 1).
 *
 * Notation: T tokens, d model width, f = d_ff, N experts, k kept experts per token,
 * r LoRA rank, s = lora_scale = alpha / r.  A "pair" is (token t, slot j < k).
 *
 * General rules for every entry point
 *   - Every data pointer is a DEVICE pointer (HIP, one GPU), row-major, 16-byte aligned,
 *     owned by the caller and not retained after the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     enqueued on it; no entry point allocates, frees or synchronises (the measurement aids at
 *     the end of this file excepted: they are not part of the block's contract).
 *   - Stream capture: the first launch of a kernel that needs more than 64 KiB of LDS sets a
 *     function attribute (hipFuncSetAttribute), once per process and kernel instance, which is
 *     not a stream operation.  Call every entry point once eagerly with the dims that will be
 *     captured before capturing it into a HIP graph; from then on its calls enqueue kernels only.
 *   - The return value is a mixlora_status.  Argument errors are detected on the host before
 *     any HIP call is made and leave all buffers untouched.  No C++ exception crosses the ABI.
 *   - Storage dtype (dims.dtype) applies to x, y, dy, dx and all weight matrices; routing
 *     weights, probabilities, losses and all returned LoRA/router gradients are float32.
 *     All accumulation is float32.
 *   - Limits: 1 <= k <= N <= 64; 1 <= r <= 64; N * (r rounded up to a multiple of 8) <= 512;
 *     d % 8 == 0; d_ff % 8 == 0; T >= 1; T*k < 2^24.  Anything else returns MIXLORA_E_SHAPE.
 *     A rank that is not a multiple of 8 (the rank study of Section 4.3 goes down to r = 2) runs
 *     on zero-padded copies of the six LoRA banks kept in the workspace; the bank and gradient
 *     arrays the caller passes keep their [N, r, .] / [N, ., r] shapes.
 */
#ifndef MIXLORA_H
#define MIXLORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define MIXLORA_API __attribute__((visibility("default")))
#else
#define MIXLORA_API
#endif

typedef enum {
  MIXLORA_OK = 0,
  MIXLORA_E_NULL = -1,      /* a required pointer is NULL                              */
  MIXLORA_E_SHAPE = -2,     /* a dimension is outside the limits above                 */
  MIXLORA_E_DTYPE = -3,     /* unknown dtype or aux_mode value                         */
  MIXLORA_E_ALIGN = -4,     /* a pointer is not 16-byte aligned                        */
  MIXLORA_E_WORKSPACE = -5, /* workspace_bytes < mixlora_workspace_bytes(...)          */
  MIXLORA_E_HIP = -6,       /* a kernel launch failed (hipGetLastError after enqueue)  */
  MIXLORA_E_SCRATCH = -7    /* the problem needs more scratch than the library's static
                               device buffer holds (mixlora_ffn_forward_static only)    */
} mixlora_status;

typedef enum { MIXLORA_F32 = 0, MIXLORA_BF16 = 1 } mixlora_dtype;

/* How F_i of Eq. 9 counts "tokens dispatched to expert i" when k > 1:
 * TOP1 = as printed (the arg-max expert only); TOPK = all k kept experts, divided by k. */
typedef enum { MIXLORA_AUX_TOP1 = 0, MIXLORA_AUX_TOPK = 1 } mixlora_aux_mode;

typedef struct {
  int32_t T, d, d_ff, N, k, r;
  float lora_scale; /* s = alpha / r (hyper-parameter table: alpha 32, r 16)           */
  float aux_coeff;  /* a of Eq. 8 (paper: 1e-2)                                        */
  int32_t aux_mode; /* mixlora_aux_mode                                                */
  int32_t dtype;    /* mixlora_dtype                                                   */
} mixlora_dims;

/* Weights, all in the storage dtype.  Frozen: W_gate, W_up, W_down (W1, W3, W2 of
 * Section 3.3).  Trainable: the LoRA banks (Eq. 1: W' = W + s B A) and the router (Eq. 7). */
typedef struct {
  const void *W_gate;   /* [f, d]                                                      */
  const void *W_up;     /* [f, d]                                                      */
  const void *W_down;   /* [d, f]                                                      */
  const void *A_gate;   /* [N, r, d]                                                   */
  const void *B_gate;   /* [N, f, r]                                                   */
  const void *A_up;     /* [N, r, d]                                                   */
  const void *B_up;     /* [N, f, r]                                                   */
  const void *A_down;   /* [N, r, f]                                                   */
  const void *B_down;   /* [N, d, r]                                                   */
  const void *W_router; /* [N, d], no bias                                             */
  /* Optional transposed copies of the frozen matrices, used by the backward pass only
   * (W_gate_T, W_up_T: [d, f]; W_down_T: [f, d]); make them once with
   * mixlora_transpose.  Where one is NULL, backward transposes that matrix into its
   * workspace on every call.                                                          */
  const void *W_gate_T;
  const void *W_up_T;
  const void *W_down_T;
} mixlora_weights;

/* Gradients of the trainable tensors: float32, same shapes as the tensors, OVERWRITTEN
 * (not accumulated).  Experts that received no token get exact zeros.                  */
typedef struct {
  float *dA_gate, *dB_gate, *dA_up, *dB_up, *dA_down, *dB_down, *dW_router;
} mixlora_grads;

/* Bytes of workspace the forward (for_backward = 0) or forward+backward (1) needs for
 * these dims; 0 if the dims are invalid.  Host-only, no HIP call. */
MIXLORA_API size_t mixlora_workspace_bytes(const mixlora_dims *dims, int for_backward);

/* Forward of the block (Eq. 6 with SwiGLU experts, Eq. 7, Algorithm 1 lines 4-15, Eq. 8-9):
 *   y[t] = sum_j topk_w[t,j] * E_{topk_idx[t,j]}(x[t]),  without the residual add of Eq. 5.
 * in : x [T,d] (storage dtype)
 * out: y [T,d] (storage dtype); topk_idx [T,k] int32, slots by descending logit, equal
 *      logits to the lower expert index; topk_w [T,k] float32 (sums to 1 per token);
 *      expert_counts [N] int32 = number of pairs routed to each expert;
 *      aux_loss [1] float32 (device) = Eq. 8 with dims.aux_coeff / dims.aux_mode.
 * workspace: scratch, and the activations the backward needs; pass the same buffer,
 *      untouched, to mixlora_ffn_backward.  Calls sharing a workspace must not overlap. */
MIXLORA_API int mixlora_ffn_forward(const mixlora_dims *dims, const mixlora_weights *w, const void *x,
                        void *y, int32_t *topk_idx, float *topk_w, int32_t *expert_counts,
                        float *aux_loss, void *workspace, size_t workspace_bytes,
                        void *stream);

/* The same forward for callers that cannot allocate or hand over device memory of their own:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Every
 * buffer that mixlora_ffn_forward takes from the caller's workspace (routing tables, grouped
 * activations, partial results of the split down projection, ...) lives instead in a device
 * array inside the library, MIXLORA_STATIC_SCRATCH_BYTES large, one copy per GPU, held until the
 * process ends.  The call allocates nothing and frees nothing; inputs and outputs are the
 * caller's as before, results are bit-identical to mixlora_ffn_forward.  Forward only: the
 * array is not a handle for mixlora_ffn_backward.
 *   - dims whose mixlora_workspace_bytes(dims, 0) exceeds MIXLORA_STATIC_SCRATCH_BYTES return
 *     MIXLORA_E_SCRATCH (checked on the host, nothing enqueued).  40 MiB covers the LLaMA-2 7B /
 *     13B and LLaMA-3 8B shapes of this block up to 128 tokens per call (decode batches).
 *   - All calls on one GPU share that GPU's array and it keeps the previous call's contents; the
 *     call itself clears what has to start at zero.  Calls that overlap on one GPU (two streams,
 *     two threads) race: serialise them.
 *   - The first call on each device looks the array's device address up (hipGetSymbolAddress) and
 *     must therefore be made outside stream capture; later calls may be captured.           */
#define MIXLORA_STATIC_SCRATCH_BYTES (40 * 1024 * 1024)
MIXLORA_API int mixlora_ffn_forward_static(const mixlora_dims *dims, const mixlora_weights *w,
                                           const void *x, void *y, int32_t *topk_idx,
                                           float *topk_w, int32_t *expert_counts, float *aux_loss,
                                           void *stream);

/* Backward of the same block for the loss  <y, dy> + d_aux * aux_loss, base matrices frozen
 * (derived from Algorithm 1 lines 4-15; the paper leaves it to autograd).
 * in : x, dy [T,d]; workspace as left by mixlora_ffn_forward for the same dims/weights/x
 *      (its size must be the for_backward = 1 size).
 * out: dx [T,d] (storage dtype, includes the paths through the router and the auxiliary
 *      loss); grads (all seven required).                                               */
MIXLORA_API int mixlora_ffn_backward(const mixlora_dims *dims, const mixlora_weights *w, const void *x,
                         const void *dy, float d_aux, void *workspace,
                         size_t workspace_bytes, void *dx, const mixlora_grads *grads,
                         void *stream);

/* ---- The paper's own execution schedules of the same block (Section 3.3, "Reducing the
 * Computational Complexity (I)", Figure 3), for measured comparison -----------------------------
 * All three compute the same function; they differ in how often the frozen matrices are applied.
 * With "unit" = one frozen d x d_ff product over T rows:
 *   MIXLORA_SCHEDULE_LINEAR_DOWN  what mixlora_ffn_forward/backward run: gate and up once per
 *       token (2 units), the pairs' activations combined with the routing weights in front of ONE
 *       frozen down product (1 unit; W_down acts linearly on the weighted sum), LoRA terms rank-r.
 *   MIXLORA_SCHEDULE_SHARED       Figure 3(b): gate and up once per token (2 units), the down
 *       projection on every routed (token, expert) pair row (k units), combined afterwards.
 *   MIXLORA_SCHEDULE_VANILLA      Figure 3(a): every expert applies gate, up and down to its own
 *       slice of token rows (3k units).
 * The backward pass mirrors the forward count (per-pair rows wherever the forward used them).
 * SHARED and VANILLA exist for bf16 only (MIXLORA_E_DTYPE otherwise), need the larger workspace
 * reported below, and the backward call must use the schedule of the forward call that filled
 * the workspace.  Other arguments, outputs and errors as in mixlora_ffn_forward / _backward;
 * an unknown schedule gives MIXLORA_E_SHAPE.                                                   */
typedef enum {
  MIXLORA_SCHEDULE_LINEAR_DOWN = 0,
  MIXLORA_SCHEDULE_SHARED = 1,
  MIXLORA_SCHEDULE_VANILLA = 2
} mixlora_schedule;

/* Workspace bytes for the given schedule (0 for invalid dims / schedule / dtype). */
MIXLORA_API size_t mixlora_schedule_workspace_bytes(const mixlora_dims *dims, int32_t schedule,
                                                    int for_backward);
MIXLORA_API int mixlora_ffn_forward_schedule(const mixlora_dims *dims, int32_t schedule,
                                 const mixlora_weights *w, const void *x, void *y,
                                 int32_t *topk_idx, float *topk_w, int32_t *expert_counts,
                                 float *aux_loss, void *workspace, size_t workspace_bytes,
                                 void *stream);
MIXLORA_API int mixlora_ffn_backward_schedule(const mixlora_dims *dims, int32_t schedule,
                                  const mixlora_weights *w, const void *x, const void *dy,
                                  float d_aux, void *workspace, size_t workspace_bytes, void *dx,
                                  const mixlora_grads *grads, void *stream);

/* ---- Weight-decomposed experts (the variant the experiments call MixDoRA, Section 4.1) ---------
 * The paper prints no formula for it; this library's reading applies the cited weight-
 * decomposition method to every expert projection P in {gate, up, down} of expert e:
 *     P'_e = diag(m_e / n_e) (W + s B_e A_e),   n_e[j] = || (W + s B_e A_e)[j, :] ||_2 ,
 * with a trainable magnitude m_e per output feature; n_e is recomputed in every forward call and
 * treated as a constant by the backward pass (no gradient through the norm), as that method does.
 * With m_e = n_e the block equals the plain MixLoRA block.
 *   m_gate, m_up [N, d_ff], m_down [N, d]: device float32, 16-byte aligned.
 *   dm_*: gradients of the magnitudes, same shapes, float32, overwritten.
 * shared != 0 selects the other reading the paper's tables allow (the "# Params" columns of
 * the rank study, Section 4.3, and of the main results are the same for MixLoRA and MixDoRA,
 * which a magnitude per expert would raise by 0.10 points on LLaMA-2 7B and one per projection
 * by 0.02): ONE magnitude vector per projection used by every expert, m_e = m.  Then m_gate,
 * m_up are [d_ff], m_down is [d], and dm_* have those shapes and hold the sum over the experts
 * (added in ascending expert order).  shared must be 0 or 1 (MIXLORA_E_SHAPE otherwise).
 * bf16 storage only (MIXLORA_E_DTYPE otherwise).  The frozen gate / up products stay shared
 * across experts; the down projection runs per routed pair (its factor depends on the expert).
 * Other arguments, outputs, workspace rules and errors as in mixlora_ffn_forward / _backward;
 * the backward call needs the workspace of a mixlora_dora_forward call with the same inputs.  */
typedef struct {
  const float *m_gate, *m_up, *m_down;
  int32_t shared;
} mixlora_dora;
typedef struct {
  float *dm_gate, *dm_up, *dm_down;
} mixlora_dora_grads;

MIXLORA_API size_t mixlora_dora_workspace_bytes(const mixlora_dims *dims, int for_backward);
MIXLORA_API int mixlora_dora_forward(const mixlora_dims *dims, const mixlora_weights *w,
                         const mixlora_dora *dora, const void *x, void *y, int32_t *topk_idx,
                         float *topk_w, int32_t *expert_counts, float *aux_loss, void *workspace,
                         size_t workspace_bytes, void *stream);
MIXLORA_API int mixlora_dora_backward(const mixlora_dims *dims, const mixlora_weights *w,
                          const mixlora_dora *dora, const void *x, const void *dy, float d_aux,
                          void *workspace, size_t workspace_bytes, void *dx,
                          const mixlora_grads *grads, const mixlora_dora_grads *dora_grads,
                          void *stream);

/* ---- Several adapters on one frozen base (Section 3.3, "Optimizing Multi-MixLoRA Training and
 * Inference (II)"; outer loop of Algorithm 1) -------------------------------------------------
 * M MixLoRA adapters, each with its own router and N LoRA experts, share W_gate / W_up / W_down.
 * Every token belongs to one adapter and is routed and processed by that adapter only; the shared
 * projections run once over the tokens of all adapters.
 *   dims->N is the number of experts PER ADAPTER (k <= N); M*N <= 64 and M*N*r <= 512.
 *   The LoRA banks, the router and their gradients hold M*N experts, adapter m's expert e at
 *   index m*N + e: A_gate [M*N,r,d], ..., W_router [M*N,d].
 *   token_model: device int32 [T], adapter of every token, values in [0, M) (not checked on the
 *   device: out-of-range values are undefined behaviour).
 *   d_aux: HOST float [M], upstream gradient of each adapter's auxiliary loss (backward only;
 *   NULL = all 1).  Read during the call, not retained. */
typedef struct {
  int32_t M;
  const int32_t *token_model;
  const float *d_aux;
} mixlora_multi;

/* Workspace bytes of the multi-adapter calls (0 for invalid dims or M). */
MIXLORA_API size_t mixlora_multi_workspace_bytes(const mixlora_dims *dims, int32_t M,
                                                 int for_backward);

/* As mixlora_ffn_forward, with: topk_idx [T,k] = expert index inside the token's adapter;
 * expert_counts [M*N] (pairs per expert of every adapter); aux_loss [M] (Eq. 8-9 per adapter,
 * over the adapter's own tokens; 0 for an adapter without tokens).  Errors as
 * mixlora_ffn_forward; MIXLORA_E_SHAPE also for M < 1 or M*N > 64. */
MIXLORA_API int mixlora_multi_forward(const mixlora_dims *dims, const mixlora_multi *multi,
                                      const mixlora_weights *w, const void *x, void *y,
                                      int32_t *topk_idx, float *topk_w, int32_t *expert_counts,
                                      float *aux_loss, void *workspace, size_t workspace_bytes,
                                      void *stream);

/* As mixlora_ffn_backward on the workspace mixlora_multi_forward filled; gradients of
 * <y, dy> + sum_m d_aux[m] * aux_loss[m].  An adapter without tokens gets zero gradients. */
MIXLORA_API int mixlora_multi_backward(const mixlora_dims *dims, const mixlora_multi *multi,
                                       const mixlora_weights *w, const void *x, const void *dy,
                                       void *workspace, size_t workspace_bytes, void *dx,
                                       const mixlora_grads *grads, void *stream);

/* Auxiliary load-balance loss alone (Eq. 8-9) from router probabilities and kept experts.
 * in : probs [T,N] float32 (full softmax), topk_idx [T,k] int32.
 * out: loss [1]; F [N], P [N] (each may be NULL); dprobs [T,N] = d loss / d probs (may be
 *      NULL; F is piecewise constant, so only P carries gradient).  All float32, device. */
MIXLORA_API int mixlora_aux_loss(const float *probs, const int32_t *topk_idx, int32_t T, int32_t N,
                     int32_t k, float coeff, int32_t mode, float *loss, float *F, float *P,
                     float *dprobs, void *stream);

/* out[cols, rows] = in[rows, cols]^T in the given dtype; for preparing the optional
 * transposed frozen copies.  rows, cols >= 1. */
MIXLORA_API int mixlora_transpose(const void *in, void *out, int32_t rows, int32_t cols, int32_t dtype,
                      void *stream);

/* Measurement hook for benchmarks.  These three and mixlora_mfma_probe are measurement aids, not
 * part of the block's contract: they are the only entry points that synchronise or create HIP
 * objects.  Between begin and end, every launch of the library is bracketed by HIP events on its
 * stream (at most max_launches of them; later launches go untimed).  end waits for those events
 * and returns, in HOST memory, the summed time in milliseconds, the number of launches and the
 * floating-point operations (2*M*N*K over their K segments) of the bf16 MFMA GEMM launches that
 * carry the frozen projections.  After end, mixlora_profile_kind returns the same three figures
 * for one kind of launch, with work in algorithmic bytes for the bandwidth-bound kinds:
 *   0 frozen-projection GEMMs (work = FLOPs), 1 per-pair SwiGLU stage forward, 2 the same
 *   backward, 3 sums over a token's pair rows, 4 grouped outer-product sums (LoRA / router
 *   gradients), 5 routing (softmax, top-k, grouping, auxiliary loss, router backward),
 *   6 re-layouts and other small launches.  Unknown kind: MIXLORA_E_SHAPE.  Not thread-safe. */
MIXLORA_API int mixlora_profile_begin(int32_t max_launches);
MIXLORA_API int mixlora_profile_end(double *ms_total, int32_t *launches, double *flops_total);
MIXLORA_API int mixlora_profile_kind(int32_t kind, double *ms_total, int32_t *launches,
                                     double *work_total);

/* ---- Plain LoRA linear (Eq. 1 with the scale alpha / r; the form the method puts on the
 * attention projections, Section 3.2):  y = x W^T + s (x A^T) B^T,  W frozen ----------------
 * Shapes (row-major, dtype = dims.dtype, device pointers, 16-byte aligned):
 *   x [T, d_in], W [d_out, d_in], A [r, d_in], B [d_out, r], y / dy [T, d_out], dx [T, d_in];
 *   dA [r, d_in], dB [d_out, r] float32, overwritten.
 * Limits: 1 <= r <= 64 (ranks off the multiples of 8 run on zero-padded copies of A and B kept
 * in the workspace), d_in % 8 == 0, d_out % 8 == 0, T < 2^24.
 * The workspace is the caller's; forward saves x A^T in it for the backward. */
typedef struct {
  int32_t T, d_in, d_out, r;
  float lora_scale;
  int32_t dtype;
} mixlora_linear_dims;

/* Bytes of workspace (0 for invalid dims). */
MIXLORA_API size_t mixlora_lora_linear_workspace_bytes(const mixlora_linear_dims *dims,
                                                       int for_backward);

/* y = x W^T + s (x A^T) B^T.  Errors: E_NULL, E_SHAPE, E_DTYPE, E_ALIGN, E_WORKSPACE, E_HIP. */
MIXLORA_API int mixlora_lora_linear_forward(const mixlora_linear_dims *dims, const void *W,
                                            const void *A, const void *B, const void *x, void *y,
                                            void *workspace, size_t workspace_bytes, void *stream);

/* Gradients of <y, dy> on the workspace the forward filled: dx = dy W + s (dy B) A,
 * dA = s (dy B)^T x, dB = s dy^T (x A^T).  W_T [d_in, d_out] is an optional pre-transposed copy
 * of W (mixlora_transpose); when NULL the transpose is made per call inside the workspace. */
MIXLORA_API int mixlora_lora_linear_backward(const mixlora_linear_dims *dims, const void *W,
                                             const void *W_T, const void *A, const void *B,
                                             const void *x, const void *dy, void *workspace,
                                             size_t workspace_bytes, void *dx, float *dA,
                                             float *dB, void *stream);

/* ---- AdamW step on adapter parameters (the optimiser named in the paper's hyper-parameter
 * table; decoupled weight decay):
 *   p <- p (1 - lr wd);  m <- b1 m + (1-b1) g;  v <- b2 v + (1-b2) g^2;
 *   p <- p - lr (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps)
 * param, grad, m, v: device float32 [n] (param, m, v updated in place); lowp: optional device
 * copy of the parameters in lowp_dtype (bf16 or f32), refreshed from the new values, or NULL.
 * step t is 1-based.  Errors: E_NULL, E_DTYPE, E_SHAPE (n < 1, step < 1, betas outside [0,1),
 * eps <= 0), E_HIP. */
typedef struct {
  float lr, beta1, beta2, eps, weight_decay;
  int32_t step;
} mixlora_adamw;
MIXLORA_API int mixlora_adamw_step(const mixlora_adamw *h, int64_t n, float *param,
                                   const float *grad, float *m, float *v, void *lowp,
                                   int32_t lowp_dtype, void *stream);

/* Measurement aid: TFLOP/s that a register-only loop of bf16 MFMA 32x32x16 on pseudo-random
 * operands sustains on the current device at waves_per_simd (1 or 2) wavefronts per SIMD - the
 * practical ceiling of the matrix pipe on a power-limited part, beside the published peak.
 * sink: device scratch of at least 2 * (number of CUs) * 1024 bytes (overwritten).
 * Creates two HIP events and WAITS for the kernel (unlike every other call here).
 * Errors: E_NULL, E_SHAPE (waves_per_simd, iters out of range), E_WORKSPACE (sink too small),
 * E_HIP. */
MIXLORA_API int mixlora_mfma_probe(void *sink, size_t sink_bytes, int32_t waves_per_simd,
                                   int32_t iters, double *tflops, void *stream);

/* Library version as major*10000 + minor*100 + patch.  Host-only. */
MIXLORA_API int mixlora_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MIXLORA_H */

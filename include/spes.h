/*
 * spes.h -- C ABI of the SPES MoE-layer hot path for AMD MI355X (gfx950).
 *
 * One node of SPES-style decentralised MoE pretraining stores every expert of a
 * routed feed-forward layer but trains only its assigned subset (paper Sec. 3.3,
 * "Expert Assignment and Local Training", Eq. 3).  This library is that node's
 * training step through one such layer, plus the periodic synchronisation of
 * node-local expert copies (Sec. 3.3 "Sparse Synchronization", Eq. 4) and the
 * expert-merging warm-up (Sec. 3.3 "Expert-Merging Warm-Up", Eq. 5-6).
 *
 * Conventions that hold for every entry point
 *  - Plain C linkage, plain pointers and sizes.  "DEVICE" pointers address GPU
 *    memory of the current HIP device, "HOST" pointers ordinary host memory.
 *  - The library allocates no device memory and the entry points declared here keep
 *    no state between calls.  Inputs, outputs, the context buffer and scratch are
 *    owned by the caller.  (The benchmark aids of spes_bench.h are the exception:
 *    they hold a process-wide set of timing events.)
 *  - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *    the default stream).  No entry point synchronises or copies device memory
 *    back to the host; per-expert token counts are consumed on the device.
 *  - HOST arrays are read before the call returns and may be freed afterwards.
 *  - Return value: SPES_OK (0) or a negative spes_status.  Arguments are checked
 *    before anything is launched, so a failed check has no side effects.
 *  - Tensors are row-major with the innermost dimension contiguous.  Weight
 *    matrices are stored [out_features, in_features].  DEVICE pointers must be
 *    16-byte aligned.  Outputs must not alias inputs.
 *  - dtype selects the storage type of parameters and activations (fp32, or
 *    bf16 with round-to-nearest-even on every store); every accumulation is fp32.
 *    Router logits, gates and all weight gradients are fp32 in both modes.
 */
#ifndef SPES_H_
#define SPES_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPES_API __attribute__((visibility("default")))

typedef enum {
  SPES_OK = 0,
  SPES_EINVAL = -1, /* null pointer, non-positive size, top_k > n_experts, bad dtype   */
  SPES_ESHAPE = -2, /* a size this build does not support (see each call)              */
  SPES_EALIGN = -3, /* a DEVICE pointer is not 16-byte aligned                         */
  SPES_EHIP = -4    /* a kernel launch failed; see hipGetLastError                     */
} spes_status;

typedef enum { SPES_F32 = 0, SPES_BF16 = 1 } spes_dtype;

/* Shape of one routed feed-forward layer (Sec. 3.1 Eq. 2; Sec. 3.2).
 * Supported: 1 <= top_k <= n_experts <= 64; d_model and d_ff multiples of 8;
 * T*top_k at most 2^22 - 4224; in bf16 storage T*d_model, T*top_k*d_ff and
 * n_experts*d_ff*d_model each below 2^31 (SPES_ESHAPE otherwise). */
typedef struct {
  int32_t T;           /* tokens in the batch                                         */
  int32_t d_model;     /* d                                                           */
  int32_t n_experts;   /* M                                                           */
  int32_t d_ff;        /* f, hidden width of one SwiGLU expert                        */
  int32_t top_k;       /* k experts per token                                         */
  int32_t dtype;       /* spes_dtype                                                  */
  int32_t renorm_topk; /* 1: gates are renormalised over the k chosen (Sec. 4,
                          upcycled model); 0: gate = softmax probability over all M   */
} spes_moe_shape;

/* Byte offsets of the regions inside the context buffer; exposed so that tests
 * can inspect routing tables and saved activations.  R = T*top_k routed rows. */
typedef struct {
  size_t total;
  size_t logits;    /* [T,M] f32 router scores                                        */
  size_t lse;       /* [T] f32 log-sum-exp of the scores                              */
  size_t topk_idx;  /* [T,k] i32 copy of the selected experts                          */
  size_t topk_gate; /* [T,k] f32 copy of their gates                                  */
  size_t offset;    /* [M+1] i32 first row of each expert in expert-contiguous order  */
  size_t perm;      /* [R] i32 row r holds routed pair perm[r] = t*k+j                */
  size_t inv;       /* [R] i32 inverse of perm                                        */
  size_t a;         /* [R,f] gate projection  W_g x, in the storage type               */
  size_t b;         /* [R,f] up projection    W_u x, in the storage type               */
  size_t h;         /* [R,f] SiLU(a)*b                                                */
  size_t yp;        /* [R,d] expert outputs before gating                             */
  size_t dlogits;   /* [T,M] f32, written by the backward                             */
  size_t dgate;     /* [T,k] f32, written by the backward                             */
} spes_moe_ctx_layout;

/* Size and layout of the context buffer that spes_moe_fwd fills and spes_moe_bwd
 * consumes (it also holds the backward's scratch).  Returns 0 on a bad shape. */
SPES_API size_t spes_moe_ctx_bytes(const spes_moe_shape* shape);
SPES_API int spes_moe_ctx_describe(const spes_moe_shape* shape, spes_moe_ctx_layout* out);

/* Forward of the routed SwiGLU layer: y_t = sum_j G_j(x_t) E_j(x_t) (Sec. 3.1 Eq. 2)
 * with softmax routing over all M experts followed by top-k selection, drop-less
 * dispatch (every selected pair is computed; Sec. 3.2) and SwiGLU experts
 * E(x) = W_d (SiLU(W_g x) * W_u x).
 *
 *  x            DEVICE [T,d]      w_router DEVICE [M,d]
 *  router_bias  DEVICE [M] f32 or NULL (added to the scores; receives no gradient)
 *  w_gate,w_up  DEVICE [M,f,d]    w_down   DEVICE [M,d,f]
 *  y            DEVICE [T,d] out
 *  topk_idx     DEVICE [T,k] i32 out: selected experts in descending score order,
 *               equal scores resolved to the lower expert id
 *  topk_gate    DEVICE [T,k] f32 out
 *  expert_count DEVICE [M] i32 out: routed pairs per expert (sums to T*k)
 *  ctx          DEVICE, spes_moe_ctx_bytes(shape) bytes, 256-byte aligned
 */
SPES_API int spes_moe_fwd(const spes_moe_shape* shape, const void* x, const void* w_router,
                          const float* router_bias, const void* w_gate, const void* w_up,
                          const void* w_down, void* y, int32_t* topk_idx, float* topk_gate,
                          int32_t* expert_count, void* ctx, void* stream);

/* The permuted copy of the input that drop-less dispatch defines (Sec. 3.2): row r of xp is
 * the input row of the routed pair that the forward placed at position r of the
 * expert-contiguous order, xp[inv[t*k+j], :] = x[t, :].  spes_moe_fwd and spes_moe_bwd do not
 * need it (their grouped GEMMs read x through the same table); this entry point materialises
 * it for callers that want the dispatched activations, and is the stand-alone form of the
 * dispatch step.
 *
 *  x    DEVICE [T,d]       ctx  DEVICE, as left by spes_moe_fwd for this shape
 *  xp   DEVICE [T*k,d] out, must not alias x
 */
SPES_API int spes_moe_permute(const spes_moe_shape* shape, const void* x, const void* ctx, void* xp,
                              void* stream);

/* Backward of the weighted combine of Eq. 2 as a stand-alone step: for the k routed pairs of
 * every token,  dyp[inv[t*k+j], :] = gate[t,j] * dy[t, :]  (the upstream gradient of each routed
 * row, in expert-contiguous order) and  dgate[t,j] = <dy[t, :], yp[inv[t*k+j], :]>  with yp the
 * expert outputs the last spes_moe_fwd left in ctx.  spes_moe_bwd does not run this kernel: it
 * gathers and scales the dy rows inside its first GEMM and takes the gate gradient from that
 * GEMM's accumulators (yp is stored in the storage type; in bf16 that rounding is too coarse for
 * the router gradient of near-identical experts).  This entry point materialises the step as the
 * chain rule states it.
 *
 *  dy     DEVICE [T,d]                 ctx    DEVICE, as left by spes_moe_fwd for this shape
 *  dyp    DEVICE [T*k, d] out          dgate  DEVICE [T,k] f32 out
 */
SPES_API int spes_moe_grad_scatter(const spes_moe_shape* shape, const void* dy, const void* ctx,
                                   void* dyp, float* dgate, void* stream);

/* Backward of the same layer for upstream gradient dy.  The selected expert set
 * is treated as constant.  The input gradient flows through every routed expert,
 * trainable or frozen; weight gradients are produced only for experts whose mask
 * byte is non-zero (Sec. 3.3 Eq. 3; App. A, block mask U_i), into compact
 * buffers with one slot per trainable expert in ascending expert id, so frozen
 * experts own no gradient memory.  The router belongs to the shared modules that
 * every node trains, so d_w_router is always produced.
 *
 *  dy, x          DEVICE [T,d]; weights as in the forward, ctx as left by it
 *  trainable_mask HOST  [M] bytes
 *  dx             DEVICE [T,d] out
 *  d_w_router     DEVICE [M,d] f32
 *  d_w_gate,d_w_up DEVICE [n_trainable,f,d] f32;  d_w_down DEVICE [n_trainable,d,f] f32
 *                 (may be NULL when no expert is trainable)
 *  accumulate     0: weight gradients are overwritten; 1: added to (micro-batches)
 */
SPES_API int spes_moe_bwd(const spes_moe_shape* shape, const void* dy, const void* x,
                          const void* w_router, const void* w_gate, const void* w_up,
                          const void* w_down, void* ctx, const uint8_t* trainable_mask, void* dx,
                          float* d_w_router, float* d_w_gate, float* d_w_up, float* d_w_down,
                          int32_t accumulate, void* stream);

/* Auxiliary router losses (Sec. 3.3 "Training Losses"; coefficients App. B: load-balancing
 * 0.01, router z-loss 0.001).  The paper names the two losses and cites their sources; the
 * formulas used are the cited ones:
 *      L_lb = M * sum_e f_e * P_e     f_e = share of the T*k routed pairs sent to expert e,
 *                                     P_e = mean over tokens of the softmax probability of e
 *      L_z  = mean over tokens of (log sum_e exp(score_te))^2
 * on the scores (router bias included) of the forward pass whose record is in ctx.
 * Call it after spes_moe_fwd and before spes_moe_bwd on the same ctx.  It writes the two loss
 * values and arms ctx so that the next spes_moe_bwd adds
 *      grad_scale * (lb_coef * dL_lb/dscores + z_coef * dL_z/dscores)
 * to the gating gradient before it reaches d_w_router and dx (f_e is a count and carries no
 * gradient).  grad_scale is whatever factor the caller's total loss applies to this layer's
 * auxiliary terms (1 for a plain sum, 1/n for n micro-batches, a loss scale).  The next
 * spes_moe_fwd on the ctx disarms it; without this call spes_moe_bwd is unchanged.
 *
 *  ctx     DEVICE, as left by spes_moe_fwd for this shape
 *  losses  DEVICE [2] f32 out: L_lb, L_z (unweighted)
 */
SPES_API int spes_moe_router_aux(const spes_moe_shape* shape, void* ctx, float lb_coef,
                                 float z_coef, float grad_scale, float* losses, void* stream);

/* AdamW step on the trainable subset of one parameter matrix of the expert store.  A node keeps
 * gradients and the two optimizer moments only for its assigned experts and for the shared
 * parameters (Sec. 3.3 "Efficiency Analysis", the 3 x |Phi_i| term of the memory model), so all
 * optimizer state is compact: one slot per expert whose mask byte is non-zero, in ascending expert
 * id, exactly like the gradient buffers of spes_moe_bwd.  Per element, with g = grad_scale * grad,
 *      m <- beta1 m + (1-beta1) g          v <- beta2 v + (1-beta2) g^2
 *      w <- w - lr ( (m / (1-beta1^step)) / (sqrt(v / (1-beta2^step)) + eps) + weight_decay w )
 * in fp32 (Table A1: beta 0.9 / 0.95, eps 1e-8, weight decay 0.1), then the expert's row of the
 * full store is overwritten with w rounded to the storage type.  Frozen experts are not touched.
 * A shared matrix such as the router is the case n_experts = 1, mask = {1}.
 *
 *  n_experts >= 1; elems = elements of the matrix per expert, a multiple of 8
 *  param        DEVICE [n_experts, elems] storage dtype, in/out
 *  trainable_mask HOST [n_experts] bytes
 *  master       DEVICE [n_trainable, elems] f32 in/out: the fp32 weights; NULL is allowed for
 *               dtype f32 only, then param itself is the weight
 *  m, v         DEVICE [n_trainable, elems] f32 in/out
 *  grad         DEVICE [n_trainable, elems] f32
 *  step         >= 1, the number of this update (bias correction)
 */
SPES_API int spes_masked_adamw(int32_t n_experts, int64_t elems, int32_t dtype, void* param,
                               const uint8_t* trainable_mask, float* master, float* m, float* v,
                               const float* grad, float lr, float beta1, float beta2, float eps,
                               float weight_decay, int32_t step, float grad_scale, void* stream);

/* Upcycling initialiser (Sec. 4, upcycling settings: the dense FFN is replicated into the experts
 * and Gaussian noise of standard deviation 0.02 is added to 50 % of the parameters), for one
 * parameter matrix:  out[e][i] = dense[i] + select(e,i) * sigma * z(e,i),  rounded to the storage type.
 * The draws are a pure function of (seed, stream_id, e*elems + i): Philox-4x64-10 with key (seed, 0)
 * and counter (g, stream_id, 0, 0) yields words w_0..w_3 for the group g of four consecutive flat
 * indices; element j is selected iff (w_j & 255) < floor(fraction * 256); z of elements 2q, 2q+1 is
 * r cos(2 pi u2), r sin(2 pi u2) with r = sqrt(-2 ln u1), u1 = ((w_2q >> 40) + 0.5) / 2^24,
 * u2 = ((w_2q+1 >> 40) + 0.5) / 2^24.  Use a different stream_id per parameter matrix.
 *
 *  n_experts >= 1; elems a multiple of 8; 0 <= fraction <= 1; sigma >= 0
 *  dense  DEVICE [elems]            out  DEVICE [n_experts, elems]
 */
SPES_API int spes_upcycle_init(int32_t n_experts, int64_t elems, int32_t dtype, const void* dense,
                               float fraction, float sigma, uint64_t seed, uint64_t stream_id,
                               void* out, void* stream);

/* Gather (to_store = 0) or scatter (to_store = 1) of the rows of the experts whose mask byte is
 * non-zero between the full store and a contiguous buffer with one row per such expert in ascending
 * expert id: what a node uploads at a synchronisation is only what it trained (Sec. 3.3, Eq. 4),
 * and the buffer has the layout spes_expert_merge reads as a node store.
 *
 *  store   DEVICE [n_experts, elems]   packed  DEVICE [n_trainable, elems]   elems a multiple of 8
 *  trainable_mask HOST [n_experts] bytes
 */
SPES_API int spes_expert_pack(int32_t n_experts, int64_t elems, int32_t dtype, void* store,
                              const uint8_t* trainable_mask, void* packed, int32_t to_store,
                              void* stream);

/* Synchronisation of node-local expert copies (Sec. 3.3 Eq. 4; App. A sync rules),
 * for one parameter matrix of every expert.  Expert j becomes the weighted mean
 * of the copies held by the nodes that trained it,
 *      dst[j] = sum_i w_i * store_i[slot[i][j]] / sum_i w_i   over i with slot[i][j] >= 0,
 * which is FedAvg when all nodes train it with equal weights and a direct
 * (bit-exact) assignment when a single node does.  An expert nobody trained keeps
 * the value already in dst.
 *
 *  n_experts >= 1; elems = elements of the matrix per expert, a multiple of 8
 *  node_store   HOST  [n_nodes] DEVICE pointers; store i is [n_i, elems]
 *  slot         HOST  [n_nodes, n_experts] i32: row of expert j in store i, or -1
 *  node_weight  HOST  [n_nodes] f32 (> 0) or NULL for equal weights
 *  dst          DEVICE [n_experts, elems] in/out
 *  trainer_count DEVICE [n_experts] i32 out or NULL: number of trainers per expert
 *  At most 224 trainers per expert (SPES_ESHAPE beyond).
 */
SPES_API int spes_expert_merge(int32_t n_experts, int64_t elems, int32_t dtype, int32_t n_nodes,
                               const void* const* node_store, const int32_t* slot,
                               const float* node_weight, void* dst, int32_t* trainer_count,
                               void* stream);

/* Expert-merging warm-up (Sec. 3.3 Eq. 5-6; App. A merge step).  Cosine similarity
 * A[j][k] between the flattened input projections w_in[j], w_in[k]; Q_j = the top_K
 * most similar experts to j, j excluded, equal similarities resolved to the lower
 * id; then for each of the n_mats parameter matrices
 *      dst[m][j] = src[m][j] + (alpha/top_K) * sum_{k in Q_j} (src[m][k] - src[m][j]),
 * every right-hand side being the pre-merge value (out of place: dst[m] != src[m]).
 *
 *  1 <= top_K < n_experts <= 64
 *  w_in     DEVICE [M, elems_in], elems_in a multiple of 8
 *  src,dst  HOST arrays of n_mats DEVICE pointers, matrix m is [M, elems[m]]
 *  elems    HOST  [n_mats], each a multiple of 8
 *  sim      DEVICE [M,M] f32 out or NULL;  nbr DEVICE [M,top_K] i32 out
 *           (a pair with a zero-norm projection, for which Eq. 5 is 0/0, gets similarity 0;
 *           every entry of nbr is a valid expert other than the row's own, whatever w_in holds)
 *  scratch  DEVICE, spes_warmup_scratch_bytes(M, elems_in) bytes
 */
SPES_API size_t spes_warmup_scratch_bytes(int32_t n_experts, int64_t elems_in);
SPES_API int spes_expert_warmup_merge(int32_t n_experts, int32_t dtype, int32_t top_K, float alpha,
                                      const void* w_in, int64_t elems_in, int32_t n_mats,
                                      const void* const* src, void* const* dst,
                                      const int64_t* elems, float* sim, int32_t* nbr,
                                      void* scratch, void* stream);

/* spes_expert_warmup_merge for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same computation with the
 * same arguments, except that the Gram partial sums go to a buffer that is part of the library's
 * own device image (8 MiB, held by every GPU the library runs on until the process ends) instead
 * of a caller-provided scratch.  The call allocates and frees nothing.  That buffer covers every
 * supported problem (n_experts <= 64, at most 512 chunks of the contraction); a problem that
 * would need more is rejected with SPES_ESHAPE.  All calls on one GPU share the buffer: calls
 * that overlap in time on one GPU (different streams) race on it; calls on one stream are safe.
 * Nothing in it needs clearing between calls: every partial a call reads was written by that call.
 */
SPES_API int spes_expert_warmup_merge_static(int32_t n_experts, int32_t dtype, int32_t top_K,
                                             float alpha, const void* w_in, int64_t elems_in,
                                             int32_t n_mats, const void* const* src,
                                             void* const* dst, const int64_t* elems, float* sim,
                                             int32_t* nbr, void* stream);

SPES_API const char* spes_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* SPES_H_ */

/*
 * smoe.h -- C ABI of libsmoe: ScatterMoE's ParallelLinear hot path on AMD MI355X (gfx950).
 *
 * The operations are the ones the paper "Scattered Mixture-of-Experts Implementation"
 * (arXiv 2403.08245) defines: routing indices (Sec. 3.1 steps 1-2), ParallelLinear
 * forward (Alg. 1) and backward (Alg. 2, Sec. 3.2.1), and the SMoE MLP built from two
 * ParallelLinears (Alg. 3).  Notation follows the paper: T tokens, E experts, top-k,
 * Tk = T*k routed slots, slot s = t*k + j.
 *
 * General conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller, on the device the
 *     context was created for.  Tensors are contiguous, row-major.  Index arrays are
 *     int32.  The library never frees or keeps a caller buffer past the call's work.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *     enqueued on it; no entry point synchronises, allocates device memory or copies to
 *     the host.  Results are ready when the stream reaches the end of the enqueued work.
 *   - `ws` / `ws_bytes`: scratch device memory supplied by the caller, at least as large
 *     as the matching *_workspace_bytes() query, 256-byte aligned.  Contents are
 *     unspecified on entry and on return.
 *   - Return value: SMOE_OK (0) or a negative smoe_status.  Argument, shape and workspace
 *     errors (INVALID_ARG, UNSUPPORTED, WORKSPACE) are found before anything is enqueued.
 *     SMOE_ERR_HIP reports a kernel launch the runtime refused: launches made earlier in
 *     the same call stay enqueued and the call's outputs are then unspecified.
 *     No entry point throws or aborts.  Index *contents* (expert ids in
 *     [0,E), a valid permutation in sorted_scattered_idxs) are the caller's contract:
 *     they live on the device and are not validated; out-of-range expert ids passed to
 *     smoe_route are clamped so that no out-of-bounds access happens.
 *   - Outputs are overwritten, never accumulated into.  All kernels are deterministic
 *     (no floating-point atomics): two identical calls give bit-identical results.
 *   - dtype: SMOE_F32 computes with fp32 FMA accumulation; SMOE_BF16 takes bf16 inputs,
 *     accumulates in fp32 on the matrix cores and rounds each stored tensor to bf16
 *     (round-to-nearest-even).  gates and dgates are always fp32.
 */
#ifndef SMOE_H_
#define SMOE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct smoe_ctx smoe_ctx; /* opaque; holds the device id and launch heuristics */

typedef enum { SMOE_F32 = 0, SMOE_BF16 = 1 } smoe_dtype;

/* Alg. 3's point-wise non-linearity.  GELU is the exact erf form.  SWIGLU reads a
 * [.., 2*d_expert] pre-activation packed as [gate | up] and yields silu(gate) * up. */
typedef enum { SMOE_ACT_NONE = 0, SMOE_ACT_GELU = 1, SMOE_ACT_SWIGLU = 2 } smoe_act;

typedef enum {
  SMOE_OK = 0,
  SMOE_ERR_INVALID_ARG = -1,   /* null pointer, non-positive size, inconsistent flags   */
  SMOE_ERR_UNSUPPORTED = -2,   /* valid request this build has no kernel for            */
  SMOE_ERR_WORKSPACE = -3,     /* ws is NULL / misaligned / smaller than required       */
  SMOE_ERR_HIP = -4,           /* a HIP runtime call (launch, device query) failed      */
  SMOE_ERR_TOO_LARGE = -5      /* beyond the fixed scratch of a no-allocation entry point */
} smoe_status;

/* The routing products of Sec. 3.1 step 2 ("sort the tokens according to the experts").
 * sorted_scattered_idxs is the paper's order-index vector o (Alg. 1-3): entry i is the
 * slot id t*k+j of the i-th row in expert-sorted order; inside an expert slots ascend. */
typedef struct {
  const int32_t *sorted_expert_idxs;    /* [Tk] expert of the i-th sorted row, non-decreasing   */
  const int32_t *sorted_scattered_idxs; /* [Tk] permutation of 0..Tk-1 (o)                      */
  const int32_t *expert_offsets;        /* [E+1] exclusive prefix sums of per-expert row counts */
  int32_t Tk;
  int32_t E;
} smoe_routing;

/* Creates a context for HIP device `device` (host call; queries device properties).
 * Also raises, on that device, the dynamic-LDS limit of the kernels that need it, so one context
 * per device is all a process needs.  *out is owned by the caller until smoe_destroy.  One context
 * may be used from several streams and threads: the entry points only read it.  The one exception
 * is smoe_set_kernel_mode below, which must not run concurrently with any other call. */
int smoe_create(smoe_ctx **out, int device);
void smoe_destroy(smoe_ctx *ctx);
/* Static string for a smoe_status value. */
const char *smoe_strerror(int status);
/* ABI version, bumped when a signature changes. */
int smoe_abi_version(void);

/* Selects the GEMM kernel family: 0 = automatic (persistent matrix-core kernels whenever the
 * shape allows), 1 = force the plain tiled kernels, 2 = matrix-core kernels with one block per
 * tile (1 and 2 are testing aids).  Host-only; writes the context, so no other call on the same
 * context may be in progress. */
int smoe_set_kernel_mode(smoe_ctx *ctx, int mode);

/* Measurement aid.  The persistent scatter2scatter kernels number their output tiles in groups of group_m M-tiles x all
 * N-tiles, and the 32 compute units of an XCD take 32 consecutive numbers, i.e. a group_m x (32 / group_m) patch of tiles
 * that shares operand panels in that XCD's L2.  The default, 4, is the measured optimum (profiles/); 1 <= group_m <= 64.
 * Results do not depend on it.  Host-only; writes the context, so no other call on it may be in progress. */
int smoe_set_tile_group(smoe_ctx *ctx, int group_m);

/* Measurement aid.  With a device array of 512 uint64 set, every launch of the persistent scatter2scatter
 * kernels (the products of smoe_plinear_fwd / _bwd, smoe_plinear_act_fwd, smoe_mlp_fwd / _bwd) makes block b
 * store, when it ends, the shader-clock cycles and the ticks of the constant 100 MHz counter between its first
 * and last instruction in entries 2b and 2b+1: cycles / ticks * 100 is the clock in MHz the compute unit ran at
 * (blocks b, b+8, ... share an XCD).  Later launches overwrite the array.  NULL (the default) turns it off.
 * Host-only; writes the context, so no other call on it may be in progress. */
int smoe_set_clock_probe(smoe_ctx *ctx, uint64_t *device_array);

/* ---- routing: Sec. 3.1 step 1 -------------------------------------------------------
 * For each token keeps the k largest of its E router logits (ties to the lower expert
 * id, slots ordered by descending logit) and the softmax over those k logits.
 *   logits      [T,E] fp32 (in)
 *   expert_idxs [T*k] int32 (out), gates [T*k] fp32 (out), both in slot order t*k+j.
 * Needs 1 <= k <= E.  T = 0 is a no-op.  A NaN logit counts as -inf; kept logits that are all
 * -inf share the weight equally, so every slot is always written. */
int smoe_topk_gate(smoe_ctx *ctx, void *stream, const float *logits, int T, int E, int k,
                   int32_t *expert_idxs, float *gates);

/* Gradient of the gate with respect to the router logits, closing the chain from Alg. 2's dp
 * (dgates) to the router of Sec. 3.1 step 1: on a token's k kept experts
 * dlogits[t,e_j] = g_j (dp_j - sum_i g_i dp_i), zero for every other expert (the selection is
 * piecewise constant).
 *   expert_idxs [T*k] int32, gates [T*k] fp32 (outputs of smoe_topk_gate), dgates [T*k] fp32 (in)
 *   dlogits [T,E] fp32 (out, every entry written). */
int smoe_topk_gate_bwd(smoe_ctx *ctx, void *stream, const int32_t *expert_idxs, const float *gates,
                       const float *dgates, int T, int E, int k, float *dlogits);

/* ---- routing: Sec. 3.1 step 2 -------------------------------------------------------
 * Stable bucket sort of the Tk = T*k slots by expert.  Outputs as in smoe_routing.
 * Integer work, bit-exact.  Experts nobody chose get an empty segment.  E <= 16384 (one
 * counter per expert in LDS), else SMOE_ERR_UNSUPPORTED. */
size_t smoe_route_workspace_bytes(int T, int k, int E);
int smoe_route(smoe_ctx *ctx, void *stream, const int32_t *expert_idxs, int T, int k, int E,
               int32_t *sorted_expert_idxs, int32_t *sorted_scattered_idxs,
               int32_t *expert_offsets, void *ws, size_t ws_bytes);

/* smoe_route for callers that cannot allocate or pass a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid device allocation.  Same inputs, outputs and results as smoe_route;
 * the per-chunk expert counts live in a fixed 1 MiB device array inside the library (one copy per GPU the
 * library runs on, held until the process ends) whose address smoe_create looks up for the context's
 * device.  Limit: ceil(T*k / 1024) * E * 4 bytes (rounded up to 256) must not exceed 1 MiB, e.g. up to
 * 1 Mi routed slots with 256 experts, else SMOE_ERR_TOO_LARGE and nothing is enqueued.  Calls no
 * allocator, no memset and no synchronisation.  Every call on one GPU uses the same array: calls that
 * overlap on one GPU (different streams, or threads) race and must be serialised by the caller; calls
 * in stream order on one stream are fine.  The array keeps the last call's contents; nothing in it needs
 * clearing, each call overwrites every counter it reads. */
int smoe_route_noalloc(smoe_ctx *ctx, void *stream, const int32_t *expert_idxs, int T, int k, int E,
                       int32_t *sorted_expert_idxs, int32_t *sorted_scattered_idxs,
                       int32_t *expert_offsets);

/* ---- ParallelLinear forward: Alg. 1 (scatter2scatter, Sec. 3.2, Fig. 2) --------------
 *   X     [x_rows, d_in]  grouped_in = 0: scattered, the row of slot s is s / k (fan-out k,
 *                         so x_rows = Tk / k); grouped_in = 1: expert-sorted, x_rows = Tk, k = 1.
 *   W     [E, d_in, d_out]
 *   Yhat  [Tk, d_out] (out) row i (grouped_out = 1) or row o[i] (grouped_out = 0) is the
 *                         i-th sorted input row times its expert's matrix.
 *   gates optional [Tk] fp32 in slot order viewed as [T, kp] with kp = gates_k; when given,
 *         grouped_out must be 0 and Y [Tk / gates_k, d_out] (out) receives
 *         Y[t] = sum_j gates[t*kp+j] * Yhat[t*kp+j]   (Alg. 1's view + bmm).
 *         gates = NULL: Y must be NULL and Yhat is the result.
 * No workspace is needed (so this entry point always runs whole output tiles; the calls that
 * take a workspace also keep 64 MiB of it for the split last round described there). */
int smoe_plinear_fwd(smoe_ctx *ctx, void *stream, smoe_dtype dtype, const void *X, int x_rows,
                     int d_in, const void *W, int d_out, const smoe_routing *r, int k,
                     const float *gates, int gates_k, int grouped_in, int grouped_out,
                     void *Yhat, void *Y);

/* ---- ParallelLinear backward: Alg. 2, Sec. 3.2.1 -------------------------------------
 * Gradients of Alg. 1's result.  dY has the shape of Alg. 1's output: [Tk/gates_k, d_out]
 * when gates were given, else [Tk, d_out] in the order grouped_out says.
 *   Yhat   forward's unweighted [Tk, d_out] (scattered); read only when gates != NULL.
 *   dX     (out) same shape as X; with scattered input the k slot gradients of a row are summed.
 *   dW     (out) [E, d_in, d_out] in the weight dtype; zeros for experts with no rows.
 *   dgates (out, nullable) [Tk] fp32, dgates[s] = <dY[s / gates_k], Yhat[s]>.
 * Either of dX / dW may be NULL to skip it.  Steps as in Alg. 2: dgates row dots, `group` of
 * dY (weighted by the gates) and of X whenever they are not already expert-sorted, groupXTY
 * for dW on the two grouped operands, scatter2scatter with W^T for dX, and the sum over a
 * row's k slots when the input was scattered.  The workspace holds the grouped copies and
 * 64 MiB for fp32 partial output tiles: when the output tiles of a product do not fill a last
 * round of the persistent grid, that round's contraction is cut into up to four chunks run
 * by otherwise idle blocks, and a second kernel adds the chunks in a fixed order. */
size_t smoe_plinear_bwd_workspace_bytes(smoe_dtype dtype, int x_rows, int d_in, int d_out, int Tk,
                                        int k, int has_gates, int grouped_in, int grouped_out);
int smoe_plinear_bwd(smoe_ctx *ctx, void *stream, smoe_dtype dtype, const void *dY, const void *X,
                     int x_rows, int d_in, const void *W, int d_out, const void *Yhat,
                     const smoe_routing *r, int k, const float *gates, int gates_k, int grouped_in,
                     int grouped_out, void *dX, void *dW, float *dgates, void *ws, size_t ws_bytes);

/* ---- first half of the SMoE MLP: Alg. 3, lines 1-2 ------------------------------------------
 * H = act(ParallelLinear(X, W1, scattered -> grouped)): the hidden activations of the Tk routed rows in
 * expert-sorted order, through the same kernels smoe_mlp_fwd uses for them (for bf16 SwiGLU the
 * activation is applied in the product's epilogue from the fp32 accumulators).
 *   X [T, d_model];  W1 [E, d_model, d_h], d_h = 2*d_expert for SWIGLU else d_expert;
 *   Hpre [Tk, d_h] (out, nullable: NULL = the pre-activation is not kept; the workspace then holds it
 *   for the paths that apply the activation in a second kernel);  H [Tk, d_expert] (out). */
size_t smoe_plinear_act_fwd_workspace_bytes(smoe_dtype dtype, smoe_act act, int T, int k, int d_model,
                                            int d_expert, int keep_hpre);
int smoe_plinear_act_fwd(smoe_ctx *ctx, void *stream, smoe_dtype dtype, smoe_act act, const void *X, int T,
                         int d_model, int d_expert, const void *W1, const smoe_routing *r, int k,
                         void *Hpre, void *H, void *ws, size_t ws_bytes);

/* ---- SMoE MLP: Alg. 3 -----------------------------------------------------------------
 * Y[t] = sum_j gates[t*k+j] * act(X[t] W1[e]) W2[e]  over the token's k experts (Sec. 3.1
 * step 5), computed as ParallelLinear(scattered->grouped), act, ParallelLinear(grouped->
 * scattered, weighted).
 *   X [T, d_model];  W1 [E, d_model, d_h] with d_h = 2*d_expert for SWIGLU else d_expert;
 *   W2 [E, d_expert, d_model];  gates [T*k] fp32;  Y [T, d_model] (out).
 *   saved_Hpre [Tk, d_h], saved_H [Tk, d_expert] (expert-sorted order) and saved_Yhat
 *   [Tk, d_model] (slot order): outputs kept for the backward pass.  Pass saved_Hpre and
 *   saved_H together or neither (inference: the workspace holds everything).  saved_Yhat
 *   (the unweighted second product, Alg. 2's input for dp) is needed by smoe_mlp_bwd only
 *   when smoe_mlp_saves_yhat says so; it may be NULL otherwise, and the workspace then holds
 *   it for the duration of the call.  `training` of the workspace query: 0 = nothing saved,
 *   1 = all three saved, 2 = Hpre and H saved, Yhat not.  The workspace always includes the
 *   64 MiB of partial tiles of a split last round (see smoe_plinear_bwd). */
size_t smoe_mlp_fwd_workspace_bytes(smoe_dtype dtype, smoe_act act, int T, int k, int d_model,
                                    int d_expert, int training);
/* 1 if smoe_mlp_bwd of this shape reads the forward's saved_Yhat, 0 if it does not (bf16 SwiGLU
 * shapes the persistent kernels take: dp[t,j] = <dY_t W2[e]^T, H_i> is then formed in the epilogue of
 * the W2^T product from its fp32 accumulators, in the spirit of Sec. 3.2.1's buffer reuse, and the
 * activation's derivative is applied there too), negative smoe_status on bad arguments. */
int smoe_mlp_saves_yhat(smoe_ctx *ctx, smoe_dtype dtype, smoe_act act, int T, int k, int E, int d_model,
                        int d_expert);
int smoe_mlp_fwd(smoe_ctx *ctx, void *stream, smoe_dtype dtype, smoe_act act, const void *X, int T,
                 int d_model, int d_expert, const void *W1, const void *W2, const smoe_routing *r,
                 int k, const float *gates, void *Y, void *saved_Hpre, void *saved_H,
                 void *saved_Yhat, void *ws, size_t ws_bytes);

/* Backward of smoe_mlp_fwd (Alg. 2 applied to both ParallelLinears, one `group` each).
 *   dY [T, d_model] upstream gradient; saved_* from the forward call (saved_Yhat may be NULL
 *   when smoe_mlp_saves_yhat returns 0).
 *   dX [T, d_model], dW1 like W1, dW2 like W2, dgates [T*k] fp32 (all out, none nullable). */
size_t smoe_mlp_bwd_workspace_bytes(smoe_dtype dtype, smoe_act act, int T, int k, int d_model,
                                    int d_expert);
int smoe_mlp_bwd(smoe_ctx *ctx, void *stream, smoe_dtype dtype, smoe_act act, const void *dY,
                 const void *X, int T, int d_model, int d_expert, const void *W1, const void *W2,
                 const smoe_routing *r, int k, const float *gates, const void *saved_Hpre,
                 const void *saved_H, const void *saved_Yhat, void *dX, void *dW1, void *dW2,
                 float *dgates, void *ws, size_t ws_bytes);

/* ---- the `group` copy of Alg. 2 --------------------------------------------------------
 * out[i] = scale_i * in[o[i] / fan] for the Tk sorted rows, scale_i = gates[o[i]] or 1 when
 * gates is NULL.  in [Tk/fan, d], out [Tk, d].  Exposed because Alg. 2 names it; the
 * forward path never needs it. */
int smoe_group(smoe_ctx *ctx, void *stream, smoe_dtype dtype, const void *in, int d,
               const smoe_routing *r, int fan, const float *gates, void *out);

/* ---- SMoE multi-head attention: Alg. 4, Sec. 3.3 ------------------------------------------
 * The attention between Alg. 4's two scattered->scattered ParallelLinears: causal scaled
 * dot-product attention softmax(q k^T / sqrt(d_head)) v inside each of the B sequences of T
 * positions, grouped-query style: Q and O hold one row per routed slot, [B, T, G, h, d_head]
 * (G = k slots per token, h = heads per expert), K and V one row per token, [B, T, h, d_head];
 * head hh of every slot attends key/value head hh (Sec. 3.3).
 *   LSE [B, T, G, h] fp32 (out): log-sum-exp of the scaled, masked scores, kept for the backward.
 * bf16 only, d_head = 128 (else SMOE_ERR_UNSUPPORTED).  No workspace. */
int smoe_attention_fwd(smoe_ctx *ctx, void *stream, smoe_dtype dtype, const void *Q, const void *K,
                       const void *V, int B, int T, int G, int h, int d_head, void *O, float *LSE);

/* Backward of smoe_attention_fwd: gradients of O with respect to Q, K and V (same shapes and
 * dtype as the inputs), from the upstream dO [B, T, G, h, d_head] and the forward's O and LSE.
 * dK and dV sum over the G slots and the later positions that attend a key.  Deterministic
 * (no atomics: one pass owns the query rows; a second one owns the key rows, cut into chunks of
 * slot rows whose fp32 partial sums a last kernel adds in a fixed order).  The workspace holds
 * one fp32 per (slot row, head) and those partial sums. */
size_t smoe_attention_bwd_workspace_bytes(int B, int T, int G, int h);
int smoe_attention_bwd(smoe_ctx *ctx, void *stream, smoe_dtype dtype, const void *dO, const void *Q,
                       const void *K, const void *V, const void *O, const float *LSE, int B, int T, int G,
                       int h, int d_head, void *dQ, void *dK, void *dV, void *ws, size_t ws_bytes);

/* SMoE multi-head attention layer, Alg. 4:
 *   V = X W_V, K = X W_K (dense), Q = ParallelLinear(X, W_Q, o, no p, scattered -> scattered),
 *   Ohat = Attention(Q, K, V), O = ParallelLinear(Ohat, W_O, o, p, scattered -> scattered).
 *   X [B*T, d_model] (B sequences of T positions, batch-time order);  d_out = h_expert * d_head;
 *   W_K, W_V [d_model, d_out];  W_Q [E, d_model, d_out];  W_O [E, d_out, d_model];
 *   r, k, gates: routing of the B*T tokens (Tk = B*T*k);  O [B*T, d_model] (out).
 *   saved_K, saved_V [B*T, d_out], saved_Q, saved_Ohat [Tk, d_out] (slot order), saved_LSE
 *   [Tk, h_expert] fp32, saved_Yhat [Tk, d_model] (slot order): kept for the backward pass; pass
 *   all six or none (inference: the workspace holds them).
 * bf16, d_head = 128.  The dense projections run through the grouped kernels as one expert. */
size_t smoe_momha_fwd_workspace_bytes(int B, int T, int k, int d_model, int h_expert, int d_head,
                                      int training);
int smoe_momha_fwd(smoe_ctx *ctx, void *stream, smoe_dtype dtype, const void *X, int B, int T, int d_model,
                   int h_expert, int d_head, const void *W_K, const void *W_V, const void *W_Q,
                   const void *W_O, const smoe_routing *r, int k, const float *gates, void *O,
                   void *saved_K, void *saved_V, void *saved_Q, void *saved_Ohat, float *saved_LSE,
                   void *saved_Yhat, void *ws, size_t ws_bytes);

/* Backward of smoe_momha_fwd: Alg. 2 for the two ParallelLinears, smoe_attention_bwd between
 * them, plain products for the dense key/value projections.
 *   dO [B*T, d_model] upstream gradient; dX like X; dW_* like W_*; dgates [Tk] fp32 (all out). */
size_t smoe_momha_bwd_workspace_bytes(int B, int T, int k, int d_model, int h_expert, int d_head);
int smoe_momha_bwd(smoe_ctx *ctx, void *stream, smoe_dtype dtype, const void *dO, const void *X, int B, int T,
                   int d_model, int h_expert, int d_head, const void *W_K, const void *W_V, const void *W_Q,
                   const void *W_O, const smoe_routing *r, int k, const float *gates, const void *saved_K,
                   const void *saved_V, const void *saved_Q, const void *saved_Ohat, const float *saved_LSE,
                   const void *saved_Yhat, void *dX, void *dW_K, void *dW_V, void *dW_Q, void *dW_O,
                   float *dgates, void *ws, size_t ws_bytes);

#ifdef __cplusplus
}
#endif
#endif /* SMOE_H_ */

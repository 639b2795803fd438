/* pp.h -- C ABI of the partial-parameter-update local training step for MI355X (gfx950).
 *
 * One node's share of "Partial Parameter Updates for Efficient Distributed Training"
 * (Algorithm 1): a full forward pass over all parameters, a restricted backward pass that forms
 * weight gradients only for the node's fixed trainable subset I_train and propagates activation
 * gradients only as far down as the lowest trainable parameter, AdamW on that subset only, and
 * the node's share of the outer pseudo-gradient step.
 *
 * Conventions
 *   - All "_dev" pointers are device (HBM) pointers owned by the CALLER; the library allocates no
 *     device memory and keeps only a host-side handle.  "host_" pointers are ordinary host memory.
 *   - All work is enqueued on the HIP stream given to pp_init_model; calls return after enqueueing
 *     unless stated otherwise.  Calls on one handle must not overlap.
 *   - Every function returning int returns PP_OK or a negative PP_E* code; pp_last_error() gives
 *     a thread-local message for the last failure.  No exception crosses this boundary.
 *
 * Model (decoder-only transformer; details the paper leaves open are fixed here):
 *   pre-norm RMSNorm  y = gamma * x * rsqrt(mean(x^2) + rms_eps);
 *   rotary embedding on q and k, half-split pairing (i, i + dh/2), angle pos * rope_base^(-2i/dh);
 *   causal softmax attention with scale 1/sqrt(dh);  SwiGLU FFN  y = (silu(x Wg^T) * (x Wu^T)) Wd;
 *   untied embedding and lm_head; no biases; loss = mean over valid positions of the next-token
 *   cross entropy (Eq. 2.2), target -1 = position ignored.
 *
 * Tensor names and canonical (row-major) shapes, element type = pp_config.dtype:
 *   "embed" [vocab x d]            "final_norm" [d]             "lm_head" [vocab x d]
 *   "layers.<l>.attn_norm" [d]     "layers.<l>.wqkv" [3d x d]   rows = [Wq; Wk; Wv], each out x in,
 *                                                                head j = rows j*dh..(j+1)*dh of its block
 *   "layers.<l>.wo" [d x d] (out x in)                          "layers.<l>.ffn_norm" [d]
 *   "layers.<l>.wg", ".wu", ".wd" [d_ff x d]  (hidden-unit major: a slice of hidden units is one
 *                                  contiguous row block of each -- the W_n / V_n blocks of the
 *                                  paper's "MLP-Only Slicing")
 *   They live back to back, in the order above (layers ascending), in the params buffer.
 */
#ifndef PP_H
#define PP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pp_model pp_model; /* opaque host-side handle */

enum { PP_OK = 0, PP_EINVAL = -1, PP_ENOMEM = -2, PP_ESTATE = -3, PP_EHIP = -4 };
enum { PP_F32 = 0, PP_BF16 = 1 };
enum { PP_BYTES_PARAMS = 0, PP_BYTES_STATE = 1, PP_BYTES_WORKSPACE = 2, PP_BYTES_SHADOW = 3,
       PP_BYTES_ACTIVATIONS = 4 };

typedef struct {
  int32_t n_layers, d_model, n_heads, d_ff, vocab;
  int32_t max_batch, max_seq; /* largest B and S any pp_local_step call will use */
  int32_t dtype;              /* PP_F32: fp32 storage and arithmetic; PP_BF16: bf16 storage, fp32 accumulate */
  float rms_eps, rope_base;
  int32_t recompute;          /* 0: every layer's activations are kept for the backward pass.  1: full activation
                                 recomputation (the memory regime of the paper's Table 1): only each layer's input is
                                 kept, the layer is run forward again when the backward pass reaches it.  Same results
                                 bit for bit; WORKSPACE shrinks by about (n_layers - 1) layers of activations. */
} pp_config;

/* I_train of Algorithm 1 as a union of row blocks (Section "Parameter Slicing").
 * all != 0: every parameter is trainable (the full-backprop step) and the other fields are ignored.
 * Otherwise: hidden units [ffn_lo, ffn_hi) of wg, wu, wd in every layer; heads [head_lo, head_hi) of
 * the Q, K and V blocks of wqkv in every layer; and the whole of wo / all norm gains / embed / lm_head
 * when the matching flag is non-zero.  lo == hi means none. */
typedef struct {
  int32_t all;
  int32_t ffn_lo, ffn_hi;
  int32_t head_lo, head_hi;
  int32_t train_wo, train_norms, train_embed, train_lm_head;
} pp_mask;

/* InnerOpt of Algorithm 1: decoupled AdamW (Experimental Setup).  Per step t = 1, 2, ...:
 *   p <- p (1 - lr*weight_decay)   [not applied to norm gains]
 *   m <- beta1 m + (1-beta1) g;  v <- beta2 v + (1-beta2) g^2
 *   p <- p - lr * (m / (1-beta1^t)) / (sqrt(v / (1-beta2^t)) + eps) */
typedef struct { float lr, beta1, beta2, eps, weight_decay; } pp_adamw;

/* OuterOpt of Algorithm 1 (SGD with Nesterov momentum, Experimental Setup) in the pseudo-gradient
 * convention: delta = (theta_g - theta_l + others_sum) / m_count;  b <- momentum*b + delta;
 * theta_g <- theta_g - lr*(delta + momentum*b) if nesterov else theta_g - lr*b.
 * m_count is the count-vector entry m[i] (number of nodes training the element), >= 1. */
typedef struct { float lr, momentum; int32_t nesterov; float m_count; } pp_outer;

/* Bytes the caller must provide.  PARAMS: canonical weights.  STATE (needs mask): fp32 master, m, v and
 * gradient for I_train only, 16 bytes per trainable element -- nothing exists for frozen elements.
 * WORKSPACE: saved activations, backward scratch and transposed read-only weight copies ("shadow");
 * SHADOW and ACTIVATIONS report those two parts of WORKSPACE.  mask may be NULL except for STATE.
 * Returns 0 on invalid arguments (and sets the error text). */
size_t pp_query_bytes(const pp_config* cfg, const pp_mask* mask, int which);

/* Creates a handle over caller-owned buffers (256-byte aligned, at least the queried sizes).
 * params_dev content is taken as is: fill it with pp_set_tensor, or directly (device copy, checkpoint load) in the canonical
 * layout BEFORE pp_set_trainable_mask, which forms the transposed read-only copies of all matrices from it.
 * hip_stream: a hipStream_t (NULL = default stream).  Blocks until its one-time tables are built. */
int pp_init_model(const pp_config* cfg, void* params_dev, size_t params_bytes, void* workspace_dev,
                  size_t workspace_bytes, void* hip_stream, pp_model** out);

/* Host <-> device copies of a named tensor (whole tensor, canonical layout, bytes must match exactly).
 * Besides the weight names, pp_get_tensor accepts "state.p", "state.m", "state.v", "state.g" (packed
 * fp32 subset, valid after pp_set_trainable_mask / a step), "state.rows" (int64 canonical element
 * offset of every packed row of d_model elements), "shadow.<weight>" (the transposed read-only copy of wqkv, wo,
 * wd or lm_head, shape [in x out]) and, for debugging, "dbg.<buffer>[.<layer>]" taps into the workspace
 * (x, n1, qkv, o, xm, n2, gu, a, lse per layer; xL, logits, dx, dn, dqkv, dgu), sized for max_batch*max_seq tokens;
 * with recompute = 1 only x is per layer, the others show the layer worked on last.
 * Both block until the copy is done.
 * pp_set_tensor on a weight after pp_set_trainable_mask leaves the fp32 masters stale: set the mask again. */
int pp_set_tensor(pp_model* m, const char* name, const void* host_src, size_t bytes);
int pp_get_tensor(pp_model* m, const char* name, void* host_dst, size_t bytes);

/* Fixes I_train (it stays fixed during local training, Section 2.2), packs the trainable rows into
 * state_dev in network order (embed, then per layer attn_norm, wqkv q/k/v head rows, wo, ffn_norm, wg,
 * wu, wd rows, then final_norm, lm_head), snapshots fp32 masters from the current weights, zeroes m and v
 * and resets the step counter; also rebuilds the transposed weight copies in the workspace from params_dev.
 * May be called again (new round, new mask, or after params_dev was rewritten by the caller). */
int pp_set_trainable_mask(pp_model* m, const pp_mask* mask, void* state_dev, size_t state_bytes);

/* One local step (Algorithm 1, inner loop body): forward over all parameters, restricted backward,
 * AdamW on I_train, write-back of the updated subset into the weights in storage dtype.  Frozen
 * parameters are never written.  tokens_dev/targets_dev: int32 [B x S] on the device; token ids in
 * [0, vocab); targets in [-1, vocab).  loss_dev: device float, receives the mean loss of this batch
 * (computed before the update).  opt == NULL: gradients are computed into "state.g" but no update is made.
 * Asynchronous on the stream.  PP_ESTATE before pp_set_trainable_mask; PP_EINVAL on bad shapes. */
int pp_local_step(pp_model* m, const int32_t* tokens_dev, const int32_t* targets_dev, int32_t B, int32_t S,
                  const pp_adamw* opt, float* loss_dev);

/* Ablation of Appendix "Additional Results" (off by default; the paper reports that it diverges or degrades):
 * which FFN hidden units enter the INPUT gradient of every later pp_local_step.
 *   mode 0: all of them (the method: frozen slices still carry the input gradient, Appendix "Partial Backward").
 *   mode 1: "detach-all-but-k": only the trainable slice of the mask, plus the units [extra_lo, extra_hi) of one more
 *           slice g ("detach-all-but-k + random"; the caller draws g and calls this before each step; an empty range
 *           = no extra slice).  dL/dH of every other hidden unit is taken as zero; with SwiGLU the appendix's
 *           activation mask I(H > 0) is the SwiGLU derivative.  Weight gradients and the forward pass are unchanged.
 * Bounds must be multiples of 8 inside [0, d_ff] (PP_EINVAL otherwise).  pp_local_step then returns PP_EINVAL if the
 * mask has no trainable FFN slice or if the extra range overlaps it.  Host-side state only; nothing is launched. */
int pp_set_jacobian_slices(pp_model* m, int32_t mode, int32_t extra_lo, int32_t extra_hi);

/* Node's share of the synchronisation (Algorithm 1, delta / normalisation / OuterOpt lines) on the
 * packed subset of n = trainable-element-count values: theta_l is read from the current weights in
 * storage dtype; theta_g_dev [n] fp32 global parameters and momentum_dev [n] fp32 are updated in place;
 * others_sum_dev [n] fp32 (nullable) is the sum of the other nodes' deltas in the same convention;
 * delta_out_dev [n] fp32 (nullable) receives the normalised delta.  Afterwards the local copy restarts
 * from the new global values: weights and fp32 masters <- theta_g, m and v are kept.  Asynchronous. */
int pp_outer_delta(pp_model* m, float* theta_g_dev, float* momentum_dev, const float* others_sum_dev,
                   const pp_outer* opt, float* delta_out_dev);

/* The same step for one group of the streaming synchronisation (Experimental Setup: the 24 layers are synchronised in
 * groups, one group every H steps, plus a group with the embeddings and the output norm): only the packed elements of
 * layers [layer_lo, layer_hi) and, if ends != 0, of embed / final_norm / lm_head are read or written; every buffer is still
 * indexed as in pp_outer_delta (full packed length n), the rest of it is left untouched.  Asynchronous. */
int pp_outer_delta_group(pp_model* m, int32_t layer_lo, int32_t layer_hi, int32_t ends, float* theta_g_dev, float* momentum_dev,
                         const float* others_sum_dev, const pp_outer* opt, float* delta_out_dev);

/* Fills dst_dev[0..n) with the sum of n_nodes seeded N(0, std) vectors from the counter-based generator
 * (splitmix64 finaliser over key + index*golden, Box-Muller pairs); stands for the all-reduced deltas of
 * the other nodes when no second GPU exists.  keys_host: n_nodes 64-bit stream keys.  Asynchronous. */
int pp_synth_delta_sum(pp_model* m, float* dst_dev, size_t n, const uint64_t* keys_host, int32_t n_nodes, float std);

/* Host-side accounting for the most recent pp_local_step: matmul FLOPs launched in forward and backward
 * (attention counted over causal pairs, recomputation inside the attention backward excluded), AdamW
 * bytes moved, and the number of trainable elements. */
int pp_get_counters(pp_model* m, double* flops_fwd, double* flops_bwd, double* adamw_bytes, int64_t* n_trainable);

/* How many contractions (GEMM calls incl. their split-K reduction, attention forward / backward calls) of the most recent
 * pp_local_step ran on the matrix-core (MFMA) kernels and how many on the plain fp32-FMA kernels.  With PP_F32 storage all
 * are plain by design; with PP_BF16 a plain call means a shape or alignment the MFMA kernels do not take (or "force_plain"):
 * the result is still correct, only slow -- tests of the bf16 benchmark shapes assert plain_calls == 0. */
int pp_get_launch_counts(pp_model* m, int64_t* matrix_core_calls, int64_t* plain_calls);

/* Options for tests and profiling.  "force_plain": 0 = automatic (MFMA kernels when shapes allow), 1 = force the
 * plain (non-MFMA) kernels.  "dw_tn": 1 (default) = weight-gradient GEMMs read their token-major operands directly
 * (LDS transpose reads), 0 = through transposed copies and the NT kernel.  "fuse_rope": 1 (default) = the rotary embedding of
 * q and k is applied in the q|k|v projection's epilogue (one rounding), 0 = as a separate pass over the stored projection.  "time_gemm": 1 = bracket every GEMM launch of later pp_local_step calls with a pair
 * of HIP events on the model's stream (host-side events only; no device memory), 0 = off; setting it resets the totals.
 * "gemm_variant" (process-wide, for tests and A/B timing only; m may be NULL; takes effect for launches issued after the
 * call returns, on any thread): 1 = direct-to-LDS MFMA GEMM (default), 0 = register-staged MFMA GEMM.
 * "gemm_persistent" (process-wide, same caveats; m may be NULL): 1 (default) = when a GEMM has more tiles than the GPU has compute
 * units, one workgroup per unit walks several tiles and requests its next tile's first operands before the current
 * tile's epilogue; 0 = one workgroup per tile.  Same results bit for bit.
 * "gemm_small_tiles" (process-wide, same caveats; m may be NULL): 1 (default) = GEMMs with at most 128 output tiles of
 * 256 x 256 (half a tile per compute unit) run on the 128 x 128-tile kernel; 0 = always 256 x 256 tiles. */
int pp_set_option(pp_model* m, const char* key, int64_t value);

/* Blocks until the stream is idle, then returns the summed duration (ms), matmul FLOPs and number of the GEMM
 * launches (forward, input-gradient and weight-gradient GEMMs, split-K reduction included) bracketed since
 * "time_gemm" was set or since the previous call, and resets the totals. */
int pp_get_gemm_timing(pp_model* m, double* total_ms, double* total_flops, int64_t* launches);

const char* pp_last_error(void);
void pp_free(pp_model* m);

#ifdef __cplusplus
}
#endif
#endif /* PP_H */

/* pp_ops.h -- op-level entry points of the same library: the dense contractions of the local step, callable
 * on their own so that each kernel can be checked against a plain definition and timed against its roofline.
 * All pointers are device pointers owned by the caller; all calls only enqueue work on `hip_stream`.
 * dtype: PP_F32 or PP_BF16 storage (see pp.h).  Return PP_OK or a negative PP_E* code (pp_last_error()).
 */
#ifndef PP_OPS_H
#define PP_OPS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* C[M x N] = A[M x K] * B[N x K]^T (+ R[M x N] if R != NULL), row-major with leading dimensions lda, ldb, ldc
 * (R uses ldc).  Every matmul of the forward pass and of the partial backward (Appendix "Partial Backward":
 * dA = V_n^T G, dX = sum_n W_n^T dH_n, dW_n = dH_n X^T, dV_n = G A_n^T) is issued in this form.
 * out_f32 != 0: C is float (weight gradients); then R must be NULL.
 * splits > 1 (needs out_f32, scratch_dev of M*N*splits floats): K is cut into `splits` equal ranges whose
 * partial products are summed in fixed order into C.
 * path: 0 = automatic (MFMA kernel when dtype is bf16 and K % 64 == 0, lda % 8 == 0, ldb % 8 == 0), 1 = plain kernel. */
int pp_op_gemm_nt(void* hip_stream, int dtype, const void* A_dev, int lda, const void* B_dev, int ldb, void* C_dev, int ldc,
                  int M, int N, int K, const void* R_dev, int out_f32, int splits, float* scratch_dev, int path);

/* The weight-gradient contraction in the layout the step has it in (Appendix "Partial Backward": dW_n = dH_n X^T,
 * dV_n = G A_n^T, with tokens as the contraction index): C[M x N] (float, ldc) = A^T B, A: [K x .] and B: [K x N] row-major
 * bf16 with leading dimensions lda, ldb -- both token-major, no transposed copies.  Column m of the product is column
 * (m / m_blk) * a_blk_stride + m % m_blk of A (m_blk = M, a_blk_stride = 0 for one contiguous column range).
 * splits > 1 (scratch_dev of M*N*splits floats): K is cut into `splits` equal ranges whose partial products are summed in
 * fixed order.  MFMA kernel only (bf16): needs M, N, lda, ldb, m_blk, a_blk_stride multiples of 8, K a multiple of
 * 64*splits, and m_blk a multiple of 128 when M > m_blk; other shapes return PP_EINVAL (pp_local_step then goes through
 * transposed copies and pp_op_gemm_nt's kernels instead). */
int pp_op_gemm_tn(void* hip_stream, const void* A_dev, int lda, int m_blk, int64_t a_blk_stride, const void* B_dev, int ldb, float* C_dev,
                  int ldc, int M, int N, int K, int splits, float* scratch_dev);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): the split-K form of pp_op_gemm_nt with fp32 output, C[M x N] (ldc) = A[M x K] * B[N x K]^T, whose
 * partial products [splits][M][N] live in a 16 MiB device array built into the library instead of a caller's scratch
 * buffer.  Same kernels, same summation order and therefore the same bits as pp_op_gemm_nt(..., out_f32 = 1, splits,
 * scratch, path).  Requirements: splits >= 2, K % splits == 0, M*N*splits <= PP_STATIC_SCRATCH_FLOATS, else PP_EINVAL
 * with a message that names the limit.  Calls no hipMalloc / hipFree and nothing that allocates; only enqueues on
 * hip_stream.  The first call on a GPU also looks up that GPU's address of the array (the HIP runtime materialises a
 * module's device variables at that moment: make one call per GPU before entering a region that must not allocate).
 * Every call on one GPU uses that GPU's one array (it keeps the previous call's partials; each call overwrites all it
 * reads): calls that overlap on one GPU -- different streams or threads -- race; calls on one stream are ordered and
 * safe.  Each GPU the library runs on holds its own 16 MiB until process exit. */
#define PP_STATIC_SCRATCH_FLOATS (4u << 20)
int pp_op_gemm_nt_splitk_static(void* hip_stream, int dtype, const void* A_dev, int lda, const void* B_dev, int ldb, float* C_dev,
                                int ldc, int M, int N, int K, int splits, int path);

/* Causal softmax attention (Appendix "MHA with frozen heads", forward of every head; mask from the autoregressive
 * factorisation of Section 2.1).  qkv_dev: [B*S x 3*h*dh], columns q | k | v, head j at columns j*dh of each part
 * (q and k already rotated).  o_dev: [B*S x h*dh].  lse_dev: float [B*h*S], log-sum-exp of the scaled scores.
 * scratch_dev: not used (the matrix-core kernels read q, k, v as stored); kept in the signature, may be NULL.
 * path: 0 = automatic (MFMA kernels for bf16 with dh 64 or 128), 1 = plain kernels. */
int pp_op_attention_fwd(void* hip_stream, int dtype, const void* qkv_dev, void* o_dev, float* lse_dev, void* scratch_dev,
                        int B, int S, int h, int dh, int path);

/* Backward of the above for all heads: dqkv_dev [B*S x 3*h*dh] receives dq | dk | dv (in the rotated frame);
 * D_dev: float [B*h*S], receives the row sums of dO * O.  scratch_dev: not used, may be NULL. */
int pp_op_attention_bwd(void* hip_stream, int dtype, const void* qkv_dev, const void* o_dev, const float* lse_dev, const void* dO_dev,
                        void* dqkv_dev, float* D_dev, void* scratch_dev, int B, int S, int h, int dh, int path);

#ifdef __cplusplus
}
#endif
#endif /* PP_OPS_H */

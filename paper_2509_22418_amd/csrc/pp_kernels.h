// Host-side launch interface of the HIP kernels.  Every function only enqueues work on `st`.
// dtype is PP_F32 (0) or PP_BF16 (1) and selects the storage type of "void*" activations/weights.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace pp {

struct RowInfo {        // one packed row (d_model elements) of the trainable subset
  int64_t canon_off;    // element offset of the row in the canonical params buffer
  float wd_on;          // 1: weight decay applies, 0: norm gain
  int32_t pad;
};
struct ShadowSeg {      // one trainable row block that also lives, transposed, in a shadow matrix
  int64_t canon_off;    // element offset of the block's first element in params
  int64_t shadow_off;   // element offset (from the shadow base) of its image: (r,c) -> shadow_off + c*shadow_ld + r
  int32_t rows, cols, shadow_ld, tile_start;   // tile_start: first 64x64 tile index of this block in the batched launch
};

enum { EPI_STORE = 0, EPI_ADD_RES = 1, EPI_SWIGLU = 2, EPI_SWIGLU_BWD = 3, EPI_ROPE = 4 };          // the last three: only inside k_gemm_swiglu_*_mfma / k_gemm_qkv_rope_mfma

void k_fill_f32(hipStream_t st, float* p, size_t n, float v);
void k_rope_tables(hipStream_t st, float* cosb, float* sinb, int S, int dh, float base);
void k_embed(hipStream_t st, int dtype, const int32_t* tok, const void* E, void* x, int T, int d, int V);
void k_rmsnorm_fwd(hipStream_t st, int dtype, const void* x, const void* gamma, void* y, float* rstd, int T, int d, float eps);
// dx = (dres ? dres : 0) + rmsnorm backward of dy ; dx may alias dres
void k_rmsnorm_bwd(hipStream_t st, int dtype, const void* dy, const void* x, const float* rstd, const void* gamma,
                   const void* dres, void* dx, int T, int d);
// dgamma[c] = sum_t dy[t,c] * x[t,c] * rstd[t]; partial: float[64*d] scratch
void k_rmsnorm_dgamma(hipStream_t st, int dtype, const void* dy, const void* x, const float* rstd, float* partial,
                      float* dgamma, int T, int d);
void k_rope(hipStream_t st, int dtype, void* qkv, const float* cosb, const float* sinb, int B, int S, int h, int dh, int inverse);
void k_swiglu_fwd(hipStream_t st, int dtype, const void* gu, void* a, int T, int F);
// dA: [T x (c1-c0)] with leading dimension ldA, holding columns c0..c1 of the activation gradient.
void k_swiglu_bwd(hipStream_t st, int dtype, const void* gu, const void* dA, int ldA, void* dgu, int T, int F, int c0, int c1);
void k_count_valid(hipStream_t st, const int32_t* targets, int T, int V, int32_t* n_valid);
// logits [T x V] are overwritten with dL/dlogits; rowloss[T] gets the per-row loss (0 on ignored rows)
// whether k_cross_entropy has a kernel for rows of V logits: bf16 rows with V % 8 == 0 stay in registers up to V = 65536,
// everything else is staged in LDS (row bytes <= 64 KB - 256)
bool ce_row_fits(int dtype, int V);
int k_cross_entropy(hipStream_t st, int dtype, void* logits, const int32_t* targets, const int32_t* n_valid, float* rowloss, int T, int V);
void k_loss_reduce(hipStream_t st, const float* rowloss, const int32_t* n_valid, float* loss, int T);
void k_transpose(hipStream_t st, int dtype, const void* src, int ld_src, void* dst, int ld_dst, int rows, int cols);
void k_shadow_refresh(hipStream_t st, int dtype, const void* params, void* shadow, const ShadowSeg* segs_dev, int n_segs, int n_tiles, int vec_ok);

// C[M x N] (ldc) = A[M x K] (lda) * B[N x K]^T (ldb)  [+ R[M x N] (ldc) if epi == EPI_ADD_RES]
// out_f32: C is float regardless of dtype.  Plain (non-MFMA) kernel, any shape.
void k_gemm_nt_plain(hipStream_t st, int dtype, const void* A, int lda, const void* B, int ldb, void* C, int ldc,
                     int M, int N, int K, int epi, const void* R, int out_f32);
// split-K variant: partial[z][M][N] float, z = 0..splits-1 over equal K chunks (K % splits == 0)
void k_gemm_nt_plain_splitk(hipStream_t st, int dtype, const void* A, int lda, const void* B, int ldb, float* partial,
                            int M, int N, int K, int splits);
void k_splitk_reduce(hipStream_t st, const float* partial, float* C, int ldc, int M, int N, int splits);

void k_attn_fwd_plain(hipStream_t st, int dtype, const void* qkv, void* o, float* lse, int B, int S, int h, int dh);
void k_attn_D(hipStream_t st, int dtype, const void* o, const void* dO, float* Dbuf, int B, int S, int h, int dh);
void k_attn_bwd_plain(hipStream_t st, int dtype, const void* qkv, const void* o, const float* lse, const void* dO, void* dqkv,
                      float* Dbuf, int B, int S, int h, int dh);

void k_embed_grad(hipStream_t st, int dtype, const int32_t* tok, const void* dx, float* gE, int T, int d, int V, int32_t* scratch);

void k_pack_master(hipStream_t st, int dtype, const void* params, const RowInfo* rows, float* p, int n_rows, int d);
void k_adamw(hipStream_t st, int dtype, void* params, const RowInfo* rows, float* p, float* m, float* v, const float* g,
             int n_rows, int d, float lr, float beta1, float beta2, float eps, float wd, float bc1, float bc2);
void k_outer(hipStream_t st, int dtype, void* params, const RowInfo* rows, float* master, float* theta_g, float* mom,
             const float* others, float* delta_out, int n_rows, int d, float lr, float mu, int nesterov, float inv_m);
void k_synth_delta_sum(hipStream_t st, float* dst, size_t n, const uint64_t* keys_dev, int n_nodes, float std);

// MFMA paths (bf16 only).  Return 0 if launched, 1 if the shape is not supported (caller falls back).
// gu[M x 2F] = X [Wg; Wu]^T (bf16, ld 2F) and a[M x F] = silu(gate) * up from the rounded gate / up, one launch.
// Returns non-zero (nothing launched) when the shapes do not fit; the caller then runs the GEMM and k_swiglu_fwd.
int k_gemm_swiglu_fwd_mfma(hipStream_t st, const void* X, int ldx, const void* Wgu, int ldw, void* gu, void* a, int M, int F, int K);
// dgu columns c0.. and F + c0.. from the product G Wd_rows^T (= dL/da for N hidden units) and the saved gate / up; see the definition
int k_gemm_swiglu_bwd_mfma(hipStream_t st, const void* G, int ldg, const void* Wd_rows, int ldw, const void* gu_c0, void* dgu_c0, int ld2f, int half,
                           int M, int N, int K);
// qkv[M x 3d] (ld 3d) = X [Wq; Wk; Wv]^T with the rotary embedding applied to the q and k columns in the epilogue (fp32, before
// the one rounding to bf16): position of row t is t % S, tables [S x dh/2] fp32.  Needs d % 256 == 0 and dh in {64, 128, 256};
// returns non-zero (nothing launched) otherwise, and the caller runs the plain projection followed by k_rope.
int k_gemm_qkv_rope_mfma(hipStream_t st, const void* X, int ldx, const void* Wqkv, int ldw, void* qkv, int M, int d, int dh, int K, int S,
                         const float* rope_cos, const float* rope_sin);
int k_gemm_nt_mfma(hipStream_t st, const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K,
                   int epi, const void* R, int out_f32, int splits, float* partial);
// Weight-gradient form: C[M x N] fp32 (ldc) = A^T B with A [K x M] (lda), B [K x N] (ldb) row-major bf16 -- no transposed
// copies.  Column m of the product is column (m / m_blk) * a_blk_stride + m % m_blk of A.  splits > 1: `partial` receives
// [splits][M][N] and C is not written.  Returns 0 if launched, 1 if the shape is not taken.
int k_gemm_tn_mfma(hipStream_t st, const void* A, int lda, int m_blk, long a_blk_stride, const void* B, int ldb, float* C, int ldc,
                   int M, int N, int K, int splits, float* partial);
// 128 x 128-tile variant for shapes with too few 256 x 256 tiles to fill the chip (bf16 out, EPI_STORE / EPI_ADD_RES)
int k_gemm_nt128_mfma(hipStream_t st, const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K, int epi, const void* R);
void gemm_set_small_tiles(int v);      // 1 (default): k_gemm_nt_mfma hands GEMMs with at most 128 tiles of 256 x 256 (half a tile per compute unit) to the 128 x 128 kernel
void gemm_set_variant(int v);          // 0: register-staged MFMA GEMM, 1: direct-to-LDS MFMA GEMM
void gemm_set_persistent(int v);       // 1 (default): a workgroup per compute unit walks several tiles when there are more tiles than units
// Causal attention on the matrix cores (bf16, head dim 64 or 128).  The backward call also fills Dbuf with rowsum(dO * O).
int k_attn_fwd_mfma(hipStream_t st, const void* qkv, void* o, float* lse, int B, int S, int h, int dh);
int k_attn_bwd_mfma(hipStream_t st, const void* qkv, const void* o, const float* lse, const void* dO, void* dqkv, float* Dbuf,
                    int B, int S, int h, int dh,
                    const float* rope_cos, const float* rope_sin);          // tables given: dq, dk come out w.r.t. the un-rotated q, k

}  // namespace pp

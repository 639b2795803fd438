// bf16 MFMA GEMM for gfx950 with the contraction index as the ROW index of both operands ("TN"):
//     C[M x N] (fp32) = A^T B,   A: [K x M] row-major (lda),  B: [K x N] row-major (ldb).
// This is the weight-gradient form of the local step (Appendix "Partial Backward": dW_n = dH_n X^T, dV_n = G A_n^T in the
// paper's features x tokens convention): K runs over tokens, and both operands are activations stored token-major, i.e.
// exactly as the forward and backward passes leave them.  No transposed copies are made: tiles go from global memory to
// LDS as they are ([k][m], rows of 256 bytes), and the MFMA operand fragments -- 8 consecutive k for one m -- are
// gathered by the LDS transpose read (ds_read_b64_tr_b16), two per fragment.
//
// Transpose read, 16-bit elements: within each group of 16 lanes, lane i receives element i % 4 of the four 8-byte
// pieces addressed by lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12.  If lane j points at T[k0 + j/4][m0 + 4 (j % 4)], lane i
// therefore gets T[k0 .. k0+3][m0 + i]: four consecutive k of one column.
//
// Tiling: 128 x 128 output tile per workgroup of 256 threads (4 waves, 2 x 2, each 64 x 64 = 2 x 2 blocks of
// v_mfma_f32_32x32x16_bf16, 64 accumulator registers); K advances in steps of 64 rows; two LDS stages of 16 KB per
// operand (64 KB per workgroup, two workgroups per compute unit), the next step's tiles in flight while the current one
// is multiplied, one barrier per step.  (A ring of four 32-row stages with three steps in flight was measured slower on
// every shape: the cost per step is the barrier and the first fragment reads behind it, not the loads.)  Within a step the
// fragment registers are double-buffered: the transpose reads of the next 16-row slice are slotted between the MFMAs of
// the current one.  Tiles are filled by direct-to-LDS loads (one wave
// load = 4 rows); the 16-byte chunk c of row r is stored at chunk c ^ ((r & 3) << 2), applied on the source side, so
// that the 4 rows x 2 x 32 bytes touched by one phase of a transpose read fall into 8 different 32-byte bank groups.
// Few output tiles and a long K: the K range is split over blockIdx.y; partial products are summed in fixed order by
// the caller (k_splitk_reduce), so the result is reproducible run to run.
#include "pp_kernels.h"
#include "pp_dev.h"

namespace pp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

constexpr int TN_BM = 128, TN_BN = 128, TN_BK = 64;
constexpr int TN_OPERAND_BYTES = TN_BK * 256;                 // 64 rows of 128 elements
constexpr int TN_STAGE_BYTES = 2 * TN_OPERAND_BYTES;          // A tile, then B tile
constexpr int TN_LDS_BYTES = 2 * TN_STAGE_BYTES;

#define PP_TN_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define PP_TN_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

// A's columns may come in blocks: column m of the product is column (m / m_blk) * a_blk_stride + m % m_blk of A
// (gate and up gradients of a hidden-unit slice sit d_ff columns apart; the Q, K, V parts of a head range d_model apart).
// A tile never straddles two blocks (the launcher requires m_blk % 128 == 0 whenever M > m_blk).
__global__ __launch_bounds__(256, 2) void gemm_tn_mfma_kernel(const bf16_t* __restrict__ A, int lda, int m_blk, long a_blk_stride,
                                                               const bf16_t* __restrict__ B, int ldb, float* __restrict__ C, int ldc,
                                                               int M, int N, int Ksplit, int tiles_m, int tiles_n) {
  extern __shared__ __align__(16) unsigned char tn_lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  // Workgroup id -> (K range z, tile).  The hardware deals workgroups to the 8 XCDs round-robin by id; XCD k = id % 8 is
  // given a contiguous range of the (z, tile) list (z slowest), so that with 8 or more K ranges an XCD reads only its own
  // rows of A and B (they then sit in that XCD's L2 for all the tiles that share them), and with fewer it works on
  // neighbouring tiles (groups of 8 M-tiles by all N-tiles) that share panels.
  const int tiles = tiles_m * tiles_n, nb = tiles * (int)gridDim.y;
  int pid = blockIdx.y * tiles + blockIdx.x;
  if ((nb & 7) == 0) pid = (pid & 7) * (nb >> 3) + (pid >> 3);
  const int z = pid / tiles, t = pid - z * tiles;
  constexpr int GROUP = 8;
  const int per_group = GROUP * tiles_n;
  const int group = t / per_group, first_m = group * GROUP;
  const int gsz = min(tiles_m - first_m, GROUP);
  const int in_group = t - group * per_group;
  const int tm = first_m + in_group % gsz, tn = in_group / gsz;
  const int m0 = tm * TN_BM, n0 = tn * TN_BN;
  const size_t kbase = (size_t)z * Ksplit;
  const int ns = Ksplit / TN_BK;

  // ---- direct-to-LDS fill: wave w moves wave-loads 4w .. 4w+3 of each operand tile; wave-load q = rows 4q .. 4q+3,
  // lane l -> row 4q + l/16, chunk position l%16, which receives source chunk (l%16) ^ ((row & 3) << 2).
  const int frow = lane >> 4;                                          // row within a wave-load (== row & 3)
  const int fchunk = (lane & 15) ^ (frow << 2);                        // source chunk of this lane
  const int a_valid = min(M, m0 + TN_BM) - m0, b_valid = min(N, n0 + TN_BN) - n0;          // columns of the tile that exist (multiples of 8)
  const int a_col = min(fchunk * 8, a_valid - 8), b_col = min(fchunk * 8, b_valid - 8);    // clamped: padded columns repeat the last chunk
  const long a_col0 = (long)(m0 / m_blk) * a_blk_stride + (m0 % m_blk);
  const bf16_t* gA = A + (kbase + (size_t)(wave * 16 + frow)) * lda + a_col0 + a_col;
  const bf16_t* gB = B + (kbase + (size_t)(wave * 16 + frow)) * ldb + n0 + b_col;
  auto issue = [&](int s, int stage) {          // K-step s into LDS stage `stage`: 8 loads per wave
    unsigned char* dst = tn_lds + stage * TN_STAGE_BYTES + wave * 4 * 1024;
    const size_t ka = (size_t)s * TN_BK * lda, kb = (size_t)s * TN_BK * ldb;
#pragma unroll
    for (int i = 0; i < 4; ++i) __builtin_amdgcn_global_load_lds(PP_TN_GPTR(gA + ka + (size_t)(4 * i) * lda), PP_TN_LPTR(dst + i * 1024), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_global_load_lds(PP_TN_GPTR(gB + kb + (size_t)(4 * i) * ldb), PP_TN_LPTR(dst + TN_OPERAND_BYTES + i * 1024), 16, 0, 0);
  };

  // ---- fragment addresses.  Lane l: j = l % 16 (position in its group of 16), grp = l / 16: column half grp & 1 of a
  // 32-column block, k half grp >> 1 of a 16-row MFMA step.  It points at row (j / 4) of a 4-row band, 8-byte piece
  // j % 4 of the 32-byte column segment: chunk (col / 8) ^ ((j / 4) << 2), byte 8 * (j & 1) within the chunk.
  const int j = lane & 15, grp = lane >> 4;
  auto frag_off = [&](int w_half, int blk) {          // byte offset inside an operand tile, for K-row 0 of the step
    const int col = w_half * 64 + blk * 32 + (grp & 1) * 16 + 4 * (j & 3);
    const int chunk = (col >> 3) ^ ((j >> 2) << 2);
    return ((grp >> 1) * 8 + (j >> 2)) * 256 + chunk * 16 + (j & 1) * 8;
  };
  const int offA0 = frag_off(wm, 0), offA1 = frag_off(wm, 1);
  const int offB0 = TN_OPERAND_BYTES + frag_off(wn, 0), offB1 = TN_OPERAND_BYTES + frag_off(wn, 1);
  auto frag = [&](const unsigned char* stage, int off, int kk) -> bf16x8 {          // 8 consecutive k (rows 16 kk + 8 (grp >> 1) ..) of one column
    const unsigned char* p = stage + off + kk * 16 * 256;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)PP_TN_LPTR(const_cast<unsigned char*>(p)));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)PP_TN_LPTR(const_cast<unsigned char*>(p + 4 * 256)));
    const s16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  bf16x8 fa[2][2], fb[2][2];
  auto read_frags = [&](int buf, const unsigned char* stage, int kk) {
    fa[buf][0] = frag(stage, offA0, kk); fa[buf][1] = frag(stage, offA1, kk);
    fb[buf][0] = frag(stage, offB0, kk); fb[buf][1] = frag(stage, offB1, kk);
  };
  auto mm = [&](int buf) {
    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][0], fb[buf][0], acc[0][0], 0, 0, 0);
    acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][0], fb[buf][1], acc[0][1], 0, 0, 0);
    acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][1], fb[buf][0], acc[1][0], 0, 0, 0);
    acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][1], fb[buf][1], acc[1][1], 0, 0, 0);
  };
  issue(0, 0);
  for (int s = 0; s < ns; ++s) {
    // this wave's loads of step s have landed; after the barrier everybody's have, and nobody reads the other stage any more
    __builtin_amdgcn_s_waitcnt(0x0070);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    if (s + 1 < ns) issue(s + 1, (s + 1) & 1);
    const unsigned char* stage = tn_lds + (s & 1) * TN_STAGE_BYTES;
    read_frags(0, stage, 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < TN_BK / 16; ++kk) {
      if (kk + 1 < TN_BK / 16) read_frags((kk + 1) & 1, stage, kk + 1);
      mm(kk & 1);
      if (kk + 1 < TN_BK / 16) {          // one MFMA, then two of the next slice's eight transpose reads, four times
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // ---- epilogue: element r of block (a, b) is row m0 + 64 wm + 32 a + 8 (r / 4) + 4 (lane / 32) + r % 4,
  //      column n0 + 64 wn + 32 b + lane % 32; 32 lanes store 128 consecutive bytes of one row
  float* Cz = C + (size_t)z * (size_t)M * (size_t)ldc;
  const int l32 = lane & 31, lh = lane >> 5;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int col = n0 + wn * 64 + b * 32 + l32;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * 64 + a * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
        if (row < M && col < N) Cz[(size_t)row * ldc + col] = acc[a][b][r];
      }
    }
}

// C[M x N] fp32 (ldc) = A^T B over K rows; splits > 1: `partial` receives [splits][M][N] (C is not written; the caller sums
// the partials in fixed order).  Returns 0 if launched, 1 if the shapes are not taken (nothing launched).
int k_gemm_tn_mfma(hipStream_t st, const void* A, int lda, int m_blk, long a_blk_stride, const void* B, int ldb, float* C, int ldc,
                   int M, int N, int K, int splits, float* partial) {
  if (M < 8 || N < 8 || (M & 7) || (N & 7) || (lda & 7) || (ldb & 7) || splits < 1 || K < 1) return 1;
  if (K % (splits * 64)) return 1;
  if (m_blk < 1 || (m_blk & 7) || (a_blk_stride & 7)) return 1;
  if (M > m_blk && (m_blk % TN_BM)) return 1;          // a tile must not straddle two column blocks of A
  if (((uintptr_t)A | (uintptr_t)B | (uintptr_t)C | (uintptr_t)partial) & 15) return 1;
  if (splits > 1 && !partial) return 1;
  static const bool ok = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_tn_mfma_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, TN_LDS_BYTES) == hipSuccess;
  if (!ok) return 1;
  const int tiles_m = (M + TN_BM - 1) / TN_BM, tiles_n = (N + TN_BN - 1) / TN_BN;
  dim3 grid(tiles_m * tiles_n, splits);
  float* out = splits > 1 ? partial : C;
  gemm_tn_mfma_kernel<<<grid, 256, TN_LDS_BYTES, st>>>((const bf16_t*)A, lda, m_blk, a_blk_stride, (const bf16_t*)B, ldb, out, splits > 1 ? N : ldc, M, N,
                                                       K / splits, tiles_m, tiles_n);
  return 0;
}

}  // namespace pp

// bf16 MFMA GEMM for gfx950, small-shape variant:  C[M x N] = A[M x K] * B[N x K]^T (+ R), both operands K-contiguous.
//
// The 256 x 256-tile kernel (one workgroup per compute unit, 160 KB of LDS) needs well over 256 tiles to fill the chip.
// The 125M-shape decoder (d_model 768) has projections with 32 x 3 = 96 such tiles for 256 compute units; for those this
// kernel cuts the output into 128 x 128 tiles: 256 threads = 4 waves (2 x 2), each 64 x 64 = 2 x 2 blocks of
// v_mfma_f32_32x32x16_bf16 (64 accumulator registers), K steps of 64, two LDS stages of 16 KB per operand (64 KB per
// workgroup, two workgroups per compute unit), tiles by direct-to-LDS loads, fragment registers double-buffered across the
// four 16-deep slices of a step.  LDS rows are 128 bytes = 8 chunks; chunk c of row r sits at c ^ ((r >> 1) & 7) (applied
// on the source side): the 16 rows of a fragment-read phase cover all 64 banks.
// The B panel is the MFMA's row operand, so an accumulator block is a 32 x 32 block of C^T: a lane owns output row
// lane % 32 and, per 4 consecutive registers, 4 consecutive columns -- stored (and the residual read) as 8-byte pieces.
// Workgroup ids are mapped so that the workgroups of one XCD (ids equal mod 8) work on neighbouring tiles.
#include "pp_kernels.h"
#include "pp_dev.h"

namespace pp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int S_BM = 128, S_BN = 128, S_BK = 64;
constexpr int S_OPERAND_BYTES = S_BM * 128;                 // 128 rows of 64 elements
constexpr int S_STAGE_BYTES = 2 * S_OPERAND_BYTES;          // A tile, then B tile
constexpr int S_LDS_BYTES = 2 * S_STAGE_BYTES;

#define PP_S_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define PP_S_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

template <int EPI>
__global__ __launch_bounds__(256, 2) void gemm_nt128_mfma_kernel(const bf16_t* __restrict__ A, int lda, const bf16_t* __restrict__ B, int ldb,
                                                                  bf16_t* __restrict__ C, int ldc, int M, int N, int K, const bf16_t* __restrict__ R,
                                                                  int tiles_m, int tiles_n) {
  extern __shared__ __align__(16) unsigned char s_lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  // XCD k = id % 8 owns a contiguous range of the tile list, ordered in groups of 8 M-tiles by all N-tiles
  const int nb = tiles_m * tiles_n;
  int pid = blockIdx.x;
  if ((nb & 7) == 0) pid = (pid & 7) * (nb >> 3) + (pid >> 3);
  constexpr int GROUP = 8;
  const int per_group = GROUP * tiles_n;
  const int group = pid / per_group, first_m = group * GROUP;
  const int gsz = min(tiles_m - first_m, GROUP);
  const int in_group = pid - group * per_group;
  const int tm = first_m + in_group % gsz, tn = in_group / gsz;
  const int m0 = tm * S_BM, n0 = tn * S_BN;
  const int ns = K / S_BK;

  // ---- direct-to-LDS fill: a wave-load is 8 rows of 128 bytes; wave w moves wave-loads 4w .. 4w+3 of each operand tile
  const int frow = lane >> 3;
  const bf16_t* gA[4];
  const bf16_t* gB[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = wave * 32 + i * 8 + frow;
    const int c = (lane & 7) ^ ((row >> 1) & 7);
    gA[i] = A + (size_t)min(m0 + row, M - 1) * lda + c * 8;
    gB[i] = B + (size_t)min(n0 + row, N - 1) * ldb + c * 8;
  }
  auto issue = [&](int s, int stage) {
    unsigned char* dst = s_lds + stage * S_STAGE_BYTES + wave * 4 * 1024;
    const size_t k = (size_t)s * S_BK;
#pragma unroll
    for (int i = 0; i < 4; ++i) __builtin_amdgcn_global_load_lds(PP_S_GPTR(gA[i] + k), PP_S_LPTR(dst + i * 1024), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) __builtin_amdgcn_global_load_lds(PP_S_GPTR(gB[i] + k), PP_S_LPTR(dst + S_OPERAND_BYTES + i * 1024), 16, 0, 0);
  };

  // ---- fragments: lane l reads, for row 32 blk + l % 32 of its wave's 64 rows, the 8 k-elements 16 kk + 8 (l / 32) ..
  const int l32 = lane & 31, lh = lane >> 5;
  auto frag = [&](const unsigned char* tile, int w_half, int blk, int kk) -> bf16x8 {
    const int row = w_half * 64 + blk * 32 + l32;
    const int chunk = (2 * kk + lh) ^ ((row >> 1) & 7);
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(tile + row * 128 + chunk * 16));
  };

  f32x16 acc[2][2];          // [A block][B block]: a 32 x 32 block of C^T (rows = output columns)
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

  bf16x8 fa[2][2], fb[2][2];
  auto read_frags = [&](int buf, const unsigned char* stage, int kk) {
    fa[buf][0] = frag(stage, wm, 0, kk); fa[buf][1] = frag(stage, wm, 1, kk);
    fb[buf][0] = frag(stage + S_OPERAND_BYTES, wn, 0, kk); fb[buf][1] = frag(stage + S_OPERAND_BYTES, wn, 1, kk);
  };
  auto mm = [&](int buf) {
    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[buf][0], fa[buf][0], acc[0][0], 0, 0, 0);
    acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[buf][1], fa[buf][0], acc[0][1], 0, 0, 0);
    acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[buf][0], fa[buf][1], acc[1][0], 0, 0, 0);
    acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[buf][1], fa[buf][1], acc[1][1], 0, 0, 0);
  };
  issue(0, 0);
  for (int s = 0; s < ns; ++s) {
    // this wave's loads of step s have landed; after the barrier everybody's have, and nobody reads the other stage any more
    __builtin_amdgcn_s_waitcnt(0x0070);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    if (s + 1 < ns) issue(s + 1, (s + 1) & 1);
    const unsigned char* stage = s_lds + (s & 1) * S_STAGE_BYTES;
    read_frags(0, stage, 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < S_BK / 16; ++kk) {
      if (kk + 1 < S_BK / 16) read_frags((kk + 1) & 1, stage, kk + 1);
      mm(kk & 1);
      if (kk + 1 < S_BK / 16) {          // one MFMA, then one of the next slice's four fragment reads, four times
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // ---- epilogue: registers 4g .. 4g+3 of block (a, b) are output row m0 + 64 wm + 32 a + lane % 32, columns
  //      n0 + 64 wn + 32 b + 8 g + 4 (lane / 32) .. + 3
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    const int row = m0 + wm * 64 + a * 32 + l32;
    if (row >= M) continue;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = n0 + wn * 64 + b * 32 + 8 * g + 4 * lh;
        if (col >= N) continue;          // N is a multiple of 4: a piece is inside or outside as a whole
        const size_t off = (size_t)row * ldc + col;
        float v[4] = {acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2], acc[a][b][4 * g + 3]};
        if constexpr (EPI == EPI_ADD_RES) {
          const u32x2 rw = *reinterpret_cast<const u32x2*>(R + off);
          v[0] += __uint_as_float(rw[0] << 16); v[1] += __uint_as_float(rw[0] & 0xffff0000u);
          v[2] += __uint_as_float(rw[1] << 16); v[3] += __uint_as_float(rw[1] & 0xffff0000u);
        }
        u32x2 w;
        w[0] = f32x2_to_bf16x2(v[0], v[1]);
        w[1] = f32x2_to_bf16x2(v[2], v[3]);
        *reinterpret_cast<u32x2*>(C + off) = w;
      }
  }
}

template <int EPI>
static int launch128(hipStream_t st, const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K, const void* R) {
  static const bool ok = hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_nt128_mfma_kernel<EPI>), hipFuncAttributeMaxDynamicSharedMemorySize, S_LDS_BYTES) == hipSuccess;
  if (!ok) return 1;
  const int tiles_m = (M + S_BM - 1) / S_BM, tiles_n = (N + S_BN - 1) / S_BN;
  gemm_nt128_mfma_kernel<EPI><<<dim3(tiles_m * tiles_n), 256, S_LDS_BYTES, st>>>((const bf16_t*)A, lda, (const bf16_t*)B, ldb, (bf16_t*)C, ldc, M, N, K, (const bf16_t*)R,
                                                                                tiles_m, tiles_n);
  return 0;
}

// bf16 output, epi = EPI_STORE or EPI_ADD_RES (R with leading dimension ldc).  Returns 0 if launched, 1 if the shape is not
// taken (K % 64, N or ldc not multiples of 4, operand rows not 16-byte aligned).
int k_gemm_nt128_mfma(hipStream_t st, const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K, int epi, const void* R) {
  if (M < 1 || N < 4 || (N & 3) || (ldc & 3) || K < S_BK || K % S_BK || (lda & 7) || (ldb & 7)) return 1;
  if (((uintptr_t)A | (uintptr_t)B) & 15) return 1;
  if (((uintptr_t)C | (uintptr_t)R) & 7) return 1;
  if (epi == EPI_ADD_RES) return R ? launch128<EPI_ADD_RES>(st, A, lda, B, ldb, C, ldc, M, N, K, R) : 1;
  if (epi == EPI_STORE) return launch128<EPI_STORE>(st, A, lda, B, ldb, C, ldc, M, N, K, nullptr);
  return 1;
}

}  // namespace pp

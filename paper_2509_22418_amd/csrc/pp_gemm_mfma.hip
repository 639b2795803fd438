// bf16 MFMA GEMM for gfx950:  C[M x N] = A[M x K] * B[N x K]^T  (both operands K-contiguous), fp32 accumulate.
//
// Every dense contraction of the local step is brought into this one form (forward projections use the weights
// as stored, input-gradient GEMMs use transposed read-only weight copies, weight-gradient GEMMs use transposed
// activations with the token dimension as K), so this is the kernel that carries the step's FLOPs.
//
// Two kernels share this file: the register-staged one described next (variant 0, kept selectable) and the
// direct-to-LDS one further down (variant 1, the default; its own comment states what differs: whole-line DMA units,
// a five-slot ring, 16 x 16 x 32 MFMAs, a tile walk with cross-tile prefetch, fused SwiGLU epilogues).
//
// Tiling: 256 x 256 output tile per workgroup of 512 threads = 8 wavefronts (2 per SIMD) arranged 2 (M) x 4 (N);
// each wavefront owns 128 x 64 = 4 x 2 MFMA tiles of v_mfma_f32_32x32x16_bf16 (128 accumulator registers).
// K advances in steps of 64: the A and B panels (256 x 64 bf16 each, 32 KB + 32 KB) are staged in LDS, two stages
// (128 KB of the CU's 160 KB); global loads run two K steps ahead in registers (see the staging comment below).
// LDS rows are 128 bytes = 8 chunks of 16 bytes; chunk c of row r is stored at chunk c ^ ((r >> 1) & 7): a 16-byte
// fragment read is served 16 lanes (= 16 consecutive rows, same logical chunk) at a time, and with this swizzle those
// 16 addresses cover all 64 four-byte banks exactly once (rows r and r+1 differ in address bit 7, rows r and r+2k in
// the chunk).
// Workgroup ids are remapped so that the workgroups resident on one XCD (ids equal mod 8) work on neighbouring
// tiles (shared A / B panels hit that XCD's L2), in groups of 8 M-tiles by all N-tiles.
#include "pp_kernels.h"
#include "pp_dev.h"

#include <atomic>
#include <mutex>

namespace pp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int STAGE_CHUNKS = (BM + BN) * 8;          // 16-byte chunks per stage
constexpr int GEMM_LDS_BYTES = 2 * STAGE_CHUNKS * 16;

template <int EPI, bool OUT_F32>
__global__ __launch_bounds__(512) void gemm_nt_mfma_kernel(const bf16_t* __restrict__ A, int lda, const bf16_t* __restrict__ B, int ldb,
                                                            void* Cv, int ldc, int M, int N, int Ksplit, const bf16_t* __restrict__ R,
                                                            int tiles_m, int tiles_n) {
  extern __shared__ u32x4 lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;

  // ---- tile assignment (XCD-aware remap, then grouped ordering)
  const int nb = tiles_m * tiles_n;
  int pid = blockIdx.x;
  if ((nb & 7) == 0) pid = (pid & 7) * (nb >> 3) + (pid >> 3);
  constexpr int GROUP = 8;
  const int per_group = GROUP * tiles_n;
  const int group = pid / per_group;
  const int first_m = group * GROUP;
  const int gsz = min(tiles_m - first_m, GROUP);
  const int in_group = pid - group * per_group;
  const int tm = first_m + in_group % gsz, tn = in_group / gsz;
  const int m0 = tm * BM, n0 = tn * BN;
  const int z = blockIdx.y;
  const size_t kbase = (size_t)z * Ksplit;

  // ---- global -> register -> LDS staging: each thread moves 4 chunks of A and 4 chunks of B per K step.
  // Two register sets: the loads for K step kt+2 are issued while step kt is multiplied (an L2 miss then has two
  // steps to land), and the set holding step kt+1 is written to the free LDS stage in between the MFMA groups.
  const int lrow = tid >> 3, lc = tid & 7;
  const bf16_t* gA[4];
  const bf16_t* gB[4];
  int sOff[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = lrow + 64 * i;
    gA[i] = A + (size_t)min(m0 + row, M - 1) * lda + kbase + lc * 8;
    gB[i] = B + (size_t)min(n0 + row, N - 1) * ldb + kbase + lc * 8;
    sOff[i] = row * 8 + (lc ^ ((row >> 1) & 7));
  }
  const int nk = Ksplit / BK;
  u32x4 r0a[4], r0b[4], r1a[4], r1b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) { r0a[i] = *reinterpret_cast<const u32x4*>(gA[i]); r0b[i] = *reinterpret_cast<const u32x4*>(gB[i]); }
  const size_t k1 = (size_t)min(1, nk - 1) * BK;
#pragma unroll
  for (int i = 0; i < 4; ++i) { r1a[i] = *reinterpret_cast<const u32x4*>(gA[i] + k1); r1b[i] = *reinterpret_cast<const u32x4*>(gB[i] + k1); }
#pragma unroll
  for (int i = 0; i < 4; ++i) { lds[sOff[i]] = r0a[i]; lds[BM * 8 + sOff[i]] = r0b[i]; }
  __syncthreads();

  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int l32 = lane & 31, lhi = lane >> 5, sw = (lane >> 1) & 7;
  const int aRow = (wm * 128 + l32) * 8, bRow = BM * 8 + (wn * 64 + l32) * 8;
  auto kstep = [&](int cur, int s) {          // one 16-deep slice of the staged panels: 6 fragment reads, 8 MFMAs
    const int pc = (2 * s + lhi) ^ sw;
    bf16x8 af[4], bfr[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) af[i] = __builtin_bit_cast(bf16x8, lds[cur + aRow + i * 32 * 8 + pc]);
#pragma unroll
    for (int j = 0; j < 2; ++j) bfr[j] = __builtin_bit_cast(bf16x8, lds[cur + bRow + j * 32 * 8 + pc]);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
  };
  // One K step: multiply step kt from stage kt&1; load step kt+2 into (la, lb); write step kt+1, held in (wa, wb), to
  // the other stage.  Past the end the loads re-read the last step and the writes land in a stage nobody reads again.
#define PP_GEMM_ITER(kt, la, lb, wa, wb)                                                              \
  {                                                                                                   \
    const int cur = ((kt) & 1) * STAGE_CHUNKS, nxt = (((kt) + 1) & 1) * STAGE_CHUNKS;                 \
    const size_t k2 = (size_t)min((kt) + 2, nk - 1) * BK;                                             \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                   \
      la[i] = *reinterpret_cast<const u32x4*>(gA[i] + k2);                                            \
      lb[i] = *reinterpret_cast<const u32x4*>(gB[i] + k2);                                            \
    }                                                                                                 \
    __builtin_amdgcn_sched_barrier(0);                                                                \
    kstep(cur, 0);                                                                                    \
    __builtin_amdgcn_sched_barrier(0);                                                                \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) lds[nxt + sOff[i]] = wa[i];                         \
    kstep(cur, 1);                                                                                    \
    __builtin_amdgcn_sched_barrier(0);                                                                \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) lds[nxt + BM * 8 + sOff[i]] = wb[i];                \
    kstep(cur, 2);                                                                                    \
    __builtin_amdgcn_sched_barrier(0);                                                                \
    kstep(cur, 3);                                                                                    \
    __syncthreads();                                                                                  \
  }
  int kt = 0;
  for (; kt + 1 < nk; kt += 2) {
    PP_GEMM_ITER(kt, r0a, r0b, r1a, r1b)
    PP_GEMM_ITER(kt + 1, r1a, r1b, r0a, r0b)
  }
  if (kt < nk) PP_GEMM_ITER(kt, r0a, r0b, r1a, r1b)
#undef PP_GEMM_ITER

  // ---- epilogue: accumulator element r of MFMA tile (i, j) is row 8*(r/4) + 4*(lane/32) + r%4, column lane%32
  const int col_base = n0 + wn * 64 + l32;
  const int row_base = m0 + wm * 128 + 4 * lhi;
  if constexpr (OUT_F32) {
    float* C = reinterpret_cast<float*>(Cv) + (size_t)z * (size_t)M * (size_t)ldc;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int col = col_base + j * 32;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = row_base + i * 32 + 8 * (r >> 2) + (r & 3);
          if (row < M && col < N) C[(size_t)row * ldc + col] = acc[i][j][r];
        }
      }
  } else {
    bf16_t* C = reinterpret_cast<bf16_t*>(Cv);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int col = col_base + j * 32;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = row_base + i * 32 + 8 * (r >> 2) + (r & 3);
          if (row < M && col < N) {
            float v = acc[i][j][r];
            if constexpr (EPI == EPI_ADD_RES) v += to_f32(R[(size_t)row * ldc + col]);
            C[(size_t)row * ldc + col] = from_f32<bf16_t>(v);
          }
        }
      }
  }
}


// ------------------------------------------------------------------------------------------ direct-to-LDS variant
// Same 256 x 256 tile and wave layout, but the panels go from global memory straight into LDS
// (global_load_lds_dwordx4: lane l's 16 bytes land at M0 base + 16 l), no staging registers and no LDS write
// instructions.  The unit of transfer is 256 rows x 64 K-elements of ONE panel (32 KB): every row piece is a whole
// 128-byte cache line, which matters because a compute unit can only keep a limited number of line requests in flight
// -- half-line requests (a 32-deep K step of both panels) were measured to cap the kernel at about 2/3 of the speed
// of this arrangement.  K advances in super-steps of 64 that consume one A unit and one B unit; five unit slots
// (160 KB) form a ring, unit u = 2s (A of super-step s) or 2s+1 (B) living in slot u % 5.  During super-step s the B
// unit of s+1 and then the A unit of s+2 are requested, so every unit has at least a whole super-step of matrix
// work to arrive, and a single barrier per super-step both publishes the arrivals and frees the two consumed slots.  LDS rows are 128 bytes = 8 chunks; a wave-load fills 8 consecutive rows; chunk c of row r
// sits at chunk c ^ ((r >> 1) & 7) (the permutation is applied on the source side), which spreads the 16 rows of a
// fragment-read phase over all 64 banks.
constexpr int DL_BK = 64, DL_SLOTS = 5;
constexpr int DL_UNIT_CHUNKS = 256 * 8;
constexpr int DL_LDS_BYTES = DL_SLOTS * DL_UNIT_CHUNKS * 16;
static_assert(BM == 256 && BN == 256, "unit geometry assumes 256-row panels");
#define PP_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define PP_LPTR(p) ((__attribute__((address_space(3))) void*)(p))

template <int EPI, bool OUT_F32>
__global__ __launch_bounds__(512) void gemm_nt_mfma_dl_kernel(const bf16_t* __restrict__ A, int lda, const bf16_t* __restrict__ B, int ldb,
                                                               void* Cv, int ldc, int M, int N, int Ksplit, const bf16_t* __restrict__ R,
                                                               int tiles_m, int tiles_n, int ldc2,
                                                               const float* __restrict__ aux0, const float* __restrict__ aux1, int aux_n, int aux_s) {
  // EPI_ROPE only: ldc2 = head dim, aux0 / aux1 = cos / sin tables [aux_s x head dim / 2], aux_n = number of leading output
  // columns that are rotated (q and k), aux_s = sequence length (position of row t is t % aux_s)
  extern __shared__ u32x4 lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;
  const int nb = tiles_m * tiles_n;
  const int z = blockIdx.y;
  const size_t kbase = (size_t)z * Ksplit;
  // Tile walk.  The grid's x extent may be smaller than the number of tiles: workgroup b then takes the tiles b,
  // b + gridDim.x, ... one after the other (gridDim.x is a multiple of 8 in that case, so a workgroup's tiles all map to
  // its own XCD below), and requests the first three units of its next tile before it starts the epilogue of the
  // current one, so that neither the launch of a new workgroup nor the first trip to memory separates two tiles.
  auto tile_of = [&](int vb, int& tm, int& tn) {
    int pid = vb;
    if ((nb & 7) == 0) pid = (pid & 7) * (nb >> 3) + (pid >> 3);          // XCD k = id % 8 owns a contiguous range of tiles
    constexpr int GROUP = 8;
    const int per_group = GROUP * tiles_n;
    const int group = pid / per_group;
    const int first_m = group * GROUP;
    const int gsz = min(tiles_m - first_m, GROUP);
    const int in_group = pid - group * per_group;
    tm = first_m + in_group % gsz;
    tn = in_group / gsz;
  };
  // wave w fills rows 32w .. 32w+31 of a unit with four loads of 8 rows (8 lanes per 128-byte row) each
  const bf16_t* gA[4];
  const bf16_t* gB[4];
  auto set_ptrs = [&](int tm, int tn) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = wave * 32 + i * 8 + (lane >> 3);
      const int c = (lane & 7) ^ ((row >> 1) & 7);
      gA[i] = A + (size_t)min(tm * BM + row, M - 1) * lda + kbase + c * 8;
      if constexpr (EPI == EPI_SWIGLU) {
        // panel rows 64q .. 64q+31 are rows of W_g, 64q+32 .. 64q+63 the same hidden units' rows of W_u (N = d_ff,
        // B = [W_g; W_u]): a wave's 64 output columns then hold gate and up of 32 units in matching registers
        const int unit = min(tn * (BN / 2) + (row >> 6) * 32 + (row & 31), N - 1);
        gB[i] = B + ((size_t)((row >> 5) & 1) * N + unit) * ldb + kbase + c * 8;
      } else if constexpr (EPI == EPI_ROPE) {
        // rotated columns: panel rows 64 w .. 64 w + 31 are 32 first-half elements i of one head, rows 64 w + 32 .. + 63 their
        // partners i + dh/2, so that a lane's accumulators (i, j) and (i, j + 2) hold the two members of a rotary pair
        int col = tn * BN + row;
        if (tn * BN < aux_n) {
          const int half = ldc2 >> 1, wph = half >> 5, wv = row >> 6, q = row & 63;
          col = tn * BN + (wv / wph) * ldc2 + (wv % wph) * 32 + (q & 31) + (q >> 5) * half;
        }
        gB[i] = B + (size_t)min(col, N - 1) * ldb + kbase + c * 8;
      } else {
        gB[i] = B + (size_t)min(tn * BN + row, N - 1) * ldb + kbase + c * 8;
      }
    }
  };
  const int wdst = wave * 32 * 8;          // chunk offset of this wave's rows inside a unit (wave-uniform)
  const int ns = Ksplit / DL_BK;
  auto issue = [&](const bf16_t* const (&g)[4], int s, int slot) {          // unit of super-step s (clamped) into `slot`
    const size_t koff = (size_t)min(s, ns - 1) * DL_BK;
    u32x4* dst = lds + slot * DL_UNIT_CHUNKS + wdst;
#pragma unroll
    for (int i = 0; i < 4; ++i) __builtin_amdgcn_global_load_lds(PP_GPTR(g[i] + koff), PP_LPTR(dst + i * 64), 16, 0, 0);
  };
  auto m5 = [](int x) { return x >= DL_SLOTS ? x - DL_SLOTS : x; };

  const int l16 = lane & 15, lq = lane >> 4, sw = (l16 >> 1) & 7;          // row in a 16-row block, 16-byte chunk within a 64-byte K32 piece
  const int aRow = (wm * 128 + l16) * 8, bRow = (wn * 64 + l16) * 8;
  // The epilogues turn the accumulators around in LDS patches of 8 KB per wave that live in ring slots 3 and 4, so that
  // slots 0..2 can already receive the next tile's first units.
  char* const wbase = reinterpret_cast<char*>(lds) + 3 * DL_UNIT_CHUNKS * 16 + wave * 8192;

  int vb = blockIdx.x, tm, tn;
  tile_of(vb, tm, tn);
  set_ptrs(tm, tn);
  issue(gA, 0, 0); issue(gB, 0, 1); issue(gA, 1, 2);
  // Plain s_barrier (no fence): a workgroup fence would force vmcnt(0), i.e. wait for ALL loads in flight.  The only
  // LDS traffic here is DMA writes (tracked by vmcnt) and fragment reads (consumed by MFMAs before the barrier).
  __builtin_amdgcn_s_waitcnt(0x0F70 | 4);          // vmcnt(4): both units of super-step 0 have landed
  for (;;) {
  const int m0 = tm * BM, n0 = tn * BN;
  __builtin_amdgcn_s_barrier();

  // 16 x 16 x 32 MFMAs: on non-trivial operand data the matrix pipe is power-limited, and this shape sustains about
  // 14 % more than 32 x 32 x 16 (2.1 vs 1.85 PFLOP/s in an MFMA-only loop on random bf16 operands; both reach 2.4 on zeros).
  // B-panel rows are the MFMA's row operand, so an accumulator tile is a 16 x 16 block of C^T: lane l holds, for output
  // row (lane % 16) of A-block i, the 4 consecutive columns 4 * (lane / 16) .. + 3 of B-block j.
  f32x4 acc[8][4];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;

  // A super-step of 64 K-elements = 2 MFMA K-steps of 32 = 4 slices of 16 MFMAs (one K-step x one half of the wave's 8 row
  // blocks of A).  Fragment registers are double-buffered: the reads of the next slice (4 A fragments, plus the 4 B
  // fragments when the K-step changes) are slotted between the MFMAs of the current one.
  bf16x8 fa[2][4], fb[2][4];
  auto readA = [&](int buf, int slot, int kk, int half) {
    const u32x4* pa = lds + slot * DL_UNIT_CHUNKS + aRow + ((4 * kk + lq) ^ sw);
#pragma unroll
    for (int i = 0; i < 4; ++i) fa[buf][i] = __builtin_bit_cast(bf16x8, pa[(half * 4 + i) * 16 * 8]);
  };
  auto readB = [&](int buf, int slot, int kk) {
    const u32x4* pb = lds + slot * DL_UNIT_CHUNKS + bRow + ((4 * kk + lq) ^ sw);
#pragma unroll
    for (int j = 0; j < 4; ++j) fb[buf][j] = __builtin_bit_cast(bf16x8, pb[j * 16 * 8]);
  };
  auto mm = [&](int abuf, int bbuf, int half) {          // the 16 MFMAs of one slice
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[half * 4 + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[bbuf][j], fa[abuf][i], acc[half * 4 + i][j], 0, 0, 0);
  };
  // R fragment reads behind the first MFMAs of a slice of 16 (the in-order LDS counter then never makes this slice's
  // MFMAs wait for the next slice's reads)
#define PP_DL_INTERLEAVE(ID, R)                                              \
  _Pragma("unroll") for (int g = 0; g < (R); ++g) {                         \
    __builtin_amdgcn_sched_group_barrier(0x008, (R) == 4 ? 2 : 1, ID);       \
    __builtin_amdgcn_sched_group_barrier(0x100, 1, ID);                      \
  }                                                                          \
  __builtin_amdgcn_sched_group_barrier(0x008, 8, ID);                        \
  __builtin_amdgcn_sched_barrier(0)

  int sa = 0;          // slot of the A unit of the current super-step; its B unit is in the next slot of the ring
  readB(0, 1, 0);
  readA(0, 0, 0, 0);
  for (int s = 0; s < ns; ++s) {
    const int sb = m5(sa + 1), na = m5(sa + 2), nb2 = m5(sa + 3), fa2 = m5(sa + 4);
    issue(gB, s + 1, nb2);          // slot of A(s-1): free since the barrier that ended super-step s-1
    __builtin_amdgcn_sched_barrier(0);
    readA(1, sa, 0, 1);
    mm(0, 0, 0);
    PP_DL_INTERLEAVE(0, 4);
    readB(1, sb, 1);
    readA(0, sa, 1, 0);
    mm(1, 0, 1);
    PP_DL_INTERLEAVE(1, 8);
    issue(gA, s + 2, fa2);          // slot of B(s-1)
    __builtin_amdgcn_sched_barrier(0);
    readA(1, sa, 1, 1);
    mm(0, 1, 0);
    PP_DL_INTERLEAVE(2, 4);
    // vmcnt(4): all but the newest unit, i.e. both units of super-step s+1, have landed in this wave's rows;
    // lgkmcnt(0): this wave's reads of the current units are done
    __builtin_amdgcn_s_waitcnt(0x0070 | 4);
    __builtin_amdgcn_s_barrier();          // everybody's super-step s+1 is in LDS; the two current slots may be refilled
    readB(0, nb2, 0);
    readA(0, na, 0, 0);
    mm(1, 1, 1);
    PP_DL_INTERLEAVE(3, 8);
    sa = na;
  }
#undef PP_DL_INTERLEAVE
  // drain the clamped tail loads (and the fragment reads issued for a super-step that does not exist) and meet: after
  // this barrier nobody reads the staged panels any more and nothing is on its way into them
  __builtin_amdgcn_s_waitcnt(0x0070);
  __builtin_amdgcn_s_barrier();
  const int vb_next = vb + gridDim.x;
  const bool has_next = vb_next < nb;
  int tm_next = 0, tn_next = 0;
  if (has_next) {
    tile_of(vb_next, tm_next, tn_next);
    set_ptrs(tm_next, tn_next);
    issue(gA, 0, 0); issue(gB, 0, 1); issue(gA, 1, 2);
  }
  __builtin_amdgcn_sched_barrier(0);

  // ---- epilogue: element r of accumulator (i, j) is output row m0 + wm*128 + 16 i + lane % 16,
  //      column n0 + wn*64 + 16 j + 4 (lane / 16) + r
  bool stored = false;
  if constexpr (EPI == EPI_SWIGLU) {
    // ---- fused SwiGLU epilogue.  acc[i][j] (j = 0, 1) and acc[i][j + 2] are gate and up pre-activations of hidden unit
    // u0 + 16 j + 4 (lane / 16) + r (u0 = tn*128 + wn*32) for output row m0 + wm*128 + 16 i + lane % 16.  Both are
    // rounded to bf16 and stored at columns u and N + u of C (ldc >= 2 N); a = silu(g) * u is formed from the ROUNDED
    // values -- exactly what a separate pass over the stored matrix would compute -- and stored at column u of C2.
    // Each wave turns 32 rows at a time around in its LDS patch (32 rows x 256 bytes: gate | up | a | unused,
    // 16-byte piece p of row r at p ^ (r & 15)), so that 4 lanes cover one 64-byte row segment of each output.
    bf16_t* C = reinterpret_cast<bf16_t*>(Cv);
    bf16_t* C2 = const_cast<bf16_t*>(R);
    const int u0 = tn * (BN / 2) + wn * 32;
#pragma unroll
    for (int qt = 0; qt < 4; ++qt) {
#pragma unroll
      for (int ii = 0; ii < 2; ++ii) {
        const int i = 2 * qt + ii, row = ii * 16 + l16;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          uint2 wg, wu, wa;
          wg.x = f32x2_to_bf16x2(acc[i][j][0], acc[i][j][1]);
          wg.y = f32x2_to_bf16x2(acc[i][j][2], acc[i][j][3]);
          wu.x = f32x2_to_bf16x2(acc[i][j + 2][0], acc[i][j + 2][1]);
          wu.y = f32x2_to_bf16x2(acc[i][j + 2][2], acc[i][j + 2][3]);
          const float gr[4] = {__uint_as_float(wg.x << 16), __uint_as_float(wg.x & 0xffff0000u), __uint_as_float(wg.y << 16), __uint_as_float(wg.y & 0xffff0000u)};
          const float ur[4] = {__uint_as_float(wu.x << 16), __uint_as_float(wu.x & 0xffff0000u), __uint_as_float(wu.y << 16), __uint_as_float(wu.y & 0xffff0000u)};
          float av[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) av[e] = silu_mul(gr[e], ur[e]);
          wa.x = f32x2_to_bf16x2(av[0], av[1]);
          wa.y = f32x2_to_bf16x2(av[2], av[3]);
          // units 16 j + 4 lq .. + 3 of the wave's 32: 8-byte piece 4 j + lq of the 64-byte segment = 16-byte piece 2 j + lq / 2, half lq % 2
          const int pc = 2 * j + (lq >> 1);
          char* rowp = wbase + row * 256 + (lq & 1) * 8;
          *reinterpret_cast<uint2*>(rowp + (((0 + pc) ^ (row & 15)) << 4)) = wg;
          *reinterpret_cast<uint2*>(rowp + (((4 + pc) ^ (row & 15)) << 4)) = wu;
          *reinterpret_cast<uint2*>(rowp + (((8 + pc) ^ (row & 15)) << 4)) = wa;
        }
      }
#pragma unroll
      for (int it = 0; it < 4; ++it) {          // gate and up: 8 pieces per row, 8 rows per wave instruction
        const int row = 8 * it + (lane >> 3), pc = lane & 7;
        const uint4 v = *reinterpret_cast<const uint4*>(wbase + row * 256 + ((pc ^ (row & 15)) << 4));
        const int grow = m0 + wm * 128 + qt * 32 + row, unit = u0 + (pc & 3) * 8;
        if (grow < M && unit < N) *reinterpret_cast<uint4*>(C + (size_t)grow * ldc + (size_t)(pc >> 2) * N + unit) = v;
      }
#pragma unroll
      for (int it = 0; it < 2; ++it) {          // a: 4 pieces per row, 16 rows per wave instruction
        const int row = 16 * it + (lane >> 2), pc = 8 + (lane & 3);
        const uint4 v = *reinterpret_cast<const uint4*>(wbase + row * 256 + ((pc ^ (row & 15)) << 4));
        const int grow = m0 + wm * 128 + qt * 32 + row, unit = u0 + (lane & 3) * 8;
        if (grow < M && unit < N) *reinterpret_cast<uint4*>(C2 + (size_t)grow * ldc2 + unit) = v;
      }
    }
    stored = true;
  } else if constexpr (!OUT_F32) {
    if ((N & 7) == 0 && (ldc & 7) == 0) {          // uniform: coalesced path through LDS
      // Each wave turns its 128 x 64 sub-tile around in its LDS patch: 8-byte pieces (4 consecutive columns of one row)
      // are written, 16-byte row chunks are read back so that 8 lanes cover one 128-byte row segment of C (and of the
      // residual).
      bf16_t* C = reinterpret_cast<bf16_t*>(Cv);
      if (EPI == EPI_ROPE && n0 < aux_n) {
        // ---- rotary epilogue (q and k columns).  acc[i][j] (j = 0, 1) holds elements p0 + 16 j + 4 (lane / 16) + r of one
        // head's first half for output row m0 + wm*128 + 16 i + lane % 16, acc[i][j + 2] their partners dh/2 further on:
        // (x1, x2) -> (x1 cos - x2 sin, x1 sin + x2 cos) with the angle of (row % aux_s, element), in fp32, rounded once.
        // The two 64-byte segments go through the wave's LDS patch like the gate / up halves of the SwiGLU epilogue.
        // (the lane index is laundered through an empty asm so that the per-lane addresses below are formed here, once per
        // tile, instead of being hoisted above the main loop, where every register is taken, and spilled)
        int ln = lane;
        asm volatile("" : "+v"(ln));
        const int e16 = ln & 15, eq = ln >> 4;
        const int half = ldc2 >> 1, wph = half >> 5;
        const int p0 = (wn % wph) * 32;                                  // first pair of this wave within its head
        const int colbase = n0 + (wn / wph) * ldc2 + p0;                 // output column of that pair's first member
#pragma unroll
        for (int qt = 0; qt < 4; ++qt) {
#pragma unroll
          for (int ii = 0; ii < 2; ++ii) {
            const int i = 2 * qt + ii, row = ii * 16 + e16;
            const int pos = min(m0 + wm * 128 + 16 * i + e16, M - 1) % aux_s;
            const float* cp = aux0 + (size_t)pos * half + p0 + 4 * eq;
            const float* sp = aux1 + (size_t)pos * half + p0 + 4 * eq;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
              const float4 cs = *reinterpret_cast<const float4*>(cp + 16 * j), sn = *reinterpret_cast<const float4*>(sp + 16 * j);
              const float cv[4] = {cs.x, cs.y, cs.z, cs.w}, sv[4] = {sn.x, sn.y, sn.z, sn.w};
              float y1[4], y2[4];
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                const float x1 = acc[i][j][e], x2 = acc[i][j + 2][e];
                y1[e] = x1 * cv[e] - x2 * sv[e];
                y2[e] = x1 * sv[e] + x2 * cv[e];
              }
              uint2 w1, w2;
              w1.x = f32x2_to_bf16x2(y1[0], y1[1]); w1.y = f32x2_to_bf16x2(y1[2], y1[3]);
              w2.x = f32x2_to_bf16x2(y2[0], y2[1]); w2.y = f32x2_to_bf16x2(y2[2], y2[3]);
              const int pc = 2 * j + (eq >> 1);
              char* rowp = wbase + row * 256 + (eq & 1) * 8;
              *reinterpret_cast<uint2*>(rowp + (((0 + pc) ^ (row & 15)) << 4)) = w1;
              *reinterpret_cast<uint2*>(rowp + (((4 + pc) ^ (row & 15)) << 4)) = w2;
            }
          }
#pragma unroll
          for (int it = 0; it < 4; ++it) {          // 8 pieces per row (4 of each half), 8 rows per wave instruction
            const int row = 8 * it + (ln >> 3), pc = ln & 7;
            const uint4 v = *reinterpret_cast<const uint4*>(wbase + row * 256 + ((pc ^ (row & 15)) << 4));
            const int grow = m0 + wm * 128 + qt * 32 + row, gcol = colbase + (pc & 3) * 8 + (pc >> 2) * half;
            if (grow < M && gcol < N) *reinterpret_cast<uint4*>(C + (size_t)grow * ldc + gcol) = v;
          }
        }
      } else if constexpr (EPI == EPI_STORE || EPI == EPI_ROPE) {
        // 64 rows x 128 bytes (bf16) at a time; chunk c of row r sits at c ^ ((r >> 1) & 7)
#pragma unroll
        for (int hi = 0; hi < 2; ++hi) {
#pragma unroll
          for (int ii = 0; ii < 4; ++ii) {
            const int i = 4 * hi + ii, row = ii * 16 + l16, sw2 = (row >> 1) & 7;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const int q = 4 * j + lq;          // 8-byte piece index within the 128-byte row
              uint2 w;
              w.x = f32x2_to_bf16x2(acc[i][j][0], acc[i][j][1]);
              w.y = f32x2_to_bf16x2(acc[i][j][2], acc[i][j][3]);
              *reinterpret_cast<uint2*>(wbase + row * 128 + (((q >> 1) ^ sw2) << 4) + (q & 1) * 8) = w;
            }
          }
#pragma unroll
          for (int it = 0; it < 8; ++it) {
            const int row = 8 * it + (lane >> 3), c = lane & 7;
            const uint4 v = *reinterpret_cast<const uint4*>(wbase + row * 128 + ((c ^ ((row >> 1) & 7)) << 4));
            const int grow = m0 + wm * 128 + hi * 64 + row, gcol = n0 + wn * 64 + c * 8;
            if (grow < M && gcol < N) *reinterpret_cast<uint4*>(C + (size_t)grow * ldc + gcol) = v;
          }
        }
      } else {
        // residual add (or SwiGLU backward): the result is formed in fp32 and rounded once, so the patch holds floats
        // (32 rows x 256 bytes at a time, 16-byte piece p of row r at p ^ (r & 15)); 8 lanes then cover one 128-byte
        // row segment of R and of C with 16-byte accesses
#pragma unroll
        for (int qt = 0; qt < 4; ++qt) {
          // The saved operands of this quarter (R, and for the SwiGLU backward the second operand ldc2 columns further
          // on) are requested first, all 4 (8) 16-byte loads of the wave at once and from clamped addresses so that no branch
          // separates them: they travel while the accumulators are turned around in LDS, instead of one dependent
          // load -> compute -> store chain per row group.
          uint4 rr[4], ru[4];
#pragma unroll
          for (int it = 0; it < 4; ++it) {
            const int grow = min(m0 + wm * 128 + qt * 32 + 8 * it + (lane >> 3), M - 1);
            const int gcol = min(n0 + wn * 64 + (lane & 7) * 8, N - 8);
            const size_t off = (size_t)grow * ldc + gcol;
            rr[it] = *reinterpret_cast<const uint4*>(R + off);
            if constexpr (EPI == EPI_SWIGLU_BWD) ru[it] = *reinterpret_cast<const uint4*>(R + off + ldc2);
          }
#pragma unroll
          for (int ii = 0; ii < 2; ++ii) {
            const int i = 2 * qt + ii, row = ii * 16 + l16;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const int q = 4 * j + lq;          // 16-byte piece (4 floats) index within the 256-byte row
              *reinterpret_cast<float4*>(wbase + row * 256 + ((q ^ (row & 15)) << 4)) =
                  make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
            }
          }
#pragma unroll
          for (int it = 0; it < 4; ++it) {          // a lane takes 8 consecutive columns of a row: 8 lanes cover a 128-byte segment of R and C
            const int row = 8 * it + (lane >> 3), c = lane & 7;
            const float4 v0 = *reinterpret_cast<const float4*>(wbase + row * 256 + (((2 * c) ^ (row & 15)) << 4));
            const float4 v1 = *reinterpret_cast<const float4*>(wbase + row * 256 + (((2 * c + 1) ^ (row & 15)) << 4));
            const int grow = m0 + wm * 128 + qt * 32 + row, gcol = n0 + wn * 64 + c * 8;
            if (grow < M && gcol < N) {
              const size_t off = (size_t)grow * ldc + gcol;
              const float v[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
              const uint32_t rw[4] = {rr[it].x, rr[it].y, rr[it].z, rr[it].w};
              if constexpr (EPI == EPI_SWIGLU_BWD) {
                // the product is dL/da; R holds the saved gate at this column and the saved up ldc2 columns further on:
                // dg = da u sig(g) (1 + g (1 - sig(g))) and du = da g sig(g) go to the same two places of C
                const uint32_t uw[4] = {ru[it].x, ru[it].y, ru[it].z, ru[it].w};
                float dg[8], du[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                  const float gg = (e & 1) ? __uint_as_float(rw[e >> 1] & 0xffff0000u) : __uint_as_float(rw[e >> 1] << 16);
                  const float uu = (e & 1) ? __uint_as_float(uw[e >> 1] & 0xffff0000u) : __uint_as_float(uw[e >> 1] << 16);
                  const float sg = sigmoid_fast(gg);
                  du[e] = v[e] * gg * sg;
                  dg[e] = v[e] * uu * sg * (1.0f + gg * (1.0f - sg));
                }
                *reinterpret_cast<uint4*>(C + off) = make_uint4(f32x2_to_bf16x2(dg[0], dg[1]), f32x2_to_bf16x2(dg[2], dg[3]),
                                                                f32x2_to_bf16x2(dg[4], dg[5]), f32x2_to_bf16x2(dg[6], dg[7]));
                *reinterpret_cast<uint4*>(C + off + ldc2) = make_uint4(f32x2_to_bf16x2(du[0], du[1]), f32x2_to_bf16x2(du[2], du[3]),
                                                                       f32x2_to_bf16x2(du[4], du[5]), f32x2_to_bf16x2(du[6], du[7]));
              } else {
                uint32_t w[4];
#pragma unroll
                for (int e = 0; e < 4; ++e)
                  w[e] = f32x2_to_bf16x2(v[2 * e] + __uint_as_float(rw[e] << 16), v[2 * e + 1] + __uint_as_float(rw[e] & 0xffff0000u));
                *reinterpret_cast<uint4*>(C + off) = make_uint4(w[0], w[1], w[2], w[3]);
              }
            }
          }
        }
      }
      stored = true;
    }
  }
  if (!stored) {          // fp32 output (weight gradients, split-K partials) and shapes the vector paths do not take
    const int row_base = m0 + wm * 128 + l16;
    const int col_base = n0 + wn * 64 + 4 * lq;
    const bool n_vec_ok = (N % 4 == 0) && (ldc % 4 == 0);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = row_base + i * 16;
      if (row >= M) continue;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int col = col_base + j * 16;
        if (col >= N) continue;
        float v[4] = {acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]};
        if constexpr (OUT_F32) {
          float* C = reinterpret_cast<float*>(Cv) + (size_t)z * (size_t)M * (size_t)ldc + (size_t)row * ldc + col;
          if (n_vec_ok) *reinterpret_cast<float4*>(C) = make_float4(v[0], v[1], v[2], v[3]);
          else for (int e = 0; e < 4 && col + e < N; ++e) C[e] = v[e];
        } else {
          bf16_t* C = reinterpret_cast<bf16_t*>(Cv) + (size_t)row * ldc + col;
          for (int e = 0; e < 4 && col + e < N; ++e) {
            float x = v[e];
            if constexpr (EPI == EPI_ADD_RES) x += to_f32(R[(size_t)row * ldc + col + e]);
            C[e] = from_f32<bf16_t>(x);
          }
        }
      }
    }
  }
  if (!has_next) break;
  vb = vb_next; tm = tm_next; tn = tn_next;
  // the next tile's first units have landed, this wave's stores are acknowledged and its patch reads are done; the
  // barrier at the top of the loop publishes all of that before any wave refills slots 3 and 4
  __builtin_amdgcn_s_waitcnt(0x0070);
  }
}

// Process-wide test / A-B switches (relaxed atomics: a launch sees the value of the last completed setter call).
static std::atomic<int> g_gemm_variant{1};          // 0: register-staged kernel, 1: direct-to-LDS kernel (default: faster on every shape measured)
void gemm_set_variant(int v) { g_gemm_variant.store(v, std::memory_order_relaxed); }
static std::atomic<int> g_gemm_persistent{1};       // 1: one workgroup per compute unit walks several tiles (see the kernel's tile walk)
void gemm_set_persistent(int v) { g_gemm_persistent.store(v, std::memory_order_relaxed); }
static std::atomic<int> g_gemm_small_tiles{1};      // 1: few-tile GEMMs go to the 128 x 128-tile kernel
void gemm_set_small_tiles(int v) { g_gemm_small_tiles.store(v, std::memory_order_relaxed); }
// One-time opt-in of a kernel to more than 64 KB of dynamic LDS; safe when several host threads launch concurrently.
struct LdsOptIn {
  std::once_flag once;
  bool ok = false;
  bool operator()(const void* kern, int bytes) {
    std::call_once(once, [&] { ok = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) == hipSuccess; });
    return ok;
  }
};
// x extent of the grid for nb tiles: all of them, or one workgroup per compute unit when there are more tiles than units
static int dl_grid_x(int nb) {
  static const int ncu = [] {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) n = 0;
    return (n >= 8 && n % 8 == 0) ? n : 0;
  }();
  return (g_gemm_persistent.load(std::memory_order_relaxed) && ncu > 0 && nb > ncu) ? ncu : nb;
}

template <int EPI, bool OUT_F32>
static int launch_dl(hipStream_t st, const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int Ksplit, const void* R, int splits) {
  static LdsOptIn opt_in;
  auto kern = gemm_nt_mfma_dl_kernel<EPI, OUT_F32>;
  if (!opt_in(reinterpret_cast<const void*>(kern), DL_LDS_BYTES)) return 1;
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  dim3 grid(splits == 1 ? dl_grid_x(tiles_m * tiles_n) : tiles_m * tiles_n, splits);
  kern<<<grid, 512, DL_LDS_BYTES, st>>>((const bf16_t*)A, lda, (const bf16_t*)B, ldb, C, ldc, M, N, Ksplit, (const bf16_t*)R, tiles_m, tiles_n, 0, nullptr, nullptr, 0, 1);
  return 0;
}

// gu[M x 2F] (ld 2F) = X[M x K] [Wg; Wu]^T and a[M x F] = silu(gate) * up in one launch; Wgu = the 2F x K stack
int k_gemm_swiglu_fwd_mfma(hipStream_t st, const void* X, int ldx, const void* Wgu, int ldw, void* gu, void* a, int M, int F, int K) {
  if (g_gemm_variant.load(std::memory_order_relaxed) != 1 || M < 1 || F < 8 || (F & 7) || K < DL_BK || K % DL_BK || (ldx & 7) || (ldw & 7)) return 1;
  if (((uintptr_t)X | (uintptr_t)Wgu | (uintptr_t)gu | (uintptr_t)a) & 15) return 1;
  static LdsOptIn opt_in;
  auto kern = gemm_nt_mfma_dl_kernel<EPI_SWIGLU, false>;
  if (!opt_in(reinterpret_cast<const void*>(kern), DL_LDS_BYTES)) return 1;
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (F + BN / 2 - 1) / (BN / 2);
  kern<<<dim3(dl_grid_x(tiles_m * tiles_n), 1), 512, DL_LDS_BYTES, st>>>((const bf16_t*)X, ldx, (const bf16_t*)Wgu, ldw, gu, 2 * F, M, F, K, (const bf16_t*)a, tiles_m, tiles_n, F, nullptr, nullptr, 0, 1);
  return 0;
}

// dgu[M x 2F] (columns c .. and F + c ..) from dA = G Wd_rows^T without materialising dA: C = dgu + c0, R = gu + c0, both
// with leading dimension ld2f = 2F; N = number of hidden units (rows of Wd_rows), half = F
int k_gemm_swiglu_bwd_mfma(hipStream_t st, const void* G, int ldg, const void* Wd_rows, int ldw, const void* gu_c0, void* dgu_c0, int ld2f, int half,
                           int M, int N, int K) {
  if (g_gemm_variant.load(std::memory_order_relaxed) != 1 || M < 1 || N < 8 || (N & 7) || (ld2f & 7) || (half & 7) || K < DL_BK || K % DL_BK || (ldg & 7) || (ldw & 7)) return 1;
  if (((uintptr_t)G | (uintptr_t)Wd_rows | (uintptr_t)gu_c0 | (uintptr_t)dgu_c0) & 15) return 1;
  static LdsOptIn opt_in;
  auto kern = gemm_nt_mfma_dl_kernel<EPI_SWIGLU_BWD, false>;
  if (!opt_in(reinterpret_cast<const void*>(kern), DL_LDS_BYTES)) return 1;
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  kern<<<dim3(dl_grid_x(tiles_m * tiles_n), 1), 512, DL_LDS_BYTES, st>>>((const bf16_t*)G, ldg, (const bf16_t*)Wd_rows, ldw, dgu_c0, ld2f, M, N, K, (const bf16_t*)gu_c0, tiles_m, tiles_n, half, nullptr, nullptr, 0, 1);
  return 0;
}

int k_gemm_qkv_rope_mfma(hipStream_t st, const void* X, int ldx, const void* Wqkv, int ldw, void* qkv, int M, int d, int dh, int K, int S,
                         const float* rope_cos, const float* rope_sin) {
  if (g_gemm_variant.load(std::memory_order_relaxed) != 1 || M < 1 || S < 1 || d < BN || d % BN || (dh != 64 && dh != 128 && dh != 256) || d % dh) return 1;
  if (K < DL_BK || K % DL_BK || (ldx & 7) || (ldw & 7) || !rope_cos || !rope_sin) return 1;
  if (((uintptr_t)X | (uintptr_t)Wqkv | (uintptr_t)qkv | (uintptr_t)rope_cos | (uintptr_t)rope_sin) & 15) return 1;
  static LdsOptIn opt_in;
  auto kern = gemm_nt_mfma_dl_kernel<EPI_ROPE, false>;
  if (!opt_in(reinterpret_cast<const void*>(kern), DL_LDS_BYTES)) return 1;
  const int N = 3 * d, tiles_m = (M + BM - 1) / BM, tiles_n = N / BN;
  kern<<<dim3(dl_grid_x(tiles_m * tiles_n), 1), 512, DL_LDS_BYTES, st>>>((const bf16_t*)X, ldx, (const bf16_t*)Wqkv, ldw, qkv, N, M, N, K, nullptr, tiles_m, tiles_n, dh,
                                                                         rope_cos, rope_sin, 2 * d, S);
  return 0;
}

template <int EPI, bool OUT_F32>
static int launch(hipStream_t st, const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int Ksplit, const void* R, int splits) {
  static LdsOptIn opt_in;          // one-time opt-in to > 64 KB of dynamic LDS for this instantiation
  auto kern = gemm_nt_mfma_kernel<EPI, OUT_F32>;
  if (!opt_in(reinterpret_cast<const void*>(kern), GEMM_LDS_BYTES)) return 1;
  if (g_gemm_variant.load(std::memory_order_relaxed) == 1) return launch_dl<EPI, OUT_F32>(st, A, lda, B, ldb, C, ldc, M, N, Ksplit, R, splits);
  const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
  dim3 grid(tiles_m * tiles_n, splits);
  kern<<<grid, 512, GEMM_LDS_BYTES, st>>>((const bf16_t*)A, lda, (const bf16_t*)B, ldb, C, ldc, M, N, Ksplit, (const bf16_t*)R, tiles_m, tiles_n);
  return 0;
}

// splits > 1: `partial` receives [splits][M][N] fp32 (C is ignored); splits == 1 writes C directly.
int k_gemm_nt_mfma(hipStream_t st, const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K,
                   int epi, const void* R, int out_f32, int splits, float* partial) {
  if (M < 1 || N < 1 || splits < 1 || K % splits) return 1;
  const int Ksplit = K / splits;
  if (Ksplit < BK || Ksplit % BK || lda % 8 || ldb % 8) return 1;
  if (((uintptr_t)A | (uintptr_t)B | (uintptr_t)C | (uintptr_t)R | (uintptr_t)partial) & 15) return 1;          // 16-byte vector accesses
  if (splits > 1) {
    if (!out_f32 || !partial || epi != EPI_STORE) return 1;
    return launch<EPI_STORE, true>(st, A, lda, B, ldb, partial, N, M, N, Ksplit, nullptr, splits);
  }
  if (out_f32) return epi == EPI_STORE ? launch<EPI_STORE, true>(st, A, lda, B, ldb, C, ldc, M, N, Ksplit, nullptr, 1) : 1;
  // At most half a tile of 256 x 256 per compute unit (d_model 768: 96 tiles for 256 units): 128 x 128 tiles, two
  // workgroups per unit, fill the chip better than a partial round of big tiles.  Measured crossover (8192 x N, K = 2048):
  // the small kernel is 6 % faster at 128 big tiles and 27 % slower at 160 -- its waves of 64 x 64 sustain about 1.0 PFLOP/s
  // against 1.4-1.5 for the big kernel's 128 x 64, so from 5/8 of a round on the big tiles win.
  const long tiles256 = (long)((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  if (tiles256 <= 128 && g_gemm_small_tiles.load(std::memory_order_relaxed) && g_gemm_variant.load(std::memory_order_relaxed) == 1 &&
      k_gemm_nt128_mfma(st, A, lda, B, ldb, C, ldc, M, N, K, epi, R) == 0)
    return 0;
  if (epi == EPI_ADD_RES) return launch<EPI_ADD_RES, false>(st, A, lda, B, ldb, C, ldc, M, N, Ksplit, R, 1);
  return launch<EPI_STORE, false>(st, A, lda, B, ldb, C, ldc, M, N, Ksplit, nullptr, 1);
}

}  // namespace pp

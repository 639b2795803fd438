// bf16 MFMA causal attention for gfx950 (head dim 64 or 128): forward with online softmax, and a backward made of
// two kernels (dQ; dK and dV) so that every output element is produced by exactly one workgroup in a fixed order
// (run-to-run reproducible, no float atomics).
//
// Orientation.  All score-shaped products are formed TRANSPOSED with respect to the quantity whose softmax
// statistics they need, so that one lane owns one softmax row:
//   forward / dQ kernel:  S^T[key][query] = K Q^T   -> lane column = query, 16 keys per lane and 32x32 tile
//   dK,dV kernel:         S[query][key]   = Q K^T   -> lane column = key (its dK/dV row), 16 queries per lane
// The 32x32 MFMA accumulator gives lane (l) the rows 8*(r/4) + 4*(l/32) + r%4 of column l%32.  Eight consecutive
// accumulator registers therefore hold, for lane half h, the rows {4h..4h+3, 8+4h..8+4h+3} of a 16-row group: exactly
// a valid K-operand of the next MFMA if the OTHER operand enumerates the contraction index in the same order, so P and
// dS never leave registers.  That other operand is a [head-dim][position] slice of V, K, Q or dO, all of which are stored
// position-major; it is gathered from the position-major LDS tile by the transpose read (ds_read_b64_tr_b16: within a
// group of 16 lanes, lane i receives element i % 4 of the four 8-byte pieces addressed by lanes i/4, i/4+4, i/4+8,
// i/4+12), one read for the positions 4h..4h+3 and one for 8+4h..8+4h+3.  The same tile serves the row-operand reads
// (16 bytes = 8 consecutive head-dim elements of one position) of the score-shaped products, so every tensor is staged
// once, in the layout it has in memory, and no transposed copies exist.
#include "pp_kernels.h"
#include "pp_dev.h"

namespace pp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0)

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) { return f32x2_to_bf16x2(a, b); }
// raw v_exp_f32: inputs here are <= 0 (or -inf); results below the normal range flush to zero, which is what softmax wants
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int base) {
  u32x4 w;
  w[0] = pack_bf16x2(v[base + 0], v[base + 1]);
  w[1] = pack_bf16x2(v[base + 2], v[base + 3]);
  w[2] = pack_bf16x2(v[base + 4], v[base + 5]);
  w[3] = pack_bf16x2(v[base + 6], v[base + 7]);
  return __builtin_bit_cast(bf16x8, w);
}
__device__ __forceinline__ void zero16(f32x16& v) {
#pragma unroll
  for (int r = 0; r < 16; ++r) v[r] = 0.f;
}

// ------------------------------------------------------------------------------------------ tile staging helpers
// A tile is ROWS positions x (CPR 16-byte chunks of 8 head-dim elements); chunk c of row r lives at r*CPR + (c ^ swz<CPR>(r)).
// The swizzle serves both kinds of read without bank conflicts (64 banks of 4 bytes):
//   * row fragments (16 bytes, 16 consecutive rows at a time, same logical chunk) need 16 different 16-byte bank groups;
//   * transpose reads (per phase 4 consecutive rows r = 4a .. 4a+3 x the 4 chunks 4q .. 4q+3 of a 32-column block) need
//     the 4 rows in 4 different 64-byte groups.
// 256-byte rows (CPR 16): the row does not enter the bank index; swz = (r & 3) << 2 | (r >> 2) & 3 is a bijection of r & 15
// whose high half separates the 4 rows of a band.  128-byte rows (CPR 8): rows r, r+1 differ in address bit 7, rows r, r+2
// do not; swz = (r & 2) << 1 | (r >> 2) & 3 is a bijection of bits 1..3 of r whose bit 2 separates rows r and r+2.
template <int CPR> __device__ __forceinline__ int swz(int r) {
  return CPR == 16 ? (((r & 3) << 2) | ((r >> 2) & 3)) : (((r & 2) << 1) | ((r >> 2) & 3));
}
#define PP_GPTR(p) ((const __attribute__((address_space(1))) void*)(p))
#define PP_LPTR(p) ((__attribute__((address_space(3))) void*)(p))
// Tiles go from global memory straight into LDS (global_load_lds_dwordx4: the 64 lanes' 16-byte pieces land at
// consecutive LDS addresses from a wave-uniform base), so one wave-load fills 64 / CPR consecutive rows and the swizzle
// is applied by choosing which source chunk each lane fetches.  No staging registers, no LDS write instructions.
// Completion is tracked by vmcnt; callers wait for it and then cross a plain s_barrier.
template <int ROWS, int CPR, int NW = 4>
struct Stage {
  static constexpr int N = ROWS * CPR / (64 * NW);          // wave-loads per wave (NW waves in the workgroup)
  template <class F>
  static __device__ __forceinline__ void issue(u32x4* tile, int wave, int lane, F&& src_of) {          // src_of(row, chunk) -> const bf16_t*
    constexpr int RPL = 64 / CPR;          // rows per wave-load
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int w = wave * N + i;
      const int row = w * RPL + lane / CPR;
      const int c = (lane % CPR) ^ swz<CPR>(row);
      __builtin_amdgcn_global_load_lds(PP_GPTR(src_of(row, c)), PP_LPTR(tile + w * 64), 16, 0, 0);
    }
  }
  // same, with the source given as a wave-uniform base pointer plus a 32-bit byte offset per lane (off_of(row, chunk)):
  // the address then needs one VGPR per load instead of a 64-bit pair, and no 64-bit vector arithmetic
  template <class F>
  static __device__ __forceinline__ void issue_u(u32x4* tile, int wave, int lane, const void* ubase, F&& off_of) {
    constexpr int RPL = 64 / CPR;
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int w = wave * N + i;
      const int row = w * RPL + lane / CPR;
      const int c = (lane % CPR) ^ swz<CPR>(row);
      const uint32_t off = off_of(row, c);
      __builtin_amdgcn_global_load_lds(PP_GPTR(reinterpret_cast<const char*>(ubase) + off), PP_LPTR(tile + w * 64), 16, 0, 0);
    }
  }
};
// wait for this wave's DMA loads (vmcnt 0) and LDS reads (lgkmcnt 0), then meet the other waves
__device__ __forceinline__ void stage_sync() {
  __builtin_amdgcn_s_waitcnt(0x0070);
  __builtin_amdgcn_s_barrier();
}
template <int CPR>
__device__ __forceinline__ bf16x8 frag(const u32x4* tile, int row, int chunk) {
  return __builtin_bit_cast(bf16x8, tile[row * CPR + (chunk ^ swz<CPR>(row))]);
}
// Transposed fragment: for head-dim column 32 colblk + lane % 32, the 8 positions row0 + {4h .. 4h+3, 8+4h .. 8+4h+3}
// (h = lane / 32, row0 a multiple of 16) -- the order in which 8 consecutive accumulator registers enumerate a 16-row group.
// Lane l = 16 grp + j points at row 4 (grp >> 1) + j / 4 of the band, 8-byte piece j % 4 of the 32-byte segment of column
// half grp & 1.  tr_lane_off() is that address for column block 0 and row0 = 0; another column block flips bits 6..7 of it
// (the block index enters the swizzled chunk by XOR), 8 rows further down flip bit 5 (bit 1 of the low swizzle field), and
// row0 adds whole rows.  Tile bases are multiples of 8 KB (the kernels have no static LDS), so the XORs commute with them.
template <int CPR>
__device__ __forceinline__ uint32_t tr_lane_off(int lane) {
  const int j = lane & 15, grp = lane >> 4;
  const int r = 4 * (grp >> 1) + (j >> 2);          // row within the 16-row group (bit 3 clear)
  const int chunk = 2 * (grp & 1) + ((j >> 1) & 1);
  return (uint32_t)(r * (CPR * 16) + ((chunk ^ swz<CPR>(r)) << 4) + (j & 1) * 8);
}
__device__ __forceinline__ uint32_t lds_byte_offset(const void* p) { return (uint32_t)(uintptr_t)PP_LPTR(const_cast<void*>(p)); }
// tl = byte offset of the tile in LDS + tr_lane_off()
template <int CPR>
__device__ __forceinline__ bf16x8 frag_tr(uint32_t tl, int row0, int colblk) {
  typedef __attribute__((address_space(3))) s16x4* lptr;
  const uint32_t lo = (tl ^ (uint32_t)(colblk << 6)) + (uint32_t)(row0 * CPR * 16);
  const uint32_t hi = (tl ^ (uint32_t)((colblk << 6) | 32)) + (uint32_t)((row0 + 8) * CPR * 16);
  const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(uintptr_t)lo);
  const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(uintptr_t)hi);
  const s16x8 v = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8, v);
}
// the same value, but opaque to the optimiser: address arithmetic that depends on it stays where it is written instead of
// being hoisted out of the tile loop into registers that live across it
__device__ __forceinline__ uint32_t launder(uint32_t v) { asm volatile("" : "+v"(v)); return v; }

constexpr float LOG2E = 1.4426950408889634f, LN2 = 0.6931471805599453f;

// Causal work is triangular: the blocks of one (batch, head) pair cost 1, 2, ..., n_blk tile passes.  The hardware
// deals workgroups to the 8 XCDs round-robin by linear id, so an id -> (pair, block) map in which the cost has a
// period of 8 or 16 ids gives some XCDs twice the work of others (measured: compute units busy 55-60 % of the kernel
// time).  Here XCD k = id % 8 owns the pairs k, k+8, ... and walks them one after the other, heaviest block first:
// every XCD gets the same work, and the blocks that run together on an XCD belong to a few pairs only, whose K/V (or
// Q/dO) tiles they share in that XCD's L2.  Each workgroup takes block `rank` and its mirror image n-1-rank (constant cost), so the order of the ranks no longer
// matters for balance.  1-D grid of n_pairs * n_blk workgroups, n_blk = number of such combined blocks per pair.
__device__ __forceinline__ void causal_block_map(int id, int n_pairs, int n_blk, int& pair, int& rank) {
  if ((n_pairs & 7) == 0) {
    const int k = id & 7, j = id >> 3;
    pair = (j / n_blk) * 8 + k;
    rank = j % n_blk;
  } else {          // fallback: equal-cost blocks at consecutive ids
    pair = id % n_pairs;
    rank = id / n_pairs;
  }
}

// MFMA phases are written with the LDS fragment reads of step i+1 ahead of the MFMAs of step i (two fragment
// buffers).  The compiler waits for ALL outstanding LDS reads whenever it needs one (it does not use partial
// counts once LDS-DMA loads are in the kernel), so each step is written as: wait for the fragments already requested
// (PP_STEP_BEGIN), request the next step's fragments, then issue this step's MFMAs -- the request then has the whole
// MFMA group to land, instead of being waited for right after it was issued.
#define PP_STEP_BEGIN()                         \
  __builtin_amdgcn_sched_barrier(0);            \
  __builtin_amdgcn_s_waitcnt(0xC07F);           \
  __builtin_amdgcn_sched_barrier(0)
#define PP_READS_THEN_MFMAS(R, M)                           \
  __builtin_amdgcn_sched_group_barrier(0x100, R, 0);        \
  __builtin_amdgcn_sched_group_barrier(0x008, M, 0);        \
  __builtin_amdgcn_sched_barrier(0)

// ------------------------------------------------------------------------------------------ forward
// B*h*ceil(S/128) workgroups (see causal_block_map), 256 threads: wave w owns queries q0 + 32w .. +31; KV tiles of 64 keys.
template <int DH>
__global__ __launch_bounds__(256, 2) void attn_fwd_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ o, float* __restrict__ lse, int S, int h,
                                                           int n_pairs, int n_blk) {
  constexpr int KS = DH / 16, CT = DH / 32, CPRK = DH / 8;
  constexpr int CH = 4;          // fragment reads (= MFMAs) per fence; divides 2 KS and 4 CT
  extern __shared__ u32x4 lds[];
  constexpr int K_CH = 64 * CPRK, ST_CH = 2 * K_CH;          // a stage = K rows, then V rows, of 64 keys
  const int d = h * DH, ld = 3 * d;
  int pair, comb;
  causal_block_map(blockIdx.x, n_pairs, (n_blk + 1) / 2, pair, comb);
  const int head = pair % h, b = pair / h;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), l32 = lane & 31, lh = lane >> 5;
  const uint32_t tr_off = tr_lane_off<CPRK>(lane);
  // a late (heavy) query block, then its early (light) mirror image: every workgroup costs the same
  for (int part = 0; part < 2; ++part) {
    const int qblk = part == 0 ? n_blk - 1 - comb : comb;
    if (part == 1 && qblk == n_blk - 1 - comb) break;
    const int q0 = qblk * 128, qw0 = q0 + wave * 32;
    const int q = qw0 + l32;
    const bf16_t* base = qkv + (size_t)b * S * ld + (size_t)head * DH;
    const int n_tiles = min((q0 + 128 + 63) / 64, (S + 63) / 64);

    bf16x8 qf[KS];
    {
      const bf16_t* qp = base + (size_t)min(q, S - 1) * ld + 8 * lh;
#pragma unroll
      for (int s = 0; s < KS; ++s) qf[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qp + 16 * s));
    }
    f32x16 oacc[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c) zero16(oacc[c]);
    float m_run = -INFINITY, l_run = 0.f;
    const float sc2 = LOG2E / sqrtf((float)DH);

    auto ksrc = [&](int kv0) { return [=](int row, int c) { return base + (size_t)min(kv0 + row, S - 1) * ld + d + c * 8; }; };
    auto vsrc = [&](int kv0) { return [=](int row, int c) { return base + (size_t)min(kv0 + row, S - 1) * ld + 2 * d + c * 8; }; };
    Stage<64, CPRK>::issue(lds, wave, lane, ksrc(0));
    Stage<64, CPRK>::issue(lds + K_CH, wave, lane, vsrc(0));
    stage_sync();

    for (int j = 0; j < n_tiles; ++j) {
      const u32x4* kt = lds + (j & 1) * ST_CH;
      const u32x4* vtile = kt + K_CH;
      u32x4* nxt = lds + ((j + 1) & 1) * ST_CH;
      const int kv0 = j * 64, kvn = min(j + 1, n_tiles - 1) * 64;
      Stage<64, CPRK>::issue(nxt, wave, lane, ksrc(kvn));
      Stage<64, CPRK>::issue(nxt + K_CH, wave, lane, vsrc(kvn));
      __builtin_amdgcn_sched_barrier(0);
      if (kv0 <= qw0 + 31) {          // wave-uniform: some key of the tile is visible to some query of this wave
        f32x16 sacc[2];
        zero16(sacc[0]); zero16(sacc[1]);
        // MFMA steps n = 0 .. 2 KS - 1: key rows (n & 1) * 32.., head-dim slice n >> 1; CH steps per fence
        auto fragK = [&](int n) { return frag<CPRK>(kt, (n & 1) * 32 + l32, 2 * (n >> 1) + lh); };
        const uint32_t vtl = lds_byte_offset(vtile) + tr_off;
        auto fragV = [&](int n) { return frag_tr<CPRK>(vtl, 16 * (n / CT), n % CT); };          // V^T block n % CT, keys 16 (n / CT) ..
        {
          bf16x8 kb[2][CH];
#pragma unroll
          for (int i = 0; i < CH; ++i) kb[0][i] = fragK(i);
#pragma unroll
          for (int c = 0; c < 2 * KS / CH; ++c) {
            PP_STEP_BEGIN();
            if (c + 1 < 2 * KS / CH) {
#pragma unroll
              for (int i = 0; i < CH; ++i) kb[(c + 1) & 1][i] = fragK((c + 1) * CH + i);
            }
#pragma unroll
            for (int i = 0; i < CH; ++i) {
              const int n = c * CH + i;
              sacc[n & 1] = MFMA(kb[c & 1][i], qf[n >> 1], sacc[n & 1]);
            }
            PP_READS_THEN_MFMAS(CH, CH);
          }
        }
        // the first V fragments are requested now, so that they arrive behind the softmax arithmetic
        bf16x8 vb[2][CH];
#pragma unroll
        for (int i = 0; i < CH; ++i) vb[0][i] = fragV(i);
        __builtin_amdgcn_sched_barrier(0);
        float tmax = -INFINITY;          // row maximum of the raw scores (the scale is positive, so it commutes with max)
        if (kv0 + 63 > qw0) {          // wave-uniform: some (key, query) pair of the tile is masked
#pragma unroll
          for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int key = kv0 + mt * 32 + 8 * (r >> 2) + 4 * lh + (r & 3);
              if (key > q) sacc[mt][r] = -INFINITY;
              tmax = fmaxf(tmax, sacc[mt][r]);
            }
        } else {
#pragma unroll
          for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, sacc[mt][r]);
        }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64)) * sc2;
        // The reference point of the exponentials only has to keep them in range, it need not be the running maximum: it is
        // moved (and the accumulators rescaled) only when a row's maximum has grown by more than 2^8 since it was set, so that
        // p <= 256 and, once the first tiles are past, the 16 CT rescaling multiplies are skipped in nearly every tile.
        const float m_new = tmax > m_run + 8.0f ? tmax : m_run;
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;          // whole row masked so far (only for padded queries)
        const float alpha = fast_exp2(m_run - m_use);
        float psum = 0.f;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int r = 0; r < 16; ++r) { const float p = fast_exp2(fmaf(sacc[mt][r], sc2, -m_use)); sacc[mt][r] = p; psum += p; }
        l_run = l_run * alpha + psum;
        m_run = m_new;
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {          // wave-uniform: some row maximum moved
#pragma unroll
          for (int c = 0; c < CT; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[c][r] *= alpha;
        }
        bf16x8 pf[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) pf[t] = pack8(sacc[t >> 1], 8 * (t & 1));
        {          // steps n run over (t, c) with c fastest: consecutive MFMAs hit different accumulators
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int c = 0; c < 4 * CT / CH; ++c) {
            PP_STEP_BEGIN();
            if (c + 1 < 4 * CT / CH) {
#pragma unroll
              for (int i = 0; i < CH; ++i) vb[(c + 1) & 1][i] = fragV((c + 1) * CH + i);
            }
#pragma unroll
            for (int i = 0; i < CH; ++i) {
              const int n = c * CH + i;
              oacc[n % CT] = MFMA(vb[c & 1][i], pf[n / CT], oacc[n % CT]);
            }
            PP_READS_THEN_MFMAS(2 * CH, CH);
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      stage_sync();
    }
    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    if (q < S) {
      const float inv = 1.0f / l_tot;
      bf16_t* op = o + ((size_t)b * S + q) * d + (size_t)head * DH + 4 * lh;
#pragma unroll
      for (int c = 0; c < CT; ++c)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          u32x2 w;
          w[0] = pack_bf16x2(oacc[c][4 * g] * inv, oacc[c][4 * g + 1] * inv);
          w[1] = pack_bf16x2(oacc[c][4 * g + 2] * inv, oacc[c][4 * g + 3] * inv);
          *reinterpret_cast<u32x2*>(op + c * 32 + 8 * g) = w;
        }
      if (lh == 0) lse[((size_t)b * h + head) * S + q] = (m_run + log2f(l_tot)) * LN2;
    }
  }
}

// Gradient of the rotary embedding (the inverse rotation), applied to an accumulator tile before it is stored: with the
// half-split pairing, elements i and i + DH/2 of a head are the same register of accumulators c and c + CT/2 of a lane.
// pos = the lane's sequence position; tables are [S x DH/2] fp32; nullptr = no rotation.
template <int DH>
__device__ __forceinline__ void unrotate_tile(f32x16 (&acc)[DH / 32], const float* __restrict__ cosb, const float* __restrict__ sinb, int pos, int lh) {
  constexpr int CT = DH / 32, HALF = DH / 2;
  if (!cosb) return;
  const float* cp = cosb + (size_t)pos * HALF + 4 * lh;
  const float* sp = sinb + (size_t)pos * HALF + 4 * lh;
#pragma unroll
  for (int c = 0; c < CT / 2; ++c)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float4 cs = *reinterpret_cast<const float4*>(cp + c * 32 + 8 * g);
      const float4 sn = *reinterpret_cast<const float4*>(sp + c * 32 + 8 * g);
      const float cv[4] = {cs.x, cs.y, cs.z, cs.w}, sv[4] = {sn.x, sn.y, sn.z, sn.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float x = acc[c][4 * g + e], y = acc[c + CT / 2][4 * g + e];
        acc[c][4 * g + e] = x * cv[e] + y * sv[e];
        acc[c + CT / 2][4 * g + e] = y * cv[e] - x * sv[e];
      }
    }
}

// ------------------------------------------------------------------------------------------ backward: dQ
// B*h*ceil(S/256) workgroups (see causal_block_map), 512 threads = 8 waves (2 per SIMD, <= 256 registers each, so every MFMA keeps its
// accumulator in ordinary VGPRs): wave w owns queries q0 + 32w .. +31.  Per KV tile of 64 keys, in two groups of 32:
// S^T = K Q^T, dP^T = V dO^T, dS^T = P^T * (dP^T - D), dQ^T += K^T dS^T (K^T gathered from the K rows by transpose reads).
// The kernel also forms D = rowsum(dO * O) for its queries (each lane already holds half of its query's dO row) and
// stores it in Dbuf for the dK/dV kernel, which runs after it.
template <int DH>
__global__ __launch_bounds__(512, 2) void attn_bwd_dq_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ o,
                                                              const bf16_t* __restrict__ dO, const float* __restrict__ lse,
                                                              float* __restrict__ Dbuf, bf16_t* __restrict__ dqkv, int S, int h, int n_pairs, int n_blk,
                                                              const float* __restrict__ cosb, const float* __restrict__ sinb) {
  constexpr int KS = DH / 16, CT = DH / 32, CPRK = DH / 8, NW = 8;
  extern __shared__ u32x4 lds[];
  constexpr int K_CH = 64 * CPRK, ST_CH = 2 * K_CH;          // a stage = K rows, then V rows, of 64 keys
  const int d = h * DH, ld = 3 * d;
  int pair, comb;
  causal_block_map(blockIdx.x, n_pairs, (n_blk + 1) / 2, pair, comb);
  const int head = pair % h, b = pair / h;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), l32 = lane & 31, lh = lane >> 5;
  const uint32_t tr_off = tr_lane_off<CPRK>(lane);
  // a late (heavy) query block, then its early (light) mirror image: every workgroup costs the same
  for (int part = 0; part < 2; ++part) {
    const int qblk = part == 0 ? n_blk - 1 - comb : comb;
    if (part == 1 && qblk == n_blk - 1 - comb) break;
    const int q0 = qblk * 256, qw0 = q0 + wave * 32;
    const int q = qw0 + l32, qc = min(q, S - 1);
    const bf16_t* base = qkv + (size_t)b * S * ld + (size_t)head * DH;
    const int n_tiles = min((q0 + 256 + 63) / 64, (S + 63) / 64);
    const float scale = 1.0f / sqrtf((float)DH), sc2 = LOG2E * scale;

    bf16x8 qf[KS], dof[KS];
    float Dq = 0.f;          // D of this lane's query: sum over the head dim of dO * O, lane halves hold alternate 8-element pieces
    {
      const bf16_t* qp = base + (size_t)qc * ld + 8 * lh;
      const bf16_t* dp = dO + ((size_t)b * S + qc) * d + (size_t)head * DH + 8 * lh;
      const bf16_t* op = o + ((size_t)b * S + qc) * d + (size_t)head * DH + 8 * lh;
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        qf[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qp + 16 * s));
        const u32x4 dw = *reinterpret_cast<const u32x4*>(dp + 16 * s), ow = *reinterpret_cast<const u32x4*>(op + 16 * s);
        dof[s] = __builtin_bit_cast(bf16x8, dw);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          Dq = fmaf(__uint_as_float(dw[e] << 16), __uint_as_float(ow[e] << 16), Dq);
          Dq = fmaf(__uint_as_float(dw[e] & 0xffff0000u), __uint_as_float(ow[e] & 0xffff0000u), Dq);
        }
      }
    }
    Dq += __shfl_xor(Dq, 32, 64);
    const size_t stat = ((size_t)b * h + head) * S + qc;
    if (lh == 0 && q < S) Dbuf[stat] = Dq;
    const float nlse2 = -lse[stat] * LOG2E;
    f32x16 dqacc[CT];
#pragma unroll
    for (int c = 0; c < CT; ++c) zero16(dqacc[c]);

    auto ksrc = [&](int kv0) { return [=](int row, int c) { return base + (size_t)min(kv0 + row, S - 1) * ld + d + c * 8; }; };
    auto vsrc = [&](int kv0) { return [=](int row, int c) { return base + (size_t)min(kv0 + row, S - 1) * ld + 2 * d + c * 8; }; };
    auto issue_all = [&](u32x4* stage, int kv0) {
      Stage<64, CPRK, NW>::issue(stage, wave, lane, ksrc(kv0));
      Stage<64, CPRK, NW>::issue(stage + K_CH, wave, lane, vsrc(kv0));
    };
    issue_all(lds, 0);
    stage_sync();

    for (int j = 0; j < n_tiles; ++j) {
      const u32x4* ktile = lds + (j & 1) * ST_CH;
      const u32x4* vtile = ktile + K_CH;
      u32x4* nxt = lds + ((j + 1) & 1) * ST_CH;
      const int kv0 = j * 64, kvn = min(j + 1, n_tiles - 1) * 64;
      issue_all(nxt, kvn);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        const int kg0 = kv0 + 32 * mt;
        if (kg0 > qw0 + 31) continue;          // wave-uniform: every key of the group lies beyond every query of this wave
        f32x16 sacc, dpacc;
        zero16(sacc); zero16(dpacc);
        {
          __builtin_amdgcn_sched_barrier(0);
          bf16x8 kb[2], vb[2];
          kb[0] = frag<CPRK>(ktile, mt * 32 + l32, lh); vb[0] = frag<CPRK>(vtile, mt * 32 + l32, lh);
#pragma unroll
          for (int s = 0; s < KS; ++s) {
            PP_STEP_BEGIN();
            if (s + 1 < KS) {
              kb[(s + 1) & 1] = frag<CPRK>(ktile, mt * 32 + l32, 2 * (s + 1) + lh);
              vb[(s + 1) & 1] = frag<CPRK>(vtile, mt * 32 + l32, 2 * (s + 1) + lh);
            }
            sacc = MFMA(kb[s & 1], qf[s], sacc);
            dpacc = MFMA(vb[s & 1], dof[s], dpacc);
            PP_READS_THEN_MFMAS(2, 2);
          }
        }
        if (kg0 + 31 > qw0) {          // wave-uniform: the group straddles the diagonal
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = kg0 + 8 * (r >> 2) + 4 * lh + (r & 3);
            const float p = key > q ? 0.f : fast_exp2(fmaf(sacc[r], sc2, nlse2));
            sacc[r] = p * (dpacc[r] - Dq);
          }
        } else {
#pragma unroll
          for (int r = 0; r < 16; ++r) sacc[r] = fast_exp2(fmaf(sacc[r], sc2, nlse2)) * (dpacc[r] - Dq);
        }
        bf16x8 dsf[2];
        dsf[0] = pack8(sacc, 0); dsf[1] = pack8(sacc, 8);
        {
          __builtin_amdgcn_sched_barrier(0);
          bf16x8 tb[2];          // K^T block n % CT for the 16 keys 32 mt + 16 (n / CT) ..
          const uint32_t ktl = launder(lds_byte_offset(ktile) + tr_off);
          tb[0] = frag_tr<CPRK>(ktl, 32 * mt, 0);
          tb[1] = frag_tr<CPRK>(ktl, 32 * mt + 16 * (1 / CT), 1 % CT);
#pragma unroll
          for (int sp = 0; sp < CT; ++sp) {          // two (u, c) steps per fence
            PP_STEP_BEGIN();
            bf16x8 cur0 = tb[0], cur1 = tb[1];
            if (sp + 1 < CT) {
              const int n0 = 2 * sp + 2, n1 = 2 * sp + 3;
              const uint32_t kt2 = launder(ktl);
              tb[0] = frag_tr<CPRK>(kt2, 32 * mt + 16 * (n0 / CT), n0 % CT);
              tb[1] = frag_tr<CPRK>(kt2, 32 * mt + 16 * (n1 / CT), n1 % CT);
            }
            const int a0 = 2 * sp, a1 = 2 * sp + 1;
            dqacc[a0 % CT] = MFMA(cur0, dsf[a0 / CT], dqacc[a0 % CT]);
            dqacc[a1 % CT] = MFMA(cur1, dsf[a1 / CT], dqacc[a1 % CT]);
            PP_READS_THEN_MFMAS(4, 2);
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      stage_sync();
    }
    if (q < S) {
      unrotate_tile<DH>(dqacc, cosb, sinb, q, lh);          // dQ w.r.t. the un-rotated query (linear: commutes with the scale below)
      bf16_t* op = dqkv + ((size_t)b * S + q) * ld + (size_t)head * DH + 4 * lh;
#pragma unroll
      for (int c = 0; c < CT; ++c)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          u32x2 w;
          w[0] = pack_bf16x2(dqacc[c][4 * g] * scale, dqacc[c][4 * g + 1] * scale);
          w[1] = pack_bf16x2(dqacc[c][4 * g + 2] * scale, dqacc[c][4 * g + 3] * scale);
          *reinterpret_cast<u32x2*>(op + c * 32 + 8 * g) = w;
        }
    }
  }
}

// ------------------------------------------------------------------------------------------ backward: dK, dV
// B*h*ceil(S/128) workgroups (see causal_block_map), 512 threads = 8 waves.  Waves w and w+4 own the same 32 keys k0 + 32(w&3) .. +31 (lane
// column = key) and split the WORK, not the data: wave w ("V-wave") forms S = Q K^T and P = exp(S - lse), hands P
// (bf16, in MFMA operand order) to its partner through an LDS mailbox and accumulates dV^T += dO^T P; wave
// w+4 ("K-wave") forms dP = dO V^T, picks P up, forms dS = P * (dP - D) and accumulates dK^T += Q^T dS (dO^T and Q^T
// are gathered from the staged dO and Q rows by transpose reads).
// Nothing is computed twice, each wave carries one 32 x dh accumulator, and everything stays in VGPRs.
// Query tiles of 64 run from the diagonal to the end of the sequence.  The K-waves run ONE TILE BEHIND the V-waves:
// in iteration i the V-waves work on tile i and fill mailbox i % 2 while the K-waves work on tile i-1 and empty mailbox
// (i-1) % 2, so the two waves that share a SIMD never wait for each other inside an iteration -- one's exponentials
// overlap the other's matrix work -- and one barrier per tile is enough.
// LDS: a ring of three tile sets (Q rows + dO rows of 64 queries; both roles read both tiles, tile i+1 is in flight while
// tiles i and i-1 are in use) and two mailboxes: 128 KB at dh = 128.
// The per-query statistics (log-sum-exp for the V-waves, D for the K-waves) travel with their tile: two 256-byte
// direct-to-LDS loads per set (wave 0: the 64 log-sum-exps, wave 4: the 64 D values), read back as four floats per
// accumulator row group when the tile is started -- no registers hold them in between, and no global load is waited
// for inside an iteration.
template <int DH, bool kwave>          // kwave false: V-wave (S, P, dV)   true: K-wave (dP, dS, dK)
__device__ __forceinline__ void attn_bwd_dkv_part(u32x4* lds, const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dO,
                                                  const float* __restrict__ lse, const float* __restrict__ Dbuf, bf16_t* __restrict__ dqkv,
                                                  int S, int h, int head, int b, int kblk, int lane, int wave,
                                                  const float* __restrict__ cosb, const float* __restrict__ sinb) {
  constexpr int KS = DH / 16, CT = DH / 32, CPRK = DH / 8, NW = 8;
  constexpr int R_CH = 64 * CPRK, SET_CH = 2 * R_CH;          // a set = Q rows, then dO rows, of 64 queries
  constexpr int MAIL_CH = 2 * 4 * 2 * 64, MAIL0 = 3 * SET_CH;          // mailbox: [query group 2][key group 4][fragment 2][lane 64] chunks
  constexpr int STAT0 = MAIL0 + 2 * MAIL_CH, STAT_CH = 2 * 16;          // per set: 64 floats of lse, then 64 floats of D
  const int d = h * DH, ld = 3 * d;
  const int l32 = lane & 31, lh = lane >> 5, kg = wave & 3;
  const uint32_t tr_off = tr_lane_off<CPRK>(lane);
  const int k0 = kblk * 128, kw0 = k0 + kg * 32;
  const int key = kw0 + l32, keyc = min(key, S - 1);
  const bf16_t* base = qkv + (size_t)b * S * ld + (size_t)head * DH;
  const bf16_t* dob = dO + (size_t)b * S * d + (size_t)head * DH;
  const float* statb = (kwave ? Dbuf : lse) + ((size_t)b * h + head) * S;          // wave 0 stages lse, wave 4 stages D
  const int t_first = k0 / 64, n_tiles = (S + 63) / 64 - t_first;
  const float scale = 1.0f / sqrtf((float)DH), sc2 = LOG2E * scale;
  const float st_mul = kwave ? -1.0f : -sqrtf((float)DH);

  bf16x8 cf[KS];          // this wave's column operand: K rows (V-wave) or V rows (K-wave) of its 32 keys
  {
    const bf16_t* cp = base + (size_t)keyc * ld + (kwave ? 2 * d : d) + 8 * lh;
#pragma unroll
    for (int s = 0; s < KS; ++s) cf[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(cp + 16 * s));
  }
  f32x16 oacc[CT];          // dV^T (V-wave) or dK^T (K-wave): rows = head-dim index, column = key
#pragma unroll
  for (int c = 0; c < CT; ++c) zero16(oacc[c]);

  // sources as wave-uniform tile base + per-lane byte offset; rows past the end of the sequence repeat the last row
  auto issue_set = [&](int slot, int qq0) {
    u32x4* set = lds + slot * SET_CH;
    const int lim = S - 1 - qq0;
    Stage<64, CPRK, NW>::issue_u(set, wave, lane, base + (size_t)qq0 * ld, [=](int row, int c) { return (uint32_t)(min(row, lim) * ld + c * 8) * 2u; });
    Stage<64, CPRK, NW>::issue_u(set + R_CH, wave, lane, dob + (size_t)qq0 * d, [=](int row, int c) { return (uint32_t)(min(row, lim) * d + c * 8) * 2u; });
    if (kg == 0)          // waves 0 and 4: the tile's 64 statistics, one float per lane (positions past the end repeat the last one)
      __builtin_amdgcn_global_load_lds(PP_GPTR(statb + qq0 + min(lane, lim)), PP_LPTR(lds + STAT0 + slot * STAT_CH + (kwave ? 16 : 0)), 4, 0, 0);
  };
  issue_set(0, t_first * 64);
  stage_sync();

  for (int it = 0; it <= n_tiles; ++it) {
    const int qv0 = (t_first + it) * 64;          // the V-waves' tile; the K-waves work on the one before it
    if (it + 1 < n_tiles) issue_set((it + 1) % 3, qv0 + 64);          // ring slot of tile it-2, last read in iteration it-1
    __builtin_amdgcn_sched_barrier(0);
    const int my_it = kwave ? it - 1 : it;          // index of the tile this wave works on now
    const int qq0 = (t_first + my_it) * 64;
    if (my_it >= 0 && my_it < n_tiles && qq0 + 63 >= kw0) {          // wave-uniform: some query of the tile sees some key of the wave
      const u32x4* set = lds + (my_it % 3) * SET_CH;
      const u32x4* rows_tile = set + (kwave ? R_CH : 0);          // row operand: Q rows (V-wave) or dO rows (K-wave)
      const u32x4* tr_tile = set + (kwave ? 0 : R_CH);            // transposed operand: dO rows (V-wave) or Q rows (K-wave)
      u32x4* mail = lds + MAIL0 + (my_it & 1) * MAIL_CH + (kg * 2) * 64 + lane;          // + mt * 512 + fragment * 64
      // The accumulators start from the row statistics instead of zero, so the products come out as S - lse / scale
      // (V-wave) or dP - D (K-wave) and the statistics need no registers while the tile is worked on.
      f32x16 x[2];
      {
        const float* stp = reinterpret_cast<const float*>(lds + STAT0 + (my_it % 3) * STAT_CH + (kwave ? 16 : 0)) + 4 * lh;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int g = 0; g < 4; ++g) {          // registers 4g .. 4g+3 are the queries 32 mt + 8 g + 4 lh .. + 3 of the tile
            const float4 v = *reinterpret_cast<const float4*>(stp + mt * 32 + 8 * g);
            x[mt][4 * g] = v.x * st_mul; x[mt][4 * g + 1] = v.y * st_mul; x[mt][4 * g + 2] = v.z * st_mul; x[mt][4 * g + 3] = v.w * st_mul;
          }
      }
      {          // both query groups at once: two independent accumulator chains
        __builtin_amdgcn_sched_barrier(0);
        bf16x8 rb[2][2];
        rb[0][0] = frag<CPRK>(rows_tile, l32, lh); rb[0][1] = frag<CPRK>(rows_tile, 32 + l32, lh);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
          PP_STEP_BEGIN();
          if (s + 1 < KS) {
            rb[(s + 1) & 1][0] = frag<CPRK>(rows_tile, l32, 2 * (s + 1) + lh);
            rb[(s + 1) & 1][1] = frag<CPRK>(rows_tile, 32 + l32, 2 * (s + 1) + lh);
          }
          x[0] = MFMA(rb[s & 1][0], cf[s], x[0]);
          x[1] = MFMA(rb[s & 1][1], cf[s], x[1]);
          PP_READS_THEN_MFMAS(2, 2);
        }
      }
      bf16x8 opf[4];
      if (!kwave) {          // P = exp(S - lse), zero outside the causal triangle and for padded queries
        if ((qq0 < kw0 + 31) || (qq0 + 63 >= S)) {          // wave-uniform: some pair of the tile is masked
          // row offset o (compile-time) of this lane's element is masked iff o < lo (query before the key) or o >= hi (padding)
          const int qb = qq0 + 4 * lh, lo = key - qb, hi = S - qb;
#pragma unroll
          for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int o = mt * 32 + 8 * (r >> 2) + (r & 3);
              const float p = fast_exp2(x[mt][r] * sc2);
              x[mt][r] = (o < lo || o >= hi) ? 0.f : p;
            }
        } else {
#pragma unroll
          for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) x[mt][r] = fast_exp2(x[mt][r] * sc2);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          opf[u] = pack8(x[u >> 1], 8 * (u & 1));
          mail[(u >> 1) * 512 + (u & 1) * 64] = __builtin_bit_cast(u32x4, opf[u]);
        }
      } else {          // dS = P * (dP - D)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const u32x4 pw = mail[(u >> 1) * 512 + (u & 1) * 64];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const int r = 8 * (u & 1) + e;
            const uint32_t w = pw[e >> 1];
            const float p = __uint_as_float((e & 1) ? (w & 0xffff0000u) : (w << 16));
            x[u >> 1][r] *= p;
          }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) opf[u] = pack8(x[u >> 1], 8 * (u & 1));
      }
      {          // oacc[c] += AT tile rows c*32.., 16-query slice u  x  opf[u]; steps run over (u, c) with c fastest
        __builtin_amdgcn_sched_barrier(0);
        bf16x8 tb[2];
        const uint32_t ttl = launder(lds_byte_offset(tr_tile) + tr_off);
        tb[0] = frag_tr<CPRK>(ttl, 0, 0);
        tb[1] = frag_tr<CPRK>(ttl, 16 * (1 / CT), 1 % CT);
#pragma unroll
        for (int sp = 0; sp < 2 * CT; ++sp) {          // two (u, c) steps per fence
          PP_STEP_BEGIN();
          bf16x8 cur0 = tb[0], cur1 = tb[1];
          if (sp + 1 < 2 * CT) {
            const int n0 = 2 * sp + 2, n1 = 2 * sp + 3;
            const uint32_t tt2 = launder(ttl);
            tb[0] = frag_tr<CPRK>(tt2, 16 * (n0 / CT), n0 % CT);
            tb[1] = frag_tr<CPRK>(tt2, 16 * (n1 / CT), n1 % CT);
          }
          const int a0 = 2 * sp, a1 = 2 * sp + 1;
          oacc[a0 % CT] = MFMA(cur0, opf[a0 / CT], oacc[a0 % CT]);
          oacc[a1 % CT] = MFMA(cur1, opf[a1 / CT], oacc[a1 % CT]);
          PP_READS_THEN_MFMAS(4, 2);
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    stage_sync();
  }
  if (key < S) {
    if constexpr (kwave) unrotate_tile<DH>(oacc, cosb, sinb, key, lh);          // dK w.r.t. the un-rotated key; V is not rotated
    const float osc = kwave ? scale : 1.0f;
    bf16_t* op = dqkv + ((size_t)b * S + key) * ld + (kwave ? d : 2 * d) + (size_t)head * DH + 4 * lh;
#pragma unroll
    for (int c = 0; c < CT; ++c)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 w;
        w[0] = pack_bf16x2(oacc[c][4 * g] * osc, oacc[c][4 * g + 1] * osc);
        w[1] = pack_bf16x2(oacc[c][4 * g + 2] * osc, oacc[c][4 * g + 3] * osc);
        *reinterpret_cast<u32x2*>(op + c * 32 + 8 * g) = w;
      }
  }
}

// The two roles are separate instantiations of the tile loop (their loop-invariant registers differ); both cross the
// same number of barriers.
template <int DH>
__global__ __launch_bounds__(512, 2) void attn_bwd_dkv_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dO,
                                                               const float* __restrict__ lse, const float* __restrict__ Dbuf,
                                                               bf16_t* __restrict__ dqkv, int S, int h, int n_pairs, int n_blk,
                                                               const float* __restrict__ cosb, const float* __restrict__ sinb) {
  extern __shared__ u32x4 lds[];
  int pair, comb;
  causal_block_map(blockIdx.x, n_pairs, (n_blk + 1) / 2, pair, comb);
  const int head = pair % h, b = pair / h;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // an early (heavy: it sees the most queries) key block, then its late (light) mirror image: every workgroup costs the same
  for (int part = 0; part < 2; ++part) {
    const int kblk = part == 0 ? comb : n_blk - 1 - comb;
    if (part == 1 && kblk == comb) break;
    if (wave >= 4) attn_bwd_dkv_part<DH, true>(lds, qkv, dO, lse, Dbuf, dqkv, S, h, head, b, kblk, lane, wave, cosb, sinb);
    else attn_bwd_dkv_part<DH, false>(lds, qkv, dO, lse, Dbuf, dqkv, S, h, head, b, kblk, lane, wave, cosb, sinb);
  }
}

// ------------------------------------------------------------------------------------------ host side
template <class K>
static bool set_lds(K kern, int bytes) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, bytes) == hipSuccess;
}

template <int DH>
static int fwd_launch(hipStream_t st, const void* qkv, void* o, float* lse, int B, int S, int h) {
  constexpr int FWD_LDS = 2 * (2 * 64 * (DH / 8)) * 16;          // two stages of K rows + V rows
  static bool ok = set_lds(attn_fwd_kernel<DH>, FWD_LDS);
  if (!ok) return 1;
  const int n_blk = (S + 127) / 128;
  attn_fwd_kernel<DH><<<dim3(B * h * ((n_blk + 1) / 2)), 256, FWD_LDS, st>>>((const bf16_t*)qkv, (bf16_t*)o, lse, S, h, B * h, n_blk);
  return 0;
}
template <int DH>
static int bwd_launch(hipStream_t st, const void* qkv, const void* o, const float* lse, const void* dO, void* dqkv, float* Dbuf,
                      int B, int S, int h, const float* cosb, const float* sinb) {
  constexpr int DQ_LDS = 2 * (2 * 64 * (DH / 8)) * 16;                                   // two stages of K rows + V rows
  constexpr int DKV_LDS = (3 * (2 * 64 * (DH / 8)) + 2 * (2 * 4 * 2 * 64) + 3 * 32) * 16;          // three sets of Q rows + dO rows, two P mailboxes, three sets of statistics
  static bool ok = set_lds(attn_bwd_dq_kernel<DH>, DQ_LDS) && set_lds(attn_bwd_dkv_kernel<DH>, DKV_LDS);
  if (!ok) return 1;
  const int nb_kv = (S + 127) / 128, nb_dq = (S + 255) / 256;
  // the dQ kernel also writes D = rowsum(dO * O), which the dK/dV kernel then reads
  attn_bwd_dq_kernel<DH><<<dim3(B * h * ((nb_dq + 1) / 2)), 512, DQ_LDS, st>>>((const bf16_t*)qkv, (const bf16_t*)o, (const bf16_t*)dO, lse, Dbuf, (bf16_t*)dqkv, S, h,
                                                                 B * h, nb_dq, cosb, sinb);
  attn_bwd_dkv_kernel<DH><<<dim3(B * h * ((nb_kv + 1) / 2)), 512, DKV_LDS, st>>>((const bf16_t*)qkv, (const bf16_t*)dO, lse, Dbuf,
                                                      (bf16_t*)dqkv, S, h, B * h, nb_kv, cosb, sinb);
  return 0;
}

// bf16, head dim 64 or 128, 16-byte aligned operands with row strides that are multiples of 8 elements
int k_attn_fwd_mfma(hipStream_t st, const void* qkv, void* o, float* lse, int B, int S, int h, int dh) {
  if ((dh != 64 && dh != 128) || S < 1) return 1;
  if (((uintptr_t)qkv | (uintptr_t)o) & 15) return 1;
  return dh == 64 ? fwd_launch<64>(st, qkv, o, lse, B, S, h) : fwd_launch<128>(st, qkv, o, lse, B, S, h);
}
// rope_cos / rope_sin ([S x dh/2] fp32, both or neither): dq and dk are returned with respect to the UN-rotated q and k
// (the inverse rotation is applied to the accumulators before they are stored).  Dbuf receives rowsum(dO * O).
int k_attn_bwd_mfma(hipStream_t st, const void* qkv, const void* o, const float* lse, const void* dO, void* dqkv, float* Dbuf,
                    int B, int S, int h, int dh, const float* rope_cos, const float* rope_sin) {
  if ((dh != 64 && dh != 128) || S < 1 || (rope_cos == nullptr) != (rope_sin == nullptr)) return 1;
  if (((uintptr_t)rope_cos | (uintptr_t)rope_sin | (uintptr_t)qkv | (uintptr_t)o | (uintptr_t)dO | (uintptr_t)dqkv) & 15) return 1;
  return dh == 64 ? bwd_launch<64>(st, qkv, o, lse, dO, dqkv, Dbuf, B, S, h, rope_cos, rope_sin)
                  : bwd_launch<128>(st, qkv, o, lse, dO, dqkv, Dbuf, B, S, h, rope_cos, rope_sin);
}

}  // namespace pp

// Plain (non-MFMA) HIP kernels for gfx950: memory-bound element-wise / reduction kernels used in every
// configuration, plus shape-agnostic GEMM and attention kernels used for fp32 models and as the
// cross-check / fallback path of the MFMA kernels.
#include "pp_kernels.h"
#include "pp_dev.h"

namespace pp {

#define PP_DISPATCH(dtype, ...)                                   \
  do {                                                            \
    if ((dtype) == 0) { using T = float; __VA_ARGS__; }           \
    else { using T = bf16_t; __VA_ARGS__; }                       \
  } while (0)

static inline unsigned cdiv(size_t a, size_t b) { return (unsigned)((a + b - 1) / b); }

// ------------------------------------------------------------------------------------------ fill
__global__ void fill_f32_kernel(float* p, size_t n, float v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = v;
}
void k_fill_f32(hipStream_t st, float* p, size_t n, float v) {
  if (n == 0) return;
  unsigned blocks = cdiv(n, 256);
  if (blocks > 8192) blocks = 8192;
  fill_f32_kernel<<<blocks, 256, 0, st>>>(p, n, v);
}

// ------------------------------------------------------------------------------------------ rotary tables
__global__ void rope_tables_kernel(float* cosb, float* sinb, int S, int half, int dh, double base) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= S * half) return;
  int pos = i / half, j = i % half;
  double ang = (double)pos * pow(base, -2.0 * (double)j / (double)dh);
  cosb[i] = (float)cos(ang);
  sinb[i] = (float)sin(ang);
}
void k_rope_tables(hipStream_t st, float* cosb, float* sinb, int S, int dh, float base) {
  int n = S * (dh / 2);
  rope_tables_kernel<<<cdiv(n, 256), 256, 0, st>>>(cosb, sinb, S, dh / 2, dh, (double)base);
}

// ------------------------------------------------------------------------------------------ embedding gather
template <class T>
__global__ void embed_kernel(const int32_t* __restrict__ tok, const T* __restrict__ E, T* __restrict__ x, int d, int V) {
  const int t = blockIdx.x;
  const int id = min(max(tok[t], 0), V - 1);          // ids outside [0, V) are clamped rather than read out of bounds
  const T* src = E + (size_t)id * d;
  T* dst = x + (size_t)t * d;
  constexpr int VEC = 16 / sizeof(T);
  for (int c = threadIdx.x * VEC; c < d; c += blockDim.x * VEC)
    *reinterpret_cast<uint4*>(dst + c) = *reinterpret_cast<const uint4*>(src + c);
}
void k_embed(hipStream_t st, int dtype, const int32_t* tok, const void* E, void* x, int T_, int d, int V) {
  PP_DISPATCH(dtype, embed_kernel<T><<<T_, 256, 0, st>>>(tok, (const T*)E, (T*)x, d, V));
}

// ------------------------------------------------------------------------------------------ RMSNorm
// One wave per row, 4 rows per block; lanes stride over the row in 8-element vectors.  NV > 0: the row has exactly
// NV * 512 elements and stays in registers between the reduction and the output pass (one read of every input);
// NV == 0: any d (multiple of 8), two passes over the inputs.  Both orders of summation are the same.
template <class T, int NV>
__global__ void rmsnorm_fwd_kernel(const T* __restrict__ x, const T* __restrict__ gamma, T* __restrict__ y,
                                   float* __restrict__ rstd_out, int T_, int d, float eps) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= T_) return;
  const T* xr = x + (size_t)row * d;
  T* yr = y + (size_t)row * d;
  float ss = 0.f, g[8];
  if constexpr (NV > 0) {
    float v[NV][8];
#pragma unroll
    for (int k = 0; k < NV; ++k) load8(xr + lane * 8 + k * 512, v[k]);
#pragma unroll
    for (int k = 0; k < NV; ++k)
#pragma unroll
      for (int i = 0; i < 8; ++i) ss += v[k][i] * v[k][i];
    ss = wave_sum(ss);
    const float rstd = 1.0f / sqrtf(ss / (float)d + eps);
    if (lane == 0) rstd_out[row] = rstd;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      load8(gamma + lane * 8 + k * 512, g);
#pragma unroll
      for (int i = 0; i < 8; ++i) v[k][i] = v[k][i] * rstd * g[i];
      store8(yr + lane * 8 + k * 512, v[k]);
    }
  } else {
    float v[8];
    for (int c = lane * 8; c < d; c += 512) {
      load8(xr + c, v);
#pragma unroll
      for (int i = 0; i < 8; ++i) ss += v[i] * v[i];
    }
    ss = wave_sum(ss);
    const float rstd = 1.0f / sqrtf(ss / (float)d + eps);
    if (lane == 0) rstd_out[row] = rstd;
    for (int c = lane * 8; c < d; c += 512) {
      load8(xr + c, v);
      load8(gamma + c, g);
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = v[i] * rstd * g[i];
      store8(yr + c, v);
    }
  }
}
#define PP_RMS_NV(d, CALL)                                              \
  do {                                                                  \
    if ((d) == 2048) { constexpr int NV = 4; CALL; }                    \
    else if ((d) == 1024) { constexpr int NV = 2; CALL; }               \
    else if ((d) == 4096) { constexpr int NV = 8; CALL; }               \
    else if ((d) == 512) { constexpr int NV = 1; CALL; }                \
    else { constexpr int NV = 0; CALL; }                                \
  } while (0)
void k_rmsnorm_fwd(hipStream_t st, int dtype, const void* x, const void* gamma, void* y, float* rstd, int T_, int d, float eps) {
  PP_RMS_NV(d, PP_DISPATCH(dtype, (rmsnorm_fwd_kernel<T, NV><<<cdiv(T_, 4), 256, 0, st>>>((const T*)x, (const T*)gamma, (T*)y, rstd, T_, d, eps))));
}

template <class T, int NV>
__global__ void rmsnorm_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ x, const float* __restrict__ rstd_in,
                                   const T* __restrict__ gamma, const T* dres, T* dx, int T_, int d) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= T_) return;
  const size_t off = (size_t)row * d;
  const float rstd = rstd_in[row];
  float dot = 0.f, g[8], r[8];
  if constexpr (NV > 0) {
    float a[NV][8], b[NV][8];          // a: gamma * dy, b: x
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      load8(dy + off + lane * 8 + k * 512, a[k]);
      load8(x + off + lane * 8 + k * 512, b[k]);
    }
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      load8(gamma + lane * 8 + k * 512, g);
#pragma unroll
      for (int i = 0; i < 8; ++i) { a[k][i] *= g[i]; dot += a[k][i] * b[k][i]; }
    }
    dot = wave_sum(dot) * rstd / (float)d;      // mean(gamma*dy*xhat)
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      if (dres) load8(dres + off + lane * 8 + k * 512, r);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float val = rstd * (a[k][i] - b[k][i] * rstd * dot);
        a[k][i] = dres ? val + r[i] : val;
      }
      store8(dx + off + lane * 8 + k * 512, a[k]);
    }
  } else {
    float a[8], b[8];
    for (int c = lane * 8; c < d; c += 512) {
      load8(dy + off + c, a);
      load8(x + off + c, b);
      load8(gamma + c, g);
#pragma unroll
      for (int i = 0; i < 8; ++i) { a[i] *= g[i]; dot += a[i] * b[i]; }
    }
    dot = wave_sum(dot) * rstd / (float)d;      // mean(gamma*dy*xhat)
    for (int c = lane * 8; c < d; c += 512) {
      load8(dy + off + c, a);
      load8(x + off + c, b);
      load8(gamma + c, g);
      if (dres) load8(dres + off + c, r);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float val = rstd * (a[i] * g[i] - b[i] * rstd * dot);
        a[i] = dres ? val + r[i] : val;
      }
      store8(dx + off + c, a);
    }
  }
}
void k_rmsnorm_bwd(hipStream_t st, int dtype, const void* dy, const void* x, const float* rstd, const void* gamma,
                   const void* dres, void* dx, int T_, int d) {
  PP_RMS_NV(d, PP_DISPATCH(dtype, (rmsnorm_bwd_kernel<T, NV><<<cdiv(T_, 4), 256, 0, st>>>((const T*)dy, (const T*)x, rstd, (const T*)gamma,
                                                                                          (const T*)dres, (T*)dx, T_, d))));
}

// dgamma: stage 1 -- block (64 columns) x (row chunk b of 64) sums its rows in fixed order; stage 2 sums the 64 chunks.
template <class T>
__global__ void dgamma_stage1_kernel(const T* __restrict__ dy, const T* __restrict__ x, const float* __restrict__ rstd,
                                     float* __restrict__ partial, int T_, int d) {
  __shared__ float red[4][64];
  const int col = blockIdx.x * 64 + (threadIdx.x & 63);
  const int sub = threadIdx.x >> 6;
  const int chunk = blockIdx.y, nchunk = gridDim.y;
  const int rows_per = (T_ + nchunk - 1) / nchunk;
  const int r0 = chunk * rows_per, r1 = min(T_, r0 + rows_per);
  float acc = 0.f;
  if (col < d)
    for (int t = r0 + sub; t < r1; t += 4) acc += to_f32(dy[(size_t)t * d + col]) * to_f32(x[(size_t)t * d + col]) * rstd[t];
  red[sub][threadIdx.x & 63] = acc;
  __syncthreads();
  if (sub == 0 && col < d) partial[(size_t)chunk * d + col] = (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
}
__global__ void dgamma_stage2_kernel(const float* __restrict__ partial, float* __restrict__ dgamma, int d, int nchunk) {
  int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= d) return;
  float s = 0.f;
  for (int i = 0; i < nchunk; ++i) s += partial[(size_t)i * d + c];
  dgamma[c] = s;
}
void k_rmsnorm_dgamma(hipStream_t st, int dtype, const void* dy, const void* x, const float* rstd, float* partial,
                      float* dgamma, int T_, int d) {
  dim3 grid(cdiv(d, 64), 64);
  PP_DISPATCH(dtype, dgamma_stage1_kernel<T><<<grid, 256, 0, st>>>((const T*)dy, (const T*)x, rstd, partial, T_, d));
  dgamma_stage2_kernel<<<cdiv(d, 256), 256, 0, st>>>(partial, dgamma, d, 64);
}

// ------------------------------------------------------------------------------------------ rotary (in place on q and k of [T x 3d])
template <class T>
__global__ void rope_kernel(T* qkv, const float* __restrict__ cosb, const float* __restrict__ sinb, int S, int h, int dh,
                            size_t total, float sgn) {
  // one thread rotates 8 consecutive pairs (i .. i+7, i+half .. i+half+7) of one (token, q|k, head)
  const int half = dh >> 1, per_head = half >> 3;
  const int d = h * dh;
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;      // over T * 2 * h * per_head
  if (idx >= total) return;
  const int i = (int)(idx % per_head) * 8;
  size_t r = idx / per_head;
  const int head = (int)(r % h); r /= h;
  const int which = (int)(r % 2);
  const size_t t = r / 2;
  const int pos = (int)(t % S);
  T* p = qkv + t * (size_t)(3 * d) + (size_t)which * d + (size_t)head * dh + i;
  float a[8], b[8], c[8], sn[8];
  load8(p, a);
  load8(p + half, b);
  load8(cosb + (size_t)pos * half + i, c);
  load8(sinb + (size_t)pos * half + i, sn);
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const float s = sgn * sn[k], x = a[k], y = b[k];
    a[k] = x * c[k] - y * s;
    b[k] = x * s + y * c[k];
  }
  store8(p, a);
  store8(p + half, b);
}
template <class T>
__global__ void rope_scalar_kernel(T* qkv, const float* __restrict__ cosb, const float* __restrict__ sinb, int S, int h, int dh,
                                   size_t total, float sgn) {
  const int half = dh >> 1;
  const int d = h * dh;
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;      // over T * 2 * h * half
  if (idx >= total) return;
  const int i = (int)(idx % half);
  size_t r = idx / half;
  const int head = (int)(r % h); r /= h;
  const int which = (int)(r % 2);
  const size_t t = r / 2;
  const int pos = (int)(t % S);
  T* p = qkv + t * (size_t)(3 * d) + (size_t)which * d + (size_t)head * dh + i;
  const float c = cosb[pos * half + i], s = sgn * sinb[pos * half + i];
  const float a = to_f32(p[0]), b = to_f32(p[half]);
  p[0] = from_f32<T>(a * c - b * s);
  p[half] = from_f32<T>(a * s + b * c);
}
void k_rope(hipStream_t st, int dtype, void* qkv, const float* cosb, const float* sinb, int B, int S, int h, int dh, int inverse) {
  const float sgn = inverse ? -1.f : 1.f;
  if ((dh / 2) % 8 == 0) {
    size_t total = (size_t)B * S * 2 * h * (dh / 16);
    PP_DISPATCH(dtype, rope_kernel<T><<<cdiv(total, 256), 256, 0, st>>>((T*)qkv, cosb, sinb, S, h, dh, total, sgn));
  } else {
    size_t total = (size_t)B * S * 2 * h * (dh / 2);
    PP_DISPATCH(dtype, rope_scalar_kernel<T><<<cdiv(total, 256), 256, 0, st>>>((T*)qkv, cosb, sinb, S, h, dh, total, sgn));
  }
}

// ------------------------------------------------------------------------------------------ SwiGLU
template <class T>
__global__ void swiglu_fwd_kernel(const T* __restrict__ gu, T* __restrict__ a, int F, size_t total8) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total8) return;
  const int per_row = F / 8;
  const size_t t = i / per_row;
  const int c = (int)(i % per_row) * 8;
  float g[8], u[8];
  load8(gu + t * (size_t)(2 * F) + c, g);
  load8(gu + t * (size_t)(2 * F) + F + c, u);
#pragma unroll
  for (int k = 0; k < 8; ++k) g[k] = silu_mul(g[k], u[k]);
  store8(a + t * (size_t)F + c, g);
}
void k_swiglu_fwd(hipStream_t st, int dtype, const void* gu, void* a, int T_, int F) {
  size_t total8 = (size_t)T_ * (F / 8);
  PP_DISPATCH(dtype, swiglu_fwd_kernel<T><<<cdiv(total8, 256), 256, 0, st>>>((const T*)gu, (T*)a, F, total8));
}

// dg = dA * u * sig(g) * (1 + g (1 - sig(g)));  du = dA * g * sig(g)   for columns [c0, c1)
template <class T>
__global__ void swiglu_bwd_kernel(const T* __restrict__ gu, const T* __restrict__ dA, int ldA, T* __restrict__ dgu, int F,
                                  int c0, int ncol8, size_t total8) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total8) return;
  const size_t t = i / ncol8;
  const int cc = (int)(i % ncol8) * 8;          // column within the range
  const int c = c0 + cc;
  float g[8], u[8], da[8], dg[8], du[8];
  load8(gu + t * (size_t)(2 * F) + c, g);
  load8(gu + t * (size_t)(2 * F) + F + c, u);
  load8(dA + t * (size_t)ldA + cc, da);
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const float sg = sigmoid_fast(g[k]);
    du[k] = da[k] * g[k] * sg;
    dg[k] = da[k] * u[k] * sg * (1.0f + g[k] * (1.0f - sg));
  }
  store8(dgu + t * (size_t)(2 * F) + c, dg);
  store8(dgu + t * (size_t)(2 * F) + F + c, du);
}
void k_swiglu_bwd(hipStream_t st, int dtype, const void* gu, const void* dA, int ldA, void* dgu, int T_, int F, int c0, int c1) {
  const int ncol8 = (c1 - c0) / 8;
  size_t total8 = (size_t)T_ * ncol8;
  if (total8 == 0) return;
  PP_DISPATCH(dtype, swiglu_bwd_kernel<T><<<cdiv(total8, 256), 256, 0, st>>>((const T*)gu, (const T*)dA, ldA, (T*)dgu, F, c0, ncol8, total8));
}

// ------------------------------------------------------------------------------------------ cross entropy
__global__ void count_valid_kernel(const int32_t* __restrict__ targets, int T_, int V, int32_t* n_valid) {
  __shared__ float red[17];
  float c = 0.f;          // exact for counts < 2^24
  for (int t = threadIdx.x; t < T_; t += blockDim.x) c += (targets[t] >= 0 && targets[t] < V) ? 1.f : 0.f;
  c = block_sum(c, red);
  if (threadIdx.x == 0) *n_valid = (int32_t)c;
}
void k_count_valid(hipStream_t st, const int32_t* targets, int T_, int V, int32_t* n_valid) {
  count_valid_kernel<<<1, 1024, 0, st>>>(targets, T_, V, n_valid);
}

// One block per row.  The row is staged in LDS once, so HBM sees one read and one write of the logits.
template <class T>
__global__ void cross_entropy_kernel(T* logits, const int32_t* __restrict__ targets, const int32_t* __restrict__ n_valid,
                                     float* __restrict__ rowloss, int V) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  T* row_s = reinterpret_cast<T*>(smem_raw);
  __shared__ float red[17];
  const int t = blockIdx.x;
  T* row = logits + (size_t)t * V;
  int tg = targets[t];
  if (tg >= V) tg = -1;          // out-of-range targets are treated as ignored
  constexpr int VEC = 16 / sizeof(T);
  const int nvec = V / VEC;
  if (tg < 0) {            // ignored position: zero gradient, zero loss (uniform branch per block)
    const uint4 z = make_uint4(0, 0, 0, 0);
    for (int i = threadIdx.x; i < nvec; i += blockDim.x) reinterpret_cast<uint4*>(row)[i] = z;
    for (int i = nvec * VEC + threadIdx.x; i < V; i += blockDim.x) row[i] = from_f32<T>(0.f);
    if (threadIdx.x == 0) rowloss[t] = 0.f;
    return;
  }
  float mx = -INFINITY;
  for (int i = threadIdx.x; i < nvec; i += blockDim.x) {
    uint4 r = reinterpret_cast<const uint4*>(row)[i];
    reinterpret_cast<uint4*>(row_s)[i] = r;
  }
  for (int i = nvec * VEC + threadIdx.x; i < V; i += blockDim.x) row_s[i] = row[i];
  __syncthreads();
  for (int i = threadIdx.x; i < V; i += blockDim.x) mx = fmaxf(mx, to_f32(row_s[i]));
  mx = block_max(mx, red);
  float sum = 0.f;
  for (int i = threadIdx.x; i < V; i += blockDim.x) sum += __expf(to_f32(row_s[i]) - mx);
  sum = block_sum(sum, red);
  const float inv_n = 1.0f / (float)max(*n_valid, 1);
  const float inv_sum = 1.0f / sum;
  if (threadIdx.x == 0) rowloss[t] = (mx + logf(sum)) - to_f32(row_s[tg]);
  for (int i = threadIdx.x; i < V; i += blockDim.x) {
    float p = __expf(to_f32(row_s[i]) - mx) * inv_sum;
    if (i == tg) p -= 1.0f;
    row[i] = from_f32<T>(p * inv_n);
  }
}
// bf16 rows of up to 512 * 8 * NV logits (NV <= 16: 65536), V % 8 == 0: the row lives in registers (NV 16-byte pieces per thread, loaded and
// stored with consecutive lanes on consecutive pieces), so there is one HBM read, one HBM write and no LDS staging.
template <int NV>
__global__ __launch_bounds__(512) void cross_entropy_reg_kernel(bf16_t* logits, const int32_t* __restrict__ targets,
                                                                const int32_t* __restrict__ n_valid, float* __restrict__ rowloss, int V) {
  __shared__ float red[17];
  const int t = blockIdx.x, nvec = V >> 3;
  uint4* row = reinterpret_cast<uint4*>(logits + (size_t)t * V);
  int tg = targets[t];
  if (tg >= V) tg = -1;          // out-of-range targets are treated as ignored
  if (tg < 0) {            // ignored position: zero gradient, zero loss (uniform branch per block)
    for (int i = threadIdx.x; i < nvec; i += 512) row[i] = make_uint4(0, 0, 0, 0);
    if (threadIdx.x == 0) rowloss[t] = 0.f;
    return;
  }
  uint4 r[NV];
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int i = threadIdx.x + 512 * k;
    r[k] = i < nvec ? row[i] : make_uint4(0xff80ff80u, 0xff80ff80u, 0xff80ff80u, 0xff80ff80u);          // -inf: no effect on max or sum
  }
  auto lo = [](uint32_t w) { return __uint_as_float(w << 16); };
  auto hi = [](uint32_t w) { return __uint_as_float(w & 0xffff0000u); };
  float mx = -INFINITY;
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const uint32_t w[4] = {r[k].x, r[k].y, r[k].z, r[k].w};
#pragma unroll
    for (int e = 0; e < 4; ++e) mx = fmaxf(mx, fmaxf(lo(w[e]), hi(w[e])));
  }
  mx = block_max(mx, red);
  float sum = 0.f;
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const uint32_t w[4] = {r[k].x, r[k].y, r[k].z, r[k].w};
#pragma unroll
    for (int e = 0; e < 4; ++e) sum += __expf(lo(w[e]) - mx) + __expf(hi(w[e]) - mx);
  }
  sum = block_sum(sum, red);
  const float inv_n = 1.0f / (float)max(*n_valid, 1);
  const float inv_sum = 1.0f / sum;
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int i = threadIdx.x + 512 * k;
    if (i >= nvec) continue;
    const uint32_t w[4] = {r[k].x, r[k].y, r[k].z, r[k].w};
    uint32_t o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float p0 = __expf(lo(w[e]) - mx) * inv_sum, p1 = __expf(hi(w[e]) - mx) * inv_sum;
      const int c = 8 * i + 2 * e;
      if (c == tg) { rowloss[t] = (mx + logf(sum)) - lo(w[e]); p0 -= 1.0f; }
      if (c + 1 == tg) { rowloss[t] = (mx + logf(sum)) - hi(w[e]); p1 -= 1.0f; }
      o[e] = f32x2_to_bf16x2(p0 * inv_n, p1 * inv_n);
    }
    row[i] = make_uint4(o[0], o[1], o[2], o[3]);
  }
}
bool ce_row_fits(int dtype, int V) {
  if (dtype == 1 && V % 8 == 0 && V <= 512 * 8 * 16) return true;
  return (size_t)V * (dtype == 0 ? 4 : 2) <= 64 * 1024 - 256;
}
int k_cross_entropy(hipStream_t st, int dtype, void* logits, const int32_t* targets, const int32_t* n_valid, float* rowloss, int T_, int V) {
  if (dtype == 1 && V % 8 == 0 && V <= 512 * 8 * 16 && ((uintptr_t)logits & 15) == 0) {
    const int nv = (V / 8 + 511) / 512;
    bf16_t* lg = (bf16_t*)logits;
    if (nv <= 1) cross_entropy_reg_kernel<1><<<T_, 512, 0, st>>>(lg, targets, n_valid, rowloss, V);
    else if (nv <= 2) cross_entropy_reg_kernel<2><<<T_, 512, 0, st>>>(lg, targets, n_valid, rowloss, V);
    else if (nv <= 4) cross_entropy_reg_kernel<4><<<T_, 512, 0, st>>>(lg, targets, n_valid, rowloss, V);
    else if (nv <= 8) cross_entropy_reg_kernel<8><<<T_, 512, 0, st>>>(lg, targets, n_valid, rowloss, V);
    else cross_entropy_reg_kernel<16><<<T_, 512, 0, st>>>(lg, targets, n_valid, rowloss, V);
    return 0;
  }
  size_t smem = (size_t)V * (dtype == 0 ? 4 : 2);
  if (smem > 64 * 1024 - 256) return 1;
  PP_DISPATCH(dtype, cross_entropy_kernel<T><<<T_, 512, smem, st>>>((T*)logits, targets, n_valid, rowloss, V));
  return 0;
}
__global__ void loss_reduce_kernel(const float* __restrict__ rowloss, const int32_t* __restrict__ n_valid, float* loss, int T_) {
  __shared__ float red[17];
  float s = 0.f;
  for (int t = threadIdx.x; t < T_; t += blockDim.x) s += rowloss[t];
  s = block_sum(s, red);
  if (threadIdx.x == 0) *loss = s / (float)max(*n_valid, 1);
}
void k_loss_reduce(hipStream_t st, const float* rowloss, const int32_t* n_valid, float* loss, int T_) {
  loss_reduce_kernel<<<1, 1024, 0, st>>>(rowloss, n_valid, loss, T_);
}

// ------------------------------------------------------------------------------------------ transpose
template <class T>
__global__ void transpose_kernel(const T* __restrict__ src, int ld_src, T* __restrict__ dst, int ld_dst, int rows, int cols) {
  __shared__ T tile[64][65];
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int i = ty; i < 64; i += 4) {
    const int r = r0 + i, c = c0 + tx;
    if (r < rows && c < cols) tile[i][tx] = src[(size_t)r * ld_src + c];
  }
  __syncthreads();
  for (int i = ty; i < 64; i += 4) {
    const int c = c0 + i, r = r0 + tx;      // dst row = c, dst col = r
    if (r < rows && c < cols) dst[(size_t)c * ld_dst + r] = tile[tx][i];
  }
}
// 64 x 64 tile of 2-byte elements with 16-byte global loads and stores; the 8 x 8 sub-blocks are turned in LDS.
// Needs rows % 8 == 0, cols % 8 == 0, leading dimensions % 8 == 0 and 16-byte aligned bases.
__global__ void transpose16_kernel(const uint16_t* __restrict__ src, int ld_src, uint16_t* __restrict__ dst, int ld_dst, int rows, int cols) {
  __shared__ uint16_t tile[64][72];          // row pitch 144 bytes: 16-byte aligned rows, column reads spread over banks
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int t = threadIdx.x;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int r = (t >> 3) + 32 * i, c8 = (t & 7) * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (r0 + r < rows && c0 + c8 < cols) v = *reinterpret_cast<const uint4*>(src + (size_t)(r0 + r) * ld_src + c0 + c8);
    *reinterpret_cast<uint4*>(&tile[r][c8]) = v;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int c = (t >> 3) + 32 * i, r8 = (t & 7) * 8;          // output row c0 + c, output columns r0 + r8 .. +7
    if (c0 + c < cols && r0 + r8 < rows) {
      uint32_t w[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) w[k] = (uint32_t)tile[r8 + 2 * k][c] | ((uint32_t)tile[r8 + 2 * k + 1][c] << 16);
      *reinterpret_cast<uint4*>(dst + (size_t)(c0 + c) * ld_dst + r0 + r8) = make_uint4(w[0], w[1], w[2], w[3]);
    }
  }
}
void k_transpose(hipStream_t st, int dtype, const void* src, int ld_src, void* dst, int ld_dst, int rows, int cols) {
  if (rows == 0 || cols == 0) return;
  dim3 grid(cdiv(cols, 64), cdiv(rows, 64));
  if (dtype == 1 && rows % 8 == 0 && cols % 8 == 0 && ld_src % 8 == 0 && ld_dst % 8 == 0 && (((uintptr_t)src | (uintptr_t)dst) & 15) == 0) {
    transpose16_kernel<<<grid, 256, 0, st>>>((const uint16_t*)src, ld_src, (uint16_t*)dst, ld_dst, rows, cols);
    return;
  }
  PP_DISPATCH(dtype, transpose_kernel<T><<<grid, 256, 0, st>>>((const T*)src, ld_src, (T*)dst, ld_dst, rows, cols));
}

// Batched transpose of the trainable row blocks into their shadow images (one launch for all blocks).
template <class T>
__global__ void shadow_refresh_kernel(const T* __restrict__ params, T* __restrict__ shadow, const ShadowSeg* __restrict__ segs, int n_segs) {
  __shared__ T tile[64][65];
  const int tileid = blockIdx.x;
  int lo = 0, hi = n_segs - 1;          // last segment with tile_start <= tileid
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (segs[mid].tile_start <= tileid) lo = mid; else hi = mid - 1;
  }
  const ShadowSeg s = segs[lo];
  const int local = tileid - s.tile_start;
  const int tiles_c = (s.cols + 63) / 64;
  const int r0 = (local / tiles_c) * 64, c0 = (local % tiles_c) * 64;
  const T* src = params + s.canon_off;
  T* dst = shadow + s.shadow_off;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int i = ty; i < 64; i += 4) {
    const int r = r0 + i, c = c0 + tx;
    if (r < s.rows && c < s.cols) tile[i][tx] = src[(size_t)r * s.cols + c];
  }
  __syncthreads();
  for (int i = ty; i < 64; i += 4) {
    const int c = c0 + i, r = r0 + tx;
    if (r < s.rows && c < s.cols) dst[(size_t)c * s.shadow_ld + r] = tile[tx][i];
  }
}
// 2-byte elements, 16-byte global accesses (block rows, columns, shadow leading dimension and offsets multiples of 8).
__global__ void shadow_refresh16_kernel(const uint16_t* __restrict__ params, uint16_t* __restrict__ shadow, const ShadowSeg* __restrict__ segs, int n_segs) {
  __shared__ uint16_t tile[64][72];
  const int tileid = blockIdx.x;
  int lo = 0, hi = n_segs - 1;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (segs[mid].tile_start <= tileid) lo = mid; else hi = mid - 1;
  }
  const ShadowSeg s = segs[lo];
  const int local = tileid - s.tile_start;
  const int tiles_c = (s.cols + 63) / 64;
  const int r0 = (local / tiles_c) * 64, c0 = (local % tiles_c) * 64;
  const uint16_t* src = params + s.canon_off;
  uint16_t* dst = shadow + s.shadow_off;
  const int t = threadIdx.x;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int r = (t >> 3) + 32 * i, c8 = (t & 7) * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (r0 + r < s.rows && c0 + c8 < s.cols) v = *reinterpret_cast<const uint4*>(src + (size_t)(r0 + r) * s.cols + c0 + c8);
    *reinterpret_cast<uint4*>(&tile[r][c8]) = v;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int c = (t >> 3) + 32 * i, r8 = (t & 7) * 8;
    if (c0 + c < s.cols && r0 + r8 < s.rows) {
      uint32_t w[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) w[k] = (uint32_t)tile[r8 + 2 * k][c] | ((uint32_t)tile[r8 + 2 * k + 1][c] << 16);
      *reinterpret_cast<uint4*>(dst + (size_t)(c0 + c) * s.shadow_ld + r0 + r8) = make_uint4(w[0], w[1], w[2], w[3]);
    }
  }
}
// vec_ok: every block has rows, cols, shadow_ld and both offsets multiples of 8 (checked by the caller on the host table)
void k_shadow_refresh(hipStream_t st, int dtype, const void* params, void* shadow, const ShadowSeg* segs_dev, int n_segs, int n_tiles, int vec_ok) {
  if (n_segs == 0 || n_tiles == 0) return;
  if (dtype == 1 && vec_ok) {
    shadow_refresh16_kernel<<<n_tiles, 256, 0, st>>>((const uint16_t*)params, (uint16_t*)shadow, segs_dev, n_segs);
    return;
  }
  PP_DISPATCH(dtype, shadow_refresh_kernel<T><<<n_tiles, 256, 0, st>>>((const T*)params, (T*)shadow, segs_dev, n_segs));
}

// ------------------------------------------------------------------------------------------ plain GEMM (NT)
// 64x64 tile, BK = 16, 256 threads, 4x4 micro-tile per thread, fp32 FMA.  Bounds-checked everywhere.
template <class T, class TO>
__global__ void gemm_nt_plain_kernel(const T* __restrict__ A, int lda, const T* __restrict__ B, int ldb, TO* C, int ldc,
                                     int M, int N, int K, int kchunk, int epi, const T* R) {
  __shared__ float As[16][68], Bs[16][68];
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int z = blockIdx.z;
  const int k_begin = z * kchunk, k_end = min(K, k_begin + kchunk);
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[4][4] = {};
  const int lr = threadIdx.x >> 2;             // 0..63: tile row loaded by this thread
  const int lk = (threadIdx.x & 3) * 4;        // 0,4,8,12
  for (int k0 = k_begin; k0 < k_end; k0 += 16) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = k0 + lk + j;
      const int am = m0 + lr, bn = n0 + lr;
      As[lk + j][lr] = (am < M && k < k_end) ? to_f32(A[(size_t)am * lda + k]) : 0.f;
      Bs[lk + j][lr] = (bn < N && k < k_end) ? to_f32(B[(size_t)bn * ldb + k]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  TO* Cz = C + (size_t)z * (size_t)M * (size_t)ldc;        // split-K partials are dense [z][M][ldc=N]
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      float v = acc[i][j];
      if (epi == EPI_ADD_RES) v += to_f32(R[(size_t)m * ldc + n]);
      Cz[(size_t)m * ldc + n] = from_f32<TO>(v);
    }
  }
}
void k_gemm_nt_plain(hipStream_t st, int dtype, const void* A, int lda, const void* B, int ldb, void* C, int ldc,
                     int M, int N, int K, int epi, const void* R, int out_f32) {
  if (M == 0 || N == 0) return;
  dim3 grid(cdiv(N, 64), cdiv(M, 64), 1);
  if (dtype == 0 || out_f32) {
    if (dtype == 0) gemm_nt_plain_kernel<float, float><<<grid, 256, 0, st>>>((const float*)A, lda, (const float*)B, ldb, (float*)C, ldc, M, N, K, K, epi, (const float*)R);
    else gemm_nt_plain_kernel<bf16_t, float><<<grid, 256, 0, st>>>((const bf16_t*)A, lda, (const bf16_t*)B, ldb, (float*)C, ldc, M, N, K, K, epi, (const bf16_t*)R);
  } else {
    gemm_nt_plain_kernel<bf16_t, bf16_t><<<grid, 256, 0, st>>>((const bf16_t*)A, lda, (const bf16_t*)B, ldb, (bf16_t*)C, ldc, M, N, K, K, epi, (const bf16_t*)R);
  }
}
void k_gemm_nt_plain_splitk(hipStream_t st, int dtype, const void* A, int lda, const void* B, int ldb, float* partial,
                            int M, int N, int K, int splits) {
  if (M == 0 || N == 0) return;
  dim3 grid(cdiv(N, 64), cdiv(M, 64), splits);
  const int kchunk = (K + splits - 1) / splits;
  if (dtype == 0) gemm_nt_plain_kernel<float, float><<<grid, 256, 0, st>>>((const float*)A, lda, (const float*)B, ldb, partial, N, M, N, K, kchunk, EPI_STORE, nullptr);
  else gemm_nt_plain_kernel<bf16_t, float><<<grid, 256, 0, st>>>((const bf16_t*)A, lda, (const bf16_t*)B, ldb, partial, N, M, N, K, kchunk, EPI_STORE, nullptr);
}
__global__ void splitk_reduce_kernel(const float* __restrict__ partial, float* __restrict__ C, int ldc, int M, int N, int splits) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t MN = (size_t)M * N;
  if (i >= MN) return;
  float s = 0.f;
  for (int z = 0; z < splits; ++z) s += partial[(size_t)z * MN + i];      // fixed order: run-to-run reproducible
  C[(i / N) * (size_t)ldc + (i % N)] = s;
}
void k_splitk_reduce(hipStream_t st, const float* partial, float* C, int ldc, int M, int N, int splits) {
  size_t MN = (size_t)M * N;
  if (MN == 0) return;
  splitk_reduce_kernel<<<cdiv(MN, 256), 256, 0, st>>>(partial, C, ldc, M, N, splits);
}

// ------------------------------------------------------------------------------------------ plain attention
// qkv: [T x 3d] (q | k | v, head j at columns j*dh), o: [T x d], lse: [(b*h + j)*S + s].
template <class T>
__global__ void attn_fwd_plain_kernel(const T* __restrict__ qkv, T* __restrict__ o, float* __restrict__ lse, int S, int h, int dh) {
  extern __shared__ float sc[];          // S floats
  __shared__ float red[17];
  const int i = blockIdx.x, head = blockIdx.y, b = blockIdx.z;
  const int d = h * dh;
  const size_t ld = (size_t)3 * d;
  const T* base = qkv + (size_t)b * S * ld + (size_t)head * dh;
  const T* qi = base + (size_t)i * ld;
  const float scale = 1.0f / sqrtf((float)dh);
  float mx = -INFINITY;
  for (int j = threadIdx.x; j <= i; j += blockDim.x) {
    const T* kj = base + (size_t)j * ld + d;
    float s = 0.f;
    for (int c = 0; c < dh; ++c) s = fmaf(to_f32(qi[c]), to_f32(kj[c]), s);
    s *= scale;
    sc[j] = s;
    mx = fmaxf(mx, s);
  }
  mx = block_max(mx, red);
  float sum = 0.f;
  for (int j = threadIdx.x; j <= i; j += blockDim.x) { float e = expf(sc[j] - mx); sc[j] = e; sum += e; }
  sum = block_sum(sum, red);
  if (threadIdx.x == 0) lse[((size_t)b * h + head) * S + i] = mx + logf(sum);
  for (int c = threadIdx.x; c < dh; c += blockDim.x) {
    float acc = 0.f;
    for (int j = 0; j <= i; ++j) acc = fmaf(sc[j], to_f32(base[(size_t)j * ld + 2 * d + c]), acc);
    o[((size_t)b * S + i) * d + (size_t)head * dh + c] = from_f32<T>(acc / sum);
  }
}
void k_attn_fwd_plain(hipStream_t st, int dtype, const void* qkv, void* o, float* lse, int B, int S, int h, int dh) {
  dim3 grid(S, h, B);
  PP_DISPATCH(dtype, attn_fwd_plain_kernel<T><<<grid, 128, S * sizeof(float), st>>>((const T*)qkv, (T*)o, lse, S, h, dh));
}

template <class T>
__global__ void attn_D_kernel(const T* __restrict__ o, const T* __restrict__ dO, float* __restrict__ Dbuf, int S, int h, int dh, size_t total) {
  // D[b, head, s] = sum_c o * dO: dh/8 lanes per (token, head), 8 consecutive elements each (dh % 8 == 0)
  const int lpr = dh >> 3;                                  // lanes per row: 2 .. 32 (power of two for dh 16, 32, 64, 128, 256)
  const size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t row = gid / lpr;                             // (token, head) index
  const int part = (int)(gid % lpr);
  float acc = 0.f;
  if (row < total) {
    float a[8], b[8];
    load8(o + row * dh + part * 8, a);
    load8(dO + row * dh + part * 8, b);
#pragma unroll
    for (int k = 0; k < 8; ++k) acc += a[k] * b[k];
  }
  for (int off = lpr >> 1; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
  if (row < total && part == 0) {
    const int head = (int)(row % h);
    const size_t t = row / h, b_ = t / S, s_ = t % S;
    Dbuf[(b_ * h + head) * S + s_] = acc;
  }
}
template <class T>
__global__ void attn_D_generic_kernel(const T* __restrict__ o, const T* __restrict__ dO, float* __restrict__ Dbuf, int S, int h, int dh, size_t total) {
  const size_t w = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (w >= total) return;
  const int head = (int)(w % h);
  const size_t t = w / h;
  const size_t off = t * (size_t)(h * dh) + (size_t)head * dh;
  float acc = 0.f;
  for (int c = lane; c < dh; c += 64) acc += to_f32(o[off + c]) * to_f32(dO[off + c]);
  acc = wave_sum(acc);
  if (lane == 0) { const size_t b = t / S, s = t % S; Dbuf[(b * h + head) * S + s] = acc; }
}
void k_attn_D(hipStream_t st, int dtype, const void* o, const void* dO, float* Dbuf, int B, int S, int h, int dh) {
  size_t total = (size_t)B * S * h;
  const int lpr = dh / 8;
  if (dh % 8 == 0 && (lpr & (lpr - 1)) == 0 && lpr <= 64) {
    size_t threads = total * lpr;
    PP_DISPATCH(dtype, attn_D_kernel<T><<<cdiv(threads, 256), 256, 0, st>>>((const T*)o, (const T*)dO, Dbuf, S, h, dh, total));
  } else {
    PP_DISPATCH(dtype, attn_D_generic_kernel<T><<<cdiv(total, 4), 256, 0, st>>>((const T*)o, (const T*)dO, Dbuf, S, h, dh, total));
  }
}

template <class T>
__global__ void attn_bwd_dq_plain_kernel(const T* __restrict__ qkv, const float* __restrict__ lse, const float* __restrict__ Dbuf,
                                         const T* __restrict__ dO, T* __restrict__ dqkv, int S, int h, int dh) {
  extern __shared__ float sc[];          // S floats: dS row
  const int i = blockIdx.x, head = blockIdx.y, b = blockIdx.z;
  const int d = h * dh;
  const size_t ld = (size_t)3 * d;
  const T* base = qkv + (size_t)b * S * ld + (size_t)head * dh;
  const T* qi = base + (size_t)i * ld;
  const T* doi = dO + ((size_t)b * S + i) * d + (size_t)head * dh;
  const float scale = 1.0f / sqrtf((float)dh);
  const size_t stat = ((size_t)b * h + head) * S + i;
  const float L = lse[stat], Di = Dbuf[stat];
  for (int j = threadIdx.x; j <= i; j += blockDim.x) {
    const T* kj = base + (size_t)j * ld + d;
    const T* vj = base + (size_t)j * ld + 2 * d;
    float s = 0.f, dp = 0.f;
    for (int c = 0; c < dh; ++c) { s = fmaf(to_f32(qi[c]), to_f32(kj[c]), s); dp = fmaf(to_f32(doi[c]), to_f32(vj[c]), dp); }
    const float p = expf(s * scale - L);
    sc[j] = p * (dp - Di);
  }
  __syncthreads();
  for (int c = threadIdx.x; c < dh; c += blockDim.x) {
    float acc = 0.f;
    for (int j = 0; j <= i; ++j) acc = fmaf(sc[j], to_f32(base[(size_t)j * ld + d + c]), acc);
    dqkv[((size_t)b * S + i) * ld + (size_t)head * dh + c] = from_f32<T>(acc * scale);
  }
}
template <class T>
__global__ void attn_bwd_dkv_plain_kernel(const T* __restrict__ qkv, const float* __restrict__ lse, const float* __restrict__ Dbuf,
                                          const T* __restrict__ dO, T* __restrict__ dqkv, int S, int h, int dh) {
  extern __shared__ float sc[];          // 2*S floats: P column and dS column for rows i >= j
  float* Pc = sc;
  float* DSc = sc + S;
  const int j = blockIdx.x, head = blockIdx.y, b = blockIdx.z;
  const int d = h * dh;
  const size_t ld = (size_t)3 * d;
  const T* base = qkv + (size_t)b * S * ld + (size_t)head * dh;
  const T* kj = base + (size_t)j * ld + d;
  const T* vj = base + (size_t)j * ld + 2 * d;
  const float scale = 1.0f / sqrtf((float)dh);
  for (int i = j + threadIdx.x; i < S; i += blockDim.x) {
    const T* qi = base + (size_t)i * ld;
    const T* doi = dO + ((size_t)b * S + i) * d + (size_t)head * dh;
    float s = 0.f, dp = 0.f;
    for (int c = 0; c < dh; ++c) { s = fmaf(to_f32(qi[c]), to_f32(kj[c]), s); dp = fmaf(to_f32(doi[c]), to_f32(vj[c]), dp); }
    const size_t stat = ((size_t)b * h + head) * S + i;
    const float p = expf(s * scale - lse[stat]);
    Pc[i] = p;
    DSc[i] = p * (dp - Dbuf[stat]);
  }
  __syncthreads();
  for (int c = threadIdx.x; c < dh; c += blockDim.x) {
    float av = 0.f, ak = 0.f;
    for (int i = j; i < S; ++i) {
      av = fmaf(Pc[i], to_f32(dO[((size_t)b * S + i) * d + (size_t)head * dh + c]), av);
      ak = fmaf(DSc[i], to_f32(base[(size_t)i * ld + c]), ak);
    }
    dqkv[((size_t)b * S + j) * ld + d + (size_t)head * dh + c] = from_f32<T>(ak * scale);
    dqkv[((size_t)b * S + j) * ld + 2 * d + (size_t)head * dh + c] = from_f32<T>(av);
  }
}
void k_attn_bwd_plain(hipStream_t st, int dtype, const void* qkv, const void* o, const float* lse, const void* dO, void* dqkv,
                      float* Dbuf, int B, int S, int h, int dh) {
  k_attn_D(st, dtype, o, dO, Dbuf, B, S, h, dh);
  dim3 grid(S, h, B);
  PP_DISPATCH(dtype, attn_bwd_dq_plain_kernel<T><<<grid, 128, S * sizeof(float), st>>>((const T*)qkv, lse, Dbuf, (const T*)dO, (T*)dqkv, S, h, dh));
  PP_DISPATCH(dtype, attn_bwd_dkv_plain_kernel<T><<<grid, 128, 2 * S * sizeof(float), st>>>((const T*)qkv, lse, Dbuf, (const T*)dO, (T*)dqkv, S, h, dh));
}

// ------------------------------------------------------------------------------------------ embedding gradient (full-backprop step only)
// One block per vocabulary row; rows of dx whose token equals the row id are summed in position order,
// so the result does not depend on scheduling.
template <class T>
__global__ void embed_grad_kernel(const int32_t* __restrict__ tok, const T* __restrict__ dx, float* __restrict__ gE, int T_, int d) {
  __shared__ int32_t hits[1024];
  __shared__ int n_hits_s;
  const int v = blockIdx.x;
  float* out = gE + (size_t)v * d;
  for (int c = threadIdx.x; c < d; c += blockDim.x) out[c] = 0.f;
  for (int t0 = 0; t0 < T_; t0 += 1024) {
    // ordered compaction of matching positions in [t0, t0+1024) by thread 0 (token reads are the cheap part)
    __syncthreads();
    if (threadIdx.x == 0) n_hits_s = 0;
    __syncthreads();
    if (threadIdx.x < 64) {          // one wave builds the ordered list with ballots
      int base = 0;
      for (int s = 0; s < 1024; s += 64) {
        const int t = t0 + s + threadIdx.x;
        const bool hit = t < T_ && tok[t] == v;
        const unsigned long long bal = __ballot(hit);
        if (hit) hits[base + __popcll(bal & ((1ull << threadIdx.x) - 1ull))] = t;
        base += __popcll(bal);
      }
      if (threadIdx.x == 0) n_hits_s = base;
    }
    __syncthreads();
    const int nh = n_hits_s;
    if (nh == 0) continue;
    for (int c = threadIdx.x; c < d; c += blockDim.x) {
      float acc = out[c];
      for (int k = 0; k < nh; ++k) acc += to_f32(dx[(size_t)hits[k] * d + c]);
      out[c] = acc;
    }
  }
}
// The same sums in the same order without every row scanning every token: positions are ranked by (token, position) --
// one thread per position counts the positions with a smaller token and the earlier ones with its own token, T^2 / 2
// comparisons from LDS -- which yields the position list of every token, in position order, as a segment of one array.
// idx: [T] sorted positions, then [V] segment starts, then [V] segment lengths (lengths zeroed beforehand).
__global__ __launch_bounds__(64) void embed_rank_kernel(const int32_t* __restrict__ tok, int32_t* __restrict__ idx, int T_, int V) {
  __shared__ int32_t chunk[1024];
  const int t = blockIdx.x * 64 + threadIdx.x;
  const int my = t < T_ ? tok[t] : -1;
  int less = 0, eq_before = 0, eq_total = 0;
  for (int t0 = 0; t0 < T_; t0 += 1024) {
    __syncthreads();
    for (int i = threadIdx.x; i < 1024; i += 64) chunk[i] = t0 + i < T_ ? tok[t0 + i] : 0x7fffffff;
    __syncthreads();
    const int n = min(1024, T_ - t0);
    for (int i = 0; i < n; ++i) {
      const int o = chunk[i];
      less += o < my;
      eq_total += o == my;
      eq_before += (o == my) & (t0 + i < t);
    }
  }
  if (t >= T_ || my < 0 || my >= V) return;          // tokens outside the vocabulary contribute nothing (as in the forward gather's clamp-free contract)
  idx[less + eq_before] = t;
  if (eq_before == 0) { idx[T_ + my] = less; idx[T_ + V + my] = eq_total; }
}
// One block per vocabulary row, 256 threads = 4 hit lanes x 64 column lanes.  Hit lane j sums the row's positions
// j, j+4, j+8, ... (in that order) for 16-byte column pieces, four loads in flight; the four partial sums are then added in
// the order ((0 + 1) + 2) + 3.  The order is fixed, so the result does not depend on scheduling; a frequent token (the
// synthetic tokens are Zipf distributed: the commonest one takes a tenth of the positions) costs a quarter of its count in
// dependent steps instead of all of it.
template <class T>
__global__ __launch_bounds__(256) void embed_grad_sorted_kernel(const int32_t* __restrict__ idx, const T* __restrict__ dx, float* __restrict__ gE, int T_, int d, int V) {
  constexpr int VEC = 16 / sizeof(T);          // elements per 16-byte piece
  __shared__ float part[3][64 * VEC];
  const int v = blockIdx.x;
  const int nh = idx[T_ + V + v], s0 = nh ? idx[T_ + v] : 0;
  const int hl = threadIdx.x >> 6, cl = threadIdx.x & 63;
  float* out = gE + (size_t)v * d;
  for (int c0 = 0; c0 < d; c0 += 64 * VEC) {          // uniform trip count: the barriers below are reached by every thread
    const int c = c0 + cl * VEC;
    float acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
    if (c < d) {
      int k = hl;
      for (; k + 12 < nh; k += 16) {          // four independent loads in flight
        uint4 w[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) w[u] = *reinterpret_cast<const uint4*>(dx + (size_t)idx[s0 + k + 4 * u] * d + c);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const T* pv = reinterpret_cast<const T*>(&w[u]);
#pragma unroll
          for (int e = 0; e < VEC; ++e) acc[e] += to_f32(pv[e]);
        }
      }
      for (; k < nh; k += 4) {
        const uint4 w = *reinterpret_cast<const uint4*>(dx + (size_t)idx[s0 + k] * d + c);
        const T* pv = reinterpret_cast<const T*>(&w);
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] += to_f32(pv[e]);
      }
    }
    __syncthreads();          // the previous piece's partials have been read
    if (hl > 0) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) part[hl - 1][cl * VEC + e] = acc[e];
    }
    __syncthreads();
    if (hl == 0 && c < d) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) out[c + e] = ((acc[e] + part[0][cl * VEC + e]) + part[1][cl * VEC + e]) + part[2][cl * VEC + e];
    }
  }
}
// scratch: (T + 2 V) ints of device memory that nothing else uses during the call, or nullptr (then every row scans the tokens)
void k_embed_grad(hipStream_t st, int dtype, const int32_t* tok, const void* dx, float* gE, int T_, int d, int V, int32_t* scratch) {
  const int vec = dtype == 0 ? 4 : 8;          // elements per 16 bytes (dtype 0 = float, else bf16)
  if (!scratch || d % vec || (reinterpret_cast<uintptr_t>(dx) & 15)) {          // no room for the index, or rows that 16-byte loads cannot take
    PP_DISPATCH(dtype, embed_grad_kernel<T><<<V, 256, 0, st>>>(tok, (const T*)dx, gE, T_, d));
    return;
  }
  k_fill_f32(st, reinterpret_cast<float*>(scratch + T_ + V), (size_t)V, 0.f);          // segment lengths := 0 (all-zero bits)
  embed_rank_kernel<<<cdiv(T_, 64), 64, 0, st>>>(tok, scratch, T_, V);
  PP_DISPATCH(dtype, embed_grad_sorted_kernel<T><<<V, 256, 0, st>>>(scratch, (const T*)dx, gE, T_, d, V));
}

// ------------------------------------------------------------------------------------------ packed-subset kernels
// Grid: (ceil(d / 1024), n_rows); 256 threads, 4 consecutive elements per thread (d % 4 == 0).
template <class T>
__global__ void pack_master_kernel(const T* __restrict__ params, const RowInfo* __restrict__ rows, float* __restrict__ p, int d) {
  const int row = blockIdx.y;
  const int c = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (c >= d) return;
  const T* src = params + rows[row].canon_off + c;
  float4 v = make_float4(to_f32(src[0]), to_f32(src[1]), to_f32(src[2]), to_f32(src[3]));
  *reinterpret_cast<float4*>(p + (size_t)row * d + c) = v;
}
void k_pack_master(hipStream_t st, int dtype, const void* params, const RowInfo* rows, float* p, int n_rows, int d) {
  if (n_rows == 0) return;
  dim3 grid(cdiv(d, 1024), n_rows);
  PP_DISPATCH(dtype, pack_master_kernel<T><<<grid, 256, 0, st>>>((const T*)params, rows, p, d));
}

template <class T> __device__ __forceinline__ void store4(T* dst, float4 v);
template <> __device__ __forceinline__ void store4<float>(float* dst, float4 v) { *reinterpret_cast<float4*>(dst) = v; }
template <> __device__ __forceinline__ void store4<bf16_t>(bf16_t* dst, float4 v) {
  uint2 w;
  w.x = f32x2_to_bf16x2(v.x, v.y);
  w.y = f32x2_to_bf16x2(v.z, v.w);
  *reinterpret_cast<uint2*>(dst) = w;
}

// Fused AdamW over the packed subset: reads g,p,m,v (fp32), writes p,m,v and the storage-dtype weight row.
template <class T>
__global__ void adamw_kernel(T* params, const RowInfo* __restrict__ rows, float* __restrict__ p, float* __restrict__ m,
                             float* __restrict__ v, const float* __restrict__ g, int d, float lr, float beta1, float beta2,
                             float eps, float wd, float inv_bc1, float inv_bc2) {
  const int row = blockIdx.y;
  const int c = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (c >= d) return;
  const RowInfo ri = rows[row];
  const size_t i = (size_t)row * d + c;
  const float4 g4 = *reinterpret_cast<const float4*>(g + i);
  float4 p4 = *reinterpret_cast<const float4*>(p + i);
  float4 m4 = *reinterpret_cast<const float4*>(m + i);
  float4 v4 = *reinterpret_cast<const float4*>(v + i);
  const float decay = 1.0f - lr * wd * ri.wd_on;
  const float gg[4] = {g4.x, g4.y, g4.z, g4.w};
  float pp[4] = {p4.x, p4.y, p4.z, p4.w}, mm[4] = {m4.x, m4.y, m4.z, m4.w}, vv[4] = {v4.x, v4.y, v4.z, v4.w};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    mm[k] = beta1 * mm[k] + (1.0f - beta1) * gg[k];
    vv[k] = beta2 * vv[k] + (1.0f - beta2) * gg[k] * gg[k];
    const float mhat = mm[k] * inv_bc1;
    const float vhat = vv[k] * inv_bc2;
    pp[k] = pp[k] * decay - lr * mhat / (sqrtf(vhat) + eps);
  }
  p4 = make_float4(pp[0], pp[1], pp[2], pp[3]);
  *reinterpret_cast<float4*>(p + i) = p4;
  *reinterpret_cast<float4*>(m + i) = make_float4(mm[0], mm[1], mm[2], mm[3]);
  *reinterpret_cast<float4*>(v + i) = make_float4(vv[0], vv[1], vv[2], vv[3]);
  store4<T>(params + ri.canon_off + c, p4);
}
void k_adamw(hipStream_t st, int dtype, void* params, const RowInfo* rows, float* p, float* m, float* v, const float* g,
             int n_rows, int d, float lr, float beta1, float beta2, float eps, float wd, float bc1, float bc2) {
  if (n_rows == 0) return;
  dim3 grid(cdiv(d, 1024), n_rows);
  PP_DISPATCH(dtype, adamw_kernel<T><<<grid, 256, 0, st>>>((T*)params, rows, p, m, v, g, d, lr, beta1, beta2, eps, wd, 1.0f / bc1, 1.0f / bc2));
}

// Outer step on the packed subset (delta, count normalisation, momentum SGD); restarts the local copy.
template <class T>
__global__ void outer_kernel(T* params, const RowInfo* __restrict__ rows, float* __restrict__ master, float* __restrict__ theta_g,
                             float* __restrict__ mom, const float* __restrict__ others, float* __restrict__ delta_out, int d,
                             float lr, float mu, int nesterov, float inv_m) {
  const int row = blockIdx.y;
  const int c = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (c >= d) return;
  const RowInfo ri = rows[row];
  const size_t i = (size_t)row * d + c;
  T* w = params + ri.canon_off + c;
  const float4 tg4 = *reinterpret_cast<const float4*>(theta_g + i);
  const float4 b4 = *reinterpret_cast<const float4*>(mom + i);
  float4 o4 = make_float4(0.f, 0.f, 0.f, 0.f);
  if (others) o4 = *reinterpret_cast<const float4*>(others + i);
  const float tg[4] = {tg4.x, tg4.y, tg4.z, tg4.w}, bb[4] = {b4.x, b4.y, b4.z, b4.w}, oo[4] = {o4.x, o4.y, o4.z, o4.w};
  float nt[4], nb[4], dl[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const float tl = to_f32(w[k]);
    dl[k] = (tg[k] - tl + oo[k]) * inv_m;
    nb[k] = mu * bb[k] + dl[k];
    const float upd = nesterov ? dl[k] + mu * nb[k] : nb[k];
    nt[k] = tg[k] - lr * upd;
  }
  const float4 nt4 = make_float4(nt[0], nt[1], nt[2], nt[3]);
  *reinterpret_cast<float4*>(theta_g + i) = nt4;
  *reinterpret_cast<float4*>(mom + i) = make_float4(nb[0], nb[1], nb[2], nb[3]);
  if (delta_out) *reinterpret_cast<float4*>(delta_out + i) = make_float4(dl[0], dl[1], dl[2], dl[3]);
  *reinterpret_cast<float4*>(master + i) = nt4;
  store4<T>(w, nt4);
}
void k_outer(hipStream_t st, int dtype, void* params, const RowInfo* rows, float* master, float* theta_g, float* mom,
             const float* others, float* delta_out, int n_rows, int d, float lr, float mu, int nesterov, float inv_m) {
  if (n_rows == 0) return;
  dim3 grid(cdiv(d, 1024), n_rows);
  PP_DISPATCH(dtype, outer_kernel<T><<<grid, 256, 0, st>>>((T*)params, rows, master, theta_g, mom, others, delta_out, d, lr, mu, nesterov, inv_m));
}

// Counter-based normal variates: x_i = mix(key + i*GOLD) (splitmix64 finaliser), u = ((x>>11)+0.5)*2^-53,
// Box-Muller on the uniform pair (2j, 2j+1): element 2j = r cos, element 2j+1 = r sin.
__device__ __forceinline__ uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
__global__ void synth_delta_sum_kernel(float* __restrict__ dst, size_t n, const uint64_t* __restrict__ keys, int n_nodes, double std) {
  const size_t pair = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t i0 = 2 * pair;
  if (i0 >= n) return;
  double a0 = 0.0, a1 = 0.0;
  for (int j = 0; j < n_nodes; ++j) {
    const uint64_t key = keys[j];
    const double u1 = ((double)(mix64(key + i0 * 0x9E3779B97F4A7C15ull) >> 11) + 0.5) * (1.0 / 9007199254740992.0);
    const double u2 = ((double)(mix64(key + (i0 + 1) * 0x9E3779B97F4A7C15ull) >> 11) + 0.5) * (1.0 / 9007199254740992.0);
    const double r = sqrt(-2.0 * log(u1)), ang = 6.283185307179586476925287 * u2;
    a0 += r * cos(ang) * std;
    a1 += r * sin(ang) * std;
  }
  dst[i0] = (float)a0;
  if (i0 + 1 < n) dst[i0 + 1] = (float)a1;
}
void k_synth_delta_sum(hipStream_t st, float* dst, size_t n, const uint64_t* keys_dev, int n_nodes, float std) {
  if (n == 0) return;
  synth_delta_sum_kernel<<<cdiv((n + 1) / 2, 256), 256, 0, st>>>(dst, n, keys_dev, n_nodes, (double)std);
}

}  // namespace pp

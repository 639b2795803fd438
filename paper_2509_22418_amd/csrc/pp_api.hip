// C ABI of the partial-parameter-update local step: handle, memory plan, and the launch sequence of one
// local step (forward over all parameters, restricted backward, AdamW on the trainable subset) and of the
// outer pseudo-gradient step.  All device memory belongs to the caller; see include/pp.h.
#include "../../include/pp.h"
#include "pp_kernels.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

using namespace pp;

static thread_local std::string g_err;
static int fail(int code, const std::string& msg) { g_err = msg; return code; }
extern "C" const char* pp_last_error(void) { return g_err.c_str(); }

#define HIPCHECK(expr)                                                                            \
  do {                                                                                            \
    hipError_t e_ = (expr);                                                                       \
    if (e_ != hipSuccess) return fail(PP_EHIP, std::string(#expr) + ": " + hipGetErrorString(e_)); \
  } while (0)

static inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

namespace {

enum TensorKind { TK_EMBED = 0, TK_ATTN_NORM, TK_WQKV, TK_WO, TK_FFN_NORM, TK_WG, TK_WU, TK_WD, TK_FINAL_NORM, TK_LM_HEAD };

struct Layout {          // element offsets
  int64_t embed, layer0, layer_stride, final_norm, lm_head, n_params;
  int64_t o_attn_norm, o_wqkv, o_wo, o_ffn_norm, o_wg, o_wu, o_wd;
  int64_t sh_layer0, sh_layer_stride, sh_wqkv, sh_wo, sh_wgu, sh_wd, sh_lm_head, n_shadow;
};

static Layout make_layout(const pp_config& c) {
  Layout L{};
  const int64_t d = c.d_model, F = c.d_ff, V = c.vocab;
  L.embed = 0;
  L.layer0 = V * d;
  L.o_attn_norm = 0;
  L.o_wqkv = d;
  L.o_wo = L.o_wqkv + 3 * d * d;
  L.o_ffn_norm = L.o_wo + d * d;
  L.o_wg = L.o_ffn_norm + d;
  L.o_wu = L.o_wg + F * d;
  L.o_wd = L.o_wu + F * d;
  L.layer_stride = L.o_wd + F * d;
  L.final_norm = L.layer0 + c.n_layers * L.layer_stride;
  L.lm_head = L.final_norm + d;
  L.n_params = L.lm_head + V * d;
  L.sh_wqkv = 0;
  L.sh_wo = 3 * d * d;
  L.sh_wgu = L.sh_wo + d * d;
  L.sh_wd = L.sh_wgu + 2 * F * d;
  L.sh_layer_stride = L.sh_wd + F * d;
  L.sh_layer0 = 0;
  L.sh_lm_head = c.n_layers * L.sh_layer_stride;
  L.n_shadow = L.sh_lm_head + V * d;
  return L;
}

struct Mask { bool emb, norms, wo, lm, heads, ffn; int fl, fh, hl, hh; };
static Mask norm_mask(const pp_config& c, const pp_mask& m) {
  Mask r{};
  if (m.all) { r.emb = r.norms = r.wo = r.lm = r.heads = r.ffn = true; r.fl = 0; r.fh = c.d_ff; r.hl = 0; r.hh = c.n_heads; return r; }
  r.emb = m.train_embed != 0; r.norms = m.train_norms != 0; r.wo = m.train_wo != 0; r.lm = m.train_lm_head != 0;
  r.fl = m.ffn_lo; r.fh = m.ffn_hi; r.hl = m.head_lo; r.hh = m.head_hi;
  r.ffn = r.fh > r.fl; r.heads = r.hh > r.hl;
  return r;
}

struct Seg { int kind, layer; int64_t canon_off; int row_lo, rows; int64_t packed_off; bool decay; int64_t shadow_off; int shadow_ld; };

struct WsPlan {          // byte offsets into the workspace
  size_t rope_cos, rope_sin, shadow, rows, segs, keys;
  size_t act0, act_stride;          // per layer (recompute: the layer input only)
  size_t act_shared;                // recompute: the one block that holds the other activations of the layer in work
  bool recompute;
  size_t a_x, a_n1, a_qkv, a_o, a_xm, a_n2, a_gu, a_a, a_rstd1, a_rstd2, a_lse;      // within a layer's block
  size_t xL, nf, rstdf, logits, rowloss, nvalid, dgpart;
  size_t dx, dn, dA, dgu, dob, dqkv, Dattn;
  size_t fixed_end;      // everything above is mask independent
  size_t tA, tB, partial, partial_bytes, total;
  size_t act_bytes, shadow_bytes;
};

static size_t esize(const pp_config& c) { return c.dtype == PP_F32 ? 4 : 2; }
static const size_t kPartialCap = 64ull << 20;

static WsPlan plan_ws(const pp_config& c, const Mask* mk) {
  WsPlan p{};
  const size_t es = esize(c), d = c.d_model, F = c.d_ff, V = c.vocab, h = c.n_heads, dh = d / h;
  const size_t T = (size_t)c.max_batch * c.max_seq;
  const Layout L = make_layout(c);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  p.rope_cos = take((size_t)c.max_seq * (dh / 2) * 4);
  p.rope_sin = take((size_t)c.max_seq * (dh / 2) * 4);
  p.shadow_bytes = (size_t)L.n_shadow * es;
  p.shadow = take(p.shadow_bytes);
  p.rows = take((size_t)(L.n_params / d) * sizeof(RowInfo));
  p.segs = take((size_t)(4 + 10 * c.n_layers) * sizeof(ShadowSeg));
  p.keys = take(256 * sizeof(uint64_t));
  // saved activations, one block per layer
  size_t lo = 0;
  auto ltake = [&](size_t bytes) { size_t o = lo; lo = align_up(lo + bytes); return o; };
  p.a_x = ltake(T * d * es); p.a_n1 = ltake(T * d * es); p.a_qkv = ltake(T * 3 * d * es); p.a_o = ltake(T * d * es);
  p.a_xm = ltake(T * d * es); p.a_n2 = ltake(T * d * es); p.a_gu = ltake(T * 2 * F * es); p.a_a = ltake(T * F * es);
  p.a_rstd1 = ltake(T * 4); p.a_rstd2 = ltake(T * 4); p.a_lse = ltake((size_t)c.max_batch * h * c.max_seq * 4);
  p.recompute = c.recompute != 0;
  if (p.recompute) {          // per layer: x only (a_x = 0 is the first field of the block); everything else lives once
    p.act_stride = align_up(T * d * es);
    p.act0 = take(p.act_stride * c.n_layers);
    p.act_shared = take(lo);
  } else {
    p.act_stride = lo;
    p.act0 = take(p.act_stride * c.n_layers);
    p.act_shared = 0;
  }
  p.xL = take(T * d * es); p.nf = take(T * d * es); p.rstdf = take(T * 4); p.logits = take(T * V * es);
  p.act_bytes = off - p.act0;
  p.rowloss = take(T * 4); p.nvalid = take(256); p.dgpart = take(64 * d * 4);
  p.dx = take(T * d * es); p.dn = take(T * d * es); p.dA = take(T * F * es); p.dgu = take(T * 2 * F * es);
  p.dob = take(T * d * es); p.dqkv = take(T * 3 * d * es); p.Dattn = take((size_t)c.max_batch * h * c.max_seq * 4);
  p.fixed_end = off;
  // mask-dependent scratch for the weight-gradient GEMMs (operands transposed to K-contiguous form)
  Mask all{}; all.emb = all.norms = all.wo = all.lm = all.heads = all.ffn = true; all.fl = 0; all.fh = c.d_ff; all.hl = 0; all.hh = c.n_heads;
  const Mask& m = mk ? *mk : all;
  size_t rowsA = 0;
  if (m.ffn) rowsA = std::max(rowsA, (size_t)2 * (m.fh - m.fl));
  if (m.heads) rowsA = std::max(rowsA, (size_t)3 * (m.hh - m.hl) * dh);
  if (m.wo) rowsA = std::max(rowsA, d);
  if (m.lm) rowsA = std::max(rowsA, V);
  const bool any_dw = rowsA > 0;
  p.tA = take(rowsA * T * es);
  p.tB = take(any_dw ? d * T * es : 0);
  p.partial_bytes = any_dw ? kPartialCap : 0;
  p.partial = take(p.partial_bytes);
  p.total = off;
  return p;
}

}  // namespace

struct pp_model {
  pp_config cfg;
  Layout lay;
  WsPlan ws;
  char* params;
  char* wsp;
  size_t ws_bytes;
  hipStream_t st;
  bool has_mask = false;
  Mask mask{};
  std::vector<Seg> segs;
  int64_t n_train = 0;
  int n_rows = 0, n_shadow_segs = 0, n_shadow_tiles = 0, shadow_vec_ok = 0;
  float *sp = nullptr, *sm = nullptr, *sv = nullptr, *sg = nullptr;
  long step = 0;
  int force_plain = 0;
  int fuse_rope = 1;      // rotary embedding inside the q | k | v projection's epilogue (0: separate pass, for A/B timing)
  int dw_tn = 1;          // weight-gradient GEMMs read token-major operands directly (0: via transposed copies, for A/B timing)
  int jac_mode = 0, jac_lo = 0, jac_hi = 0;          // ablation: FFN input Jacobian over the trainable slice (+ units jac_lo..jac_hi-1) only
  double flops_fwd = 0, flops_bwd = 0, flops_recompute = 0, adamw_bytes = 0;
  int64_t n_mfma = 0, n_plain = 0;          // contractions (GEMM / attention calls) of the last step by kernel family
  double* flop_acc = nullptr;
  // optional GEMM timing: one event pair per GEMM launch, summed by pp_get_gemm_timing
  int time_gemm = 0;
  std::vector<hipEvent_t> ev;
  size_t ev_used = 0;
  double timed_flops = 0;
  ~pp_model() { for (hipEvent_t e : ev) hipEventDestroy(e); }
};

namespace {
struct GemmTimer {          // brackets the launches issued during its lifetime
  pp_model* m; double flops; bool on = false; size_t idx = 0;
  GemmTimer(pp_model* m_, double flops_) : m(m_), flops(flops_) {
    if (!m->time_gemm) return;
    if (m->ev_used + 2 > m->ev.size()) {
      hipEvent_t a, b;
      if (hipEventCreate(&a) != hipSuccess) return;
      if (hipEventCreate(&b) != hipSuccess) { hipEventDestroy(a); return; }
      m->ev.push_back(a); m->ev.push_back(b);
    }
    idx = m->ev_used; m->ev_used += 2; on = true;
    hipEventRecord(m->ev[idx], m->st);
  }
  void cancel() { if (on) { on = false; m->ev_used -= 2; } }          // nothing was launched: give the event pair back
  ~GemmTimer() { if (on) { hipEventRecord(m->ev[idx + 1], m->st); m->timed_flops += flops; } }
};
}  // namespace

// ------------------------------------------------------------------------------------------------ helpers
static int check_cfg(const pp_config* c) {
  if (!c) return fail(PP_EINVAL, "config is NULL");
  if (c->n_layers < 1 || c->d_model < 8 || c->n_heads < 1 || c->d_ff < 8 || c->vocab < 8 || c->max_batch < 1 || c->max_seq < 1)
    return fail(PP_EINVAL, "config: non-positive dimension");
  if (c->dtype != PP_F32 && c->dtype != PP_BF16) return fail(PP_EINVAL, "config: dtype must be PP_F32 or PP_BF16");
  if (c->recompute != 0 && c->recompute != 1) return fail(PP_EINVAL, "config: recompute must be 0 or 1");
  if (c->d_model % c->n_heads) return fail(PP_EINVAL, "config: d_model must be a multiple of n_heads");
  const int dh = c->d_model / c->n_heads;
  if (dh % 2 || dh > 256) return fail(PP_EINVAL, "config: head dim must be even and <= 256");
  if (c->d_model % 8 || c->d_ff % 8 || c->vocab % 8) return fail(PP_EINVAL, "config: d_model, d_ff and vocab must be multiples of 8");
  if (!ce_row_fits(c->dtype, c->vocab))
    return fail(PP_EINVAL, c->dtype == PP_BF16 ? "config: vocab > 65536 is not supported by the cross-entropy kernels (bf16)"
                                               : "config: vocab row does not fit the cross-entropy LDS stage (fp32: vocab <= 16320)");
  if (c->max_seq > 8192) return fail(PP_EINVAL, "config: max_seq > 8192 not supported");
  if ((double)c->max_batch * c->max_seq > 1e8) return fail(PP_EINVAL, "config: max_batch*max_seq too large");
  if (!(c->rms_eps > 0.f) || !(c->rope_base > 1.f)) return fail(PP_EINVAL, "config: rms_eps must be > 0 and rope_base > 1");
  return PP_OK;
}
static int check_mask(const pp_config* c, const pp_mask* m) {
  if (!m) return fail(PP_EINVAL, "mask is NULL");
  if (m->all) return PP_OK;
  if (m->ffn_lo < 0 || m->ffn_hi < m->ffn_lo || m->ffn_hi > c->d_ff) return fail(PP_EINVAL, "mask: ffn range outside [0, d_ff]");
  if (m->head_lo < 0 || m->head_hi < m->head_lo || m->head_hi > c->n_heads) return fail(PP_EINVAL, "mask: head range outside [0, n_heads]");
  if (m->ffn_lo % 8 || m->ffn_hi % 8) return fail(PP_EINVAL, "mask: ffn range bounds must be multiples of 8");
  return PP_OK;
}

static std::vector<Seg> build_segs(const pp_config& c, const Layout& L, const Mask& m, int64_t* n_train) {
  std::vector<Seg> s;
  const int64_t d = c.d_model, F = c.d_ff;
  const int dh = c.d_model / c.n_heads;
  int64_t poff = 0;
  auto add = [&](int kind, int layer, int64_t tensor_off, int row_lo, int rows, bool decay, int64_t sh_off, int sh_ld) {
    Seg g{kind, layer, tensor_off + (int64_t)row_lo * d, row_lo, rows, poff, decay, sh_off, sh_ld};
    s.push_back(g);
    poff += (int64_t)rows * d;
  };
  if (m.emb) add(TK_EMBED, -1, L.embed, 0, c.vocab, true, -1, 0);
  for (int l = 0; l < c.n_layers; ++l) {
    const int64_t lb = L.layer0 + l * L.layer_stride, sb = L.sh_layer0 + l * L.sh_layer_stride;
    if (m.norms) add(TK_ATTN_NORM, l, lb + L.o_attn_norm, 0, 1, false, -1, 0);
    if (m.heads)
      for (int blk = 0; blk < 3; ++blk) {
        const int r0 = blk * (int)d + m.hl * dh;
        add(TK_WQKV, l, lb + L.o_wqkv, r0, (m.hh - m.hl) * dh, true, sb + L.sh_wqkv + r0, 3 * (int)d);
      }
    if (m.wo) add(TK_WO, l, lb + L.o_wo, 0, (int)d, true, sb + L.sh_wo, (int)d);
    if (m.norms) add(TK_FFN_NORM, l, lb + L.o_ffn_norm, 0, 1, false, -1, 0);
    if (m.ffn) {
      add(TK_WG, l, lb + L.o_wg, m.fl, m.fh - m.fl, true, sb + L.sh_wgu + m.fl, 2 * (int)F);
      add(TK_WU, l, lb + L.o_wu, m.fl, m.fh - m.fl, true, sb + L.sh_wgu + F + m.fl, 2 * (int)F);
      add(TK_WD, l, lb + L.o_wd, m.fl, m.fh - m.fl, true, sb + L.sh_wd + m.fl, (int)F);
    }
  }
  if (m.norms) add(TK_FINAL_NORM, -1, L.final_norm, 0, 1, false, -1, 0);
  if (m.lm) add(TK_LM_HEAD, -1, L.lm_head, 0, c.vocab, true, L.sh_lm_head, c.vocab);
  *n_train = poff;
  return s;
}

static const Seg* find_seg(const pp_model* m, int kind, int layer, int nth = 0) {
  for (const Seg& s : m->segs)
    if (s.kind == kind && s.layer == layer) { if (nth == 0) return &s; --nth; }
  return nullptr;
}

struct TensorRef { int64_t off, count; int64_t sh_off; int rows, cols, sh_ld; };
static bool lookup_tensor(const pp_model* m, const char* name, TensorRef* r) {
  const pp_config& c = m->cfg;
  const Layout& L = m->lay;
  const int64_t d = c.d_model, F = c.d_ff, V = c.vocab;
  std::string n(name);
  auto set = [&](int64_t off, int rows, int cols, int64_t sh, int shld) { *r = TensorRef{off, (int64_t)rows * cols, sh, rows, cols, shld}; return true; };
  if (n == "embed") return set(L.embed, (int)V, (int)d, -1, 0);
  if (n == "final_norm") return set(L.final_norm, 1, (int)d, -1, 0);
  if (n == "lm_head") return set(L.lm_head, (int)V, (int)d, L.sh_lm_head, (int)V);
  int l = -1, consumed = 0;
  if (sscanf(name, "layers.%d.%n", &l, &consumed) == 1 && consumed > 0 && l >= 0 && l < c.n_layers) {
    std::string t(name + consumed);
    const int64_t lb = L.layer0 + l * L.layer_stride, sb = L.sh_layer0 + l * L.sh_layer_stride;
    if (t == "attn_norm") return set(lb + L.o_attn_norm, 1, (int)d, -1, 0);
    if (t == "wqkv") return set(lb + L.o_wqkv, 3 * (int)d, (int)d, sb + L.sh_wqkv, 3 * (int)d);
    if (t == "wo") return set(lb + L.o_wo, (int)d, (int)d, sb + L.sh_wo, (int)d);
    if (t == "ffn_norm") return set(lb + L.o_ffn_norm, 1, (int)d, -1, 0);
    if (t == "wg") return set(lb + L.o_wg, (int)F, (int)d, sb + L.sh_wgu, 2 * (int)F);
    if (t == "wu") return set(lb + L.o_wu, (int)F, (int)d, sb + L.sh_wgu + F, 2 * (int)F);
    if (t == "wd") return set(lb + L.o_wd, (int)F, (int)d, sb + L.sh_wd, (int)F);
  }
  return false;
}

// ------------------------------------------------------------------------------------------------ queries / lifetime
extern "C" size_t pp_query_bytes(const pp_config* cfg, const pp_mask* mask, int which) {
  if (check_cfg(cfg) != PP_OK) return 0;
  if (mask && check_mask(cfg, mask) != PP_OK) return 0;
  const Layout L = make_layout(*cfg);
  Mask mk{};
  if (mask) mk = norm_mask(*cfg, *mask);
  switch (which) {
    case PP_BYTES_PARAMS: return align_up((size_t)L.n_params * esize(*cfg));
    case PP_BYTES_STATE: {
      if (!mask) { fail(PP_EINVAL, "pp_query_bytes(STATE) needs a mask"); return 0; }
      int64_t n = 0;
      build_segs(*cfg, L, mk, &n);
      return align_up((size_t)n * 4) * 4;
    }
    case PP_BYTES_WORKSPACE: return plan_ws(*cfg, mask ? &mk : nullptr).total;
    case PP_BYTES_SHADOW: return plan_ws(*cfg, mask ? &mk : nullptr).shadow_bytes;
    case PP_BYTES_ACTIVATIONS: return plan_ws(*cfg, mask ? &mk : nullptr).act_bytes;
    default: fail(PP_EINVAL, "pp_query_bytes: unknown selector"); return 0;
  }
}

extern "C" int pp_init_model(const pp_config* cfg, void* params_dev, size_t params_bytes, void* workspace_dev,
                             size_t workspace_bytes, void* hip_stream, pp_model** out) {
  if (int rc = check_cfg(cfg)) return rc;
  if (!params_dev || !workspace_dev || !out) return fail(PP_EINVAL, "pp_init_model: NULL pointer");
  if (((uintptr_t)params_dev | (uintptr_t)workspace_dev) & 255) return fail(PP_EINVAL, "pp_init_model: buffers must be 256-byte aligned");
  const Layout L = make_layout(*cfg);
  if (params_bytes < (size_t)L.n_params * esize(*cfg)) return fail(PP_EINVAL, "pp_init_model: params buffer too small");
  Mask none{};
  const WsPlan base = plan_ws(*cfg, &none);
  if (workspace_bytes < base.total) return fail(PP_EINVAL, "pp_init_model: workspace smaller than the minimum for this config");
  pp_model* m = new (std::nothrow) pp_model();
  if (!m) return fail(PP_ENOMEM, "pp_init_model: host allocation failed");
  m->cfg = *cfg; m->lay = L; m->ws = base;
  m->params = (char*)params_dev; m->wsp = (char*)workspace_dev; m->ws_bytes = workspace_bytes;
  m->st = (hipStream_t)hip_stream;
  k_rope_tables(m->st, (float*)(m->wsp + base.rope_cos), (float*)(m->wsp + base.rope_sin), cfg->max_seq, cfg->d_model / cfg->n_heads, cfg->rope_base);
  hipError_t e = hipStreamSynchronize(m->st);
  if (e == hipSuccess) e = hipGetLastError();
  if (e != hipSuccess) { delete m; return fail(PP_EHIP, std::string("pp_init_model: ") + hipGetErrorString(e)); }
  *out = m;
  return PP_OK;
}

extern "C" void pp_free(pp_model* m) { delete m; }

extern "C" int pp_set_option(pp_model* m, const char* key, int64_t value) {
  if (key && !strcmp(key, "gemm_variant")) { gemm_set_variant((int)value); return PP_OK; }          // process-wide, no model needed
  if (key && !strcmp(key, "gemm_persistent")) { gemm_set_persistent(value != 0); return PP_OK; }
  if (key && !strcmp(key, "gemm_small_tiles")) { gemm_set_small_tiles(value != 0); return PP_OK; }
  if (!m || !key) return fail(PP_EINVAL, "pp_set_option: NULL");
  if (!strcmp(key, "force_plain")) { m->force_plain = value != 0; return PP_OK; }
  if (!strcmp(key, "dw_tn")) { m->dw_tn = value != 0; return PP_OK; }
  if (!strcmp(key, "fuse_rope")) { m->fuse_rope = value != 0; return PP_OK; }
  if (!strcmp(key, "gemm_variant")) { gemm_set_variant((int)value); return PP_OK; }
  if (!strcmp(key, "time_gemm")) {
    if (hipStreamSynchronize(m->st) != hipSuccess) return fail(PP_EHIP, "pp_set_option: stream sync failed");
    m->time_gemm = value != 0; m->ev_used = 0; m->timed_flops = 0;
    return PP_OK;
  }
  return fail(PP_EINVAL, std::string("pp_set_option: unknown key ") + key);
}

extern "C" int pp_set_jacobian_slices(pp_model* m, int32_t mode, int32_t extra_lo, int32_t extra_hi) {
  if (!m) return fail(PP_EINVAL, "pp_set_jacobian_slices: NULL");
  if (mode != 0 && mode != 1) return fail(PP_EINVAL, "pp_set_jacobian_slices: mode must be 0 (full Jacobian) or 1 (trainable slice + extra range only)");
  if (mode == 0) { m->jac_mode = 0; m->jac_lo = m->jac_hi = 0; return PP_OK; }
  if (extra_lo < 0 || extra_hi < extra_lo || extra_hi > m->cfg.d_ff) return fail(PP_EINVAL, "pp_set_jacobian_slices: extra range outside [0, d_ff]");
  if (extra_lo % 8 || extra_hi % 8) return fail(PP_EINVAL, "pp_set_jacobian_slices: extra range bounds must be multiples of 8");
  m->jac_mode = 1; m->jac_lo = extra_lo; m->jac_hi = extra_hi;
  return PP_OK;
}

// ------------------------------------------------------------------------------------------------ tensor I/O
extern "C" int pp_set_tensor(pp_model* m, const char* name, const void* host_src, size_t bytes) {
  if (!m || !name || !host_src) return fail(PP_EINVAL, "pp_set_tensor: NULL");
  TensorRef r;
  if (!lookup_tensor(m, name, &r)) return fail(PP_EINVAL, std::string("pp_set_tensor: unknown tensor ") + name);
  const size_t es = esize(m->cfg);
  if (bytes != (size_t)r.count * es) return fail(PP_EINVAL, std::string("pp_set_tensor: byte count mismatch for ") + name);
  HIPCHECK(hipMemcpyAsync(m->params + r.off * es, host_src, bytes, hipMemcpyHostToDevice, m->st));
  if (r.sh_off >= 0)
    k_transpose(m->st, m->cfg.dtype, m->params + r.off * es, r.cols, m->wsp + m->ws.shadow + r.sh_off * es, r.sh_ld, r.rows, r.cols);
  HIPCHECK(hipStreamSynchronize(m->st));
  HIPCHECK(hipGetLastError());
  return PP_OK;
}

extern "C" int pp_get_tensor(pp_model* m, const char* name, void* host_dst, size_t bytes) {
  if (!m || !name || !host_dst) return fail(PP_EINVAL, "pp_get_tensor: NULL");
  const size_t es = esize(m->cfg);
  const void* src = nullptr;
  size_t want = 0;
  std::vector<int64_t> rowoffs;
  std::string n(name);
  TensorRef r;
  if (n.rfind("state.", 0) == 0) {
    if (!m->has_mask) return fail(PP_ESTATE, "pp_get_tensor: no trainable mask set");
    want = (size_t)m->n_train * 4;
    if (n == "state.p") src = m->sp; else if (n == "state.m") src = m->sm; else if (n == "state.v") src = m->sv;
    else if (n == "state.g") src = m->sg;
    else if (n == "state.rows") {
      for (const Seg& s : m->segs) for (int i = 0; i < s.rows; ++i) rowoffs.push_back(s.canon_off + (int64_t)i * m->cfg.d_model);
      want = rowoffs.size() * 8;
      if (bytes != want) return fail(PP_EINVAL, "pp_get_tensor: byte count mismatch for state.rows");
      memcpy(host_dst, rowoffs.data(), want);
      return PP_OK;
    } else return fail(PP_EINVAL, std::string("pp_get_tensor: unknown tensor ") + name);
  } else if (n.rfind("dbg.", 0) == 0) {
    // debugging taps into the workspace: dbg.<buffer>[.<layer>], sized for max_batch*max_seq tokens
    const pp_config& c = m->cfg;
    const size_t T = (size_t)c.max_batch * c.max_seq, d = c.d_model, F = c.d_ff;
    char buf[32]; int l = 0;
    if (sscanf(name, "dbg.%31[a-z0-9A-Z_].%d", buf, &l) < 1) return fail(PP_EINVAL, "pp_get_tensor: bad dbg name");
    if (l < 0 || l >= c.n_layers) return fail(PP_EINVAL, "pp_get_tensor: dbg layer out of range");
    std::string b(buf);
    const char* lx = m->wsp + m->ws.act0 + (size_t)l * m->ws.act_stride;          // the layer's own block
    const char* lb = m->ws.recompute ? m->wsp + m->ws.act_shared : lx;                // where its other activations are
    if (b == "x") { src = lx + m->ws.a_x; want = T * d * es; }
    else if (b == "n1") { src = lb + m->ws.a_n1; want = T * d * es; }
    else if (b == "qkv") { src = lb + m->ws.a_qkv; want = T * 3 * d * es; }
    else if (b == "o") { src = lb + m->ws.a_o; want = T * d * es; }
    else if (b == "xm") { src = lb + m->ws.a_xm; want = T * d * es; }
    else if (b == "n2") { src = lb + m->ws.a_n2; want = T * d * es; }
    else if (b == "gu") { src = lb + m->ws.a_gu; want = T * 2 * F * es; }
    else if (b == "a") { src = lb + m->ws.a_a; want = T * F * es; }
    else if (b == "lse") { src = lb + m->ws.a_lse; want = (size_t)c.max_batch * c.n_heads * c.max_seq * 4; }
    else if (b == "xL") { src = m->wsp + m->ws.xL; want = T * d * es; }
    else if (b == "logits") { src = m->wsp + m->ws.logits; want = T * (size_t)c.vocab * es; }
    else if (b == "dx") { src = m->wsp + m->ws.dx; want = T * d * es; }
    else if (b == "dn") { src = m->wsp + m->ws.dn; want = T * d * es; }
    else if (b == "dqkv") { src = m->wsp + m->ws.dqkv; want = T * 3 * d * es; }
    else if (b == "dgu") { src = m->wsp + m->ws.dgu; want = T * 2 * F * es; }
    else return fail(PP_EINVAL, std::string("pp_get_tensor: unknown dbg buffer ") + name);
  } else if (n.rfind("shadow.", 0) == 0) {
    if (!lookup_tensor(m, name + 7, &r) || r.sh_off < 0) return fail(PP_EINVAL, std::string("pp_get_tensor: no shadow for ") + name);
    // shadow images are strided (row length sh_ld); only whole-matrix images are contiguous: wqkv, wo, wd, lm_head
    if (r.sh_ld != r.rows) return fail(PP_EINVAL, "pp_get_tensor: shadow of wg/wu is interleaved; read shadow via wd/wqkv/wo/lm_head only");
    src = m->wsp + m->ws.shadow + r.sh_off * es; want = (size_t)r.count * es;
  } else {
    if (!lookup_tensor(m, name, &r)) return fail(PP_EINVAL, std::string("pp_get_tensor: unknown tensor ") + name);
    src = m->params + r.off * es; want = (size_t)r.count * es;
  }
  if (bytes != want) return fail(PP_EINVAL, std::string("pp_get_tensor: byte count mismatch for ") + name);
  if (want == 0) return PP_OK;
  HIPCHECK(hipMemcpyAsync(host_dst, src, bytes, hipMemcpyDeviceToHost, m->st));
  HIPCHECK(hipStreamSynchronize(m->st));
  return PP_OK;
}

// ------------------------------------------------------------------------------------------------ mask / state
// Every transposed read-only weight copy is formed again from the canonical parameter buffer (one transpose per matrix).
static void rebuild_shadows(pp_model* m) {
  const pp_config& c = m->cfg;
  const Layout& L = m->lay;
  const size_t es = esize(c);
  const int d = c.d_model, F = c.d_ff, V = c.vocab;
  char* sh = m->wsp + m->ws.shadow;
  auto tr = [&](int64_t off, int rows, int cols, int64_t sh_off, int sh_ld) {
    k_transpose(m->st, c.dtype, m->params + off * es, cols, sh + sh_off * es, sh_ld, rows, cols);
  };
  for (int l = 0; l < c.n_layers; ++l) {
    const int64_t lb = L.layer0 + l * L.layer_stride, sb = L.sh_layer0 + l * L.sh_layer_stride;
    tr(lb + L.o_wqkv, 3 * d, d, sb + L.sh_wqkv, 3 * d);
    tr(lb + L.o_wo, d, d, sb + L.sh_wo, d);
    tr(lb + L.o_wg, F, d, sb + L.sh_wgu, 2 * F);
    tr(lb + L.o_wu, F, d, sb + L.sh_wgu + F, 2 * F);
    tr(lb + L.o_wd, F, d, sb + L.sh_wd, F);
  }
  tr(L.lm_head, V, d, L.sh_lm_head, V);
}

extern "C" int pp_set_trainable_mask(pp_model* m, const pp_mask* mask, void* state_dev, size_t state_bytes) {
  if (!m) return fail(PP_EINVAL, "pp_set_trainable_mask: NULL model");
  if (int rc = check_mask(&m->cfg, mask)) return rc;
  const Mask mk = norm_mask(m->cfg, *mask);
  int64_t n = 0;
  std::vector<Seg> segs = build_segs(m->cfg, m->lay, mk, &n);
  const size_t quarter = align_up((size_t)n * 4);
  if (n > 0 && (!state_dev || state_bytes < quarter * 4)) return fail(PP_EINVAL, "pp_set_trainable_mask: state buffer too small");
  if ((uintptr_t)state_dev & 255) return fail(PP_EINVAL, "pp_set_trainable_mask: state buffer must be 256-byte aligned");
  const WsPlan plan = plan_ws(m->cfg, &mk);
  if (plan.total > m->ws_bytes) return fail(PP_EINVAL, "pp_set_trainable_mask: workspace too small for this mask (see pp_query_bytes)");
  const int d = m->cfg.d_model;
  // host tables: one RowInfo per packed row, one ShadowSeg per trainable block with a shadow image
  std::vector<RowInfo> rows;
  std::vector<ShadowSeg> ssegs;
  int tiles = 0, vec_ok = 1;
  for (const Seg& s : segs) {
    for (int i = 0; i < s.rows; ++i) rows.push_back(RowInfo{s.canon_off + (int64_t)i * d, s.decay ? 1.f : 0.f, 0});
    if (s.shadow_off >= 0) {
      ssegs.push_back(ShadowSeg{s.canon_off, s.shadow_off, s.rows, d, s.shadow_ld, tiles});
      if ((s.rows | d | s.shadow_ld) & 7 || (s.canon_off | s.shadow_off) & 7) vec_ok = 0;
      tiles += ((s.rows + 63) / 64) * ((d + 63) / 64);
    }
  }
  if (ssegs.size() > (size_t)(4 + 10 * m->cfg.n_layers)) return fail(PP_EINVAL, "internal: too many shadow segments");
  HIPCHECK(hipStreamSynchronize(m->st));
  if (!rows.empty()) HIPCHECK(hipMemcpy(m->wsp + plan.rows, rows.data(), rows.size() * sizeof(RowInfo), hipMemcpyHostToDevice));
  if (!ssegs.empty()) HIPCHECK(hipMemcpy(m->wsp + plan.segs, ssegs.data(), ssegs.size() * sizeof(ShadowSeg), hipMemcpyHostToDevice));
  m->ws = plan; m->mask = mk; m->segs = std::move(segs); m->n_train = n; m->n_rows = (int)rows.size();
  m->n_shadow_segs = (int)ssegs.size(); m->n_shadow_tiles = tiles; m->shadow_vec_ok = vec_ok;
  char* sb = (char*)state_dev;
  m->sp = (float*)sb; m->sm = (float*)(sb + quarter); m->sv = (float*)(sb + 2 * quarter); m->sg = (float*)(sb + 3 * quarter);
  rebuild_shadows(m);          // the parameter buffer may have been filled without pp_set_tensor (device copy, checkpoint load)
  k_pack_master(m->st, m->cfg.dtype, m->params, (const RowInfo*)(m->wsp + plan.rows), m->sp, m->n_rows, d);
  k_fill_f32(m->st, m->sm, (size_t)n, 0.f);
  k_fill_f32(m->st, m->sv, (size_t)n, 0.f);
  k_fill_f32(m->st, m->sg, (size_t)n, 0.f);
  m->step = 0; m->has_mask = true;
  HIPCHECK(hipStreamSynchronize(m->st));
  HIPCHECK(hipGetLastError());
  return PP_OK;
}

// ------------------------------------------------------------------------------------------------ GEMM dispatch
static void gemm_nt(pp_model* m, const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K,
                    int epi = EPI_STORE, const void* R = nullptr) {
  if (m->flop_acc) *m->flop_acc += 2.0 * M * N * K;
  GemmTimer timer(m, 2.0 * M * N * K);
  if (m->cfg.dtype == PP_BF16 && !m->force_plain &&
      k_gemm_nt_mfma(m->st, A, lda, B, ldb, C, ldc, M, N, K, epi, R, 0, 1, nullptr) == 0) { m->n_mfma++; return; }
  m->n_plain++;
  k_gemm_nt_plain(m->st, m->cfg.dtype, A, lda, B, ldb, C, ldc, M, N, K, epi, R, 0);
}

// gate/up projection with the SwiGLU product formed in the GEMM's epilogue; false = not launched (shape or path)
static bool gemm_swiglu(pp_model* m, const void* X, const void* Wgu, void* gu, void* a, int T, int F, int d) {
  if (m->cfg.dtype != PP_BF16 || m->force_plain) return false;
  GemmTimer timer(m, 2.0 * T * (2.0 * F) * d);
  if (k_gemm_swiglu_fwd_mfma(m->st, X, d, Wgu, d, gu, a, T, F, d) != 0) { timer.cancel(); return false; }
  if (m->flop_acc) *m->flop_acc += 2.0 * T * (2.0 * F) * d;
  m->n_mfma++;
  return true;
}

// q | k | v projection with the rotary embedding of q and k applied in the GEMM's epilogue; false = not launched (shape or path)
static bool gemm_qkv_rope(pp_model* m, const void* X, const void* Wqkv, void* qkv, int T, int d, int dh, int S, const float* cosb, const float* sinb) {
  if (m->cfg.dtype != PP_BF16 || m->force_plain || !m->fuse_rope) return false;
  GemmTimer timer(m, 2.0 * T * (3.0 * d) * d);
  if (k_gemm_qkv_rope_mfma(m->st, X, d, Wqkv, d, qkv, T, d, dh, d, S, cosb, sinb) != 0) { timer.cancel(); return false; }
  if (m->flop_acc) *m->flop_acc += 2.0 * T * (3.0 * d) * d;
  m->n_mfma++;
  return true;
}

// dA = G Wd_rows^T with the SwiGLU backward formed in the epilogue (dA itself is never stored); false = not launched
static bool gemm_swiglu_bwd(pp_model* m, const void* G, const void* Wd_rows, const void* gu_c0, void* dgu_c0, int T, int nc, int F, int d) {
  if (m->cfg.dtype != PP_BF16 || m->force_plain) return false;
  GemmTimer timer(m, 2.0 * T * (double)nc * d);
  if (k_gemm_swiglu_bwd_mfma(m->st, G, d, Wd_rows, d, gu_c0, dgu_c0, 2 * F, F, T, nc, d) != 0) { timer.cancel(); return false; }
  if (m->flop_acc) *m->flop_acc += 2.0 * T * (double)nc * d;
  m->n_mfma++;
  return true;
}

// Weight-gradient GEMM: G[M x N] (fp32, ld = N) = At[M x K] * Bt[N x K]^T with K = tokens.  Few output tiles and
// a long K: the K range is split over `splits` workgroup columns and summed in fixed order.
static void gemm_dw(pp_model* m, const void* At, const void* Bt, float* G, int M, int N, int K) {
  if (m->flop_acc) *m->flop_acc += 2.0 * M * N * K;
  GemmTimer timer(m, 2.0 * M * N * K);
  const size_t out_bytes = (size_t)M * N * 4;
  const long tiles = (long)((M + 127) / 128) * ((N + 127) / 128);
  int splits = 1;
  while (splits < 32 && tiles * splits < 1024 && K % (splits * 2) == 0 && K / (splits * 2) >= 256 &&
         out_bytes * (size_t)(splits * 2) <= m->ws.partial_bytes) splits *= 2;
  float* partial = (float*)(m->wsp + m->ws.partial);
  if (m->cfg.dtype == PP_BF16 && !m->force_plain &&
      k_gemm_nt_mfma(m->st, At, K, Bt, K, G, N, M, N, K, EPI_STORE, nullptr, 1, splits, partial) == 0) {
    if (splits > 1) k_splitk_reduce(m->st, partial, G, N, M, N, splits);
    m->n_mfma++;
    return;
  }
  m->n_plain++;
  if (splits == 1) { k_gemm_nt_plain(m->st, m->cfg.dtype, At, K, Bt, K, G, N, M, N, K, EPI_STORE, nullptr, 1); return; }
  k_gemm_nt_plain_splitk(m->st, m->cfg.dtype, At, K, Bt, K, partial, M, N, K, splits);
  k_splitk_reduce(m->st, partial, G, N, M, N, splits);
}

// Weight gradient from token-major operands: G[M x N] (fp32, ld N) = A^T B, A [K x M'] (lda) and B [K x N] (ldb) as the
// forward / backward passes left them, K = tokens; column m of the product is column (m / m_blk) * a_blk_stride + m % m_blk
// of A.  The MFMA kernel gathers its operands with LDS transpose reads; shapes it does not take (and fp32 storage) go
// through transposed copies and gemm_dw.
static void gemm_dw_tn(pp_model* m, const void* A, int lda, int m_blk, long a_blk_stride, const void* B, int ldb, float* G, int M, int N, int K) {
  const size_t es = esize(m->cfg);
  // (measured at K = 16384: up to 256 tiles of 128 x 128 -- the row-block slices, which need split-K anyway, and d x d --
  // the transpose-read kernel beats transposing both operands and running the 256 x 256-tile NT kernel; above that the
  // NT kernel's higher rate outweighs the two extra passes)
  const long tiles = (long)((M + 127) / 128) * ((N + 127) / 128);
  if (m->cfg.dtype == PP_BF16 && !m->force_plain && m->dw_tn && tiles <= 256) {
    const size_t out_bytes = (size_t)M * N * 4;
    int splits = 1;
    while (splits < 32 && tiles * splits < 512 && K % (splits * 2 * 64) == 0 && K / (splits * 2) >= 256 &&
           out_bytes * (size_t)(splits * 2) <= m->ws.partial_bytes) splits *= 2;
    float* partial = (float*)(m->wsp + m->ws.partial);
    GemmTimer timer(m, 2.0 * M * N * K);
    if (k_gemm_tn_mfma(m->st, A, lda, m_blk, a_blk_stride, B, ldb, G, N, M, N, K, splits, partial) == 0) {
      if (splits > 1) k_splitk_reduce(m->st, partial, G, N, M, N, splits);
      if (m->flop_acc) *m->flop_acc += 2.0 * M * N * K;
      m->n_mfma++;
      return;
    }
    timer.cancel();
  }
  char* tA = m->wsp + m->ws.tA;
  char* tB = m->wsp + m->ws.tB;
  for (int b0 = 0; b0 < M; b0 += m_blk)
    k_transpose(m->st, m->cfg.dtype, (const char*)A + (size_t)(b0 / m_blk) * a_blk_stride * es, lda, tA + (size_t)b0 * K * es, K, K, std::min(m_blk, M - b0));
  k_transpose(m->st, m->cfg.dtype, B, ldb, tB, K, K, N);
  gemm_dw(m, tA, tB, G, M, N, K);
}

static void attn_fwd(pp_model* m, const void* qkv, void* o, float* lse, int B, int S) {
  const int h = m->cfg.n_heads, dh = m->cfg.d_model / h;
  if (m->flop_acc) *m->flop_acc += 4.0 * ((double)B * S * (S + 1) / 2) * m->cfg.d_model;
  if (m->cfg.dtype == PP_BF16 && !m->force_plain && k_attn_fwd_mfma(m->st, qkv, o, lse, B, S, h, dh) == 0) { m->n_mfma++; return; }
  m->n_plain++;
  k_attn_fwd_plain(m->st, m->cfg.dtype, qkv, o, lse, B, S, h, dh);
}
// attention backward followed by the rotary embedding's backward on dq, dk (fused into the MFMA kernels' epilogues)
static void attn_bwd(pp_model* m, const void* qkv, const void* o, const float* lse, const void* dO, void* dqkv, float* Dbuf, int B, int S,
                     const float* cosb, const float* sinb) {
  const int h = m->cfg.n_heads, dh = m->cfg.d_model / h;
  if (m->flop_acc) *m->flop_acc += 8.0 * ((double)B * S * (S + 1) / 2) * m->cfg.d_model;
  if (m->cfg.dtype == PP_BF16 && !m->force_plain &&
      k_attn_bwd_mfma(m->st, qkv, o, lse, dO, dqkv, Dbuf, B, S, h, dh, cosb, sinb) == 0) { m->n_mfma++; return; }
  m->n_plain++;
  k_attn_bwd_plain(m->st, m->cfg.dtype, qkv, o, lse, dO, dqkv, Dbuf, B, S, h, dh);
  k_rope(m->st, m->cfg.dtype, dqkv, cosb, sinb, B, S, h, dh, 1);
}

// ------------------------------------------------------------------------------------------------ the local step
extern "C" int pp_local_step(pp_model* m, const int32_t* tokens_dev, const int32_t* targets_dev, int32_t B, int32_t S,
                             const pp_adamw* opt, float* loss_dev) {
  if (!m || !tokens_dev || !targets_dev || !loss_dev) return fail(PP_EINVAL, "pp_local_step: NULL pointer");
  if (!m->has_mask) return fail(PP_ESTATE, "pp_local_step: call pp_set_trainable_mask first");
  const pp_config& c = m->cfg;
  if (B < 1 || S < 1 || B > c.max_batch || S > c.max_seq) return fail(PP_EINVAL, "pp_local_step: B or S outside [1, max]");
  if (opt && (!(opt->lr >= 0.f) || !(opt->beta1 >= 0.f && opt->beta1 < 1.f) || !(opt->beta2 >= 0.f && opt->beta2 < 1.f) || !(opt->eps > 0.f) || !(opt->weight_decay >= 0.f)))
    return fail(PP_EINVAL, "pp_local_step: bad AdamW hyper-parameters");
  const int T = B * S, d = c.d_model, F = c.d_ff, V = c.vocab, h = c.n_heads, dh = d / h, L = c.n_layers, dt = c.dtype;
  const size_t es = esize(c);
  const Layout& ly = m->lay;
  const WsPlan& w = m->ws;
  const Mask& mk = m->mask;
  if (m->jac_mode == 1) {
    if (!mk.ffn) return fail(PP_EINVAL, "pp_local_step: the reduced FFN Jacobian (pp_set_jacobian_slices) needs a mask with a trainable FFN slice");
    if (m->jac_hi > m->jac_lo && m->jac_lo < mk.fh && mk.fl < m->jac_hi)
      return fail(PP_EINVAL, "pp_local_step: the extra Jacobian range overlaps the trainable FFN slice");
  }
  hipStream_t st = m->st;
  char* P = m->params;
  char* W = m->wsp;
  char* shadow = W + w.shadow;
  const float* cosb = (const float*)(W + w.rope_cos);
  const float* sinb = (const float*)(W + w.rope_sin);
  auto canon = [&](int64_t off) { return (void*)(P + off * es); };
  auto shad = [&](int64_t off) { return (void*)(shadow + off * es); };
  auto act = [&](int l, size_t o) {          // activation `o` of layer l (recompute: only the layer input is per layer)
    return (void*)((w.recompute && o != w.a_x) ? W + w.act_shared + o : W + w.act0 + (size_t)l * w.act_stride + o);
  };
  auto ofs = [&](void* p, size_t elems) { return (void*)((char*)p + elems * es); };

  // ---------------- forward over all parameters (Section 2.2: "the forward pass is standard")
  m->flops_fwd = 0; m->flops_bwd = 0; m->flops_recompute = 0;
  m->n_mfma = 0; m->n_plain = 0;
  m->flop_acc = &m->flops_fwd;
  k_embed(st, dt, tokens_dev, canon(ly.embed), act(0, w.a_x), T, d, V);
  // one layer forward; xnext == nullptr: stop after the SwiGLU product (all that a recomputation needs)
  auto layer_forward = [&](int l, void* xnext) {
    const int64_t lb = ly.layer0 + l * ly.layer_stride, sb = ly.sh_layer0 + l * ly.sh_layer_stride;
    void* x = act(l, w.a_x);
    k_rmsnorm_fwd(st, dt, x, canon(lb + ly.o_attn_norm), act(l, w.a_n1), (float*)act(l, w.a_rstd1), T, d, c.rms_eps);
    if (!gemm_qkv_rope(m, act(l, w.a_n1), canon(lb + ly.o_wqkv), act(l, w.a_qkv), T, d, dh, S, cosb, sinb)) {
      gemm_nt(m, act(l, w.a_n1), d, canon(lb + ly.o_wqkv), d, act(l, w.a_qkv), 3 * d, T, 3 * d, d);
      k_rope(st, dt, act(l, w.a_qkv), cosb, sinb, B, S, h, dh, 0);
    }
    attn_fwd(m, act(l, w.a_qkv), act(l, w.a_o), (float*)act(l, w.a_lse), B, S);
    gemm_nt(m, act(l, w.a_o), d, canon(lb + ly.o_wo), d, act(l, w.a_xm), d, T, d, d, EPI_ADD_RES, x);
    k_rmsnorm_fwd(st, dt, act(l, w.a_xm), canon(lb + ly.o_ffn_norm), act(l, w.a_n2), (float*)act(l, w.a_rstd2), T, d, c.rms_eps);
    if (!gemm_swiglu(m, act(l, w.a_n2), canon(lb + ly.o_wg), act(l, w.a_gu), act(l, w.a_a), T, F, d)) {      // [Wg; Wu] are adjacent
      gemm_nt(m, act(l, w.a_n2), d, canon(lb + ly.o_wg), d, act(l, w.a_gu), 2 * F, T, 2 * F, d);
      k_swiglu_fwd(st, dt, act(l, w.a_gu), act(l, w.a_a), T, F);
    }
    if (xnext) gemm_nt(m, act(l, w.a_a), F, shad(sb + ly.sh_wd), F, xnext, d, T, d, F, EPI_ADD_RES, act(l, w.a_xm));
  };
  for (int l = 0; l < L; ++l) layer_forward(l, (l + 1 < L) ? act(l + 1, w.a_x) : (void*)(W + w.xL));
  void* xL = W + w.xL;
  void* nf = W + w.nf;
  void* logits = W + w.logits;
  float* rstdf = (float*)(W + w.rstdf);
  k_rmsnorm_fwd(st, dt, xL, canon(ly.final_norm), nf, rstdf, T, d, c.rms_eps);
  gemm_nt(m, nf, d, canon(ly.lm_head), d, logits, V, T, V, d);
  int32_t* nvalid = (int32_t*)(W + w.nvalid);
  float* rowloss = (float*)(W + w.rowloss);
  k_count_valid(st, targets_dev, T, V, nvalid);
  if (k_cross_entropy(st, dt, logits, targets_dev, nvalid, rowloss, T, V)) return fail(PP_EINVAL, "pp_local_step: vocab too large for cross entropy kernel");
  k_loss_reduce(st, rowloss, nvalid, loss_dev, T);

  // ---------------- restricted backward (Appendix "Partial Backward"): dW only for trainable row blocks, dX through
  // every slice and head, nothing below the lowest trainable parameter.
  m->flop_acc = &m->flops_bwd;
  const bool any_layer = mk.norms || mk.heads || mk.wo || mk.ffn;
  auto below_layer = [&](int l) { return mk.emb || (l > 0 && any_layer); };
  void* dx = W + w.dx;
  void* dn = W + w.dn;
  void* dA = W + w.dA;
  void* dgu = W + w.dgu;
  void* dob = W + w.dob;
  void* dqkv = W + w.dqkv;
  float* Dattn = (float*)(W + w.Dattn);
  float* dgpart = (float*)(W + w.dgpart);
  float* g = m->sg;
  void* dz = logits;
  bool reached_bottom = false;
  if (any_layer || mk.emb || mk.lm) {
    if (mk.lm) gemm_dw_tn(m, dz, V, V, 0, nf, d, g + find_seg(m, TK_LM_HEAD, -1)->packed_off, V, d, T);
    if (any_layer || mk.emb) {
      gemm_nt(m, dz, V, shad(ly.sh_lm_head), V, dn, d, T, d, V);
      if (mk.norms) k_rmsnorm_dgamma(st, dt, dn, xL, rstdf, dgpart, g + find_seg(m, TK_FINAL_NORM, -1)->packed_off, T, d);
      k_rmsnorm_bwd(st, dt, dn, xL, rstdf, canon(ly.final_norm), nullptr, dx, T, d);
      for (int l = L - 1; l >= 0; --l) {
        const int64_t lb = ly.layer0 + l * ly.layer_stride, sb = ly.sh_layer0 + l * ly.sh_layer_stride;
        const bool below_ffn_w = mk.norms || mk.wo || mk.heads || below_layer(l);
        if (w.recompute && (mk.ffn || below_ffn_w)) {          // run the layer forward again from its saved input (not counted as executed FLOPs)
          double* keep = m->flop_acc; m->flop_acc = &m->flops_recompute;
          layer_forward(l, nullptr);
          m->flop_acc = keep;
        }
        if (mk.ffn || below_ffn_w) {
          const int c0 = below_ffn_w ? 0 : mk.fl, c1 = below_ffn_w ? F : mk.fh, nc = c1 - c0, Fk = mk.fh - mk.fl;
          if (mk.ffn)      // dWd_k = A_k^T G
            gemm_dw_tn(m, ofs(act(l, w.a_a), mk.fl), F, Fk, 0, dx, d, g + find_seg(m, TK_WD, l)->packed_off, Fk, d, T);
          // dG, dU of hidden units r0..r1-1 into their columns of dgu
          auto ffn_dgu = [&](int r0, int r1) {
            if (!gemm_swiglu_bwd(m, dx, canon(lb + ly.o_wd + (int64_t)r0 * d), ofs(act(l, w.a_gu), r0), ofs(dgu, r0), T, r1 - r0, F, d)) {
              gemm_nt(m, dx, d, canon(lb + ly.o_wd + (int64_t)r0 * d), d, dA, r1 - r0, T, r1 - r0, d);        // dA = G Wd^T (rows r0..r1 of Wd)
              k_swiglu_bwd(st, dt, act(l, w.a_gu), dA, r1 - r0, dgu, T, F, r0, r1);
            }
          };
          const bool detach = below_ffn_w && m->jac_mode == 1;
          if (!detach) ffn_dgu(c0, c1);
          else { ffn_dgu(mk.fl, mk.fh); if (m->jac_hi > m->jac_lo) ffn_dgu(m->jac_lo, m->jac_hi); }
          if (mk.ffn)      // [dWg_k; dWu_k] = [dG_k; dU_k]^T Xn: the two column blocks of dgu sit d_ff columns apart
            gemm_dw_tn(m, ofs(dgu, mk.fl), 2 * F, Fk, F, act(l, w.a_n2), d, g + find_seg(m, TK_WG, l)->packed_off, 2 * Fk, d, T);
          if (below_ffn_w && !detach) gemm_nt(m, dgu, 2 * F, shad(sb + ly.sh_wgu), 2 * F, dn, d, T, d, 2 * F);   // dXn over ALL slices
          if (detach) {
            // Appendix "Additional Results" (detach-all-but-k, + one more slice): dXn summed over the kept units only.
            // Gate and up columns of a range are K-slices of the same product; the pieces are chained through the
            // residual input, alternating between dn and the (idle) attention-gradient buffer so that the last lands in dn.
            const int rng[2][2] = {{mk.fl, mk.fh}, {m->jac_lo, m->jac_hi}};
            const int n_rng = m->jac_hi > m->jac_lo ? 2 : 1, n_pc = 2 * n_rng;
            void* prev = nullptr;
            for (int i = 0; i < n_pc; ++i) {
              const size_t col = (size_t)(i & 1) * F + rng[i >> 1][0];
              void* out = ((n_pc - 1 - i) & 1) ? dob : dn;
              gemm_nt(m, ofs(dgu, col), 2 * F, ofs(shad(sb + ly.sh_wgu), col), 2 * F, out, d, T, d, rng[i >> 1][1] - rng[i >> 1][0],
                      i ? EPI_ADD_RES : EPI_STORE, prev);
              prev = out;
            }
          }
        }
        if (!below_ffn_w) break;
        if (mk.norms) k_rmsnorm_dgamma(st, dt, dn, act(l, w.a_xm), (float*)act(l, w.a_rstd2), dgpart, g + find_seg(m, TK_FFN_NORM, l)->packed_off, T, d);
        const bool below_norm2 = mk.wo || mk.heads || mk.norms || below_layer(l);
        if (!below_norm2) break;
        k_rmsnorm_bwd(st, dt, dn, act(l, w.a_xm), (float*)act(l, w.a_rstd2), canon(lb + ly.o_ffn_norm), dx, dx, T, d);   // dx := dL/dx_mid
        if (mk.wo) gemm_dw_tn(m, dx, d, d, 0, act(l, w.a_o), d, g + find_seg(m, TK_WO, l)->packed_off, d, d, T);
        const bool below_wo = mk.heads || mk.norms || below_layer(l);
        if (!below_wo) break;
        gemm_nt(m, dx, d, shad(sb + ly.sh_wo), d, dob, d, T, d, d);
        attn_bwd(m, act(l, w.a_qkv), act(l, w.a_o), (float*)act(l, w.a_lse), dob, dqkv, Dattn, B, S, cosb, sinb);
        if (mk.heads) {      // the Q, K and V parts of the head range sit d_model columns apart in dqkv
          const int nhd = (mk.hh - mk.hl) * dh;
          gemm_dw_tn(m, ofs(dqkv, (size_t)mk.hl * dh), 3 * d, nhd, d, act(l, w.a_n1), d, g + find_seg(m, TK_WQKV, l)->packed_off, 3 * nhd, d, T);
        }
        const bool below_wqkv = mk.norms || below_layer(l);
        if (!below_wqkv) break;
        gemm_nt(m, dqkv, 3 * d, shad(sb + ly.sh_wqkv), 3 * d, dn, d, T, d, 3 * d);
        if (mk.norms) k_rmsnorm_dgamma(st, dt, dn, act(l, w.a_x), (float*)act(l, w.a_rstd1), dgpart, g + find_seg(m, TK_ATTN_NORM, l)->packed_off, T, d);
        if (!below_layer(l)) break;
        k_rmsnorm_bwd(st, dt, dn, act(l, w.a_x), (float*)act(l, w.a_rstd1), canon(lb + ly.o_attn_norm), dx, dx, T, d);     // dx := dL/dx_l
        if (l == 0) reached_bottom = true;
      }
      if (reached_bottom && mk.emb) {
        // the dL/da block is idle by now (the last layer's backward is done): room for the position index
        const bool fits = ((size_t)T + 2 * (size_t)V) * 4 <= (size_t)T * F * esize(m->cfg);
        k_embed_grad(st, dt, tokens_dev, dx, g + find_seg(m, TK_EMBED, -1)->packed_off, T, d, V, fits ? (int32_t*)(m->wsp + w.dA) : nullptr);
      }
    }
  }
  m->flop_acc = nullptr;

  // ---------------- InnerOpt on theta[I_train] only (Algorithm 1, inner update line)
  m->adamw_bytes = 0;
  if (opt && m->n_train > 0) {
    m->step += 1;
    const double bc1 = 1.0 - std::pow((double)opt->beta1, (double)m->step), bc2 = 1.0 - std::pow((double)opt->beta2, (double)m->step);
    k_adamw(st, dt, P, (const RowInfo*)(W + w.rows), m->sp, m->sm, m->sv, m->sg, m->n_rows, d, opt->lr, opt->beta1, opt->beta2,
            opt->eps, opt->weight_decay, (float)bc1, (float)bc2);
    k_shadow_refresh(st, dt, P, shadow, (const ShadowSeg*)(W + w.segs), m->n_shadow_segs, m->n_shadow_tiles, m->shadow_vec_ok);
    m->adamw_bytes = (double)m->n_train * (28.0 + es);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PP_EHIP, std::string("pp_local_step: ") + hipGetErrorString(e));
  return PP_OK;
}

// ------------------------------------------------------------------------------------------------ outer step
extern "C" int pp_outer_delta(pp_model* m, float* theta_g_dev, float* momentum_dev, const float* others_sum_dev,
                              const pp_outer* opt, float* delta_out_dev) {
  if (!m || !theta_g_dev || !momentum_dev || !opt) return fail(PP_EINVAL, "pp_outer_delta: NULL pointer");
  if (!m->has_mask) return fail(PP_ESTATE, "pp_outer_delta: call pp_set_trainable_mask first");
  if (!(opt->m_count >= 1.0f)) return fail(PP_EINVAL, "pp_outer_delta: m_count must be >= 1");
  if (!(opt->lr >= 0.f) || !(opt->momentum >= 0.f)) return fail(PP_EINVAL, "pp_outer_delta: bad hyper-parameters");
  k_outer(m->st, m->cfg.dtype, m->params, (const RowInfo*)(m->wsp + m->ws.rows), m->sp, theta_g_dev, momentum_dev, others_sum_dev,
          delta_out_dev, m->n_rows, m->cfg.d_model, opt->lr, opt->momentum, opt->nesterov != 0, 1.0f / opt->m_count);
  k_shadow_refresh(m->st, m->cfg.dtype, m->params, m->wsp + m->ws.shadow, (const ShadowSeg*)(m->wsp + m->ws.segs), m->n_shadow_segs, m->n_shadow_tiles, m->shadow_vec_ok);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PP_EHIP, std::string("pp_outer_delta: ") + hipGetErrorString(e));
  return PP_OK;
}

// Streaming synchronisation (Experimental Setup: layers synchronised group by group): the same update restricted to the
// packed rows of layers [layer_lo, layer_hi) and, if ends != 0, of embed / final_norm / lm_head.  The packed order is the
// network order, so the selection is at most three contiguous row ranges.
extern "C" int pp_outer_delta_group(pp_model* m, int32_t layer_lo, int32_t layer_hi, int32_t ends, float* theta_g_dev, float* momentum_dev,
                                    const float* others_sum_dev, const pp_outer* opt, float* delta_out_dev) {
  if (!m || !theta_g_dev || !momentum_dev || !opt) return fail(PP_EINVAL, "pp_outer_delta_group: NULL pointer");
  if (!m->has_mask) return fail(PP_ESTATE, "pp_outer_delta_group: call pp_set_trainable_mask first");
  if (!(opt->m_count >= 1.0f)) return fail(PP_EINVAL, "pp_outer_delta_group: m_count must be >= 1");
  if (!(opt->lr >= 0.f) || !(opt->momentum >= 0.f)) return fail(PP_EINVAL, "pp_outer_delta_group: bad hyper-parameters");
  if (layer_lo < 0 || layer_hi < layer_lo || layer_hi > m->cfg.n_layers) return fail(PP_EINVAL, "pp_outer_delta_group: bad layer range");
  const int d = m->cfg.d_model;
  int64_t run_lo = -1, run_hi = -1;          // current run of selected packed rows
  auto flush = [&]() {
    if (run_lo < 0) return;
    const size_t e0 = (size_t)run_lo * d;
    k_outer(m->st, m->cfg.dtype, m->params, (const RowInfo*)(m->wsp + m->ws.rows) + run_lo, m->sp + e0, theta_g_dev + e0, momentum_dev + e0,
            others_sum_dev ? others_sum_dev + e0 : nullptr, delta_out_dev ? delta_out_dev + e0 : nullptr, (int)(run_hi - run_lo), d,
            opt->lr, opt->momentum, opt->nesterov != 0, 1.0f / opt->m_count);
    run_lo = run_hi = -1;
  };
  for (const Seg& s : m->segs) {
    const bool sel = s.layer >= 0 ? (s.layer >= layer_lo && s.layer < layer_hi) : (ends != 0);
    const int64_t r0 = s.packed_off / d, r1 = r0 + s.rows;
    if (sel && s.rows > 0) {
      if (run_lo >= 0 && run_hi == r0) run_hi = r1;
      else { flush(); run_lo = r0; run_hi = r1; }
    } else flush();
  }
  flush();
  k_shadow_refresh(m->st, m->cfg.dtype, m->params, m->wsp + m->ws.shadow, (const ShadowSeg*)(m->wsp + m->ws.segs), m->n_shadow_segs, m->n_shadow_tiles, m->shadow_vec_ok);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PP_EHIP, std::string("pp_outer_delta_group: ") + hipGetErrorString(e));
  return PP_OK;
}

extern "C" int pp_synth_delta_sum(pp_model* m, float* dst_dev, size_t n, const uint64_t* keys_host, int32_t n_nodes, float std) {
  if (!m || !dst_dev || !keys_host) return fail(PP_EINVAL, "pp_synth_delta_sum: NULL pointer");
  if (n_nodes < 1 || n_nodes > 256) return fail(PP_EINVAL, "pp_synth_delta_sum: n_nodes must be in [1, 256]");
  uint64_t* keys_dev = (uint64_t*)(m->wsp + m->ws.keys);
  HIPCHECK(hipMemcpyAsync(keys_dev, keys_host, (size_t)n_nodes * 8, hipMemcpyHostToDevice, m->st));
  HIPCHECK(hipStreamSynchronize(m->st));
  k_synth_delta_sum(m->st, dst_dev, n, keys_dev, n_nodes, std);
  HIPCHECK(hipGetLastError());
  return PP_OK;
}

extern "C" int pp_get_gemm_timing(pp_model* m, double* total_ms, double* total_flops, int64_t* launches) {
  if (!m) return fail(PP_EINVAL, "pp_get_gemm_timing: NULL model");
  HIPCHECK(hipStreamSynchronize(m->st));
  double ms = 0;
  for (size_t i = 0; i + 1 < m->ev_used; i += 2) {
    float t = 0.f;
    HIPCHECK(hipEventElapsedTime(&t, m->ev[i], m->ev[i + 1]));
    ms += t;
  }
  if (total_ms) *total_ms = ms;
  if (total_flops) *total_flops = m->timed_flops;
  if (launches) *launches = (int64_t)(m->ev_used / 2);
  m->ev_used = 0; m->timed_flops = 0;
  return PP_OK;
}

extern "C" int pp_get_counters(pp_model* m, double* flops_fwd, double* flops_bwd, double* adamw_bytes, int64_t* n_trainable) {
  if (!m) return fail(PP_EINVAL, "pp_get_counters: NULL model");
  if (flops_fwd) *flops_fwd = m->flops_fwd;
  if (flops_bwd) *flops_bwd = m->flops_bwd;
  if (adamw_bytes) *adamw_bytes = m->adamw_bytes;
  if (n_trainable) *n_trainable = m->n_train;
  return PP_OK;
}

extern "C" int pp_get_launch_counts(pp_model* m, int64_t* matrix_core_calls, int64_t* plain_calls) {
  if (!m) return fail(PP_EINVAL, "pp_get_launch_counts: NULL model");
  if (matrix_core_calls) *matrix_core_calls = m->n_mfma;
  if (plain_calls) *plain_calls = m->n_plain;
  return PP_OK;
}

// ------------------------------------------------------------------------------------------------ op-level entry points
#include "../../include/pp_ops.h"

extern "C" int pp_op_gemm_nt(void* hip_stream, int dtype, const void* A, int lda, const void* B, int ldb, void* C, int ldc,
                             int M, int N, int K, const void* R, int out_f32, int splits, float* scratch, int path) {
  if (!A || !B || !C) return fail(PP_EINVAL, "pp_op_gemm_nt: NULL pointer");
  if (dtype != PP_F32 && dtype != PP_BF16) return fail(PP_EINVAL, "pp_op_gemm_nt: bad dtype");
  if (M < 1 || N < 1 || K < 1 || lda < K || ldb < K || ldc < N) return fail(PP_EINVAL, "pp_op_gemm_nt: bad shape or leading dimension");
  if (splits < 1 || K % splits) return fail(PP_EINVAL, "pp_op_gemm_nt: K must be a multiple of splits");
  if (splits > 1 && (!out_f32 || !scratch || R)) return fail(PP_EINVAL, "pp_op_gemm_nt: split-K needs out_f32, scratch and no residual");
  if (out_f32 && R) return fail(PP_EINVAL, "pp_op_gemm_nt: residual with float output is not supported");
  hipStream_t st = (hipStream_t)hip_stream;
  const int epi = R ? EPI_ADD_RES : EPI_STORE;
  const bool f32out = out_f32 || dtype == PP_F32;
  bool done = false;
  if (path == 0 && dtype == PP_BF16)
    done = k_gemm_nt_mfma(st, A, lda, B, ldb, C, ldc, M, N, K, epi, R, out_f32, splits, scratch) == 0;
  if (!done) {
    if (splits > 1) k_gemm_nt_plain_splitk(st, dtype, A, lda, B, ldb, scratch, M, N, K, splits);
    else k_gemm_nt_plain(st, dtype, A, lda, B, ldb, C, ldc, M, N, K, epi, R, f32out ? 1 : 0);
  }
  if (splits > 1) k_splitk_reduce(st, scratch, (float*)C, ldc, M, N, splits);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PP_EHIP, std::string("pp_op_gemm_nt: ") + hipGetErrorString(e));
  return PP_OK;
}

extern "C" int pp_op_gemm_tn(void* hip_stream, const void* A, int lda, int m_blk, int64_t a_blk_stride, const void* B, int ldb, float* C, int ldc,
                             int M, int N, int K, int splits, float* scratch) {
  if (!A || !B || !C) return fail(PP_EINVAL, "pp_op_gemm_tn: NULL pointer");
  if (M < 1 || N < 1 || K < 1 || ldb < N || ldc < N || m_blk < 1) return fail(PP_EINVAL, "pp_op_gemm_tn: bad shape or leading dimension");
  if ((int64_t)((M - 1) / m_blk) * a_blk_stride + std::min(M, m_blk) > lda) return fail(PP_EINVAL, "pp_op_gemm_tn: column blocks of A exceed lda");
  if (splits < 1 || (splits > 1 && !scratch)) return fail(PP_EINVAL, "pp_op_gemm_tn: split-K needs a scratch buffer");
  hipStream_t st = (hipStream_t)hip_stream;
  if (k_gemm_tn_mfma(st, A, lda, m_blk, (long)a_blk_stride, B, ldb, C, ldc, M, N, K, splits, scratch) != 0)
    return fail(PP_EINVAL, "pp_op_gemm_tn: shape or alignment not taken by the MFMA kernel (see pp_ops.h)");
  if (splits > 1) k_splitk_reduce(st, scratch, C, ldc, M, N, splits);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PP_EHIP, std::string("pp_op_gemm_tn: ") + hipGetErrorString(e));
  return PP_OK;
}

// ---- split-K GEMM for callers that cannot allocate: the partial products live in a file-scope device array
constexpr size_t kStaticScratchFloats = PP_STATIC_SCRATCH_FLOATS;          // 16 MiB per GPU, held until the process ends
static __device__ __align__(256) float scratch[kStaticScratchFloats];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static float* g_scratch_ptr[kMaxDevices];          // device address of `scratch` on each GPU (each GPU has its own copy), nullptr = not asked yet

// Device address of the current GPU's copy of `scratch` (looked up once per device, with that device current).
static int static_scratch(float** out) {
  int dev = -1;
  HIPCHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(PP_EINVAL, "static scratch: device index out of range");
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    float* p = nullptr;
    HIPCHECK(hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(PP_EHIP, "static scratch: hipGetSymbolAddress returned a null address");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return PP_OK;
}

extern "C" int pp_op_gemm_nt_splitk_static(void* hip_stream, int dtype, const void* A, int lda, const void* B, int ldb, float* C, int ldc,
                                           int M, int N, int K, int splits, int path) {
  if (!A || !B || !C) return fail(PP_EINVAL, "pp_op_gemm_nt_splitk_static: NULL pointer");
  if (dtype != PP_F32 && dtype != PP_BF16) return fail(PP_EINVAL, "pp_op_gemm_nt_splitk_static: bad dtype");
  if (M < 1 || N < 1 || K < 1 || lda < K || ldb < K || ldc < N) return fail(PP_EINVAL, "pp_op_gemm_nt_splitk_static: bad shape or leading dimension");
  if (splits < 2 || K % splits) return fail(PP_EINVAL, "pp_op_gemm_nt_splitk_static: splits must be >= 2 and divide K");
  if ((size_t)M * (size_t)N > kStaticScratchFloats / (size_t)splits)
    return fail(PP_EINVAL, "pp_op_gemm_nt_splitk_static: M*N*splits exceeds the built-in scratch of " + std::to_string(kStaticScratchFloats) +
                               " floats (use pp_op_gemm_nt with a scratch buffer of your own)");
  float* part = nullptr;
  if (int rc = static_scratch(&part)) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  // every element [z][row < M][col < N] of the partials is written by the GEMM before the reduction reads it: nothing to clear
  if (!(path == 0 && dtype == PP_BF16 && k_gemm_nt_mfma(st, A, lda, B, ldb, C, ldc, M, N, K, EPI_STORE, nullptr, 1, splits, part) == 0))
    k_gemm_nt_plain_splitk(st, dtype, A, lda, B, ldb, part, M, N, K, splits);
  k_splitk_reduce(st, part, C, ldc, M, N, splits);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PP_EHIP, std::string("pp_op_gemm_nt_splitk_static: ") + hipGetErrorString(e));
  return PP_OK;
}

static int check_attn(int dtype, int B, int S, int h, int dh) {
  if (dtype != PP_F32 && dtype != PP_BF16) return fail(PP_EINVAL, "attention: bad dtype");
  if (B < 1 || S < 1 || h < 1 || dh < 2 || dh % 2 || dh > 256 || S > 8192) return fail(PP_EINVAL, "attention: bad shape");
  return PP_OK;
}
extern "C" int pp_op_attention_fwd(void* hip_stream, int dtype, const void* qkv, void* o, float* lse, void* scratch, int B, int S, int h, int dh, int path) {
  if (!qkv || !o || !lse) return fail(PP_EINVAL, "pp_op_attention_fwd: NULL pointer");
  if (int rc = check_attn(dtype, B, S, h, dh)) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  if (!(path == 0 && dtype == PP_BF16 && k_attn_fwd_mfma(st, qkv, o, lse, B, S, h, dh) == 0)) k_attn_fwd_plain(st, dtype, qkv, o, lse, B, S, h, dh);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PP_EHIP, std::string("pp_op_attention_fwd: ") + hipGetErrorString(e));
  return PP_OK;
}
extern "C" int pp_op_attention_bwd(void* hip_stream, int dtype, const void* qkv, const void* o, const float* lse, const void* dO,
                                   void* dqkv, float* Dbuf, void* scratch, int B, int S, int h, int dh, int path) {
  if (!qkv || !o || !lse || !dO || !dqkv || !Dbuf) return fail(PP_EINVAL, "pp_op_attention_bwd: NULL pointer");
  if (int rc = check_attn(dtype, B, S, h, dh)) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  if (!(path == 0 && dtype == PP_BF16 && k_attn_bwd_mfma(st, qkv, o, lse, dO, dqkv, Dbuf, B, S, h, dh, nullptr, nullptr) == 0))
    k_attn_bwd_plain(st, dtype, qkv, o, lse, dO, dqkv, Dbuf, B, S, h, dh);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PP_EHIP, std::string("pp_op_attention_bwd: ") + hipGetErrorString(e));
  return PP_OK;
}

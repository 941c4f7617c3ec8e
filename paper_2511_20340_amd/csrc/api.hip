// C ABI of libspecformer: context, argument validation, workspace planning and the three step
// schedulers (draft / verify / accept) that enqueue the HIP kernels on the caller's stream.
#include <math.h>
#include <string.h>
#include <new>
#include <vector>
#include "sf_internal.h"
#include "../../include/specformer_aux.h"

#include <cstddef>

using namespace sf;

// Optional per-kernel-class timing (sf_profile_begin / sf_profile_end): every launch is bracketed
// by a pair of HIP events on the launch stream.
enum { K_GEMM = 0, K_ATTN, K_ATTN_COMBINE, K_NORM, K_ROPE, K_SILU, K_EMBED_HOOK, K_ARGMAX, K_ACCEPT, K_NCLASS };
struct Prof {
  bool on = false;
  std::vector<hipEvent_t> ev;  // pairs
  std::vector<int> cls;
  size_t used = 0;             // pairs in use
};

struct sf_ctx {
  mutable Prof prof;
  sf_model_cfg tc, dc;
  int max_B, max_k;
  bool bound, has_draft;
  sf_target_weights tw;
  sf_draft_weights dw;
  std::vector<const void *> attn_norm, wqkv, wo, ffn_norm, w_gate_up, w_down;
  mutable int hip_err;
  // call order: the block that sf_verify_step wrote behind the prefixes and that no sf_accept_commit has
  // committed yet (state identified by its kv_len buffer); k < 0: none
  const void *verified_state = nullptr;
  int verified_k = -1;
  // tuning overrides of this context (0 = automatic)
  int tune_tile = 0, tune_split = 0, tune_chunk = 0;
};

namespace {

constexpr size_t ALIGN = 256;
size_t up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }
size_t esize(int dtype) { return dtype == SF_BF16 ? 2 : 4; }

// Workspace arena.  Buffers are sized for the larger of the verify (B*(k+1) rows), draft-context
// (B*(max_k+1) rows) and draft-slot (B*k rows) uses; draft and verify run back to back on one
// stream, so they share it.
struct Arena {
  size_t h, hb, a, qkv, qr, ao, gu, act, table, order, part_o, part_ml, pmax, pidx, logits;  // shared
  size_t f4, x, kvc, xl, s0, s0b;                                        // draft only
  size_t x_last, id_last, q1, qr1, ao1, len_m1, zeros, kc2, vc2;         // draft, two-stage wiring
  size_t gemm_ws, gemm_ws_bytes, dev_err;
  size_t total;
};

Arena plan(const sf_ctx *c, int B, int k, int cap) {
  const sf_model_cfg &m = c->tc;
  const size_t es = esize(m.dtype);
  const size_t qm = c->max_k + 1;
  const size_t M = (size_t)B * (k + 1), Mh = (size_t)B * qm, Ms = (size_t)B * (k > 0 ? k : 1);
  const size_t Mx = M > Mh ? M : Mh;
  const size_t d = m.d_model, F = m.d_ffn, V = m.vocab;
  const size_t nq = (size_t)m.n_q_heads * m.head_dim, nkv = (size_t)m.n_kv_heads * m.head_dim;
  Arena a;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += up(bytes); return o; };
  // first, at an offset that does not depend on k: the split-K ticket counters must stay zero
  // between calls, so no other buffer of any call shape may ever overlap them
  a.gemm_ws_bytes = m.dtype == SF_BF16 ? gemm_workspace_bytes((int)Mx) : 0;
  a.gemm_ws = take(a.gemm_ws_bytes);
  a.zeros = take((size_t)B * sizeof(int32_t));  // likewise never written: the empty prefix of a slot-only attention
  a.dev_err = take(sizeof(int32_t));            // sticky SF_DEVERR_* bits, read and cleared by sf_check_state
  a.h = take(M * d * sizeof(float));  // the residual stream
  a.hb = take(m.dtype == SF_BF16 ? M * d * es : 0);
  a.a = take(Mx * d * es);
  a.qkv = take(M * (nq + 2 * nkv) * es);
  a.qr = take(M * nq * es);
  a.ao = take(M * nq * es);
  a.gu = take(m.dtype == SF_F32 ? M * 2 * F * sizeof(float) : 0);  // bf16 gates in the GEMM epilogue
  a.act = take(M * F * es);
  a.table = take((Mx + Ms) * (m.head_dim / 2) * sizeof(float2));  // block rows, then the draft's slot rows
  a.order = take((size_t)B * sizeof(int32_t));
  const int G = m.n_q_heads / m.n_kv_heads;
  size_t part = m.dtype == SF_BF16 ? attn_workspace_bytes(B, m.n_kv_heads, m.head_dim, G, k + 1, cap) : 0;
  const size_t rows_part = part / ((m.head_dim + 2) * sizeof(float));
  a.part_o = take(rows_part * m.head_dim * sizeof(float));
  a.part_ml = take(rows_part * 2 * sizeof(float));
  // arg-max partials: per row one entry per column tile of the LM head (bf16) or per segment (fp32)
  const size_t parts = m.dtype == SF_BF16 ? (size_t)gemm_argmax_parts((int)V) : (size_t)ARGMAX_SEGS;
  a.pmax = take(Mx * parts * sizeof(float));
  a.pidx = take(Mx * parts * sizeof(int32_t));
  a.logits = take(m.dtype == SF_F32 ? Mx * V * sizeof(float) : 0);  // fp32 mode materialises them
  a.f4 = take(Mh * 4 * d * es);
  a.x = take(Mh * d * es);
  a.kvc = take(Mh * 2 * nkv * es);
  a.xl = take((size_t)B * d * es);
  a.s0 = take(Ms * d * sizeof(float));  // the slot layer's residual stream
  a.s0b = take(m.dtype == SF_BF16 ? Ms * d * es : 0);
  a.x_last = take((size_t)B * d * es);
  a.id_last = take((size_t)B * d * sizeof(float));
  a.q1 = take((size_t)B * nq * es);
  a.qr1 = take((size_t)B * nq * es);
  a.ao1 = take((size_t)B * nq * es);
  a.len_m1 = take((size_t)B * sizeof(int32_t));
  a.kc2 = take((size_t)B * nkv * TK * es);      // one 32-key tile per (sequence, kv head)
  a.vc2 = take((size_t)B * nkv * TK * es);
  a.total = off;
  return a;
}

bool same_shape(const sf_model_cfg &a, const sf_model_cfg &b) {
  return a.d_model == b.d_model && a.n_q_heads == b.n_q_heads && a.n_kv_heads == b.n_kv_heads &&
         a.head_dim == b.head_dim && a.d_ffn == b.d_ffn && a.vocab == b.vocab && a.dtype == b.dtype &&
         a.rope_theta == b.rope_theta && a.rms_eps == b.rms_eps;
}

sf_status check_attn_shape(const sf_model_cfg &m, int n_q) {
  const int G = m.n_q_heads / m.n_kv_heads;
  if (m.dtype == SF_BF16) {
    if (G * n_q > 1024) return SF_EUNSUPPORTED;  // 32 row tiles of 32 rows per (sequence, kv head)
  } else {
    if (n_q * m.head_dim > 2048) return SF_EUNSUPPORTED;
  }
  return SF_OK;
}

struct Run {
  const sf_ctx *c;
  hipStream_t s;
  sf_status st = SF_OK;
  void *gemm_ws = nullptr;
  size_t gemm_ws_bytes = 0;
  int plan_rows = 0;  // rows the linear layers' K partition is chosen for (0: the launch's own M)
  // a stale error left by an earlier, unrelated HIP call of the process must not be blamed on us
  Run(const sf_ctx *ctx, hipStream_t stream) : c(ctx), s(stream) { (void)hipGetLastError(); }
  bool ok(hipError_t e) {
    if (st != SF_OK) return false;
    if (e != hipSuccess) { c->hip_err = (int)e; st = SF_EHIP; return false; }
    return true;
  }
  // enqueue one kernel launch of class `cls`, timed when profiling is on
  template <class F> void launch(int cls, F f) {
    if (st != SF_OK) return;
    Prof &p = c->prof;
    if (!p.on) { ok(f()); return; }
    if (p.ev.size() < 2 * (p.used + 1)) {
      hipEvent_t a, b;
      if (!ok(hipEventCreate(&a)) || !ok(hipEventCreate(&b))) return;
      p.ev.push_back(a); p.ev.push_back(b);
    }
    if (!ok(hipEventRecord(p.ev[2 * p.used], s))) return;
    if (!ok(f())) return;
    if (!ok(hipEventRecord(p.ev[2 * p.used + 1], s))) return;
    if (p.cls.size() <= p.used) p.cls.resize(p.used + 1);
    p.cls[p.used++] = cls;
  }
};
#define LAUNCH(cls, expr) r.launch(cls, [&] { return (expr); })

// optional extras of one linear launch (bf16 mode)
struct GemmExtra {
  int res_f32 = 0;               // residual (and, with out_f32, y) are rows of the float residual stream
  void *y2 = nullptr;            // bf16 copy of y
  void *hooks = nullptr;         // hooked copies of the block rows
  int hook_mask = 0, hook_q = 1, hook_qmax = 1;
  float *am_val = nullptr;       // arg-max partials per column tile
  int32_t *am_idx = nullptr;
  int am_stride = 0;
  int *am_parts_out = nullptr;
};

void gemm(Run &r, int dtype, const void *x, const void *w, const void *bias, const void *res, void *y, int M, int N,
          int K, int out_f32, int glu = 0, int fused_norm = 0, float norm_eps = 0.f, const GemmExtra *ex = nullptr) {
  if (r.st != SF_OK) return;
  GemmArgs g{x, w, bias, res, y, M, N, K, out_f32, glu, r.gemm_ws, r.gemm_ws_bytes};
  g.plan_M = r.plan_rows;
  g.tile = r.c->tune_tile; g.split = r.c->tune_split;
  g.fused_norm = fused_norm; g.norm_eps = norm_eps;
  if (ex && dtype == SF_BF16) {
    g.res_f32 = ex->res_f32; g.y2 = ex->y2; g.hooks = ex->hooks; g.hook_mask = ex->hook_mask; g.hook_q = ex->hook_q;
    g.hook_qmax = ex->hook_qmax; g.am_val = ex->am_val; g.am_idx = ex->am_idx; g.am_stride = ex->am_stride;
    g.am_parts_out = ex->am_parts_out;
  }
  LAUNCH(K_GEMM, dtype == SF_BF16 ? launch_gemm_bf16(g, r.s) : launch_gemm_f32(g, r.s));
}

// LM head + arg-max: ids[row] = argmax_v (a . lm_head^T)[row][v].  bf16: the linear kernel's epilogue leaves
// per-column-tile partials and the logits are stored only when `logits` is given; fp32: the logits are
// materialised (in `logits`, else in `scratch_logits`) and scanned in segments.
void lm_head_argmax(Run &r, const sf_model_cfg &m, const void *a, const void *lm_head, float *logits,
                    float *scratch_logits, float *pmax, int32_t *pidx, int32_t *ids, int M) {
  if (m.dtype == SF_BF16) {
    GemmExtra ex;
    int parts = 0;  // column tiles of the launch's tile shape: the partials it writes per row
    ex.am_val = pmax; ex.am_idx = pidx; ex.am_stride = gemm_argmax_parts(m.vocab); ex.am_parts_out = &parts;
    gemm(r, m.dtype, a, lm_head, nullptr, nullptr, logits, M, m.vocab, m.d_model, 1, 0, 0, 0.f, &ex);
    LAUNCH(K_ACCEPT, launch_argmax_final(pmax, pidx, M, parts, ex.am_stride, ids, r.s));
  } else {
    float *lg = logits ? logits : scratch_logits;
    gemm(r, m.dtype, a, lm_head, nullptr, nullptr, lg, M, m.vocab, m.d_model, 1);
    LAUNCH(K_ARGMAX, launch_argmax_partial(lg, M, m.vocab, pmax, pidx, r.s));
    LAUNCH(K_ACCEPT, launch_argmax_final(pmax, pidx, M, ARGMAX_SEGS, ARGMAX_SEGS, ids, r.s));
  }
}

// act[M][F] = silu(a . Wg^T) * (a . Wu^T): one kernel in bf16 mode (weight packed with glu = 1), GEMM to
// fp32 + gating kernel in fp32 mode
void swiglu_in(Run &r, int dtype, const void *a, const void *w_gate_up, float *gu, void *act, int M, int F, int K,
               int fused_norm = 0, float norm_eps = 0.f) {
  if (dtype == SF_BF16) {
    gemm(r, dtype, a, w_gate_up, nullptr, nullptr, act, M, 2 * F, K, 0, 1, fused_norm, norm_eps);
  } else {
    gemm(r, dtype, a, w_gate_up, nullptr, nullptr, gu, M, 2 * F, K, 1);
    LAUNCH(K_SILU, launch_silu_mul(gu, act, M, F, dtype, r.s));
  }
}

void norm(Run &r, const sf_model_cfg &m, const void *x, const void *gain, void *y, int M, int n_gain = 1,
          int map = 0, int q = 1, int q_max = 1, const int32_t *n_new = nullptr, int x_f32 = 0) {
  if (r.st != SF_OK) return;
  NormArgs n{x, gain, y, M, m.d_model, n_gain, m.rms_eps, map, q, q_max, n_new, x_f32};
  LAUNCH(K_NORM, launch_rmsnorm(n, m.dtype, r.s));
}

// y = RMSNorm(x; gain) . w^T.  bf16: ONE kernel -- w was packed with the gain folded into its columns,
// the linear kernel takes the raw rows, sums their squares while staging them and scales its
// accumulators by the row factor.  fp32: the norm kernel into `tmp`, then the linear kernel.
// x: the rows in fp32 mode; xb: their bf16 copy in bf16 mode (rows of the residual stream are kept as float
// plus a bf16 copy for exactly this use).
void norm_gemm(Run &r, const sf_model_cfg &m, const void *x, const void *xb, const void *gain, void *tmp,
               const void *w, void *y, int M, int N, int K, int out_f32) {
  if (m.dtype == SF_BF16) {
    gemm(r, m.dtype, xb, w, nullptr, nullptr, y, M, N, K, out_f32, 0, 1, m.rms_eps);
  } else {
    norm(r, m, x, gain, tmp, M);
    gemm(r, m.dtype, tmp, w, nullptr, nullptr, y, M, N, K, out_f32);
  }
}

void norm_swiglu_in(Run &r, const sf_model_cfg &m, const void *x, const void *xb, const void *gain, void *tmp,
                    const void *w_gate_up, float *gu, void *act, int M, int F, int K) {
  if (m.dtype == SF_BF16) {
    swiglu_in(r, m.dtype, xb, w_gate_up, gu, act, M, F, K, 1, m.rms_eps);
  } else {
    norm(r, m, x, gain, tmp, M);
    swiglu_in(r, m.dtype, tmp, w_gate_up, gu, act, M, F, K);
  }
}

void attention(Run &r, const sf_model_cfg &m, const void *q, const void *kc, const void *vc, const int32_t *kv_len,
               void *out, float *part_o, float *part_ml, int B, int n_q, int cap, int mode, int len_upper,
               const void *qkv = nullptr, const float2 *table = nullptr, const int32_t *order = nullptr) {
  if (r.st != SF_OK) return;
  AttnArgs a{};
  a.q = q; a.qkv = qkv; a.table = table; a.order = order; a.kc = kc; a.vc = vc; a.kv_len = kv_len; a.out = out; a.part_o = part_o; a.part_ml = part_ml;
  a.B = B; a.n_q = n_q; a.Hq = m.n_q_heads; a.Hkv = m.n_kv_heads; a.hd = m.head_dim; a.cap = cap; a.mode = mode;
  const int n_rt = (m.n_q_heads / m.n_kv_heads * n_q + 31) / 32;
  a.chunk_tiles = r.c->tune_chunk > 0 ? r.c->tune_chunk : attn_chunk_tiles(B * m.n_kv_heads * n_rt, len_upper + n_q);
  const int n_tiles = (len_upper + n_q + TK - 1) / TK;
  a.n_chunks = (n_tiles + a.chunk_tiles - 1) / a.chunk_tiles;
  LAUNCH(K_ATTN, m.dtype == SF_BF16 ? launch_attention_bf16(a, r.s) : launch_attention_f32(a, r.s));
  if (m.dtype == SF_BF16 && a.n_chunks > 1) LAUNCH(K_ATTN_COMBINE, launch_attention_combine(a, r.s));
}

size_t kv_layer_bytes(const sf_model_cfg &m, int B, int cap) {
  return (size_t)B * m.n_kv_heads * cap * m.head_dim * esize(m.dtype);
}

sf_status check_state(const sf_ctx *c, const sf_state *st, int k, bool need_draft) {
  if (!c || !st) return SF_EINVAL;
  if (!c->bound) return SF_ESTATE;
  if (need_draft && !c->has_draft) return SF_ESTATE;
  if (k < 0 || k > c->max_k || st->B < 1 || st->B > c->max_B) return SF_EINVAL;
  if (st->cap < TK || st->cap % TK) return SF_EINVAL;
  if (!st->kv_len || !st->pending || !st->hooks || !st->n_new || !st->cu_new || !st->workspace) return SF_EINVAL;
  if (!st->tk || !st->tv) return SF_EINVAL;
  if (need_draft && (!st->dk || !st->dv)) return SF_EINVAL;
  if (((uintptr_t)st->workspace) % ALIGN) return SF_EINVAL;
  if (st->workspace_bytes < plan(c, st->B, k, st->cap).total) return SF_ECAPACITY;
  return SF_OK;
}

}  // namespace

extern "C" {

sf_status sf_create(const sf_model_cfg *t, const sf_model_cfg *d, int32_t max_B, int32_t max_k, sf_ctx **out) {
  if (!t || !d || !out) return SF_EINVAL;
  if (max_B < 1 || max_B > 4096 || max_k < 0 || max_k > 127) return SF_EINVAL;
  if (t->n_layers < 1 || d->n_layers != 1 || !same_shape(*t, *d)) return SF_EINVAL;
  if (t->d_model < 8 || t->n_q_heads < 1 || t->n_kv_heads < 1 || t->head_dim < 8 || t->d_ffn < 8 || t->vocab < 1)
    return SF_EINVAL;
  if (t->n_q_heads % t->n_kv_heads) return SF_EINVAL;
  if (t->dtype != SF_BF16 && t->dtype != SF_F32) return SF_EINVAL;
  if (!(t->rms_eps >= 0.f) || !(t->rope_theta > 1.f)) return SF_EINVAL;
  if (t->d_model % 8 || t->d_ffn % 32 || (t->n_q_heads * t->head_dim) % 32) return SF_EUNSUPPORTED;
  if (t->dtype == SF_BF16 && t->head_dim != 64 && t->head_dim != 128) return SF_EUNSUPPORTED;
  if (t->dtype == SF_F32 && (t->head_dim % 8 || t->head_dim > 256)) return SF_EUNSUPPORTED;
  sf_status s = check_attn_shape(*t, max_k + 1);
  if (s != SF_OK) return s;
  sf_ctx *c = new (std::nothrow) sf_ctx();
  if (!c) return SF_EINVAL;
  c->tc = *t; c->dc = *d; c->max_B = max_B; c->max_k = max_k;
  c->bound = false; c->has_draft = false; c->hip_err = 0;
  *out = c;
  return SF_OK;
}

sf_status sf_destroy(sf_ctx *c) {
  if (!c) return SF_EINVAL;
  for (hipEvent_t e : c->prof.ev) (void)hipEventDestroy(e);
  delete c;
  return SF_OK;
}

size_t sf_workspace_bytes(const sf_ctx *c, int32_t B, int32_t k, int32_t cap) {
  if (!c || B < 1 || B > c->max_B || k < 0 || k > c->max_k || cap < TK || cap % TK) return 0;
  return plan(c, B, k, cap).total;
}

size_t sf_kv_cache_bytes(const sf_ctx *c, int32_t which, int32_t B, int32_t cap) {
  if (!c || B < 1 || cap < TK || cap % TK || (which != 0 && which != 1)) return 0;
  return kv_layer_bytes(c->tc, B, cap) * (which == 0 ? c->tc.n_layers : 1);
}

sf_status sf_bind(sf_ctx *c, const sf_target_weights *t, const sf_draft_weights *d) {
  if (!c || !t) return SF_EINVAL;
  if (!t->embed || !t->lm_head || !t->final_norm || !t->attn_norm || !t->wqkv || !t->wo || !t->ffn_norm ||
      !t->w_gate_up || !t->w_down)
    return SF_EINVAL;
  const int L = c->tc.n_layers;
  for (int l = 0; l < L; ++l)
    if (!t->attn_norm[l] || !t->wqkv[l] || !t->wo[l] || !t->ffn_norm[l] || !t->w_gate_up[l] || !t->w_down[l])
      return SF_EINVAL;
  if (d) {
    // every pointer up to out_norm is required; the slot attention's own set (sa_*) comes whole or not at all
    const void *const *p = reinterpret_cast<const void *const *>(d);
    for (size_t i = 0; i < offsetof(sf_draft_weights, sa_norm) / sizeof(void *); ++i)
      if (!p[i]) return SF_EINVAL;
    const int n_sa = (d->sa_norm != nullptr) + (d->sa_wqkv != nullptr) + (d->sa_wo != nullptr);
    if (n_sa != 0 && n_sa != 3) return SF_EINVAL;
  }
  c->tw = *t;
  c->attn_norm.assign(t->attn_norm, t->attn_norm + L);
  c->wqkv.assign(t->wqkv, t->wqkv + L);
  c->wo.assign(t->wo, t->wo + L);
  c->ffn_norm.assign(t->ffn_norm, t->ffn_norm + L);
  c->w_gate_up.assign(t->w_gate_up, t->w_gate_up + L);
  c->w_down.assign(t->w_down, t->w_down + L);
  c->has_draft = d != nullptr;
  if (d) c->dw = *d;
  // function attributes of the tall linear tiles, set here so that the first launch (possibly under stream
  // capture) has nothing left to set; best effort -- a launch repeats the call and reports its error
  if (c->tc.dtype == SF_BF16) (void)gemm_prepare_device();
  c->bound = true;
  return SF_OK;
}

sf_status sf_verify_step(sf_ctx *c, const sf_state *st, int32_t k, const int32_t *draft, int32_t len_upper,
                         float *logits, int32_t *target_ids, void *stream) {
  sf_status v = check_state(c, st, k, false);
  if (v != SF_OK) return v;
  if (!target_ids || (k > 0 && !draft) || len_upper < 0) return SF_EINVAL;
  const sf_model_cfg &m = c->tc;
  const int B = st->B, q = k + 1, M = B * q, cap = st->cap, qm = c->max_k + 1;
  if ((long)len_upper + q > cap) return SF_ECAPACITY;
  if ((v = check_attn_shape(m, q)) != SF_OK) return v;
  const Arena A = plan(c, B, k, cap);
  char *ws = (char *)st->workspace;
  float *h = (float *)(ws + A.h);                                    // the residual stream
  void *hb = m.dtype == SF_BF16 ? (void *)(ws + A.hb) : (void *)h;   // bf16: its copy for the matrix products
  void *a = ws + A.a, *qkv = ws + A.qkv, *qr = ws + A.qr, *ao = ws + A.ao, *act = ws + A.act;
  float *gu = (float *)(ws + A.gu);
  const int d = m.d_model, F = m.d_ffn, L = m.n_layers;
  const int nq = m.n_q_heads * m.head_dim, nkv = m.n_kv_heads * m.head_dim;
  const bool bf = m.dtype == SF_BF16;
  Run r{c, (hipStream_t)stream};
  r.gemm_ws = ws + A.gemm_ws; r.gemm_ws_bytes = A.gemm_ws_bytes;
  // the target's logits for a position must not depend on how many draft positions are verified
  // with it: every k of this state uses the K partition chosen for the largest block
  r.plan_rows = B * qm;
  // hooked states: group g holds the stream after layer hook_layer[g] (0 = the embedding)
  const int hook_layer[4] = {0, L / 2, L - 1, L};
  auto hook_mask_of = [&](int l) {
    int mask = 0;
    for (int g = 0; g < 4; ++g) mask |= (hook_layer[g] == l) << g;
    return mask;
  };
  LAUNCH(K_EMBED_HOOK, launch_embed(c->tw.embed, st->pending, draft, h, bf ? hb : nullptr, st->hooks, hook_mask_of(0),
                                    B, k, qm, d, m.vocab, m.dtype, r.s));
  RopeArgs ra{};
  ra.qkv = qkv; ra.q_out = qr; ra.kv_len = st->kv_len; ra.n_new = nullptr; ra.table = (float2 *)(ws + A.table);
  ra.B = B; ra.n_q = q; ra.Hq = m.n_q_heads; ra.Hkv = m.n_kv_heads; ra.hd = m.head_dim; ra.cap = cap;
  ra.kv_only = 0; ra.pos_mode = 0; ra.theta = m.rope_theta;
  // bf16, more attention workgroups than the chip holds at once (2 per CU): the table kernel also ranks
  // the sequences by length, and the attention launches of this call start the longest first
  const int attn_groups = B * m.n_kv_heads * ((m.n_q_heads / m.n_kv_heads * q + 31) / 32);
  ra.order = bf && attn_groups > 512 ? (int32_t *)(ws + A.order) : nullptr;
  ra.dev_err = (int32_t *)(ws + A.dev_err); ra.len_upper = len_upper;
  LAUNCH(K_ROPE, launch_rope_table(ra, r.s));
  const size_t lb = kv_layer_bytes(m, B, cap);
  for (int l = 0; l < L && r.st == SF_OK; ++l) {
    void *kc = (char *)st->tk + l * lb, *vc = (char *)st->tv + l * lb;
    norm_gemm(r, m, h, hb, c->attn_norm[l], a, c->wqkv[l], qkv, M, nq + 2 * nkv, d, 0);
    ra.kc = kc; ra.vc = vc;
    // bf16: the attention kernel rotates Q and K and appends the block's K, V rows itself
    if (!bf) LAUNCH(K_ROPE, launch_rope_kv(ra, m.dtype, r.s));
    attention(r, m, qr, kc, vc, st->kv_len, ao, (float *)(ws + A.part_o), (float *)(ws + A.part_ml), B, q, cap,
              SF_MASK_CAUSAL, len_upper, bf ? qkv : nullptr, ra.table, ra.order);
    // h += attention . W_O, and h += W_down . act: float sums; bf16 mode also refreshes the bf16 copy
    GemmExtra ex;
    ex.res_f32 = 1; ex.y2 = hb;
    gemm(r, m.dtype, ao, c->wo[l], nullptr, h, h, M, d, nq, 1, 0, 0, 0.f, &ex);
    norm_swiglu_in(r, m, h, hb, c->ffn_norm[l], a, c->w_gate_up[l], gu, act, M, F, d);
    const int mask = hook_mask_of(l + 1);  // the stream after this layer is hooked state(s) `mask`
    if (mask) { ex.hooks = st->hooks; ex.hook_mask = mask; ex.hook_q = q; ex.hook_qmax = qm; }
    gemm(r, m.dtype, act, c->w_down[l], nullptr, h, h, M, d, F, 1, 0, 0, 0.f, &ex);
    if (!bf)
      for (int g = 1; g < 4; ++g)
        if (mask >> g & 1) LAUNCH(K_EMBED_HOOK, launch_hook_copy(h, st->hooks, B, q, qm, d, g, m.dtype, r.s));
  }
  // the LM head serves two norms (this one and the draft's), so no gain is folded into it
  norm(r, m, h, c->tw.final_norm, a, M, 1, 0, 1, 1, nullptr, 1);
  lm_head_argmax(r, m, a, c->tw.lm_head, logits, (float *)(ws + A.logits), (float *)(ws + A.pmax),
                 (int32_t *)(ws + A.pidx), target_ids, M);
  if (r.st == SF_OK) { c->verified_state = st->kv_len; c->verified_k = k; }
  return r.st;
}

sf_status sf_draft_step(sf_ctx *c, const sf_state *st, int32_t k, int32_t mask, int32_t len_upper,
                        int32_t *draft_tokens, float *draft_logits, void *stream) {
  sf_status v = check_state(c, st, k, true);
  if (v != SF_OK) return v;
  if (k == 0) return SF_OK;
  const bool two_stage = (mask & SF_DRAFT_TWO_STAGE) != 0;
  mask &= ~SF_DRAFT_TWO_STAGE;
  if (!draft_tokens || len_upper < 0 || (mask != SF_MASK_CAUSAL && mask != SF_MASK_BIDIR)) return SF_EINVAL;
  const sf_model_cfg &m = c->dc;
  const int B = st->B, cap = st->cap, qm = c->max_k + 1, Mh = B * qm, Ms = B * k;
  if ((long)len_upper + k > cap) return SF_ECAPACITY;
  if ((v = check_attn_shape(m, k)) != SF_OK) return v;
  const sf_draft_weights &w = c->dw;
  if (two_stage && (!w.sa_norm || !w.sa_wqkv || !w.sa_wo)) return SF_ESTATE;
  if (two_stage && k > TK) return SF_EUNSUPPORTED;
  const Arena A = plan(c, B, k, cap);
  char *ws = (char *)st->workspace;
  const bool bf = m.dtype == SF_BF16;
  void *a = ws + A.a, *qkv = ws + A.qkv, *qr = ws + A.qr, *ao = ws + A.ao, *act = ws + A.act;
  void *f4 = ws + A.f4, *x = ws + A.x, *kvc = ws + A.kvc, *xl = ws + A.xl;
  float *s0 = (float *)(ws + A.s0);                                    // the slot layer's residual stream
  void *s0b = bf ? (void *)(ws + A.s0b) : (void *)s0;                  // bf16: its copy for the matrix products
  float *gu = (float *)(ws + A.gu);
  float *part_o = (float *)(ws + A.part_o), *part_ml = (float *)(ws + A.part_ml);
  const int d = m.d_model, F = m.d_ffn;
  const int nq = m.n_q_heads * m.head_dim, nkv = m.n_kv_heads * m.head_dim;
  const size_t es = esize(m.dtype);
  Run r{c, (hipStream_t)stream};
  r.gemm_ws = ws + A.gemm_ws; r.gemm_ws_bytes = A.gemm_ws_bytes;
  // context rows: Grouped RMSNorm -> W_D -> K,V of the draft attention layer at the rows' positions
  norm(r, m, st->hooks, w.group_norm, f4, Mh * 4, 4, 1, qm, qm, nullptr);
  gemm(r, m.dtype, f4, w.w_ds, nullptr, nullptr, x, Mh, d, 4 * d, 0);
  // K and V rows of wqkv start after the nq query rows (a whole number of packed 32-row blocks)
  const size_t kv_off = bf ? packed_weight_bytes(nq, d, m.dtype) : (size_t)nq * d * es;
  norm_gemm(r, m, x, x, w.attn_norm, a, (const char *)w.wqkv + kv_off, kvc, Mh, 2 * nkv, d, 0);
  RopeArgs ra{};
  ra.qkv = kvc; ra.q_out = nullptr; ra.kc = st->dk; ra.vc = st->dv; ra.kv_len = st->kv_len; ra.n_new = st->n_new;
  ra.table = (float2 *)(ws + A.table);
  ra.B = B; ra.n_q = qm; ra.Hq = m.n_q_heads; ra.Hkv = m.n_kv_heads; ra.hd = m.head_dim; ra.cap = cap;
  ra.kv_only = 1; ra.pos_mode = 1; ra.theta = m.rope_theta;
  // the same launch fills the slots' table (positions kv_len[b] + s) when they sit behind the cached context
  float2 *slot_table = ra.table + (size_t)Mh * (m.head_dim / 2);
  if (!two_stage) {
    ra.table2 = slot_table; ra.n_q2 = k;
    ra.dev_err = (int32_t *)(ws + A.dev_err); ra.len_upper = len_upper;
  }
  LAUNCH(K_ROPE, launch_rope_table(ra, r.s));
  LAUNCH(K_ROPE, launch_rope_kv(ra, m.dtype, r.s));
  ra.table2 = nullptr; ra.dev_err = nullptr;
  const void *norm_s = w.attn_norm, *wqkv_s = w.wqkv, *wo_s = w.wo;  // the slot attention's parameters
  const void *kc_s = st->dk, *vc_s = st->dv;
  const int32_t *len_s = st->kv_len;
  int cap_s = cap, len_upper_s = len_upper;
  if (!two_stage) {
    // positional FFN on the newest committed row -> k slot states
    norm(r, m, x, w.pos_norm, xl, B, 1, 2, qm, qm, st->n_new);
  } else {
    // The context attention's own output at the newest row (its K/V are in the cache by now):
    // I_D = X + W_O . attention(RoPE(W_Q . RMS(X)), keys up to and including the row itself).
    void *x_last = ws + A.x_last, *q1 = ws + A.q1, *qr1 = ws + A.qr1, *ao1 = ws + A.ao1;
    float *id_last = (float *)(ws + A.id_last);
    int32_t *len_m1 = (int32_t *)(ws + A.len_m1);
    LAUNCH(K_EMBED_HOOK, launch_gather_last(x, x_last, st->n_new, st->kv_len, len_m1, B, qm, d, m.dtype, r.s));
    norm_gemm(r, m, x_last, x_last, w.attn_norm, a, w.wqkv, q1, B, nq, d, 0);  // the nq query rows lead wqkv
    RopeArgs rq{};
    rq.qkv = q1; rq.q_out = qr1; rq.kc = nullptr; rq.vc = nullptr; rq.kv_len = len_m1; rq.n_new = nullptr;
    rq.table = ra.table; rq.B = B; rq.n_q = 1; rq.Hq = m.n_q_heads; rq.Hkv = 0; rq.hd = m.head_dim; rq.cap = cap;
    rq.kv_only = 0; rq.pos_mode = 0; rq.theta = m.rope_theta;
    LAUNCH(K_ROPE, launch_rope_table(rq, r.s));
    LAUNCH(K_ROPE, launch_rope_kv(rq, m.dtype, r.s));
    attention(r, m, qr1, st->dk, st->dv, len_m1, ao1, part_o, part_ml, B, 1, cap, SF_MASK_CAUSAL, len_upper);
    gemm(r, m.dtype, ao1, w.wo, nullptr, x_last, id_last, B, d, nq, 1);  // float row of the stream
    norm(r, m, id_last, w.pos_norm, xl, B, 1, 3, 1, 1, st->n_new, 1);
    // the slots attend to each other only: an empty prefix in a one-tile cache of their own
    norm_s = w.sa_norm; wqkv_s = w.sa_wqkv; wo_s = w.sa_wo;
    kc_s = ws + A.kc2; vc_s = ws + A.vc2; len_s = (const int32_t *)(ws + A.zeros);
    cap_s = TK; len_upper_s = 0;
  }
  GemmExtra ex;
  ex.y2 = s0b;
  gemm(r, m.dtype, xl, w.w_pos, w.b_pos, nullptr, s0, B, k * d, d, 1, 0, 0, 0.f, &ex);
  // one attention + SwiGLU layer over the slots
  norm_gemm(r, m, s0, s0b, norm_s, a, wqkv_s, qkv, Ms, nq + 2 * nkv, d, 0);
  ra.qkv = qkv; ra.q_out = qr; ra.kc = (void *)kc_s; ra.vc = (void *)vc_s; ra.kv_len = len_s; ra.n_new = nullptr;
  ra.n_q = k; ra.cap = cap_s; ra.kv_only = 0; ra.pos_mode = 0; ra.table = slot_table;
  if (two_stage) LAUNCH(K_ROPE, launch_rope_table(ra, r.s));  // slots at positions 0..k-1 of their own tile
  // bf16: the attention kernel rotates the slots' Q and K and appends their K, V rows itself
  if (!bf) LAUNCH(K_ROPE, launch_rope_kv(ra, m.dtype, r.s));
  attention(r, m, qr, kc_s, vc_s, len_s, ao, part_o, part_ml, B, k, cap_s, mask, len_upper_s, bf ? qkv : nullptr,
            ra.table);
  ex.res_f32 = 1;
  gemm(r, m.dtype, ao, wo_s, nullptr, s0, s0, Ms, d, nq, 1, 0, 0, 0.f, &ex);
  norm_swiglu_in(r, m, s0, s0b, w.ffn_norm, a, w.w_gate_up, gu, act, Ms, F, d);
  ex.y2 = nullptr;
  gemm(r, m.dtype, act, w.w_down, nullptr, s0, s0, Ms, d, F, 1, 0, 0, 0.f, &ex);
  norm(r, m, s0, w.out_norm, a, Ms, 1, 0, 1, 1, nullptr, 1);
  lm_head_argmax(r, m, a, c->tw.lm_head, draft_logits, (float *)(ws + A.logits), (float *)(ws + A.pmax),
                 (int32_t *)(ws + A.pidx), draft_tokens, Ms);
  return r.st;
}

sf_status sf_accept_commit(sf_ctx *c, const sf_state *st, int32_t k, const int32_t *draft, const int32_t *target_ids,
                           const int32_t *force_len, int32_t *accept_len, int32_t *out_tokens, void *stream) {
  sf_status v = check_state(c, st, k, false);
  if (v != SF_OK) return v;
  if (!target_ids || !accept_len || !out_tokens || (k > 0 && !draft && !force_len)) return SF_EINVAL;
  // nothing to commit unless sf_verify_step wrote this very block (same state, same k) since the last commit
  if (c->verified_state != st->kv_len || c->verified_k != k) return SF_ESTATE;
  Run r{c, (hipStream_t)stream};
  AcceptArgs a{target_ids, draft, force_len, accept_len, out_tokens, st->kv_len, st->pending, st->n_new, st->cu_new,
               st->B, k};
  LAUNCH(K_ACCEPT, launch_accept(a, r.s));
  if (r.st == SF_OK) { c->verified_state = nullptr; c->verified_k = -1; }
  return r.st;
}

sf_status sf_op_accept(const sf_ctx *c, int32_t B, int32_t k, const int32_t *draft, const int32_t *target_ids,
                       const int32_t *force_len, int32_t *accept_len, int32_t *out_tokens, int32_t *kv_len,
                       int32_t *pending, int32_t *n_new, int32_t *cu_new, void *stream) {
  if (!c || B < 1 || k < 0 || k > 127) return SF_EINVAL;
  if (!target_ids || !accept_len || !out_tokens || !kv_len || !pending || !n_new || !cu_new) return SF_EINVAL;
  if (k > 0 && !draft && !force_len) return SF_EINVAL;
  Run r{c, (hipStream_t)stream};
  AcceptArgs a{target_ids, draft, force_len, accept_len, out_tokens, kv_len, pending, n_new, cu_new, B, k};
  LAUNCH(K_ACCEPT, launch_accept(a, r.s));
  return r.st;
}

sf_status sf_check_state(const sf_ctx *c, const sf_state *st, int32_t *flags, void *stream) {
  if (!c || !st || !flags || !st->workspace || st->B < 1 || st->B > c->max_B || st->cap < TK || st->cap % TK)
    return SF_EINVAL;
  const Arena A = plan(c, st->B, 0, st->cap);  // the word sits in the k-independent head of the arena
  if (st->workspace_bytes < A.dev_err + sizeof(int32_t)) return SF_ECAPACITY;
  int32_t *word = (int32_t *)((char *)st->workspace + A.dev_err);
  hipStream_t s = (hipStream_t)stream;
  hipError_t e = hipMemcpyAsync(flags, word, sizeof(int32_t), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e == hipSuccess && *flags != 0) {
    e = hipMemsetAsync(word, 0, sizeof(int32_t), s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
  }
  if (e != hipSuccess) { c->hip_err = (int)e; return SF_EHIP; }
  return *flags ? SF_ECAPACITY : SF_OK;
}

sf_status sf_kv_import(const sf_ctx *c, const void *plain, void *tiled, int32_t is_v, int32_t B, int32_t cap,
                       void *stream) {
  if (!c || !plain || !tiled || B < 1 || cap < TK || cap % TK) return SF_EINVAL;
  hipError_t e = launch_kv_convert(plain, tiled, is_v, 1, B, c->tc.n_kv_heads, cap, c->tc.head_dim, c->tc.dtype,
                                   (hipStream_t)stream);
  if (e != hipSuccess) { c->hip_err = (int)e; return SF_EHIP; }
  return SF_OK;
}

sf_status sf_kv_export(const sf_ctx *c, const void *tiled, void *plain, int32_t is_v, int32_t B, int32_t cap,
                       void *stream) {
  if (!c || !plain || !tiled || B < 1 || cap < TK || cap % TK) return SF_EINVAL;
  hipError_t e = launch_kv_convert(tiled, plain, is_v, 0, B, c->tc.n_kv_heads, cap, c->tc.head_dim, c->tc.dtype,
                                   (hipStream_t)stream);
  if (e != hipSuccess) { c->hip_err = (int)e; return SF_EHIP; }
  return SF_OK;
}

size_t sf_attention_workspace_bytes(const sf_ctx *c, int32_t B, int32_t n_q, int32_t len_upper) {
  if (!c || B < 1 || n_q < 1 || len_upper < 0 || c->tc.dtype != SF_BF16) return 0;
  return attn_workspace_bytes(B, c->tc.n_kv_heads, c->tc.head_dim, c->tc.n_q_heads / c->tc.n_kv_heads, n_q,
                              len_upper);
}

sf_status sf_op_attention(const sf_ctx *c, const void *q, const void *kc, const void *vc, const int32_t *kv_len,
                          int32_t B, int32_t n_q, int32_t cap, int32_t mask, int32_t len_upper, void *out,
                          void *workspace, size_t workspace_bytes, void *stream) {
  if (!c || !q || !kc || !vc || !kv_len || !out) return SF_EINVAL;
  if (B < 1 || n_q < 1 || cap < TK || cap % TK || len_upper < 0) return SF_EINVAL;
  if (mask != SF_MASK_CAUSAL && mask != SF_MASK_BIDIR) return SF_EINVAL;
  if ((long)len_upper + n_q > cap) return SF_ECAPACITY;
  const sf_model_cfg &m = c->tc;
  sf_status v = check_attn_shape(m, n_q);
  if (v != SF_OK) return v;
  const size_t need = sf_attention_workspace_bytes(c, B, n_q, len_upper);
  if (need && (!workspace || workspace_bytes < need || ((uintptr_t)workspace) % ALIGN)) return SF_ECAPACITY;
  const size_t rows = need / ((m.head_dim + 2) * sizeof(float));
  float *part_o = (float *)workspace, *part_ml = part_o ? part_o + rows * m.head_dim : nullptr;
  Run r{c, (hipStream_t)stream};
  attention(r, m, q, kc, vc, kv_len, out, part_o, part_ml, B, n_q, cap, mask, len_upper);
  return r.st;
}

size_t sf_packed_weight_bytes(const sf_ctx *c, int32_t N, int32_t K) {
  if (!c || N < 1 || K < 1) return 0;
  return packed_weight_bytes(N, K, c->tc.dtype);
}

sf_status sf_pack_weight(const sf_ctx *c, const void *w, void *packed, int32_t N, int32_t K, int32_t glu,
                         const void *col_gain, void *stream) {
  if (!c || !w || !packed || N < 1 || K < 1) return SF_EINVAL;
  if (((uintptr_t)packed) % 16) return SF_EINVAL;
  if (glu && (N % 64)) return SF_EUNSUPPORTED;  // F = N/2 must be a multiple of 32
  hipError_t e = launch_pack_weight(w, packed, N, K, glu, c->tc.dtype == SF_BF16 ? col_gain : nullptr, c->tc.dtype,
                                    (hipStream_t)stream);
  if (e != hipSuccess) { c->hip_err = (int)e; return SF_EHIP; }
  return SF_OK;
}

size_t sf_linear_workspace_bytes(const sf_ctx *c, int32_t M) {
  if (!c || M < 1 || c->tc.dtype != SF_BF16) return 0;
  return gemm_workspace_bytes(M);
}

sf_status sf_tune_attention(sf_ctx *c, int32_t chunk_tiles) {
  if (!c || chunk_tiles < 0 || (chunk_tiles > 0 && chunk_tiles < 16)) return SF_EINVAL;
  c->tune_chunk = chunk_tiles;
  return SF_OK;
}

sf_status sf_tune_linear(sf_ctx *c, int32_t tile, int32_t split_k) {
  if (!c || tile < 0 || tile > gemm_num_tiles() || split_k < 0 || split_k > 64) return SF_EINVAL;
  c->tune_tile = tile; c->tune_split = split_k;
  return SF_OK;
}

int32_t sf_linear_num_tiles(void) { return gemm_num_tiles(); }

sf_status sf_linear_config(int32_t M, int32_t plan_M, int32_t N, int32_t K, size_t workspace_bytes, int32_t *tile,
                           int32_t *split_k, int32_t *tile_rows) {
  if (M < 1 || plan_M < M || N < 1 || K < 1 || !tile || !split_k || !tile_rows) return SF_EINVAL;
  const GemmConfig c = gemm_heuristic(M, plan_M, N, K, workspace_bytes);
  *tile = c.tile; *split_k = c.split; *tile_rows = gemm_tile_rows(c.tile);
  return SF_OK;
}

sf_status sf_op_linear(const sf_ctx *c, const void *x, const void *w, const void *bias, const void *residual,
                       void *y, int32_t M, int32_t N, int32_t K, int32_t out_f32, void *workspace,
                       size_t workspace_bytes, void *stream) {
  if (!c || !x || !w || !y || M < 1 || N < 1 || K < 1) return SF_EINVAL;
  if (K % 8 || N % 8) return SF_EUNSUPPORTED;
  if (((uintptr_t)x | (uintptr_t)w) % 16) return SF_EINVAL;
  if (workspace && ((uintptr_t)workspace) % ALIGN) return SF_EINVAL;
  Run r{c, (hipStream_t)stream};
  r.gemm_ws = workspace; r.gemm_ws_bytes = workspace ? workspace_bytes : 0;
  gemm(r, c->tc.dtype, x, w, bias, residual, y, M, N, K, out_f32);
  return r.st;
}

size_t sf_linear_argmax_workspace_bytes(const sf_ctx *c, int32_t M, int32_t N) {
  if (!c || M < 1 || N < 1) return 0;
  const bool bf = c->tc.dtype == SF_BF16;
  const size_t parts = bf ? (size_t)gemm_argmax_parts(N) : (size_t)ARGMAX_SEGS;
  return up(bf ? gemm_workspace_bytes(M) : 0) + 2 * up((size_t)M * parts * 4) + up(bf ? 0 : (size_t)M * N * sizeof(float));
}

sf_status sf_op_linear_argmax(const sf_ctx *c, const void *x, const void *w, int32_t M, int32_t N, int32_t K,
                              int32_t *ids, float *logits, void *workspace, size_t workspace_bytes, void *stream) {
  if (!c || !x || !w || !ids || !workspace || M < 1 || N < 1 || K < 1) return SF_EINVAL;
  if (K % 8 || N % 8) return SF_EUNSUPPORTED;
  if (((uintptr_t)x | (uintptr_t)w) % 16 || ((uintptr_t)workspace) % ALIGN) return SF_EINVAL;
  if (workspace_bytes < sf_linear_argmax_workspace_bytes(c, M, N)) return SF_ECAPACITY;
  const bool bf = c->tc.dtype == SF_BF16;
  const size_t parts = bf ? (size_t)gemm_argmax_parts(N) : (size_t)ARGMAX_SEGS;
  char *ws = (char *)workspace;
  const size_t lin = up(bf ? gemm_workspace_bytes(M) : 0), pb = up((size_t)M * parts * 4);
  sf_model_cfg m = c->tc;
  m.vocab = N; m.d_model = K;
  Run r{c, (hipStream_t)stream};
  if (bf) { r.gemm_ws = ws; r.gemm_ws_bytes = lin; }
  lm_head_argmax(r, m, x, w, logits, (float *)(ws + lin + 2 * pb), (float *)(ws + lin), (int32_t *)(ws + lin + pb), ids,
                 M);
  return r.st;
}

sf_status sf_op_rmsnorm_linear(const sf_ctx *c, const void *x, const void *w, void *y, int32_t M, int32_t N,
                               int32_t K, int32_t out_f32, void *workspace, size_t workspace_bytes, void *stream) {
  if (!c || !x || !w || !y || M < 1 || N < 1 || K < 1) return SF_EINVAL;
  if (c->tc.dtype != SF_BF16 || K % 8 || N % 8) return SF_EUNSUPPORTED;
  if (((uintptr_t)x | (uintptr_t)w) % 16) return SF_EINVAL;
  if (workspace && ((uintptr_t)workspace) % ALIGN) return SF_EINVAL;
  Run r{c, (hipStream_t)stream};
  r.gemm_ws = workspace; r.gemm_ws_bytes = workspace ? workspace_bytes : 0;
  gemm(r, SF_BF16, x, w, nullptr, nullptr, y, M, N, K, out_f32, 0, 1, c->tc.rms_eps);
  return r.st;
}

sf_status sf_op_linear_swiglu(const sf_ctx *c, const void *x, const void *w_gate_up, void *act, int32_t M, int32_t F,
                              int32_t K, void *workspace, size_t workspace_bytes, void *stream) {
  if (!c || !x || !w_gate_up || !act || M < 1 || F < 1 || K < 1) return SF_EINVAL;
  if (K % 8 || F % 32) return SF_EUNSUPPORTED;
  if (workspace && ((uintptr_t)workspace) % ALIGN) return SF_EINVAL;
  const bool bf = c->tc.dtype == SF_BF16;
  const size_t lin = bf ? gemm_workspace_bytes(M) : 0, gu_bytes = bf ? 0 : up((size_t)M * 2 * F * sizeof(float));
  if (!bf && (!workspace || workspace_bytes < gu_bytes)) return SF_ECAPACITY;
  Run r{c, (hipStream_t)stream};
  if (bf && workspace && workspace_bytes >= lin) { r.gemm_ws = workspace; r.gemm_ws_bytes = workspace_bytes; }
  swiglu_in(r, c->tc.dtype, x, w_gate_up, (float *)workspace, act, M, F, K);
  return r.st;
}

sf_status sf_op_rmsnorm(const sf_ctx *c, const void *x, const void *gain, void *y, int32_t M, int32_t d,
                        int32_t n_gain, void *stream) {
  if (!c || !x || !gain || !y || M < 1 || d < 1 || n_gain < 1) return SF_EINVAL;
  NormArgs n{x, gain, y, M, d, n_gain, c->tc.rms_eps, 0, 1, 1, nullptr};
  Run r{c, (hipStream_t)stream};
  LAUNCH(K_NORM, launch_rmsnorm(n, c->tc.dtype, r.s));
  return r.st;
}

sf_status sf_op_rope_kv_append(const sf_ctx *c, const void *qkv, const int32_t *kv_len, int32_t B, int32_t n_q,
                               int32_t cap, void *q_out, void *kc, void *vc, void *workspace, size_t workspace_bytes,
                               void *stream) {
  if (!c || !qkv || !kv_len || !q_out || !kc || !vc || !workspace) return SF_EINVAL;
  if (B < 1 || n_q < 1 || cap < TK || cap % TK) return SF_EINVAL;
  const sf_model_cfg &m = c->tc;
  if (workspace_bytes < (size_t)B * n_q * (m.head_dim / 2) * sizeof(float2)) return SF_ECAPACITY;
  RopeArgs ra{};
  ra.qkv = qkv; ra.q_out = q_out; ra.kc = kc; ra.vc = vc; ra.kv_len = kv_len; ra.table = (float2 *)workspace;
  ra.B = B; ra.n_q = n_q; ra.Hq = m.n_q_heads; ra.Hkv = m.n_kv_heads; ra.hd = m.head_dim; ra.cap = cap;
  ra.theta = m.rope_theta;
  Run r{c, (hipStream_t)stream};
  LAUNCH(K_ROPE, launch_rope_table(ra, r.s));
  LAUNCH(K_ROPE, launch_rope_kv(ra, m.dtype, r.s));
  return r.st;
}

size_t sf_rope_attention_workspace_bytes(const sf_ctx *c, int32_t B, int32_t n_q, int32_t len_upper) {
  if (!c || B < 1 || n_q < 1 || len_upper < 0) return 0;
  return up((size_t)B * n_q * (c->tc.head_dim / 2) * sizeof(float2)) + up((size_t)B * sizeof(int32_t)) +
         sf_attention_workspace_bytes(c, B, n_q, len_upper);
}

sf_status sf_op_rope_attention(const sf_ctx *c, const void *qkv, const int32_t *kv_len, int32_t B, int32_t n_q,
                               int32_t cap, int32_t mask, int32_t len_upper, void *kc, void *vc, void *out,
                               void *workspace, size_t workspace_bytes, void *stream) {
  if (!c || !qkv || !kv_len || !kc || !vc || !out || !workspace) return SF_EINVAL;
  if (B < 1 || n_q < 1 || cap < TK || cap % TK || len_upper < 0) return SF_EINVAL;
  if (mask != SF_MASK_CAUSAL && mask != SF_MASK_BIDIR) return SF_EINVAL;
  if ((long)len_upper + n_q > cap) return SF_ECAPACITY;
  const sf_model_cfg &m = c->tc;
  if (m.dtype != SF_BF16) return SF_EUNSUPPORTED;  // fp32 keeps the two separate kernels
  sf_status v = check_attn_shape(m, n_q);
  if (v != SF_OK) return v;
  if (workspace_bytes < sf_rope_attention_workspace_bytes(c, B, n_q, len_upper) || ((uintptr_t)workspace) % ALIGN)
    return SF_ECAPACITY;
  const size_t table_bytes = up((size_t)B * n_q * (m.head_dim / 2) * sizeof(float2));
  const size_t order_bytes = up((size_t)B * sizeof(int32_t));
  const size_t need = sf_attention_workspace_bytes(c, B, n_q, len_upper);
  const size_t rows = need / ((m.head_dim + 2) * sizeof(float));
  float *part_o = need ? (float *)((char *)workspace + table_bytes + order_bytes) : nullptr;
  float *part_ml = part_o ? part_o + rows * m.head_dim : nullptr;
  RopeArgs ra{};
  ra.kv_len = kv_len; ra.table = (float2 *)workspace; ra.order = (int32_t *)((char *)workspace + table_bytes);
  ra.B = B; ra.n_q = n_q; ra.Hq = m.n_q_heads; ra.Hkv = m.n_kv_heads; ra.hd = m.head_dim; ra.cap = cap;
  ra.theta = m.rope_theta;
  Run r{c, (hipStream_t)stream};
  LAUNCH(K_ROPE, launch_rope_table(ra, r.s));
  attention(r, m, nullptr, kc, vc, kv_len, out, part_o, part_ml, B, n_q, cap, mask, len_upper, qkv, ra.table, ra.order);
  return r.st;
}

sf_status sf_op_silu_mul(const sf_ctx *c, const float *gu, void *act, int32_t M, int32_t F, void *stream) {
  if (!c || !gu || !act || M < 1 || F < 1) return SF_EINVAL;
  Run r{c, (hipStream_t)stream};
  LAUNCH(K_SILU, launch_silu_mul(gu, act, M, F, c->tc.dtype, r.s));
  return r.st;
}

size_t sf_argmax_workspace_bytes(int32_t M) {
  return M < 1 ? 0 : up((size_t)M * ARGMAX_SEGS * sizeof(float)) + up((size_t)M * ARGMAX_SEGS * sizeof(int32_t));
}

sf_status sf_op_argmax(const sf_ctx *c, const float *logits, int32_t M, int32_t V, int32_t *ids, void *workspace,
                       size_t workspace_bytes, void *stream) {
  if (!c || !logits || !ids || !workspace || M < 1 || V < 1) return SF_EINVAL;
  if (workspace_bytes < sf_argmax_workspace_bytes(M) || ((uintptr_t)workspace) % ALIGN) return SF_ECAPACITY;
  float *pmax = (float *)workspace;
  int32_t *pidx = (int32_t *)((char *)workspace + up((size_t)M * ARGMAX_SEGS * sizeof(float)));
  Run r{c, (hipStream_t)stream};
  LAUNCH(K_ARGMAX, launch_argmax_partial(logits, M, V, pmax, pidx, r.s));
  LAUNCH(K_ACCEPT, launch_argmax_final(pmax, pidx, M, ARGMAX_SEGS, ARGMAX_SEGS, ids, r.s));
  return r.st;
}

sf_status sf_op_argmax_noalloc(const sf_ctx *c, const float *logits, int32_t M, int32_t V, int32_t *ids, void *stream) {
  if (!c || !logits || !ids || M < 1 || V < 1) return SF_EINVAL;
  if (M > ARGMAX_NOALLOC_MAX_ROWS) return SF_ECAPACITY;
  (void)hipGetLastError();
  const hipError_t e = launch_argmax_noalloc(logits, M, V, ids, (hipStream_t)stream);
  if (e != hipSuccess) { c->hip_err = (int)e; return SF_EHIP; }
  return SF_OK;
}

sf_status sf_calib_copy(void *dst, const void *src, size_t bytes, void *stream) {
  if (!dst || !src || bytes % 16 || (((uintptr_t)dst | (uintptr_t)src) % 16)) return SF_EINVAL;
  return launch_calib_copy(src, dst, bytes, (hipStream_t)stream) == hipSuccess ? SF_OK : SF_EHIP;
}

sf_status sf_profile_begin(sf_ctx *c) {
  if (!c) return SF_EINVAL;
  c->prof.on = true;
  c->prof.used = 0;
  return SF_OK;
}

sf_status sf_profile_end(sf_ctx *c, double *ms, int32_t *launches, int32_t n_class) {
  if (!c || !ms || !launches || n_class < K_NCLASS) return SF_EINVAL;
  Prof &p = c->prof;
  p.on = false;
  for (int i = 0; i < n_class; ++i) { ms[i] = 0.0; launches[i] = 0; }
  if (p.used == 0) return SF_OK;
  hipError_t e = hipEventSynchronize(p.ev[2 * p.used - 1]);
  for (size_t i = 0; i < p.used && e == hipSuccess; ++i) {
    float t = 0.f;
    e = hipEventElapsedTime(&t, p.ev[2 * i], p.ev[2 * i + 1]);
    ms[p.cls[i]] += t;
    launches[p.cls[i]] += 1;
  }
  p.used = 0;
  if (e != hipSuccess) { c->hip_err = (int)e; return SF_EHIP; }
  return SF_OK;
}

const char *sf_strerror(sf_status s) {
  switch (s) {
    case SF_OK: return "ok";
    case SF_EINVAL: return "invalid argument";
    case SF_ECAPACITY: return "capacity exceeded (cache or workspace too small)";
    case SF_ESTATE: return "call order: weights not bound, or no verified block to commit";
    case SF_EHIP: return "HIP error";
    case SF_EUNSUPPORTED: return "shape not supported by the kernels";
  }
  return "unknown status";
}

int sf_last_hip_error(const sf_ctx *c) { return c ? c->hip_err : 0; }
const char *sf_version(void) { return "specformer-mi355x 0.1 (gfx950)"; }

}  // extern "C"

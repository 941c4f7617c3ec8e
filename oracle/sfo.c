/*
 * CPU oracle for the SpecFormer draft / verify / accept step (test infrastructure only;
 * see sfo.h).  Plain definitions in double precision: triple-loop linear maps, softmax
 * attention that materialises the whole score row, an explicit visibility predicate for
 * the mask, strict-greater argmax.  OpenMP only splits independent output rows; every
 * output element is summed in a fixed left-to-right order.
 */
#include "sfo.h"
#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ---------------------------------------------------------------------- */
/* bf16 rounding: double -> float (RNE) -> bf16 (RNE on the upper 16 bits) */
double sfo_round_bf16(double x) {
  float f = (float)x;
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7f800000u) == 0x7f800000u) return (double)f; /* inf / nan unchanged */
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7fffu + lsb;
  u &= 0xffff0000u;
  memcpy(&f, &u, 4);
  return (double)f;
}

static void round_buf(double *x, long n, int on) {
  if (!on) return;
  for (long i = 0; i < n; ++i) x[i] = sfo_round_bf16(x[i]);
}

/* y = RMSNorm(x; g) . w^T for the norm + linear pairs of the decoder layers.  Exact mode: the two
 * definitions one after the other.  bf16 emulation: the path under test stores neither the normalised
 * rows nor the gains separately -- the gain vector is folded into the weight's columns once (rounded
 * to bf16), the matrix product runs on the raw rows as a bf16 pipeline sees them (its bf16 copy of
 * the row: the residual stream itself is kept wider, see sfo.h), and the row factor
 * 1/sqrt(mean(x^2)+eps), taken from that same bf16 copy, commutes with the sum over the features and
 * is applied unrounded -- so the emulation rounds w*g and x, and nothing else. */
void sfo_norm_linear(const double *x, const float *g, const float *w, int M, int K, int N, double eps, int on,
                     double *y) {
  if (!on) {
    double *a = (double *)malloc(sizeof(double) * (size_t)M * K);
    sfo_rmsnorm(x, g, M, K, eps, a);
    sfo_linear(a, w, NULL, M, K, N, y);
    free(a);
    return;
  }
  float *wf = (float *)malloc(sizeof(float) * (size_t)N * K);
  double *xr = (double *)malloc(sizeof(double) * (size_t)M * K);
  for (long n = 0; n < N; ++n)
    for (int k = 0; k < K; ++k) wf[n * K + k] = (float)sfo_round_bf16((double)w[n * K + k] * (double)g[k]);
  for (long i = 0; i < (long)M * K; ++i) xr[i] = sfo_round_bf16(x[i]);
  sfo_linear(xr, wf, NULL, M, K, N, y);
  free(wf);
  for (int r = 0; r < M; ++r) {
    double ss = 0.0;
    for (int e = 0; e < K; ++e) ss += xr[(long)r * K + e] * xr[(long)r * K + e];
    double rinv = 1.0 / sqrt(ss / K + eps);
    for (int n = 0; n < N; ++n) y[(long)r * N + n] *= rinv;
  }
  free(xr);
}

void sfo_rmsnorm(const double *x, const float *g, int M, int d, double eps, double *y) {
  for (int r = 0; r < M; ++r) {
    const double *xr = x + (long)r * d;
    double ss = 0.0;
    for (int i = 0; i < d; ++i) ss += xr[i] * xr[i];
    double inv = 1.0 / sqrt(ss / d + eps);
    for (int i = 0; i < d; ++i) y[(long)r * d + i] = (double)g[i] * (xr[i] * inv);
  }
}

/* Grouped RMS Norm (Context Causal Attention, hook + down-sampler paragraph): RMS over the
 * last dimension, one gain vector per slice of the second-to-last dimension. x:[M][ng][d]. */
void sfo_group_rmsnorm(const double *x, const float *g, int M, int ng, int d, double eps, double *y) {
  for (int r = 0; r < M; ++r)
    for (int s = 0; s < ng; ++s)
      sfo_rmsnorm(x + ((long)r * ng + s) * d, g + (long)s * d, 1, d, eps, y + ((long)r * ng + s) * d);
}

/* y[m][n] = sum_k x[m][k] * w[n][k] (+ bias[n]) */
void sfo_linear(const double *x, const float *w, const float *bias, int M, int K, int N, double *y) {
#pragma omp parallel for schedule(static)
  for (long n = 0; n < N; ++n) {
    const float *wn = w + n * K;
    for (int m = 0; m < M; ++m) {
      const double *xm = x + (long)m * K;
      double acc = 0.0;
      for (int kk = 0; kk < K; ++kk) acc += xm[kk] * (double)wn[kk];
      if (bias) acc += (double)bias[n];
      y[(long)m * N + n] = acc;
    }
  }
}

/* Rotary position embedding, rotate-half pairing (i, i+hd/2), angle = pos * theta^(-2i/hd).
 * x:[M][H][hd], one position per row m. */
void sfo_rope(double *x, const int32_t *pos, int M, int H, int hd, double theta) {
  int half = hd / 2;
  for (int m = 0; m < M; ++m)
    for (int h = 0; h < H; ++h) {
      double *v = x + ((long)m * H + h) * hd;
      for (int i = 0; i < half; ++i) {
        double ang = (double)pos[m] * pow(theta, -2.0 * i / hd);
        double c = cos(ang), s = sin(ang);
        double a = v[i], b = v[i + half];
        v[i] = a * c - b * s;
        v[i + half] = b * c + a * s;
      }
    }
}

/* SwiGLU inner product: silu(gate) * up, silu(x) = x * sigmoid(x). */
void sfo_silu_mul(const double *gate, const double *up, long n, double *y) {
  for (long i = 0; i < n; ++i) y[i] = gate[i] / (1.0 + exp(-gate[i])) * up[i];
}

/* Which cache positions a block row may look at.  Positions [0,len) are the committed
 * prefix (always visible: causal along the context).  Positions [len, len+nq) are the
 * block itself: row i sees block key j when j<=i (CAUSAL: verify / "+Att Mask" ablation)
 * or always (BIDIR: bidirectional along the draft dimension).  Everything else is dead. */
static int visible(int len, int nq, int mode, int i, int pos) {
  if (pos < len) return 1;
  int j = pos - len;
  if (j >= nq) return 0;
  return mode == SFO_MASK_BIDIR ? 1 : (j <= i);
}

/* Softmax attention with grouped KV heads; scale 1/sqrt(hd); two-pass softmax. */
void sfo_attention(const double *q, const double *kc, const double *vc, const int32_t *len,
                   int B, int nq, int Hq, int Hkv, int hd, int cap, int mode, double *out) {
  int G = Hq / Hkv;
  double scale = 1.0 / sqrt((double)hd);
#pragma omp parallel for schedule(dynamic, 1) collapse(2)
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < Hq; ++h) {
      double *sc = (double *)malloc(sizeof(double) * (size_t)cap);
      int g = h / G;
      const double *K = kc + ((long)b * Hkv + g) * cap * hd;
      const double *Vv = vc + ((long)b * Hkv + g) * cap * hd;
      for (int i = 0; i < nq; ++i) {
        const double *qv = q + (((long)b * nq + i) * Hq + h) * hd;
        double *o = out + (((long)b * nq + i) * Hq + h) * hd;
        double mx = -INFINITY;
        for (int p = 0; p < cap; ++p) {
          if (!visible(len[b], nq, mode, i, p)) continue;
          double s = 0.0;
          for (int e = 0; e < hd; ++e) s += qv[e] * K[(long)p * hd + e];
          sc[p] = s * scale;
          if (sc[p] > mx) mx = sc[p];
        }
        double den = 0.0;
        for (int p = 0; p < cap; ++p)
          if (visible(len[b], nq, mode, i, p)) { sc[p] = exp(sc[p] - mx); den += sc[p]; }
        for (int e = 0; e < hd; ++e) o[e] = 0.0;
        for (int p = 0; p < cap; ++p)
          if (visible(len[b], nq, mode, i, p)) {
            double pw = sc[p] / den;
            for (int e = 0; e < hd; ++e) o[e] += pw * Vv[(long)p * hd + e];
          }
      }
      free(sc);
    }
}

/* Lowest index among the maxima; NaN never wins. */
int32_t sfo_argmax(const double *x, int n) {
  int32_t best = 0;
  double bv = -INFINITY;
  int have = 0;
  for (int i = 0; i < n; ++i) {
    if (x[i] != x[i]) continue;
    if (!have || x[i] > bv) { bv = x[i]; best = i; have = 1; }
  }
  return best;
}

/* ---------------------------------------------------------------------- */
static double *dalloc(long n) { return (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1)); }

/* Pre-norm residual unit (Eq. "Ops.Norm + I"): h += Ops(Norm(h)) for the attention half of a
 * decoder layer.  rows: M = B*nq, row (b,i) sits at position len_b + i.  Writes K,V of every
 * row into the cache at its position, then attends with the given mask. */
static void attn_half(const sfo_cfg *c, const float *norm_g, const float *wqkv, const float *wo,
                      double *h /*[M][d] in/out*/, int B, int nq, const int32_t *len, int cap,
                      double *kc, double *vc, int mode) {
  int d = c->d_model, Hq = c->n_q_heads, Hkv = c->n_kv_heads, hd = c->head_dim;
  int M = B * nq, NQ = Hq * hd, NKV = Hkv * hd, N = NQ + 2 * NKV, R = c->round_bf16;
  double *qkv = dalloc((long)M * N);
  double *q = dalloc((long)M * NQ), *kk = dalloc((long)M * NKV), *o = dalloc((long)M * NQ);
  double *proj = dalloc((long)M * d);
  int32_t *pos = (int32_t *)malloc(sizeof(int32_t) * (size_t)M);
  sfo_norm_linear(h, norm_g, wqkv, M, d, N, c->rms_eps, R, qkv);
  round_buf(qkv, (long)M * N, R);
  for (int b = 0; b < B; ++b)
    for (int i = 0; i < nq; ++i) pos[b * nq + i] = len[b] + i;
  for (int m = 0; m < M; ++m) {
    memcpy(q + (long)m * NQ, qkv + (long)m * N, sizeof(double) * NQ);
    memcpy(kk + (long)m * NKV, qkv + (long)m * N + NQ, sizeof(double) * NKV);
  }
  sfo_rope(q, pos, M, Hq, hd, c->rope_theta);
  sfo_rope(kk, pos, M, Hkv, hd, c->rope_theta);
  round_buf(q, (long)M * NQ, R);
  round_buf(kk, (long)M * NKV, R);
  for (int b = 0; b < B; ++b)
    for (int i = 0; i < nq; ++i) {
      int m = b * nq + i, p = len[b] + i;
      for (int g = 0; g < Hkv; ++g) {
        long dst = (((long)b * Hkv + g) * cap + p) * hd;
        memcpy(kc + dst, kk + (long)m * NKV + (long)g * hd, sizeof(double) * hd);
        memcpy(vc + dst, qkv + (long)m * N + NQ + NKV + (long)g * hd, sizeof(double) * hd);
      }
    }
  sfo_attention(q, kc, vc, len, B, nq, Hq, Hkv, hd, cap, mode, o);
  round_buf(o, (long)M * NQ, R);
  sfo_linear(o, wo, NULL, M, NQ, d, proj);
  for (long i = 0; i < (long)M * d; ++i) h[i] += proj[i]; /* the residual stream stays unrounded */
  free(qkv); free(q); free(kk); free(o); free(proj); free(pos);
}

/* h += W_down( silu(W_gate n) * (W_up n) ), n = RMS(h)   (SwiGLU feed-forward, pre-norm residual) */
static void ffn_half(const sfo_cfg *c, const float *norm_g, const float *wg, const float *wu,
                     const float *wd, double *h, int M) {
  int d = c->d_model, F = c->d_ffn, R = c->round_bf16;
  double *g = dalloc((long)M * F), *u = dalloc((long)M * F);
  double *proj = dalloc((long)M * d);
  sfo_norm_linear(h, norm_g, wg, M, d, F, c->rms_eps, R, g);
  sfo_norm_linear(h, norm_g, wu, M, d, F, c->rms_eps, R, u);
  sfo_silu_mul(g, u, (long)M * F, g);
  round_buf(g, (long)M * F, R);
  sfo_linear(g, wd, NULL, M, F, d, proj);
  for (long i = 0; i < (long)M * d; ++i) h[i] += proj[i]; /* the residual stream stays unrounded */
  free(g); free(u); free(proj);
}

/* Multi-token verification (Introduction, step 2): the unmodified target decoder runs over
 * the block [pending, draft_0..draft_{k-1}] of every sequence at positions len_b+i with a
 * causal mask, writes the block's K/V behind the committed prefix, records the four hooked
 * hidden states HS[0], HS[L/2], HS[L-1], HS[L] (General Notations; hook paragraph) and
 * returns the logits of every block row. */
int sfo_verify_step(const sfo_cfg *c, const sfo_target_weights *w, sfo_state *s, int k,
                    const int32_t *draft, double *logits) {
  int B = s->B, nq = k + 1, d = c->d_model, L = c->n_layers, V = c->vocab, M = B * nq;
  if (nq > s->q_max) return -1;
  for (int b = 0; b < B; ++b)
    if (s->kv_len[b] + nq > s->cap) return -1;
  double *h = dalloc((long)M * d), *a = dalloc((long)M * d);
  for (int b = 0; b < B; ++b)
    for (int i = 0; i < nq; ++i) {
      int tok = i == 0 ? s->pending[b] : draft[b * k + (i - 1)];
      if (tok < 0 || tok >= V) { free(h); free(a); return -1; }
      for (int e = 0; e < d; ++e) h[((long)b * nq + i) * d + e] = (double)w->embed[(long)tok * d + e];
    }
  int hook_layer[4] = {0, L / 2, L - 1, L};
  long cache_l = (long)B * c->n_kv_heads * s->cap * c->head_dim;
  for (int l = 0; l <= L; ++l) {
    for (int g = 0; g < 4; ++g)
      if (hook_layer[g] == l)
        for (int b = 0; b < B; ++b)
          for (int i = 0; i < nq; ++i) {
            double *dst = s->hooks + (((long)b * s->q_max + i) * 4 + g) * d;
            memcpy(dst, h + ((long)b * nq + i) * d, sizeof(double) * d);
            round_buf(dst, d, c->round_bf16); /* the hooked copies are stored in the model dtype */
          }
    if (l == L) break;
    attn_half(c, w->attn_norm[l], w->wqkv[l], w->wo[l], h, B, nq, s->kv_len, s->cap,
              s->tk + l * cache_l, s->tv + l * cache_l, SFO_MASK_CAUSAL);
    ffn_half(c, w->ffn_norm[l], w->w_gate[l], w->w_up[l], w->w_down[l], h, M);
  }
  sfo_rmsnorm(h, w->final_norm, M, d, c->rms_eps, a);
  round_buf(a, (long)M * d, c->round_bf16);
  sfo_linear(a, w->lm_head, NULL, M, d, V, logits);
  if (c->round_bf16) /* a bf16 pipeline keeps logits as fp32 accumulators */
    for (long i = 0; i < (long)M * V; ++i) logits[i] = (double)(float)logits[i];
  free(h); free(a);
  return 0;
}

/* Multi-token generation (Introduction, step 1) by the SpecFormer draft block.
 *  1. Grouped RMSNorm of the hooked states of the rows committed by the last accept,
 *     concatenated to 4d, down-sampled by W_D (first equation of Context Causal Attention).
 *  2. Those context rows enter the draft attention layer ("an additional (L+1)-th layer"
 *     with its own KV cache): K,V of RMS(X) at the rows' absolute positions.
 *  3. Positional FFN: the newest context row, RMS-normed, times W_P plus b_P gives k
 *     position-specific slot states (second equation).
 *  4. The slots run one pre-norm attention + SwiGLU layer (Draft Bi-directional Attention);
 *     a slot sees the whole cached context and, with BIDIR, all k slots.
 *  5. Output norm, the target's LM head, argmax.
 *
 * With SFO_DRAFT_TWO_STAGE in mask_mode the two attentions stay apart as the section writes them
 * (its first and third equations): the context attention is a residual unit of its own,
 * I_D = X + MSA(RMS(X)), causal over the cached context, and only its newest row feeds the
 * Positional FFN; the slot attention then sees the k slots only (positions 0..k-1, no cached
 * keys) and has its own norm, QKV and output weights. */
int sfo_draft_step(const sfo_cfg *c, const sfo_draft_weights *w, const float *lm_head, sfo_state *s,
                   int k, int mask_mode, int32_t *draft, double *draft_logits) {
  int B = s->B, d = c->d_model, Hq = c->n_q_heads, Hkv = c->n_kv_heads, hd = c->head_dim;
  int V = c->vocab, R = c->round_bf16, cap = s->cap;
  int NQ = Hq * hd, NKV = Hkv * hd, N = NQ + 2 * NKV;
  int two_stage = (mask_mode & SFO_DRAFT_TWO_STAGE) != 0;
  mask_mode &= ~SFO_DRAFT_TWO_STAGE;
  if (two_stage && (!w->sa_norm || !w->sa_wqkv || !w->sa_wo)) return -1;
  if (k < 1) return 0;
  for (int b = 0; b < B; ++b) {
    if (s->n_new[b] < 0 || s->n_new[b] > s->q_max || s->n_new[b] > s->kv_len[b]) return -1;
    if (s->kv_len[b] + k > cap) return -1;
  }
  double *xlast = dalloc((long)B * d);
  /* steps 1-2, sequence by sequence over its newly committed rows */
  for (int b = 0; b < B; ++b) {
    int n = s->n_new[b];
    if (n == 0) { /* nothing committed (a sequence idle during ragged prefill): zero state */
      for (int e = 0; e < d; ++e) xlast[(long)b * d + e] = 0.0;
      continue;
    }
    double *f = dalloc((long)n * 4 * d), *x = dalloc((long)n * d);
    double *qkv = dalloc((long)n * N), *kk = dalloc((long)n * NKV);
    int32_t *pos = (int32_t *)malloc(sizeof(int32_t) * (size_t)n);
    sfo_group_rmsnorm(s->hooks + (long)b * s->q_max * 4 * d, w->group_norm, n, 4, d, c->rms_eps, f);
    round_buf(f, (long)n * 4 * d, R);
    sfo_linear(f, w->w_ds, NULL, n, 4 * d, d, x);
    round_buf(x, (long)n * d, R);
    sfo_norm_linear(x, w->attn_norm, w->wqkv, n, d, N, c->rms_eps, R, qkv);
    round_buf(qkv, (long)n * N, R);
    for (int r = 0; r < n; ++r) {
      pos[r] = s->kv_len[b] - n + r;
      memcpy(kk + (long)r * NKV, qkv + (long)r * N + NQ, sizeof(double) * NKV);
    }
    sfo_rope(kk, pos, n, Hkv, hd, c->rope_theta);
    round_buf(kk, (long)n * NKV, R);
    for (int r = 0; r < n; ++r)
      for (int g = 0; g < Hkv; ++g) {
        long dst = (((long)b * Hkv + g) * cap + pos[r]) * hd;
        memcpy(s->dk + dst, kk + (long)r * NKV + (long)g * hd, sizeof(double) * hd);
        memcpy(s->dv + dst, qkv + (long)r * N + NQ + NKV + (long)g * hd, sizeof(double) * hd);
      }
    memcpy(xlast + (long)b * d, x + (long)(n - 1) * d, sizeof(double) * d);
    if (two_stage) {
      /* the context attention's own output at the newest row: its query against every cached
       * context key up to and including itself, projected and added to the row (residual) */
      double *q = dalloc(NQ), *o = dalloc(NQ), *proj = dalloc(d);
      int32_t last_pos = pos[n - 1], before = last_pos; /* keys before the row = its position */
      memcpy(q, qkv + (long)(n - 1) * N, sizeof(double) * NQ);
      sfo_rope(q, &last_pos, 1, Hq, hd, c->rope_theta);
      round_buf(q, NQ, R);
      sfo_attention(q, s->dk + (long)b * Hkv * cap * hd, s->dv + (long)b * Hkv * cap * hd, &before, 1, 1, Hq, Hkv,
                    hd, cap, SFO_MASK_CAUSAL, o);
      round_buf(o, NQ, R);
      sfo_linear(o, w->wo, NULL, 1, NQ, d, proj);
      for (int e = 0; e < d; ++e) xlast[(long)b * d + e] += proj[e]; /* residual stream: unrounded */
      free(q); free(o); free(proj);
    }
    free(f); free(x); free(qkv); free(kk); free(pos);
  }
  /* step 3 */
  int M = B * k;
  double *an = dalloc((long)B * d), *S = dalloc((long)M * d), *o = dalloc((long)M * d);
  sfo_rmsnorm(xlast, w->pos_norm, B, d, c->rms_eps, an);
  round_buf(an, (long)B * d, R);
  sfo_linear(an, w->w_pos, w->b_pos, B, d, k * d, S); /* row b = [slot0 | slot1 | ...] = rows b*k+s of S */
  /* S is the residual stream of the slot layer: unrounded */
  /* step 4 */
  if (two_stage) {
    /* the slots alone: an empty prefix in a k-slot cache of their own */
    int32_t *len0 = (int32_t *)calloc((size_t)B, sizeof(int32_t));
    double *kc2 = dalloc((long)B * Hkv * k * hd), *vc2 = dalloc((long)B * Hkv * k * hd);
    attn_half(c, w->sa_norm, w->sa_wqkv, w->sa_wo, S, B, k, len0, k, kc2, vc2, mask_mode);
    free(len0); free(kc2); free(vc2);
  } else {
    attn_half(c, w->attn_norm, w->wqkv, w->wo, S, B, k, s->kv_len, cap, s->dk, s->dv, mask_mode);
  }
  ffn_half(c, w->ffn_norm, w->w_gate, w->w_up, w->w_down, S, M);
  /* step 5 */
  sfo_rmsnorm(S, w->out_norm, M, d, c->rms_eps, o);
  round_buf(o, (long)M * d, R);
  double *lg = draft_logits ? draft_logits : dalloc((long)M * V);
  sfo_linear(o, lm_head, NULL, M, d, V, lg);
  if (R) for (long i = 0; i < (long)M * V; ++i) lg[i] = (double)(float)lg[i];
  for (int m = 0; m < M; ++m) draft[m] = sfo_argmax(lg + (long)m * V, V);
  if (!draft_logits) free(lg);
  free(xlast); free(an); free(S); free(o);
  return 0;
}

/* Multi-token acceptance (Introduction, step 3; lossless condition 1): a draft token is
 * accepted only while it equals the target's own greedy choice; the first disagreement
 * (or the row after the last slot) contributes the target's token as a bonus, so
 * 1 <= a_b <= k+1.  Written as the definition reads: slot i counts when it and every slot
 * before it agree with the target, i.e. n_b = sum_i prod_{j<=i} [draft_j == p_j].  The K/V of
 * the accepted rows already sit behind the prefix, so the commit is kv_len += a_b.  force_len
 * (prefill) commits a fixed number of rows instead; the pending token is then the target's
 * choice after the last committed row.  cu_new is the exclusive prefix sum of the a_b. */
int sfo_accept_commit(sfo_state *s, int k, int V, const int32_t *draft, const double *logits,
                      const int32_t *force_len, int32_t *accept_len, int32_t *out_tokens) {
  int B = s->B, nq = k + 1;
  if (force_len)
    for (int b = 0; b < B; ++b)
      if (force_len[b] < 0 || force_len[b] > nq) return -1;
  /* the target's greedy choice at every block row */
  int32_t *p = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * nq);
  for (long r = 0; r < (long)B * nq; ++r) p[r] = sfo_argmax(logits + r * V, V);
  /* accept lengths */
  for (int b = 0; b < B; ++b) {
    if (force_len) { accept_len[b] = force_len[b]; continue; }
    int agree_so_far = 1, n = 0;
    for (int i = 0; i < k; ++i) {
      agree_so_far *= (draft[b * k + i] == p[b * nq + i]);
      n += agree_so_far;
    }
    accept_len[b] = n + 1;
  }
  /* emitted tokens, commit */
  for (int b = 0; b < B; ++b) {
    int a = accept_len[b];
    for (int i = 0; i < nq; ++i) out_tokens[b * nq + i] = i < a ? p[b * nq + i] : -1;
    if (a > 0) s->pending[b] = p[b * nq + a - 1];
    s->kv_len[b] += a;
    s->n_new[b] = a;
  }
  s->cu_new[0] = 0;
  for (int b = 0; b < B; ++b) s->cu_new[b + 1] = s->cu_new[b] + accept_len[b];
  free(p);
  return 0;
}

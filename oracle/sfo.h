/*
 * SpecFormer draft / verify / accept step -- CPU ORACLE (test infrastructure).
 *
 * This is the slow, plain definition of what one speculative-decoding step of
 * arXiv 2511.20340 (SpecFormer) computes.  It exists only so that tests, the
 * smoke check and the bench's cpu_baseline leg can compare the GPU library
 * against it; the product never calls it.  It shares no source, header, table
 * or helper with the HIP path.
 *
 * Arithmetic: every floating-point operation is IEEE double.  Weights are
 * passed as float arrays (they hold bf16- or fp32-representable values),
 * activations, caches and logits as double arrays.  With cfg.round_bf16 != 0
 * the tensors that a bf16 pipeline stores to memory in bf16 are rounded to bf16
 * (round-to-nearest-even) at exactly those points; accumulation stays double.
 * The residual stream of the decoder layers (the running sum h that every
 * attention and feed-forward block adds to, and the slot states of the draft
 * block) is NOT among them: a bf16 pipeline keeps that one sum in a wider type,
 * so it is left unrounded here; what is read from it is rounded where it is
 * consumed (the hooked copies, the operand of a matrix product, a norm's output).
 *
 * Pins (tests/test_oracle_*.py): brute-force softmax attention on tiny shapes,
 * k=1 hybrid mask == causal decode, block-causal rows == successive decodes,
 * visibility perturbation tests, closed forms for RMSNorm / RoPE / SwiGLU,
 * all 2^k match patterns for acceptance, and the lossless invariant (Intro,
 * "lossless SD" conditions): speculative greedy output == plain greedy output.
 * Draft-token VALUES on random-init weights have no reference in the paper:
 * parity unpinned against the paper for those (structural pins only).
 *
 * Layouts (all row-major, last index fastest):
 *   linear weight   w[N][K]          y = x . w^T  (out-features major)
 *   K/V cache       [B][Hkv][cap][hd]   (per layer; target cache [L][B][Hkv][cap][hd])
 *   q / attn out    [B][n_q][Hq][hd]
 *   hooks           [B][q_max][4][d]    HS[0], HS[L/2], HS[L-1], HS[L]
 */
#ifndef SFO_H
#define SFO_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

enum { SFO_MASK_CAUSAL = 0, SFO_MASK_BIDIR = 1 };
/* OR-ed into the draft step's mask mode: the two attentions of the SpecFormer section kept apart
 * (Context Causal Attention with its own output, then a prefix-free Draft Bi-directional Attention
 * with a parameter set of its own) instead of one attention over cached context + slots. */
enum { SFO_DRAFT_TWO_STAGE = 16 };

typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  double rope_theta, rms_eps;
  int32_t round_bf16;
} sfo_cfg;

typedef struct {
  const float *embed;      /* [V][d] */
  const float *lm_head;    /* [V][d] */
  const float *final_norm; /* [d] */
  const float *const *attn_norm; /* L x [d] */
  const float *const *wqkv;      /* L x [(Hq+2Hkv)*hd][d]  rows: Q heads, K heads, V heads */
  const float *const *wo;        /* L x [d][Hq*hd] */
  const float *const *ffn_norm;  /* L x [d] */
  const float *const *w_gate;    /* L x [F][d] */
  const float *const *w_up;      /* L x [F][d] */
  const float *const *w_down;    /* L x [d][F] */
} sfo_target_weights;

typedef struct {
  const float *group_norm; /* [4][d]   Grouped RMSNorm gains           */
  const float *w_ds;       /* [d][4d]  down-sampler W_D                */
  const float *pos_norm;   /* [d]                                         */
  const float *w_pos;      /* [k_max*d][d]  positional FFN W_P, slot s = rows [s*d,(s+1)*d) */
  const float *b_pos;      /* [k_max*d]                                   */
  const float *attn_norm;  /* [d] */
  const float *wqkv;       /* [(Hq+2Hkv)*hd][d] */
  const float *wo;         /* [d][Hq*hd] */
  const float *ffn_norm;   /* [d] */
  const float *w_gate, *w_up; /* [F][d] */
  const float *w_down;     /* [d][F] */
  const float *out_norm;   /* [d] */
  /* two-stage wiring only (may be NULL otherwise): the slot attention's own parameters */
  const float *sa_norm;    /* [d] */
  const float *sa_wqkv;    /* [(Hq+2Hkv)*hd][d] */
  const float *sa_wo;      /* [d][Hq*hd] */
} sfo_draft_weights;

typedef struct {
  int32_t B, cap, q_max;
  double *tk, *tv;   /* [L][B][Hkv][cap][hd] */
  double *dk, *dv;   /* [B][Hkv][cap][hd]    */
  int32_t *kv_len;   /* [B] committed positions */
  int32_t *pending;  /* [B] token whose KV is not yet computed */
  double *hooks;     /* [B][q_max][4][d] */
  int32_t *n_new;    /* [B]   rows of hooks committed by the last accept */
  int32_t *cu_new;   /* [B+1] exclusive prefix sum of n_new */
} sfo_state;

/* ---- primitives ------------------------------------------------------- */
double sfo_round_bf16(double x);
void sfo_rmsnorm(const double *x, const float *g, int M, int d, double eps, double *y);
void sfo_group_rmsnorm(const double *x, const float *g, int M, int ng, int d, double eps, double *y);
void sfo_linear(const double *x, const float *w, const float *bias, int M, int K, int N, double *y);
/* RMSNorm(x; g) . w^T; round_bf16 != 0: as a bf16 pipeline that folds g into w computes it (sfo.c) */
void sfo_norm_linear(const double *x, const float *g, const float *w, int M, int K, int N, double eps,
                     int round_bf16, double *y);
void sfo_rope(double *x, const int32_t *pos, int M, int H, int hd, double theta);
void sfo_silu_mul(const double *gate, const double *up, long n, double *y);
void sfo_attention(const double *q, const double *kc, const double *vc, const int32_t *len,
                   int B, int nq, int Hq, int Hkv, int hd, int cap, int mode, double *out);
int32_t sfo_argmax(const double *x, int n);

/* ---- the three steps --------------------------------------------------- */
/* returns 0, or -1 on a capacity / argument error */
int sfo_verify_step(const sfo_cfg *c, const sfo_target_weights *w, sfo_state *s, int k,
                    const int32_t *draft /*[B][k]*/, double *logits /*[B][k+1][V]*/);
int sfo_draft_step(const sfo_cfg *c, const sfo_draft_weights *w, const float *lm_head, sfo_state *s,
                   int k, int mask_mode, int32_t *draft /*[B][k]*/, double *draft_logits /*[B][k][V] or NULL*/);
int sfo_accept_commit(sfo_state *s, int k, int V, const int32_t *draft, const double *logits,
                      const int32_t *force_len /*[B] or NULL*/, int32_t *accept_len /*[B]*/,
                      int32_t *out_tokens /*[B][k+1]*/);

#ifdef __cplusplus
}
#endif
#endif

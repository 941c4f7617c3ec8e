/*
 * specformer.h -- C ABI of the MI355X (gfx950) library for the batched draft-and-verify step of
 * SpecFormer-style lossless speculative decoding (arXiv 2511.20340).
 *
 * One decoding step is the three calls, in this order (Introduction, the three steps of SD):
 *     sf_draft_step    multi-token generation by the SpecFormer draft block (Methods, SpecFormer:
 *                      Context Causal Attention + Draft Bi-directional Attention)
 *     sf_verify_step   multi-token verification: the unmodified target decoder over the block
 *                      [pending, draft_0 .. draft_{k-1}] of every sequence
 *     sf_accept_commit multi-token acceptance: lossless greedy longest-prefix match + commit
 *
 * General rules
 *  - Every pointer marked "dev" is device memory of the current HIP device, owned by the caller
 *    (e.g. PyTorch tensors); the library borrows it and never frees it.  Pointers marked "host"
 *    are ordinary host memory.  The library allocates no device memory at all.
 *  - Every call enqueues work on `stream` (a hipStream_t passed as void*, NULL = default stream)
 *    and returns without synchronising; integer results (accept lengths, lengths, token ids) stay
 *    on the device.  Calls on one sf_ctx must be issued from one thread at a time.
 *  - Tensors are dense row-major, last index fastest.  "elem" is the model dtype: 2-byte bf16 for
 *    SF_BF16, 4-byte IEEE float for SF_F32.  Logits are always float.
 *  - Linear weights are logically [out_features][in_features] (y = x . W^T) and are passed PACKED:
 *    sf_pack_weight turns a row-major matrix into the MFMA-operand-ordered form the kernels stream
 *    (bf16; for SF_F32 packing is a plain copy).  The shapes in the weight structs are logical.
 *  - Errors: argument / state problems are reported synchronously by the return code and nothing
 *    is enqueued; a failed HIP launch gives SF_EHIP and sf_last_hip_error() holds the HIP code.
 *
 * K/V cache layout.  The caches are opaque byte buffers whose size sf_kv_cache_bytes() gives; the
 * kernels keep them in an MFMA-operand-ordered tiling (32 positions per tile) so that attention
 * streams them with fully coalesced 16-byte loads.  sf_kv_import / sf_kv_export convert from / to
 * the plain layout [B][Hkv][cap][head_dim].  `cap` must be a multiple of 32.
 */
#ifndef SPECFORMER_H
#define SPECFORMER_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

typedef struct sf_ctx sf_ctx;

typedef enum {
  SF_OK = 0,
  SF_EINVAL = 1,       /* null pointer, size out of range, inconsistent shapes, misaligned pointer */
  SF_ECAPACITY = 2,    /* host_len_upper + block does not fit the cache capacity / workspace      */
  SF_ESTATE = 3,       /* call order: a step before sf_bind; sf_accept_commit without a preceding
                          sf_verify_step of the same state and k (or a second commit of one block)   */
  SF_EHIP = 4,         /* a HIP call failed; see sf_last_hip_error                                 */
  SF_EUNSUPPORTED = 5  /* shape outside what the kernels cover (e.g. head_dim, rows per KV head)   */
} sf_status;

typedef enum { SF_BF16 = 0, SF_F32 = 1 } sf_dtype;

/* Block mask of the ragged attention (SpecFormer: unidirectional along the context, bidirectional
 * along the draft).  Cached prefix positions are always visible.  CAUSAL: block row i sees block
 * keys j <= i (verify pass; the "+Att Mask" ablation of the draft).  BIDIR: every block key. */
typedef enum { SF_MASK_CAUSAL = 0, SF_MASK_BIDIR = 1 } sf_mask_mode;
/* OR-ed into sf_draft_step's mask argument: run the draft block with its two attentions kept apart,
 * as the SpecFormer section writes them (first and third equation): the Context Causal Attention is
 * a residual unit of its own, I_D = X + MSA(RMS(X)), whose newest row feeds the Positional FFN, and
 * the Draft Bi-directional Attention then sees the k slots only (positions 0..k-1, no cached keys)
 * with the parameter set sa_* of sf_draft_weights.  Without the flag one attention layer serves both:
 * the slots attend to the cached context and to each other. */
enum { SF_DRAFT_TWO_STAGE = 16 };

/* A pre-norm decoder with grouped-query attention, rotary embedding (rotate-half pairing) and a
 * SwiGLU feed-forward.  The draft block uses the same widths with n_layers = 1. */
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rope_theta, rms_eps;
  int32_t dtype; /* sf_dtype */
} sf_model_cfg;

/* Target weights, all dev, elem dtype.  Per-layer arrays are HOST arrays of n_layers dev pointers
 * (copied by sf_bind). */
typedef struct {
  const void *embed;              /* [vocab][d]  row-major (gathered, not multiplied) */
  const void *lm_head;            /* [vocab][d]  packed                            */
  const void *final_norm;         /* [d]                                           */
  const void *const *attn_norm;   /* L x [d]                                       */
  const void *const *wqkv;        /* L x [(Hq+2Hkv)*hd][d]  rows: Q heads, K heads, V heads; bf16: attn_norm folded */
  const void *const *wo;          /* L x [d][Hq*hd]                                */
  const void *const *ffn_norm;    /* L x [d]                                       */
  const void *const *w_gate_up;   /* L x [2F][d]  rows [0,F) gate, [F,2F) up; packed with glu=1; bf16: ffn_norm folded */
  const void *const *w_down;      /* L x [d][F]                                    */
} sf_target_weights;

/* Draft-block weights (SpecFormer, Context Causal Attention and Draft Bi-directional Attention). */
typedef struct {
  const void *group_norm; /* [4][d]        Grouped RMSNorm gains, one vector per hooked layer     */
  const void *w_ds;       /* [d][4d]       down-sampler W_D, no bias                               */
  const void *pos_norm;   /* [d]                                                                   */
  const void *w_pos;      /* [k_max*d][d]  positional FFN W_P; slot s = rows [s*d,(s+1)*d)         */
  const void *b_pos;      /* [k_max*d]     positional FFN bias b_P                                 */
  const void *attn_norm;  /* [d]                                                                   */
  const void *wqkv;       /* [(Hq+2Hkv)*hd][d]  bf16: attn_norm folded                              */
  const void *wo;         /* [d][Hq*hd]                                                            */
  const void *ffn_norm;   /* [d]                                                                   */
  const void *w_gate_up;  /* [2F][d]  packed with glu = 1; bf16: ffn_norm folded                   */
  const void *w_down;     /* [d][F]                                                                */
  const void *out_norm;   /* [d]  the draft's own output norm; logits use the target's lm_head     */
  /* SF_DRAFT_TWO_STAGE only, NULL otherwise: the slot attention's own parameters                  */
  const void *sa_norm;    /* [d]                                                                   */
  const void *sa_wqkv;    /* [(Hq+2Hkv)*hd][d]  packed; bf16: sa_norm folded                        */
  const void *sa_wo;      /* [d][Hq*hd]         packed                                             */
} sf_draft_weights;

/* Decoding state, every buffer dev and caller-owned.  Per sequence b:
 *   kv_len[b]  positions whose K/V are committed in both caches' prefix
 *   pending[b] the newest emitted token: its id is known, its K/V not yet computed
 *   hooks      the four hooked hidden states HS[0], HS[L/2], HS[L-1], HS[L] of the last verify
 *              block's rows (SpecFormer, hook paragraph); rows [0, n_new[b]) are the committed ones
 *   n_new[b]   rows committed by the last sf_accept_commit; cu_new = exclusive prefix sum       */
typedef struct {
  int32_t B;          /* sequences                                                     */
  int32_t cap;        /* K/V capacity per sequence, multiple of 32                     */
  void *tk, *tv;      /* target caches, sf_kv_cache_bytes(ctx, 0, B, cap) bytes each   */
  void *dk, *dv;      /* draft caches,  sf_kv_cache_bytes(ctx, 1, B, cap) bytes each   */
  int32_t *kv_len;    /* [B]   in/out */
  int32_t *pending;   /* [B]   in/out */
  void *hooks;        /* [B][max_k+1][4][d] elem; written by verify, read by draft     */
  int32_t *n_new;     /* [B]   written by accept, read by draft                        */
  int32_t *cu_new;    /* [B+1] written by accept                                       */
  void *workspace;    /* >= sf_workspace_bytes(ctx, B, k, cap) bytes, 256-byte aligned,
                         zero-filled once by the caller after allocation            */
  size_t workspace_bytes;
} sf_state;

/* Context.  host.  max_B <= 4096, 0 <= max_k <= 127 (decoding uses a handful of slots; blocks of up to 128
 * rows serve chunked prefill: sf_verify_step over prompt tokens + sf_accept_commit with force_len).  target and draft must agree on every field
 * but n_layers (draft: 1).  SF_EUNSUPPORTED unless head_dim in {64,128} for SF_BF16 (any multiple
 * of 8 up to 256 for SF_F32), d_model % 8 == 0, d_ffn % 32 == 0, (n_q_heads * head_dim) % 32 == 0. */
sf_status sf_create(const sf_model_cfg *target, const sf_model_cfg *draft, int32_t max_B, int32_t max_k,
                    sf_ctx **out);
sf_status sf_destroy(sf_ctx *ctx);
/* Bytes of workspace the three step calls need for batch B, draft length k and cache capacity cap
 * (0 on bad args). */
size_t sf_workspace_bytes(const sf_ctx *ctx, int32_t B, int32_t k, int32_t cap);
/* Bytes of ONE of the K or V cache buffers: which = 0 target (all layers), 1 draft. */
size_t sf_kv_cache_bytes(const sf_ctx *ctx, int32_t which, int32_t B, int32_t cap);
/* Borrow the weight pointers until sf_destroy or the next sf_bind.  draft may be NULL when only
 * sf_verify_step / sf_accept_commit are used (plain autoregressive decoding, k = 0). */
sf_status sf_bind(sf_ctx *ctx, const sf_target_weights *target, const sf_draft_weights *draft);

/* Multi-token generation (SpecFormer, Eq. dec1 / dec2 / enc).  Reads hooks rows [0,n_new[b]) --
 * the rows at positions [kv_len[b]-n_new[b], kv_len[b]) -- and:
 *   Grouped RMSNorm -> W_D -> K,V of the draft attention layer appended to the draft cache at
 *   those positions (the "(L+1)-th layer" cache); the newest row -> RMS -> W_P + b_P -> k slot
 *   states; slots run one attention (+W_O, residual) and SwiGLU layer at positions kv_len[b]+s,
 *   seeing the whole cached context and the k slots under `mask`; output norm -> target LM head
 *   -> argmax.  draft_tokens: dev [B][k] out.  draft_logits: dev float [B][k][vocab] out, or NULL to
 *   keep them in the workspace.  Slot s predicts the token that follows the pending token by s+1
 *   places.  n_new[b] == 0 leaves that sequence's cache alone (its draft is then
 *   computed from a zero context row and is meaningless).  k == 0: no-op.
 * host_len_upper: any host-known upper bound of max_b kv_len[b]; it sizes the launch grids, so
 * no device read-back is needed.  SF_ECAPACITY when host_len_upper + k > cap. */
sf_status sf_draft_step(sf_ctx *ctx, const sf_state *st, int32_t k, int32_t mask, int32_t host_len_upper,
                        int32_t *draft_tokens, float *draft_logits, void *stream);

/* Multi-token verification.  Block row i of sequence b is token (i == 0 ? pending[b] :
 * draft_tokens[b][i-1]) at position kv_len[b]+i.  Runs the target decoder over the B*(k+1) rows
 * with the CAUSAL block mask, writes the rows' K/V into the target caches at their positions
 * (rows beyond what accept later commits stay dead), writes hooks[b][i][0..3] and
 * target_ids: dev [B][k+1] out, the target's greedy choice after every block row,
 *   target_ids[b][i] = argmax_v logits[b][i][v] (lowest index on ties, NaN never wins).  In SF_BF16 mode
 *   the arg-max is taken on the LM-head kernel's fp32 accumulators, tile by tile, so the logits need not
 *   be stored at all;
 * logits: dev float [B][k+1][vocab] out, or NULL when only target_ids are wanted.
 * draft_tokens: dev [B][k] (ignored when k == 0).  SF_ECAPACITY when host_len_upper + k + 1 > cap. */
sf_status sf_verify_step(sf_ctx *ctx, const sf_state *st, int32_t k, const int32_t *draft_tokens,
                         int32_t host_len_upper, float *logits, int32_t *target_ids, void *stream);

/* Multi-token acceptance (lossless SD, condition 1: only draft tokens equal to the target's own
 * output are accepted).  p = target_ids (dev [B][k+1], as sf_verify_step wrote them);
 * n_b = longest prefix with draft_tokens[b][i] == p[b][i]; a_b = n_b + 1 (the target's token at
 * the first mismatch, or after the last slot, is the bonus);  out_tokens[b][i] = p[b][i] for
 * i < a_b else -1;  accept_len[b] = a_b;  pending[b] = p[b][a_b-1];  kv_len[b] += a_b;
 * n_new[b] = a_b;  cu_new = exclusive scan of a.  The accepted rows' K/V already sit behind the
 * prefix, so nothing is moved.  force_len (dev [B] or NULL): commit exactly force_len[b] in
 * [0,k+1] rows instead of matching (prefill); with 0 the sequence's pending token is kept.
 * accept_len: dev [B] out; out_tokens: dev [B][k+1] out.
 * SF_ESTATE unless the last step call on this context that touched the caches was
 * sf_verify_step(ctx, st, k, ...) with this state (identified by st->kv_len) and this k: there is
 * nothing else to commit, and one block is committed once. */
sf_status sf_accept_commit(sf_ctx *ctx, const sf_state *st, int32_t k, const int32_t *draft_tokens,
                           const int32_t *target_ids, const int32_t *force_len, int32_t *accept_len,
                           int32_t *out_tokens, void *stream);

/* What the device saw that contradicts the host's promises.  The step calls size their launch grids from
 * host_len_upper and never read lengths back, so a kv_len[b] above that bound (the tail of that sequence is
 * then not attended to, and nothing reports it) or a block that does not fit the cache (lengths are clamped
 * to cap - block, older rows get overwritten) cannot fail synchronously.  Instead the first kernel of
 * sf_verify_step and sf_draft_step ORs SF_DEVERR_* bits into a sticky word inside the workspace, and this
 * call reads it back: it WAITS for `stream`, copies the word to *flags (host), clears it, and returns
 * SF_ECAPACITY when any bit was set, SF_OK otherwise.  A caller that replays a captured step with a pinned
 * bound must stop before kv_len can reach cap - (k+1), and may poll this call to be sure. */
enum { SF_DEVERR_LEN_ABOVE_BOUND = 1, SF_DEVERR_CACHE_FULL = 2 };
sf_status sf_check_state(const sf_ctx *ctx, const sf_state *st, int32_t *flags, void *stream);

/* Plain <-> tiled K/V layout, one layer: plain is dev elem [B][Hkv][cap][hd]; `tiled` points at
 * the layer's slab inside a cache buffer: (char*)cache + layer * sf_kv_cache_bytes(ctx,1,B,cap).
 * is_v selects the V tiling (K and V are tiled differently). */
sf_status sf_kv_import(const sf_ctx *ctx, const void *plain, void *tiled, int32_t is_v, int32_t B,
                       int32_t cap, void *stream);
sf_status sf_kv_export(const sf_ctx *ctx, const void *tiled, void *plain, int32_t is_v, int32_t B,
                       int32_t cap, void *stream);

/* ---- single operations of the path (what the steps are built from; used by tests / bench) ---- */

/* Hybrid-mask ragged attention (SpecFormer: MSA over the cached context + SA over the block).
 * q, out: dev elem [B][n_q][Hq][hd]; kc, vc: one layer's tiled caches with the block's own K/V
 * already stored at positions [kv_len[b], kv_len[b]+n_q); softmax(q.k/sqrt(hd)) in fp32.
 * Requires (Hq/Hkv)*n_q <= 1024 for SF_BF16 (row tiles of 32 rows; every row tile streams the keys once).  workspace as in sf_state (split-KV partials);
 * sf_attention_workspace_bytes gives its size. */
size_t sf_attention_workspace_bytes(const sf_ctx *ctx, int32_t B, int32_t n_q, int32_t host_len_upper);
sf_status sf_op_attention(const sf_ctx *ctx, const void *q, const void *kc, const void *vc,
                          const int32_t *kv_len, int32_t B, int32_t n_q, int32_t cap, int32_t mask,
                          int32_t host_len_upper, void *out, void *workspace, size_t workspace_bytes,
                          void *stream);

/* Weight packing.  w: dev elem row-major [N][K]; packed: dev, sf_packed_weight_bytes(ctx,N,K) bytes,
 * 16-byte aligned.  bf16: 32-row x 16-column units of 1 KiB in the lane order of the 32x32x16 MFMA,
 * rows and columns zero-padded to multiples of 32 / 16; a prefix of whole 32-row blocks of a packed
 * matrix is itself a packed matrix (used for the K/V rows of wqkv and the first k slots of W_P).
 * glu != 0 (only for w_gate_up = [gate; up], N = 2F, F % 32 == 0): gate and up rows are interleaved 16 by
 * 16 so that the linear kernel's epilogue can form silu(gate)*up in registers.
 * col_gain (dev elem [K], or NULL): SF_BF16 only -- the gain vector of the RMSNorm whose output this
 * layer consumes, folded into the weight's columns (w[n][k] * col_gain[k], rounded to bf16 once).  The
 * decoder's norm + linear pairs run as ONE kernel on such weights (see sf_op_rmsnorm_linear), which is
 * why, in SF_BF16 mode, the weight structs below want wqkv, w_gate_up and sa_wqkv packed with their
 * norm's gains; SF_F32 mode ignores col_gain and applies the gains in its norm kernel. */
size_t sf_packed_weight_bytes(const sf_ctx *ctx, int32_t N, int32_t K);
sf_status sf_pack_weight(const sf_ctx *ctx, const void *w, void *packed, int32_t N, int32_t K, int32_t glu,
                         const void *col_gain, void *stream);

/* y[M][N] = x[M][K] . w[N][K]^T (+ bias[N]) (+ residual[M][N]); x, bias, residual: dev elem; w: packed;
 * fp32 accumulation; y: dev elem, or float when out_f32 != 0.  K % 8 == 0, N % 8 == 0.
 * residual may alias y.  workspace (dev, 256-byte aligned, may be NULL): lets skinny shapes split the
 * K dimension over several workgroups; its first 64 KiB are ticket counters that must be ZERO before
 * the first use and are left zero by every launch (the same holds for sf_state.workspace, which the
 * caller zero-fills once after allocating it).  sf_linear_workspace_bytes gives the size to pass. */
size_t sf_linear_workspace_bytes(const sf_ctx *ctx, int32_t M);
sf_status sf_op_linear(const sf_ctx *ctx, const void *x, const void *w, const void *bias,
                       const void *residual, void *y, int32_t M, int32_t N, int32_t K, int32_t out_f32,
                       void *workspace, size_t workspace_bytes, void *stream);
/* Fused y = RMSNorm(x; gain, eps of the target configuration) . w^T, SF_BF16 only (SF_EUNSUPPORTED
 * otherwise): what the decoder layers run in place of a norm kernel followed by a linear kernel.  w must
 * have been packed with col_gain = gain; the kernel streams the raw x, accumulates every row's sum of
 * squares on the way, and scales its fp32 accumulators by the row factor 1/sqrt(mean(x^2)+eps), which
 * commutes with the K sum; the normalised activations never reach HBM.  x: dev bf16 [M][K]; other
 * arguments as sf_op_linear. */
sf_status sf_op_rmsnorm_linear(const sf_ctx *ctx, const void *x, const void *w, void *y, int32_t M, int32_t N,
                               int32_t K, int32_t out_f32, void *workspace, size_t workspace_bytes,
                               void *stream);
/* SwiGLU input half: act[M][F] = silu(x . Wg^T) * (x . Wu^T); w_gate_up packed with glu = 1 (SF_BF16:
 * one kernel, gate/up never leave registers; SF_F32: workspace must hold M*2F floats). act: dev elem. */
sf_status sf_op_linear_swiglu(const sf_ctx *ctx, const void *x, const void *w_gate_up, void *act, int32_t M,
                              int32_t F, int32_t K, void *workspace, size_t workspace_bytes, void *stream);
/* The LM head with its arg-max, as the step calls run it: ids[m] = argmax_n (x . w^T)[m][n] (lowest index
 * on ties, NaN never wins).  SF_BF16: one linear launch whose epilogue reduces every column tile of its
 * fp32 accumulators to (largest value, its column), then one small launch that finishes each row; logits
 * (dev float [M][N], or NULL) are stored only when given.  SF_F32: logits are materialised (in `logits`, or
 * in the workspace) and scanned.  x: dev elem [M][K]; w: packed [N][K]; ids: dev [M];
 * workspace: dev, 256-byte aligned, sf_linear_argmax_workspace_bytes. */
size_t sf_linear_argmax_workspace_bytes(const sf_ctx *ctx, int32_t M, int32_t N);
sf_status sf_op_linear_argmax(const sf_ctx *ctx, const void *x, const void *w, int32_t M, int32_t N, int32_t K,
                              int32_t *ids, float *logits, void *workspace, size_t workspace_bytes, void *stream);

/* RMS normalisation over the last dimension with `n_gain` gain vectors: row r uses gain[r % n_gain]
 * (n_gain = 4 over rows [.,4,d] is the Grouped RMSNorm of the down-sampler).  x, y: dev elem [M][d];
 * gain: dev elem [n_gain][d].  Statistics in fp32. */
sf_status sf_op_rmsnorm(const sf_ctx *ctx, const void *x, const void *gain, void *y, int32_t M, int32_t d,
                        int32_t n_gain, void *stream);

/* Rotary embedding of q and k (rotate-half pairing, angle = pos * theta^(-2i/hd)) and append of k, v
 * to one layer's tiled caches.  qkv: dev elem [B*n_q][(Hq+2Hkv)*hd]; row (b,i) has position
 * kv_len[b]+i.  q_out: dev elem [B*n_q][Hq*hd]. */
sf_status sf_op_rope_kv_append(const sf_ctx *ctx, const void *qkv, const int32_t *kv_len, int32_t B,
                               int32_t n_q, int32_t cap, void *q_out, void *kc, void *vc, void *workspace,
                               size_t workspace_bytes, void *stream);

/* The two operations above in one kernel, as the target's layers run them (SF_BF16 only, else
 * SF_EUNSUPPORTED): rotary embedding of the block's q and k rows, append of k, v at positions
 * [kv_len[b], kv_len[b]+n_q) of one layer's tiled caches (kc, vc: dev, written), and the hybrid-mask
 * attention of the rotated rows over the cached context plus the block.  qkv: dev elem
 * [B*n_q][(Hq+2Hkv)*hd] (read only); out: dev elem [B][n_q][Hq][hd].  workspace: dev, 256-byte
 * aligned, sf_rope_attention_workspace_bytes (cos/sin table, length ranking, split-KV partials); host_len_upper
 * >= max kv_len, host_len_upper + n_q <= cap (SF_ECAPACITY otherwise). */
size_t sf_rope_attention_workspace_bytes(const sf_ctx *ctx, int32_t B, int32_t n_q, int32_t host_len_upper);
sf_status sf_op_rope_attention(const sf_ctx *ctx, const void *qkv, const int32_t *kv_len, int32_t B,
                               int32_t n_q, int32_t cap, int32_t mask, int32_t host_len_upper, void *kc,
                               void *vc, void *out, void *workspace, size_t workspace_bytes, void *stream);

/* act[M][F] = silu(gu[M][0:F]) * gu[M][F:2F];  gu: dev float [M][2F]; act: dev elem. */
sf_status sf_op_silu_mul(const sf_ctx *ctx, const float *gu, void *act, int32_t M, int32_t F, void *stream);

/* ids[r] = argmax_v logits[r][v] over dev float [M][V] (lowest index on ties); ids: dev [M].
 * workspace >= sf_argmax_workspace_bytes(M). */
size_t sf_argmax_workspace_bytes(int32_t M);
sf_status sf_op_argmax(const sf_ctx *ctx, const float *logits, int32_t M, int32_t V, int32_t *ids,
                       void *workspace, size_t workspace_bytes, void *stream);

/* sf_op_argmax for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments without the workspace, same
 * result.  The partials live in a static device array of the library (512 KiB, held on every GPU the library
 * runs on until the process ends), sized for M <= SF_ARGMAX_NOALLOC_MAX_ROWS rows: SF_ECAPACITY beyond that.
 * The call allocates nothing and frees nothing.  All calls on one GPU share that array: calls that overlap
 * in time on one GPU (different streams, or different threads) race -- serialise them. */
#define SF_ARGMAX_NOALLOC_MAX_ROWS 4096
sf_status sf_op_argmax_noalloc(const sf_ctx *ctx, const float *logits, int32_t M, int32_t V, int32_t *ids,
                               void *stream);

/* The acceptance rule alone, on explicit state arrays (what sf_accept_commit launches after its call-order
 * check): all pointers dev; kv_len, pending: [B] in/out; n_new: [B] out; cu_new: [B+1] out. */
sf_status sf_op_accept(const sf_ctx *ctx, int32_t B, int32_t k, const int32_t *draft_tokens,
                       const int32_t *target_ids, const int32_t *force_len, int32_t *accept_len,
                       int32_t *out_tokens, int32_t *kv_len, int32_t *pending, int32_t *n_new, int32_t *cu_new,
                       void *stream);

const char *sf_strerror(sf_status s);
/* HIP error code (hipError_t) of the last SF_EHIP on this context, 0 if none. host. */
int sf_last_hip_error(const sf_ctx *ctx);
/* Library version, and the code-object architecture it was built for ("gfx950"). host. */
const char *sf_version(void);

#ifdef __cplusplus
}
#endif
#endif

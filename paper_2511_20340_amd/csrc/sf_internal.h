// Internal declarations shared by the HIP translation units of libspecformer (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/specformer.h"

namespace sf {

typedef uint16_t bf16_t;  // raw bf16 bits in memory
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
// round-to-nearest-even (gfx950 converts in hardware: v_cvt_pk_bf16_f32); NaN stays NaN
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16_t f2bf(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
__device__ __forceinline__ uint32_t pack2bf(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// One RoPE pair (x[e], x[e + hd/2]) turned by the angle whose (cos, sin) is cs.  Explicit fused
// multiply-adds: every kernel that rotates must round the same way.
__device__ __forceinline__ void rope_pair(float a, float b, float2 cs, float &lo, float &hi) {
  lo = __builtin_fmaf(a, cs.x, -(b * cs.y));
  hi = __builtin_fmaf(b, cs.x, a * cs.y);
}

template <typename T> struct Elem;
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float ld(const bf16_t *p) { return bf2f(*p); }
  static __device__ __forceinline__ void st(bf16_t *p, float v) { *p = f2bf(v); }
};
template <> struct Elem<float> {
  static __device__ __forceinline__ float ld(const float *p) { return *p; }
  static __device__ __forceinline__ void st(float *p, float v) { *p = v; }
};

// ---------------------------------------------------------------------------------------------
// Tiled K/V cache (bf16).  A tile holds TK = 32 consecutive positions of one (sequence, kv head)
// as one contiguous blob of 32*HD elements, ordered so that a wavefront's MFMA operand loads are
// `blob[i*64 + lane]` in 16-byte units.
//
// 32x32x16 MFMA accumulator layout: lane l, register v holds row c_row(v, l/32), column l%32.
__host__ __device__ constexpr int c_row(int v, int h) { return 8 * (v >> 2) + 4 * h + (v & 3); }

constexpr int TK = 32;

// K tile: element (key a in [0,32), feature c) -> element offset inside the blob.
// 16-byte unit index = (c/8)*32 + a : k-step s of the QK^T product reads units [s*64, s*64+64).
__host__ __device__ constexpr int k_tile_off(int a, int c) { return ((c >> 3) * 32 + a) * 8 + (c & 7); }

// V tile: element (key a, feature c) -> element offset.  The P.V product runs as O^T = V^T.P^T with
// the keys as the MFMA reduction dimension, 16 keys per MFMA (u = a/16).  Inside a 16-key group,
// lane half h and operand element e hold key 16u + 8*(e/4) + 4h + e%4 (the accumulator layout of the
// preceding S^T = K.Q^T product, so P needs no shuffle).  16-byte unit = ((u*NT + c/32)*2 + h)*32 + c%32.
__host__ __device__ constexpr int v_tile_off(int a, int c, int hd) {
  int u = a >> 4, a16 = a & 15;
  int h = (a16 >> 2) & 1, e = ((a16 >> 3) << 2) | (a16 & 3);
  return ((((u * (hd >> 5) + (c >> 5)) * 2 + h) * 32) + (c & 31)) * 8 + e;
}

// fp32 mode keeps the plain layout [B][Hkv][cap][hd].

// ---- kernel launchers (defined in the .hip files) ---------------------------------------------
struct AttnArgs {
  const void *q;
  // bf16 only, optional: the raw QKV projection rows [q | k | v] and the cos/sin table of their
  // positions.  When set, q is ignored and the kernel rotates Q and K and appends K, V itself.
  const void *qkv;
  const float2 *table;
  const int32_t *order;  // bf16 only, optional [B]: a permutation of the sequences, workgroups of order[0] start first
  const void *kc, *vc;
  const int32_t *kv_len;
  void *out;
  float *part_o;   // [B][Hkv][n_chunks][64][HD]
  float *part_ml;  // [B][Hkv][n_chunks][64][2]
  int B, n_q, Hq, Hkv, hd, cap, mode;
  int chunk_tiles;  // tiles of 32 keys per workgroup chunk
  int n_chunks;     // grid.x
};
int attn_chunk_tiles(int groups, int keys_upper);  // groups = B * Hkv * row tiles
size_t attn_workspace_bytes(int B, int Hkv, int hd, int G, int n_q, int len_upper);
hipError_t launch_attention_bf16(const AttnArgs &a, hipStream_t s);
// merges the split-KV partials (only needed when a.n_chunks > 1)
hipError_t launch_attention_combine(const AttnArgs &a, hipStream_t s);
hipError_t launch_attention_f32(const AttnArgs &a, hipStream_t s);

struct GemmArgs {
  const void *x, *w, *bias, *residual;
  void *y;
  int M, N, K;
  int out_f32;
  int glu;          // bf16 only: w packed with glu=1, y = silu(gate) * up as elem [M][N/2]
  void *ws;         // split-K tickets (first GEMM_TICKET_BYTES, zero between launches) + partial tiles
  size_t ws_bytes;  // 0: no split-K
  // bf16 kernel choice; 0 = heuristic.  plan_M: the row count the split factor is chosen for (the
  // largest M this weight is used with), so that every M gets the same K partition; 0 = M.
  int tile = 0, split = 0, plan_M = 0;
  // bf16 only: y = RMSNorm(x) . w^T with x the un-normalised input and the norm's gain vector already
  // folded into w's columns at pack time; the kernel supplies the row factor 1/sqrt(mean(x^2)+eps)
  int fused_norm = 0;
  float norm_eps = 0.f;
  // bf16 only, the residual stream: residual (and with out_f32 the output) is float [M][N]; y2, when
  // set, receives a bf16 copy of the output (what the next norm + linear pair multiplies with)
  int res_f32 = 0;
  void *y2 = nullptr;
  // bf16 only: the output rows are block rows (b, i) = (row / hook_q, row % hook_q); their bf16 copy also
  // goes to hooks[b][i][g][:] ([B][hook_qmax][4][N]) for every group g in hook_mask
  void *hooks = nullptr;
  int hook_mask = 0, hook_q = 1, hook_qmax = 1;
  // bf16 only: per output row and column tile the largest value and its column (lowest on ties, NaN never
  // wins, (-inf, INT_MAX) when the tile holds no comparable value): am_val/am_idx [M][am_stride], entry
  // [row][column tile]; y may then be NULL (logits not materialised).  Forces split 1.
  float *am_val = nullptr;
  int32_t *am_idx = nullptr;
  int am_stride = 0;
  int *am_parts_out = nullptr;  // host: receives the number of column tiles the launch wrote partials for
};
// column tiles the arg-max partials of an N-column layer can have at most (narrowest tile: 128 columns)
inline int gemm_argmax_parts(int N) { return (N + 127) / 128; }
struct GemmConfig {
  int tile, split;
};
constexpr size_t GEMM_TICKET_BYTES = 64 * 1024;
constexpr size_t GEMM_PARTIAL_BYTES = 96u * 1024 * 1024;
constexpr size_t GEMM_SSQ_BYTES = 1024 * 1024;  // split-K: per-split row sums of squares of the fused norm
size_t gemm_workspace_bytes(int M_max);
hipError_t gemm_prepare_device();
int gemm_num_tiles();
int gemm_tile_rows(int tile);
GemmConfig gemm_heuristic(int M, int plan_M, int N, int K, size_t ws_bytes);
bool gemm_config_fits(const GemmConfig &c, const GemmArgs &a);  // split-K partials fit a.ws?
// bf16 weights are consumed in MFMA-operand-packed form (see gemm.hip); fp32 weights stay row-major
size_t packed_weight_bytes(int N, int K, int dtype);
hipError_t launch_pack_weight(const void *w, void *packed, int N, int K, int glu, const void *col_gain, int dtype,
                              hipStream_t s);
hipError_t launch_gemm_bf16(const GemmArgs &a, hipStream_t s);
hipError_t launch_gemm_f32(const GemmArgs &a, hipStream_t s);

// row-mapped RMSNorm: output row r reads input row in_row(r), see elementwise.hip
struct NormArgs {
  const void *x, *gain;
  void *y;
  int M, d, n_gain;
  float eps;
  // input row mapping: 0 identity; 1 hooks rows: r=(b*q+i)*4+g -> ((b*q_max+i)*4+g);
  // 2 newest committed row of x[B*q][d]: r=b -> b*q + n_new[b]-1 (zero row when n_new[b]==0)
  // 3 identity, but a zero row when n_new[r]==0
  int map;
  int q, q_max;
  const int32_t *n_new;
  int x_f32 = 0;  // x is float whatever the model dtype (rows of the residual stream)
};
hipError_t launch_rmsnorm(const NormArgs &a, int dtype, hipStream_t s);
hipError_t launch_calib_copy(const void *src, void *dst, size_t bytes, hipStream_t s);

struct RopeArgs {
  const void *qkv;  // [M][(Hq+2Hkv)*hd] or, kv_only, [M][2*Hkv*hd]
  void *q_out;      // [M][Hq*hd] (ignored when kv_only)
  void *kc, *vc;
  const int32_t *kv_len;
  const int32_t *n_new;  // pos_mode 1
  float2 *table;         // [M][hd/2] cos,sin scratch
  float2 *table2 = nullptr;  // optional second table of the same launch: n_q2 rows per sequence at kv_len[b] + r
  int n_q2 = 0;
  int32_t *order;        // optional [B]: filled with the sequences in descending kv_len order
  // optional: a sticky word that collects SF_DEVERR_* bits when a device-side length contradicts what the
  // host promised (len_upper >= every kv_len, kv_len + n_q <= cap)
  int32_t *dev_err = nullptr;
  int len_upper = 0;
  int B, n_q, Hq, Hkv, hd, cap;
  int kv_only;   // rows carry only K,V
  int pos_mode;  // 0: pos = kv_len[b]+i, all rows valid; 1: pos = kv_len[b]-n_new[b]+i, valid iff i<n_new[b]
  float theta;
};
// fills a.table for the rows' positions; launch_rope_kv then rotates and appends using it
hipError_t launch_rope_table(const RopeArgs &a, hipStream_t s);
hipError_t launch_rope_kv(const RopeArgs &a, int dtype, hipStream_t s);

hipError_t launch_silu_mul(const float *gu, void *act, int M, int F, int dtype, hipStream_t s);
// h (float) = embedding rows of the block tokens; hb (bf16 mode, may be null) their bf16 copy; hooks
// groups in hook_mask receive the rows too
hipError_t launch_embed(const void *embed, const int32_t *pending, const int32_t *draft, float *h, void *hb,
                        void *hooks, int hook_mask, int B, int k, int q_max, int d, int vocab, int dtype,
                        hipStream_t s);
// out[b] = x[b*q + n_new[b]-1] (zero row when n_new[b]==0); len_m1[b] = max(kv_len[b]-1, 0)
hipError_t launch_gather_last(const void *x, void *out, const int32_t *n_new, const int32_t *kv_len, int32_t *len_m1,
                              int B, int q, int d, int dtype, hipStream_t s);
hipError_t launch_hook_copy(const float *h, void *hooks, int B, int q, int q_max, int d, int group, int dtype,
                            hipStream_t s);
hipError_t launch_kv_convert(const void *src, void *dst, int is_v, int to_tiled, int B, int Hkv, int cap, int hd,
                             int dtype, hipStream_t s);

constexpr int ARGMAX_SEGS = 16;
constexpr int ARGMAX_NOALLOC_MAX_ROWS = 4096;  // rows the allocation-free arg-max entry point accepts
// arg-max over stored logits with its partials in a static device array (no workspace argument)
hipError_t launch_argmax_noalloc(const float *logits, int M, int V, int32_t *ids, hipStream_t s);
hipError_t launch_argmax_partial(const float *logits, int M, int V, float *pmax, int32_t *pidx, hipStream_t s);
// ids[row] = column of the best of the row's n_part partials pmax/pidx[row * stride + 0..n_part)
hipError_t launch_argmax_final(const float *pmax, const int32_t *pidx, int M, int n_part, int stride, int32_t *ids,
                               hipStream_t s);
struct AcceptArgs {
  const int32_t *target_ids;  // [B][k+1] the target's greedy choice at every block row
  const int32_t *draft, *force_len;
  int32_t *accept_len, *out_tokens, *kv_len, *pending, *n_new, *cu_new;
  int B, k;
};
hipError_t launch_accept(const AcceptArgs &a, hipStream_t s);

}  // namespace sf

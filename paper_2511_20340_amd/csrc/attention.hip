// Hybrid-mask ragged-prefix attention for gfx950 (SpecFormer: causal along the cached context,
// bidirectional -- or causal -- inside the block of n_q new rows).
//
// bf16 path.  One workgroup (4 wavefronts) owns one chunk of `chunk_tiles` 32-key tiles of one
// (sequence, kv head, 32-row group).  All G*n_q query rows that share the kv head form the N side
// of a 32x32x16 MFMA, so every K/V byte is read from HBM once for the whole GQA group and block.
// Per tile a wave computes   S^T = K . Q^T   (keys on the MFMA M side, loaded straight from the
// tiled cache into operand registers: `blob[i*64+lane]`, 1 KiB contiguous per instruction),
// an online softmax in fp32 registers with the mask built from (key position, row's block
// index), and   O^T += V^T . P^T   whose P operand is exactly the S^T accumulator layout.
// The 4 waves interleave tiles; they merge (m, l, O) through LDS at the end.  A sequence that
// spans several chunks leaves fp32 partials that a small combine kernel merges.
#include "sf_internal.h"

namespace sf {

namespace {

constexpr int WAVES = 4;
constexpr float NEG_INF = -__builtin_huge_valf();

//
// FUSE = 1 (the target's layers): Q is the raw output of the QKV projection, rows [q | k | v].  The
// workgroup first rotates the block's new K rows that fall into its own tiles (RoPE, cos/sin from
// `table`) and appends them and the V rows to the cache, then rotates its Q rows in registers (a
// rotation pair (e, e + HD/2) sits in the same lane, k-steps s and s + KS/2).  The appended rows are
// read back by the same workgroup after a barrier; workgroups that share (sequence, kv head) own
// disjoint tiles, or (several row groups) write identical values.
template <int HD, int FUSE>
__global__ __launch_bounds__(256, HD == 64 ? 4 : 2) void attn_bf16_kernel(
    const bf16_t *__restrict__ Q, const uint4 *Kc, const uint4 *Vc,
    const int32_t *__restrict__ kv_len, bf16_t *__restrict__ O, float *__restrict__ part_o,
    float *__restrict__ part_ml, int n_q, int Hq, int Hkv, int cap, int mode, int chunk_tiles,
    int n_chunks, int n_rt, float scale_log2e, const float2 *__restrict__ table,
    const int32_t *__restrict__ order) {
  constexpr int KS = HD / 16;       // k-steps of the QK^T product
  constexpr int NT = HD / 32;       // 32-column tiles of the output
  constexpr int TILE_U4 = HD * 4;   // 16-byte units per 32-key tile (32*HD*2/16)
  constexpr int LROW = HD + 4;      // padded LDS row (floats)
  extern __shared__ float lds[];    // [WAVES][32][LROW] + [WAVES][32][2]

  const int b = order ? order[blockIdx.z] : blockIdx.z;  // longest sequences first, if the caller ranked them
  const int g = blockIdx.y / n_rt, rt = blockIdx.y % n_rt;
  const int chunk = blockIdx.x;
  const int G = Hq / Hkv;
  const int R = G * n_q;
  const int len = min(kv_len[b], cap - n_q);  // never read past the slab, whatever the caller stored
  const int total = len + n_q;
  const int n_tiles = (total + TK - 1) / TK;
  const int t_begin = chunk * chunk_tiles;
  if (t_begin >= n_tiles) return;  // whole workgroup leaves before any barrier
  const int t_end = min(t_begin + chunk_tiles, n_tiles);
  const int seq_chunks = (n_tiles + chunk_tiles - 1) / chunk_tiles;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, h = lane >> 5;
  const int r = rt * 32 + n;            // query row inside the (kv head) group
  const bool row_ok = r < R;
  const int qi = row_ok ? r / G : 0;    // block index of the row
  const int qh = g * G + (row_ok ? r % G : 0);

  const size_t seq_base = ((size_t)b * Hkv + g) * (size_t)(cap / TK) * TILE_U4;
  const uint4 *Kb = Kc + seq_base + lane;
  const uint4 *Vb = Vc + seq_base + lane;
  int t = t_begin + wave;
  uint4 kf[KS];
  // first K tile of this wave: before the append below when the tile lies wholly in the prefix
  const bool early = !FUSE || (t + 1) * TK <= len;
  if (t < t_end && early) {
#pragma unroll
    for (int s = 0; s < KS; ++s) kf[s] = Kb[(size_t)t * TILE_U4 + s * 64];
  }

  // Q^T operand: lane (n, h), k-step s holds features [(2s+h)*8, +8) of row r
  bf16x8 qf[KS];
  if (FUSE) {
    constexpr int HALF = HD / 2;
    const size_t row_stride = (size_t)(Hq + 2 * Hkv) * HD;
    // the block's new rows that live in this workgroup's tiles: rotate K, append K and V
    bf16_t *Vw = reinterpret_cast<bf16_t *>(const_cast<uint4 *>(Vc)) + seq_base * 8;
    // K: one thread per (new row, 8 features of the lower half): both halves of the rotation pairs leave as
    // whole 16-byte units
    for (int x = tid; x < n_q * (HALF / 8); x += 256) {
      const int j = x / (HALF / 8), c8 = x % (HALF / 8);
      const int pos = len + j, tile = pos / TK, a_in = pos % TK;
      if (tile < t_begin || tile >= t_end) continue;
      const bf16_t *src = Q + ((size_t)b * n_q + j) * row_stride + (size_t)(Hq + g) * HD;
      const uint4 lo4 = *reinterpret_cast<const uint4 *>(src + c8 * 8);
      const uint4 hi4 = *reinterpret_cast<const uint4 *>(src + HALF + c8 * 8);
      const unsigned lo[4] = {lo4.x, lo4.y, lo4.z, lo4.w}, hi[4] = {hi4.x, hi4.y, hi4.z, hi4.w};
      const float2 *cs = table + ((size_t)b * n_q + j) * HALF + c8 * 8;
      unsigned k0[4], k1[4];
#pragma unroll
      for (int w = 0; w < 4; ++w) {  // two features per 32-bit word
        float a0, a1, b0, b1;
        rope_pair(bf2f((bf16_t)(lo[w] & 0xffffu)), bf2f((bf16_t)(hi[w] & 0xffffu)), cs[2 * w], a0, a1);
        rope_pair(bf2f((bf16_t)(lo[w] >> 16)), bf2f((bf16_t)(hi[w] >> 16)), cs[2 * w + 1], b0, b1);
        k0[w] = (unsigned)f2bf(a0) | ((unsigned)f2bf(b0) << 16);
        k1[w] = (unsigned)f2bf(a1) | ((unsigned)f2bf(b1) << 16);
      }
      const uint4 o0 = make_uint4(k0[0], k0[1], k0[2], k0[3]), o1 = make_uint4(k1[0], k1[1], k1[2], k1[3]);
      uint4 *Ku = const_cast<uint4 *>(Kc) + seq_base + (size_t)tile * TILE_U4;
      Ku[c8 * 32 + a_in] = o0;
      Ku[(HALF / 8 + c8) * 32 + a_in] = o1;
    }
    // V: one thread per (feature, aligned group of four positions); a group's keys are 8 consecutive bytes of
    // one 16-byte unit, written at once when all four are new
    const int quad0 = len >> 2, n_quads = ((len + n_q - 1) >> 2) - quad0 + 1;
    for (int x = tid; x < n_quads * HD; x += 256) {
      const int quad = quad0 + x / HD, c = x % HD;
      const int p0 = quad * 4, tile = p0 / TK;
      if (tile < t_begin || tile >= t_end) continue;
      const size_t base = (size_t)tile * (TK * HD);
      const bf16_t *vsrc = Q + (size_t)b * n_q * row_stride + (size_t)(Hq + Hkv + g) * HD + c;
      const int j0 = p0 - len;  // block row of the group's first position (negative: still prefix)
      if (j0 >= 0 && j0 + 4 <= n_q) {
        ushort4 v;
        v.x = vsrc[(size_t)j0 * row_stride];
        v.y = vsrc[(size_t)(j0 + 1) * row_stride];
        v.z = vsrc[(size_t)(j0 + 2) * row_stride];
        v.w = vsrc[(size_t)(j0 + 3) * row_stride];
        *reinterpret_cast<ushort4 *>(Vw + base + v_tile_off(p0 % TK, c, HD)) = v;
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int j = j0 + i;
          if (j >= 0 && j < n_q) Vw[base + v_tile_off((p0 + i) % TK, c, HD)] = vsrc[(size_t)j * row_stride];
        }
      }
    }
    // this lane's Q features: a rotation pair sits in k-steps s and s + KS/2 of the same lane
    const uint4 *qp = reinterpret_cast<const uint4 *>(Q + ((size_t)b * n_q + qi) * row_stride + (size_t)qh * HD);
    const float2 *tab = table + ((size_t)b * n_q + qi) * HALF;
#pragma unroll
    for (int s = 0; s < KS / 2; ++s) {
      const uint4 lo4 = row_ok ? qp[2 * s + h] : make_uint4(0, 0, 0, 0);
      const uint4 hi4 = row_ok ? qp[2 * (s + KS / 2) + h] : make_uint4(0, 0, 0, 0);
      const bf16x8 lo = __builtin_bit_cast(bf16x8, lo4), hi = __builtin_bit_cast(bf16x8, hi4);
      bf16x8 rl, rh;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float2 cs = tab[(2 * s + h) * 8 + i];
        float q0, q1;
        rope_pair((float)lo[i], (float)hi[i], cs, q0, q1);
        rl[i] = (__bf16)q0;
        rh[i] = (__bf16)q1;
      }
      qf[s] = rl;
      qf[s + KS / 2] = rh;
    }
    __syncthreads();  // the appended rows are visible to every wave of the workgroup
  } else {
    const uint4 *qp = reinterpret_cast<const uint4 *>(Q + (((size_t)b * n_q + qi) * Hq + qh) * HD);
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      uint4 v = row_ok ? qp[2 * s + h] : make_uint4(0, 0, 0, 0);
      qf[s] = __builtin_bit_cast(bf16x8, v);
    }
  }

  f32x16 acc[NT];
#pragma unroll
  for (int c = 0; c < NT; ++c)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;
  float m_run = NEG_INF, l_run = 0.f;

  auto tile_step = [&](const int t, const int t_lim) __attribute__((always_inline)) {
    uint4 vf[KS];  // 2*NT == KS units
#pragma unroll
    for (int s = 0; s < KS; ++s) vf[s] = Vb[(size_t)t * TILE_U4 + s * 64];

    f32x16 sacc;
#pragma unroll
    for (int v = 0; v < 16; ++v) sacc[v] = 0.f;
#pragma unroll
    for (int s = 0; s < KS; ++s)
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[s]), qf[s], sacc, 0, 0, 0);

    // prefetch the next tile's K while the softmax runs
    const int tn = t + WAVES;
    if (tn < t_lim) {
#pragma unroll
      for (int s = 0; s < KS; ++s) kf[s] = Kb[(size_t)tn * TILE_U4 + s * 64];
    }

    const int p0 = t * TK;
    const bool tail = p0 + TK > len;  // tile touches the block or dead slots: wave-uniform
    float sv[16];
    float mx = NEG_INF;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      float s = sacc[v] * scale_log2e;
      if (tail) {
        const int j = p0 + c_row(v, h) - len;  // block index of the key (<0: prefix)
        const bool vis = j < 0 || (j < n_q && (mode == SF_MASK_BIDIR || j <= qi));
        s = vis ? s : NEG_INF;
      }
      sv[v] = s;
      mx = fmaxf(mx, s);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    const float m_use = m_new == NEG_INF ? 0.f : m_new;  // nothing visible yet: keep exp finite
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
    float psum = 0.f;
    bf16x8 pf[2];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const float p = __builtin_amdgcn_exp2f(sv[v] - m_use);
      psum += p;
      pf[v >> 3][v & 7] = (__bf16)p;
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int c = 0; c < NT; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[c][v] *= alpha;

    if (tail) {
      // dead slots may hold anything (even NaN): zero the V operand of invisible-to-all keys
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const int u = s / NT;  // unit index = (u*NT + ct)*64 + lane
        uint32_t w[4] = {vf[s].x, vf[s].y, vf[s].z, vf[s].w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int key = p0 + 16 * u + 8 * (e >> 2) + 4 * h + (e & 3);
          if (key >= total) w[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
        }
        vf[s] = make_uint4(w[0], w[1], w[2], w[3]);
      }
    }
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int c = 0; c < NT; ++c)
        acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf[u * NT + c]), pf[u],
                                                         acc[c], 0, 0, 0);
  };
  if (FUSE && t < t_end && !early) {
#pragma unroll
    for (int s = 0; s < KS; ++s) kf[s] = Kb[(size_t)t * TILE_U4 + s * 64];
  }
  for (; t < t_end; t += WAVES) tile_step(t, t_end);

  // ---- merge the 4 waves through LDS --------------------------------------------------------
  float *lds_o = lds;                           // [WAVES][32][LROW]
  float *lds_ml = lds + WAVES * 32 * LROW;      // [WAVES][32][2]
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  if (h == 0) {
    lds_ml[(wave * 32 + n) * 2 + 0] = m_run;
    lds_ml[(wave * 32 + n) * 2 + 1] = l_tot;
  }
  __syncthreads();
  float m_all = NEG_INF;
#pragma unroll
  for (int w = 0; w < WAVES; ++w) m_all = fmaxf(m_all, lds_ml[(w * 32 + n) * 2]);
  const float m_fin = m_all == NEG_INF ? 0.f : m_all;
  const float f_own = __builtin_amdgcn_exp2f(m_run - m_fin);
#pragma unroll
  for (int c = 0; c < NT; ++c)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float4 o4 = make_float4(acc[c][4 * j] * f_own, acc[c][4 * j + 1] * f_own, acc[c][4 * j + 2] * f_own,
                              acc[c][4 * j + 3] * f_own);
      *reinterpret_cast<float4 *>(&lds_o[(wave * 32 + n) * LROW + 32 * c + 8 * j + 4 * h]) = o4;
    }
  __syncthreads();

  const bool direct = seq_chunks == 1;
  const int rows_here = min(32, R - rt * 32);
  // 256 threads sweep the [rows_here][HD] outputs, 4 consecutive features per thread
  for (int idx = tid; idx < rows_here * (HD / 4); idx += 256) {
    const int row = idx / (HD / 4), c4 = (idx % (HD / 4)) * 4;
    float l_all = 0.f, m_row = NEG_INF;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) m_row = fmaxf(m_row, lds_ml[(w * 32 + row) * 2]);
    const float m_r = m_row == NEG_INF ? 0.f : m_row;
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      l_all += lds_ml[(w * 32 + row) * 2 + 1] * __builtin_amdgcn_exp2f(lds_ml[(w * 32 + row) * 2] - m_r);
      const float4 x = *reinterpret_cast<const float4 *>(&lds_o[(w * 32 + row) * LROW + c4]);
      o.x += x.x; o.y += x.y; o.z += x.z; o.w += x.w;
    }
    const int rr = rt * 32 + row;
    if (direct) {
      const float inv = 1.f / l_all;
      const int i = rr / G, hq = g * G + rr % G;
      uint2 pk = make_uint2(pack2bf(o.x * inv, o.y * inv), pack2bf(o.z * inv, o.w * inv));
      *reinterpret_cast<uint2 *>(O + (((size_t)b * n_q + i) * Hq + hq) * HD + c4) = pk;
    } else {
      const size_t slot = (((size_t)b * Hkv + g) * n_chunks + chunk) * (size_t)(n_rt * 32) + rr;
      *reinterpret_cast<float4 *>(part_o + slot * HD + c4) = o;
      if (c4 == 0) {
        part_ml[slot * 2 + 0] = m_row;
        part_ml[slot * 2 + 1] = l_all;
      }
    }
  }
}

// Merge the split-KV partials of sequences that span more than one chunk.
template <int HD>
__global__ __launch_bounds__(HD / 4) void attn_combine_kernel(
    const float *__restrict__ part_o, const float *__restrict__ part_ml, const int32_t *__restrict__ kv_len,
    bf16_t *__restrict__ O, int n_q, int Hq, int Hkv, int cap, int chunk_tiles, int n_chunks, int n_rt) {
  const int hq = blockIdx.x, i = blockIdx.y, b = blockIdx.z;
  const int G = Hq / Hkv, g = hq / G, rr = i * G + hq % G;
  const int n_tiles = (min(kv_len[b], cap - n_q) + n_q + TK - 1) / TK;
  const int sc = min((n_tiles + chunk_tiles - 1) / chunk_tiles, n_chunks);
  if (sc <= 1) return;
  const size_t base = ((size_t)b * Hkv + g) * n_chunks;
  float m = NEG_INF;
  for (int c = 0; c < sc; ++c) m = fmaxf(m, part_ml[((base + c) * (n_rt * 32) + rr) * 2]);
  const float m_use = m == NEG_INF ? 0.f : m;
  float l = 0.f;
  float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
  const int c4 = threadIdx.x * 4;
  for (int c = 0; c < sc; ++c) {
    const size_t slot = (base + c) * (n_rt * 32) + rr;
    const float f = __builtin_amdgcn_exp2f(part_ml[slot * 2] - m_use);
    l += part_ml[slot * 2 + 1] * f;
    const float4 x = *reinterpret_cast<const float4 *>(part_o + slot * HD + c4);
    o.x += x.x * f; o.y += x.y * f; o.z += x.z * f; o.w += x.w * f;
  }
  const float inv = 1.f / l;
  uint2 pk = make_uint2(pack2bf(o.x * inv, o.y * inv), pack2bf(o.z * inv, o.w * inv));
  *reinterpret_cast<uint2 *>(O + (((size_t)b * n_q + i) * Hq + hq) * HD + c4) = pk;
}

// fp32 path (small models): plain cache layout, one workgroup per (sequence, query head).
// Keys are processed in chunks of CK with a workgroup-wide online softmax.
constexpr int CK = 512;
__global__ __launch_bounds__(256) void attn_f32_kernel(const float *__restrict__ Q, const float *__restrict__ Kc,
                                                       const float *__restrict__ Vc,
                                                       const int32_t *__restrict__ kv_len, float *__restrict__ O,
                                                       int n_q, int Hq, int Hkv, int hd, int cap, int mode,
                                                       float scale) {
  extern __shared__ float sm[];
  // sm: q[n_q][hd] | sc[n_q][CK] | red[256] | m[n_q] | l[n_q] | alpha[n_q]
  float *sq = sm, *sc = sq + n_q * hd, *red = sc + n_q * CK, *sm_m = red + 256, *sm_l = sm_m + n_q,
        *sm_a = sm_l + n_q;
  const int hq = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int g = hq / (Hq / Hkv);
  const int len = min(kv_len[b], cap - n_q), total = len + n_q;
  const float *K = Kc + ((size_t)b * Hkv + g) * (size_t)cap * hd;
  const float *V = Vc + ((size_t)b * Hkv + g) * (size_t)cap * hd;
  for (int x = tid; x < n_q * hd; x += 256) sq[x] = Q[(((size_t)b * n_q + x / hd) * Hq + hq) * hd + x % hd];
  if (tid < n_q) { sm_m[tid] = NEG_INF; sm_l[tid] = 0.f; }
  // each thread owns up to 2 (row, feature) outputs per 256-stride sweep
  float oacc[8];
#pragma unroll
  for (int x = 0; x < 8; ++x) oacc[x] = 0.f;
  __syncthreads();
  for (int p0 = 0; p0 < total; p0 += CK) {
    const int nk = min(CK, total - p0);
    for (int x = tid; x < n_q * nk; x += 256) {
      const int i = x / nk, p = p0 + x % nk;
      const int j = p - len;
      const bool vis = j < 0 || (mode == SF_MASK_BIDIR || j <= i);
      float s = NEG_INF;
      if (vis) {
        s = 0.f;
        const float *kr = K + (size_t)p * hd;
        for (int e = 0; e < hd; ++e) s += sq[i * hd + e] * kr[e];
        s *= scale;
      }
      sc[i * CK + x % nk] = s;
    }
    __syncthreads();
    // per-row max and sum: wave w handles rows w, w+4, ...
    const int lane = tid & 63, wave = tid >> 6;
    for (int i = wave; i < n_q; i += 4) {
      float mx = NEG_INF;
      for (int x = lane; x < nk; x += 64) mx = fmaxf(mx, sc[i * CK + x]);
      for (int o = 32; o; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
      const float m_new = fmaxf(sm_m[i], mx);
      const float m_use = m_new == NEG_INF ? 0.f : m_new;
      float sum = 0.f;
      for (int x = lane; x < nk; x += 64) {
        const float p = expf(sc[i * CK + x] - m_use);
        sc[i * CK + x] = p;
        sum += p;
      }
      for (int o = 32; o; o >>= 1) sum += __shfl_xor(sum, o);
      if (lane == 0) {
        const float a = expf(sm_m[i] - m_use);
        sm_a[i] = a;
        sm_l[i] = sm_l[i] * a + sum;
        sm_m[i] = m_new;
      }
    }
    __syncthreads();
    int slot = 0;
    for (int x = tid; x < n_q * hd; x += 256, ++slot) {
      const int i = x / hd, e = x % hd;
      float o = oacc[slot] * sm_a[i];
      for (int kk = 0; kk < nk; ++kk) o += sc[i * CK + kk] * V[(size_t)(p0 + kk) * hd + e];
      oacc[slot] = o;
    }
    __syncthreads();
  }
  int slot = 0;
  for (int x = tid; x < n_q * hd; x += 256, ++slot) {
    const int i = x / hd, e = x % hd;
    O[(((size_t)b * n_q + i) * Hq + hq) * hd + e] = oacc[slot] / sm_l[i];
  }
}

}  // namespace

// Chunk size (in 32-key tiles) of the split-KV decomposition.  The grid is sized from the host's
// upper bound of the lengths: split only when there are fewer (sequence, head, row tile) groups
// than CUs, and never below 16 tiles (4 per wave) per chunk; with >= 256 groups every group is one
// workgroup and no combine pass is needed (measured fastest at every batch >= 32).
int attn_chunk_tiles(int groups, int keys_upper) {
  const int n_tiles = (keys_upper + TK - 1) / TK;
  const int want_chunks = (256 + groups - 1) / (groups > 0 ? groups : 1);
  int ct = (n_tiles + want_chunks - 1) / want_chunks;
  return ct < 16 ? 16 : ct;
}

size_t attn_workspace_bytes(int B, int Hkv, int hd, int G, int n_q, int len_upper) {
  const int n_rt = (G * n_q + 31) / 32;
  // sized for the smallest chunk any launch may pick (16 tiles)
  const int ct = 16;
  const int n_tiles = (len_upper + n_q + TK - 1) / TK;
  const int n_chunks = (n_tiles + ct - 1) / ct;
  if (n_chunks <= 1) return 0;
  return (size_t)B * Hkv * n_chunks * (n_rt * 32) * (hd + 2) * sizeof(float);
}

hipError_t launch_attention_bf16(const AttnArgs &a, hipStream_t s) {
  const int G = a.Hq / a.Hkv;
  const int n_rt = (G * a.n_q + 31) / 32;
  const float scale_log2e = 1.4426950408889634f / sqrtf((float)a.hd);
  dim3 grid(a.n_chunks, a.Hkv * n_rt, a.B), block(256);
  const size_t lds = (size_t)WAVES * 32 * (a.hd + 4 + 2) * sizeof(float);
  static bool attr_done = false;
  if (!attr_done) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(attn_bf16_kernel<128, 0>),
                        hipFuncAttributeMaxDynamicSharedMemorySize, WAVES * 32 * (128 + 6) * 4);
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(attn_bf16_kernel<128, 1>),
                        hipFuncAttributeMaxDynamicSharedMemorySize, WAVES * 32 * (128 + 6) * 4);
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(attn_bf16_kernel<64, 0>),
                        hipFuncAttributeMaxDynamicSharedMemorySize, WAVES * 32 * (64 + 6) * 4);
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(attn_bf16_kernel<64, 1>),
                        hipFuncAttributeMaxDynamicSharedMemorySize, WAVES * 32 * (64 + 6) * 4);
    attr_done = true;
  }
  // a.qkv: the raw QKV projection; the kernel rotates and appends the block's rows itself
  const bf16_t *q = (const bf16_t *)(a.qkv ? a.qkv : a.q);
#define SF_ATTN_LAUNCH(HD_, FUSE_)                                                                              \
  attn_bf16_kernel<HD_, FUSE_><<<grid, block, lds, s>>>(q, (const uint4 *)a.kc, (const uint4 *)a.vc, a.kv_len, \
                                                        (bf16_t *)a.out, a.part_o, a.part_ml, a.n_q, a.Hq,     \
                                                        a.Hkv, a.cap, a.mode, a.chunk_tiles, a.n_chunks, n_rt, \
                                                        scale_log2e, a.table, a.order)
  if (a.hd == 128) {
    if (a.qkv) SF_ATTN_LAUNCH(128, 1); else SF_ATTN_LAUNCH(128, 0);
  } else {
    if (a.qkv) SF_ATTN_LAUNCH(64, 1); else SF_ATTN_LAUNCH(64, 0);
  }
#undef SF_ATTN_LAUNCH
  return hipGetLastError();
}

hipError_t launch_attention_combine(const AttnArgs &a, hipStream_t s) {
  const int G = a.Hq / a.Hkv;
  const int n_rt = (G * a.n_q + 31) / 32;
  dim3 cgrid(a.Hq, a.n_q, a.B);
  if (a.hd == 128)
    attn_combine_kernel<128><<<cgrid, 32, 0, s>>>(a.part_o, a.part_ml, a.kv_len, (bf16_t *)a.out, a.n_q, a.Hq,
                                                  a.Hkv, a.cap, a.chunk_tiles, a.n_chunks, n_rt);
  else
    attn_combine_kernel<64><<<cgrid, 16, 0, s>>>(a.part_o, a.part_ml, a.kv_len, (bf16_t *)a.out, a.n_q, a.Hq,
                                                 a.Hkv, a.cap, a.chunk_tiles, a.n_chunks, n_rt);
  return hipGetLastError();
}

hipError_t launch_attention_f32(const AttnArgs &a, hipStream_t s) {
  const size_t lds = ((size_t)a.n_q * a.hd + (size_t)a.n_q * CK + 256 + 3 * a.n_q) * sizeof(float);
  dim3 grid(a.Hq, a.B);
  static bool attr_done = false;
  if (!attr_done) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(attn_f32_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                        64 * 1024);
    attr_done = true;
  }
  attn_f32_kernel<<<grid, 256, lds, s>>>((const float *)a.q, (const float *)a.kc, (const float *)a.vc, a.kv_len,
                                         (float *)a.out, a.n_q, a.Hq, a.Hkv, a.hd, a.cap, a.mode,
                                         1.f / sqrtf((float)a.hd));
  return hipGetLastError();
}

}  // namespace sf

// Bandwidth-trivial row kernels of the SpecFormer step for gfx950: RMSNorm / Grouped RMSNorm,
// rotary embedding + K/V append into the tiled caches, SwiGLU gating, embedding gather,
// hook capture, cache layout conversion.  All statistics and rotations in fp32.
#include "sf_internal.h"

namespace sf {
namespace {

__device__ __forceinline__ float block_sum_256(float v, float *red) {
  for (int o = 32; o; o >>= 1) v += __shfl_xor(v, o);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) red[wave] = v;
  __syncthreads();
  const float t = red[0] + red[1] + red[2] + red[3];
  __syncthreads();
  return t;
}

// 8 consecutive elements of a row of T, as floats
template <typename T> struct Vec8;
template <> struct Vec8<bf16_t> {
  static __device__ __forceinline__ void ld(const bf16_t *p, float (&v)[8]) {
    const uint4 u = *reinterpret_cast<const uint4 *>(p);
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) { v[2 * i] = __uint_as_float(w[i] << 16); v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u); }
  }
  static __device__ __forceinline__ void st(bf16_t *p, const float (&v)[8]) {
    *reinterpret_cast<uint4 *>(p) = make_uint4(pack2bf(v[0], v[1]), pack2bf(v[2], v[3]), pack2bf(v[4], v[5]),
                                               pack2bf(v[6], v[7]));
  }
};
template <> struct Vec8<float> {
  static __device__ __forceinline__ void ld(const float *p, float (&v)[8]) {
    const float4 a = *reinterpret_cast<const float4 *>(p), b = *reinterpret_cast<const float4 *>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
  static __device__ __forceinline__ void st(float *p, const float (&v)[8]) {
    *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4 *>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
  }
};

// One workgroup per output row.  y = gain[r % n_gain] * x / sqrt(mean(x^2) + eps).  TI: type of x (float for
// rows of the residual stream), TO: type of the gains and of y.
// The row stays in registers between the two passes (up to 4 x 8 elements per thread, i.e. d <= 8192);
// longer or unaligned rows take the scalar path.
template <typename TI, typename TO>
__global__ __launch_bounds__(256) void rmsnorm_kernel(const TI *__restrict__ X, const TO *__restrict__ gain,
                                                      TO *__restrict__ Y, int d, int n_gain, float eps, int map,
                                                      int q, int q_max, const int32_t *__restrict__ n_new) {
  __shared__ float red[4];
  const int r = blockIdx.x;
  long in_row = r;
  bool zero = false;
  if (map == 1) {  // hooks rows: r = (b*q + i)*4 + g
    const int g = r & 3, bi = r >> 2, b = bi / q, i = bi % q;
    in_row = ((long)b * q_max + i) * 4 + g;
  } else if (map == 2) {  // newest committed row of sequence r
    const int nn = n_new[r];
    zero = nn <= 0;
    in_row = (long)r * q + (zero ? 0 : min(nn, q) - 1);
  } else if (map == 3) {  // row r itself, silenced when sequence r committed nothing
    zero = n_new[r] <= 0;
  }
  const TI *x = X + in_row * d;
  const TO *gv = gain + (size_t)(r % n_gain) * d;
  TO *y = Y + (size_t)r * d;
  if (d % 8 == 0 && d <= 8 * 256 * 4) {
    float v[4][8];
    float ss = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int e = (threadIdx.x + 256 * j) * 8;
      if (e < d && !zero) {
        Vec8<TI>::ld(x + e, v[j]);
#pragma unroll
        for (int i = 0; i < 8; ++i) ss += v[j][i] * v[j][i];
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[j][i] = 0.f;
      }
    }
    ss = block_sum_256(ss, red);
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int e = (threadIdx.x + 256 * j) * 8;
      if (e < d) {
        float g[8], o[8];
        Vec8<TO>::ld(gv + e, g);
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = g[i] * (v[j][i] * inv);
        Vec8<TO>::st(y + e, o);
      }
    }
    return;
  }
  float ss = 0.f;
  if (!zero)
    for (int e = threadIdx.x; e < d; e += 256) {
      const float v = Elem<TI>::ld(x + e);
      ss += v * v;
    }
  ss = block_sum_256(ss, red);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
  for (int e = threadIdx.x; e < d; e += 256) {
    const float v = zero ? 0.f : Elem<TI>::ld(x + e);
    Elem<TO>::st(y + e, Elem<TO>::ld(gv + e) * (v * inv));
  }
}

// cos/sin of pos * theta^(-2i/hd), evaluated in double so that large positions stay exact to fp32.
// One extra workgroup (when `order` is given) ranks the sequences by descending length, ties by
// index: order[rank] = b.  The attention kernel starts the longest sequences first, which evens out
// the tail of a ragged batch.
// A second table (table2: n_q2 rows per sequence at positions kv_len[b] + r) can be filled by the same launch.
__global__ void rope_table_kernel(float2 *__restrict__ table, const int32_t *__restrict__ kv_len,
                                  const int32_t *__restrict__ n_new, int B, int n_q, int half, int pos_mode,
                                  double log2_theta, int32_t *__restrict__ order, int32_t *__restrict__ dev_err,
                                  int len_upper, int cap, float2 *__restrict__ table2, int n_q2) {
  if (dev_err && blockIdx.x == 0) {
    // the launch grids of this step were sized from the host's bound: say so if a length breaks it
    const bool fwd = pos_mode == 0 || table2;        // rows that extend the sequences are part of this launch
    const int rows = table2 ? n_q2 : n_q;
    for (int b = threadIdx.x; b < B; b += blockDim.x) {
      const int len = kv_len[b];
      int bits = 0;
      if (fwd && len > len_upper) bits |= SF_DEVERR_LEN_ABOVE_BOUND;
      if (fwd && len + rows > cap) bits |= SF_DEVERR_CACHE_FULL;
      if (len < 0) bits |= SF_DEVERR_LEN_ABOVE_BOUND;
      if (bits) atomicOr(dev_err, bits);
    }
  }
  if (order && blockIdx.x == gridDim.x - 1) {
    for (int b = threadIdx.x; b < B; b += blockDim.x) {
      const int mine = kv_len[b];
      int rank = 0;
      for (int j = 0; j < B; ++j) {
        const int other = kv_len[j];
        rank += (other > mine || (other == mine && j < b)) ? 1 : 0;
      }
      order[rank] = b;
    }
    return;
  }
  int idx = blockIdx.x * blockDim.x + threadIdx.x;
  const int n1 = B * n_q * half;
  if (idx >= n1) {  // the second table, if any
    idx -= n1;
    if (!table2 || idx >= B * n_q2 * half) return;
    table = table2; n_q = n_q2; pos_mode = 0;
  }
  const int i = idx % half, row = idx / half, b = row / n_q, r = row % n_q;
  const int pos = pos_mode == 0 ? kv_len[b] + r : kv_len[b] - n_new[b] + r;
  const double inv_freq = exp2(-(double)(2 * i) / (double)(2 * half) * log2_theta);
  double s, c;
  sincos((double)pos * inv_freq, &s, &c);
  table[idx] = make_float2((float)c, (float)s);
}

// One workgroup per row (b,i).  Rotates q and k (pairs (e, e+hd/2)), writes q to q_out, k and v into
// the caches at position pos.  bf16: tiled cache; fp32: plain cache.
template <typename T>
__global__ __launch_bounds__(256) void rope_kv_kernel(const T *__restrict__ QKV, T *__restrict__ Qo,
                                                      T *__restrict__ Kc, T *__restrict__ Vc,
                                                      const int32_t *__restrict__ kv_len,
                                                      const int32_t *__restrict__ n_new,
                                                      const float2 *__restrict__ table, int n_q, int Hq, int Hkv,
                                                      int hd, int cap, int kv_only, int pos_mode) {
  const int row = blockIdx.x, b = row / n_q, i = row % n_q;
  const int half = hd >> 1;
  const int nq_cols = kv_only ? 0 : Hq * hd, nkv = Hkv * hd;
  const T *src = QKV + (size_t)row * (nq_cols + 2 * nkv);
  const float2 *tab = table + (size_t)row * half;
  int pos;
  bool valid = true;
  if (pos_mode == 0) pos = kv_len[b] + i;
  else { const int nn = n_new[b]; pos = kv_len[b] - nn + i; valid = i < nn; }
  if (pos < 0 || pos >= cap) valid = false;
  // q: pairs
  for (int x = threadIdx.x; x < Hq * half && !kv_only; x += 256) {
    const int hh = x / half, e = x % half;
    const float2 cs = tab[e];
    const float a = Elem<T>::ld(src + hh * hd + e), bb = Elem<T>::ld(src + hh * hd + e + half);
    float q0, q1;
    rope_pair(a, bb, cs, q0, q1);
    Elem<T>::st(Qo + (size_t)row * nq_cols + hh * hd + e, q0);
    Elem<T>::st(Qo + (size_t)row * nq_cols + hh * hd + e + half, q1);
  }
  if (!valid) return;
  const size_t tile = pos / TK;
  const int a_in = pos % TK;
  for (int x = threadIdx.x; x < Hkv * half; x += 256) {
    const int g = x / half, e = x % half;
    const float2 cs = tab[e];
    const float a = Elem<T>::ld(src + nq_cols + g * hd + e), bb = Elem<T>::ld(src + nq_cols + g * hd + e + half);
    float k0, k1;
    rope_pair(a, bb, cs, k0, k1);
    const float v0 = Elem<T>::ld(src + nq_cols + nkv + g * hd + e);
    const float v1 = Elem<T>::ld(src + nq_cols + nkv + g * hd + e + half);
    if (sizeof(T) == 2) {
      const size_t base = (((size_t)b * Hkv + g) * (cap / TK) + tile) * (size_t)(TK * hd);
      Elem<T>::st(Kc + base + k_tile_off(a_in, e), k0);
      Elem<T>::st(Kc + base + k_tile_off(a_in, e + half), k1);
      Elem<T>::st(Vc + base + v_tile_off(a_in, e, hd), v0);
      Elem<T>::st(Vc + base + v_tile_off(a_in, e + half, hd), v1);
    } else {
      const size_t base = (((size_t)b * Hkv + g) * cap + pos) * (size_t)hd;
      Elem<T>::st(Kc + base + e, k0);
      Elem<T>::st(Kc + base + e + half, k1);
      Elem<T>::st(Vc + base + e, v0);
      Elem<T>::st(Vc + base + e + half, v1);
    }
  }
}

template <typename T>
__global__ void silu_mul_kernel(const float *__restrict__ gu, T *__restrict__ act, int M, int F) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)M * F) return;
  const size_t m = idx / F, f = idx % F;
  const float g = gu[m * 2 * F + f], u = gu[m * 2 * F + F + f];
  Elem<T>::st(act + idx, g / (1.0f + expf(-g)) * u);
}

// h[row] = embed[token(row)] as float (the residual stream), hb its copy in the model dtype (optional), and
// the same row as hooked state g for every group g in hook_mask.  Out-of-range ids read row 0.
template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(const T *__restrict__ E, const int32_t *__restrict__ pending,
                                                    const int32_t *__restrict__ draft, float *__restrict__ H,
                                                    T *__restrict__ Hb, T *__restrict__ hooks, int hook_mask, int k,
                                                    int q_max, int d, int vocab) {
  const int row = blockIdx.x, q = k + 1, b = row / q, i = row % q;
  int tok = i == 0 ? pending[b] : draft[b * k + i - 1];
  if (tok < 0 || tok >= vocab) tok = 0;
  const T *src = E + (size_t)tok * d;
  float *h = H + (size_t)row * d;
  T *hk = hooks + ((size_t)b * q_max + i) * 4 * d;
  for (int e = threadIdx.x; e < d; e += 256) {
    const T v = src[e];
    h[e] = Elem<T>::ld(&v);
    if (Hb) Hb[(size_t)row * d + e] = v;
#pragma unroll
    for (int g = 0; g < 4; ++g)
      if (hook_mask >> g & 1) hk[(size_t)g * d + e] = v;
  }
}

// The newest committed context row of every sequence, raw (the residual input of the context
// attention's own output), and the number of keys that row sees before itself.
template <typename T>
__global__ __launch_bounds__(256) void gather_last_kernel(const T *__restrict__ X, T *__restrict__ out,
                                                          const int32_t *__restrict__ n_new,
                                                          const int32_t *__restrict__ kv_len,
                                                          int32_t *__restrict__ len_m1, int q, int d) {
  const int b = blockIdx.x, nn = n_new[b];
  const T *src = X + ((size_t)b * q + (nn > 0 ? min(nn, q) - 1 : 0)) * d;
  for (int e = threadIdx.x; e < d; e += 256) out[(size_t)b * d + e] = nn > 0 ? src[e] : T(0);
  if (threadIdx.x == 0) len_m1[b] = max(kv_len[b] - 1, 0);
}

template <typename T>
__global__ __launch_bounds__(256) void hook_copy_kernel(const float *__restrict__ H, T *__restrict__ hooks, int q,
                                                        int q_max, int d, int group) {
  const int row = blockIdx.x, b = row / q, i = row % q;
  const float *h = H + (size_t)row * d;
  T *hk = hooks + (((size_t)b * q_max + i) * 4 + group) * d;
  for (int e = threadIdx.x; e < d; e += 256) Elem<T>::st(hk + e, h[e]);
}

// plain [B][Hkv][cap][hd] <-> tiled (bf16) / plain (fp32: straight copy)
template <typename T>
__global__ void kv_convert_kernel(const T *__restrict__ src, T *__restrict__ dst, int is_v, int to_tiled,
                                  size_t n, int cap, int hd) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n) return;
  size_t t_idx = idx;
  if (sizeof(T) == 2) {
    const int c = idx % hd;
    const size_t pos_all = idx / hd;  // (b*Hkv+g)*cap + pos
    const int pos = pos_all % cap;
    const size_t slab = pos_all / cap;
    const size_t base = (slab * (cap / TK) + pos / TK) * (size_t)(TK * hd);
    t_idx = base + (is_v ? v_tile_off(pos % TK, c, hd) : k_tile_off(pos % TK, c));
  }
  if (to_tiled) dst[t_idx] = src[idx];
  else dst[idx] = src[t_idx];
}

// plain streaming copy of 16-byte units: the reference dispatch for scaling profiler byte counters
__global__ __launch_bounds__(256) void calib_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                                         size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

template <typename TI, typename TO>
hipError_t rmsnorm_t(const NormArgs &a, hipStream_t s) {
  rmsnorm_kernel<TI, TO><<<a.M, 256, 0, s>>>((const TI *)a.x, (const TO *)a.gain, (TO *)a.y, a.d, a.n_gain, a.eps,
                                             a.map, a.q, a.q_max, a.n_new);
  return hipGetLastError();
}

template <typename T>
hipError_t rope_kv_t(const RopeArgs &a, hipStream_t s) {
  const int M = a.B * a.n_q;
  rope_kv_kernel<T><<<M, 256, 0, s>>>((const T *)a.qkv, (T *)a.q_out, (T *)a.kc, (T *)a.vc, a.kv_len, a.n_new,
                                      a.table, a.n_q, a.Hq, a.Hkv, a.hd, a.cap, a.kv_only, a.pos_mode);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_calib_copy(const void *src, void *dst, size_t bytes, hipStream_t s) {
  calib_copy_kernel<<<8192, 256, 0, s>>>((const uint4 *)src, (uint4 *)dst, bytes / 16);
  return hipGetLastError();
}

hipError_t launch_rmsnorm(const NormArgs &a, int dtype, hipStream_t s) {
  if (dtype != SF_BF16) return rmsnorm_t<float, float>(a, s);
  return a.x_f32 ? rmsnorm_t<float, bf16_t>(a, s) : rmsnorm_t<bf16_t, bf16_t>(a, s);
}

hipError_t launch_rope_table(const RopeArgs &a, hipStream_t s) {
  const int half = a.hd / 2;
  const int n = a.B * (a.n_q + (a.table2 ? a.n_q2 : 0)) * half;
  rope_table_kernel<<<(n + 255) / 256 + (a.order ? 1 : 0), 256, 0, s>>>(a.table, a.kv_len, a.n_new, a.B, a.n_q, half,
                                                                        a.pos_mode, log2((double)a.theta), a.order,
                                                                        a.dev_err, a.len_upper, a.cap, a.table2, a.n_q2);
  return hipGetLastError();
}

hipError_t launch_rope_kv(const RopeArgs &a, int dtype, hipStream_t s) {
  return dtype == SF_BF16 ? rope_kv_t<bf16_t>(a, s) : rope_kv_t<float>(a, s);
}

hipError_t launch_silu_mul(const float *gu, void *act, int M, int F, int dtype, hipStream_t s) {
  const size_t n = (size_t)M * F;
  const unsigned blocks = (unsigned)((n + 255) / 256);
  if (dtype == SF_BF16) silu_mul_kernel<bf16_t><<<blocks, 256, 0, s>>>(gu, (bf16_t *)act, M, F);
  else silu_mul_kernel<float><<<blocks, 256, 0, s>>>(gu, (float *)act, M, F);
  return hipGetLastError();
}

hipError_t launch_embed(const void *embed, const int32_t *pending, const int32_t *draft, float *h, void *hb,
                        void *hooks, int hook_mask, int B, int k, int q_max, int d, int vocab, int dtype,
                        hipStream_t s) {
  const int M = B * (k + 1);
  if (dtype == SF_BF16)
    embed_kernel<bf16_t><<<M, 256, 0, s>>>((const bf16_t *)embed, pending, draft, h, (bf16_t *)hb, (bf16_t *)hooks,
                                           hook_mask, k, q_max, d, vocab);
  else
    embed_kernel<float><<<M, 256, 0, s>>>((const float *)embed, pending, draft, h, nullptr, (float *)hooks,
                                          hook_mask, k, q_max, d, vocab);
  return hipGetLastError();
}

hipError_t launch_gather_last(const void *x, void *out, const int32_t *n_new, const int32_t *kv_len, int32_t *len_m1,
                              int B, int q, int d, int dtype, hipStream_t s) {
  if (dtype == SF_BF16)
    gather_last_kernel<bf16_t><<<B, 256, 0, s>>>((const bf16_t *)x, (bf16_t *)out, n_new, kv_len, len_m1, q, d);
  else
    gather_last_kernel<float><<<B, 256, 0, s>>>((const float *)x, (float *)out, n_new, kv_len, len_m1, q, d);
  return hipGetLastError();
}

hipError_t launch_hook_copy(const float *h, void *hooks, int B, int q, int q_max, int d, int group, int dtype,
                            hipStream_t s) {
  if (dtype == SF_BF16) hook_copy_kernel<bf16_t><<<B * q, 256, 0, s>>>(h, (bf16_t *)hooks, q, q_max, d, group);
  else hook_copy_kernel<float><<<B * q, 256, 0, s>>>(h, (float *)hooks, q, q_max, d, group);
  return hipGetLastError();
}

hipError_t launch_kv_convert(const void *src, void *dst, int is_v, int to_tiled, int B, int Hkv, int cap, int hd,
                             int dtype, hipStream_t s) {
  const size_t n = (size_t)B * Hkv * cap * hd;
  const unsigned blocks = (unsigned)((n + 255) / 256);
  if (dtype == SF_BF16)
    kv_convert_kernel<bf16_t><<<blocks, 256, 0, s>>>((const bf16_t *)src, (bf16_t *)dst, is_v, to_tiled, n, cap, hd);
  else
    kv_convert_kernel<float><<<blocks, 256, 0, s>>>((const float *)src, (float *)dst, is_v, to_tiled, n, cap, hd);
  return hipGetLastError();
}

}  // namespace sf

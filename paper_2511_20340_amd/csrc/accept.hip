// Lossless greedy acceptance for gfx950: arg-max over the vocabulary (the only HBM-heavy part: one
// streaming read of the fp32 logits), draft/target comparison, longest accepted prefix, commit of
// lengths / pending tokens, exclusive scan of the accept lengths.
//
// The arg-max normally arrives as per-column-tile partials from the LM-head kernel's epilogue (the
// logits are then never stored); argmax_partial_kernel produces the same kind of partials from
// materialised logits (16 segments per row, thousands of workgroups).  argmax_final_kernel finishes
// a row's partials; accept_kernel is one workgroup that compares, commits and scans.
// Ties resolve to the lowest index; NaN never wins; a row without any comparable value gives 0.
#include "sf_internal.h"
#include <limits.h>
#include <mutex>

// Scratch of the entry point that must not allocate (sf_op_argmax_noalloc): the arg-max partials of up to
// ARGMAX_NOALLOC_MAX_ROWS logits rows, [rows][ARGMAX_SEGS] values followed by [rows][ARGMAX_SEGS] indices.
// Every GPU the library runs on holds its own copy of this array until the process ends; host code reaches
// it only through the per-device address that hipGetSymbolAddress returns.
static __device__ __align__(256) unsigned char scratch[(size_t)sf::ARGMAX_NOALLOC_MAX_ROWS * sf::ARGMAX_SEGS * 8];

namespace sf {
namespace {

struct Best {
  float v;
  int32_t i;
};
__device__ __forceinline__ void take(Best &b, float v, int32_t i) {
  if (v != v) return;
  if (v > b.v || (v == b.v && i < b.i)) { b.v = v; b.i = i; }
}
__device__ __forceinline__ Best better(Best a, Best b) {
  return (b.v > a.v || (b.v == a.v && b.i < a.i)) ? b : a;
}

__global__ __launch_bounds__(256) void argmax_partial_kernel(const float *__restrict__ logits, int V,
                                                             float *__restrict__ pmax, int32_t *__restrict__ pidx) {
  __shared__ float sv[4];
  __shared__ int32_t si[4];
  const int seg = blockIdx.x, row = blockIdx.y;
  int seg_len = (V + ARGMAX_SEGS - 1) / ARGMAX_SEGS;
  seg_len = (seg_len + 3) & ~3;
  const int lo = seg * seg_len, hi = min(V, lo + seg_len);
  const float *x = logits + (size_t)row * V;
  Best b{-__builtin_huge_valf(), INT_MAX};
  if ((V & 3) == 0) {
    for (int i = lo + threadIdx.x * 4; i < hi; i += 1024) {
      const float4 v = *reinterpret_cast<const float4 *>(x + i);
      take(b, v.x, i); take(b, v.y, i + 1); take(b, v.z, i + 2); take(b, v.w, i + 3);
    }
  } else {
    for (int i = lo + threadIdx.x; i < hi; i += 256) take(b, x[i], i);
  }
  for (int o = 32; o; o >>= 1) {
    Best other{__shfl_xor(b.v, o), __shfl_xor(b.i, o)};
    b = better(b, other);
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) { sv[wave] = b.v; si[wave] = b.i; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w) b = better(b, Best{sv[w], si[w]});
    pmax[row * ARGMAX_SEGS + seg] = b.v;
    pidx[row * ARGMAX_SEGS + seg] = b.i;
  }
}

// One wavefront per row: the best of the row's n_part partials (ascending column ranges, so the
// lowest index wins among equal values).
__global__ __launch_bounds__(256) void argmax_final_kernel(const float *__restrict__ pmax,
                                                           const int32_t *__restrict__ pidx, int M, int n_part,
                                                           int stride, int32_t *__restrict__ ids) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= M) return;
  Best b{-__builtin_huge_valf(), INT_MAX};
  for (int s = lane; s < n_part; s += 64) {
    const int32_t i = pidx[(size_t)row * stride + s];
    if (i != INT_MAX) b = better(b, Best{pmax[(size_t)row * stride + s], i});
  }
  for (int o = 32; o; o >>= 1) {
    Best other{__shfl_xor(b.v, o), __shfl_xor(b.i, o)};
    b = better(b, other);
  }
  if (lane == 0) ids[row] = b.i == INT_MAX ? 0 : b.i;
}

// One workgroup.  Thread t owns the sequences [t*per, (t+1)*per): their accept lengths from the
// target's choices p and the draft, the commit, and a workgroup-wide scan for the offsets.
__global__ __launch_bounds__(256) void accept_kernel(const int32_t *__restrict__ target_ids,
                                                     const int32_t *__restrict__ draft,
                                                     const int32_t *__restrict__ force_len,
                                                     int32_t *__restrict__ accept_len, int32_t *__restrict__ out_tokens,
                                                     int32_t *__restrict__ kv_len, int32_t *__restrict__ pending,
                                                     int32_t *__restrict__ n_new, int32_t *__restrict__ cu_new, int B,
                                                     int k) {
  __shared__ int32_t scan[256];
  const int q = k + 1;
  const int per = (B + 255) / 256;
  const int b0 = threadIdx.x * per, b1 = min(B, b0 + per);
  int32_t local = 0;
  for (int b = b0; b < b1; ++b) {
    const int32_t *p = target_ids + (size_t)b * q;
    int a;
    if (force_len) {
      a = min(max(force_len[b], 0), q);
    } else {
      a = 1;
      for (int n = 0; n < k && draft[b * k + n] == p[n]; ++n) a = n + 2;
    }
    for (int i = 0; i < q; ++i) out_tokens[b * q + i] = i < a ? p[i] : -1;
    accept_len[b] = a;
    if (a > 0) pending[b] = p[a - 1];
    kv_len[b] += a;
    n_new[b] = a;
    local += a;
  }
  scan[threadIdx.x] = local;
  __syncthreads();
  for (int o = 1; o < 256; o <<= 1) {  // inclusive Hillis-Steele scan
    const int32_t v = threadIdx.x >= o ? scan[threadIdx.x - o] : 0;
    __syncthreads();
    scan[threadIdx.x] += v;
    __syncthreads();
  }
  int32_t run = scan[threadIdx.x] - local;  // exclusive offset of this thread's first sequence
  for (int b = b0; b < b1; ++b) {
    cu_new[b] = run;
    run += n_new[b];
  }
  if (b1 == B && b0 < B) cu_new[B] = run;
}

}  // namespace

hipError_t launch_argmax_partial(const float *logits, int M, int V, float *pmax, int32_t *pidx, hipStream_t s) {
  argmax_partial_kernel<<<dim3(ARGMAX_SEGS, M), 256, 0, s>>>(logits, V, pmax, pidx);
  return hipGetLastError();
}

hipError_t launch_argmax_final(const float *pmax, const int32_t *pidx, int M, int n_part, int stride, int32_t *ids,
                               hipStream_t s) {
  argmax_final_kernel<<<(M + 3) / 4, 256, 0, s>>>(pmax, pidx, M, n_part, stride, ids);
  return hipGetLastError();
}

hipError_t launch_argmax_noalloc(const float *logits, int M, int V, int32_t *ids, hipStream_t s) {
  constexpr int MAX_DEVICES = 64;
  static void *dev_scratch[MAX_DEVICES];  // the array's address on each device, resolved once
  static std::mutex mu;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  void *p;
  {
    std::lock_guard<std::mutex> lock(mu);
    if (!dev_scratch[dev]) {
      void *sym = nullptr;
      e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
      if (e != hipSuccess) return e;
      dev_scratch[dev] = sym;
    }
    p = dev_scratch[dev];
  }
  float *pmax = reinterpret_cast<float *>(p);
  int32_t *pidx = reinterpret_cast<int32_t *>(static_cast<char *>(p) + (size_t)ARGMAX_NOALLOC_MAX_ROWS * ARGMAX_SEGS * 4);
  // every partial the finish reads is written by the first pass of the same call: nothing to clear
  argmax_partial_kernel<<<dim3(ARGMAX_SEGS, M), 256, 0, s>>>(logits, V, pmax, pidx);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  argmax_final_kernel<<<(M + 3) / 4, 256, 0, s>>>(pmax, pidx, M, ARGMAX_SEGS, ARGMAX_SEGS, ids);
  return hipGetLastError();
}

hipError_t launch_accept(const AcceptArgs &a, hipStream_t s) {
  accept_kernel<<<1, 256, 0, s>>>(a.target_ids, a.draft, a.force_len, a.accept_len, a.out_tokens, a.kv_len,
                                  a.pending, a.n_new, a.cu_new, a.B, a.k);
  return hipGetLastError();
}

}  // namespace sf

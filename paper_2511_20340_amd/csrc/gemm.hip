// Linear layers  y[M][N] = x[M][K] . w[N][K]^T (+bias) (+residual)  for gfx950.
//
// bf16 path: 256-thread workgroups, BMxBN output tile, BK = 64 slices staged through LDS
// (register-prefetched double buffer, rows padded to 72 elements so the 16-byte MFMA operand
// reads are bank-conflict free), 32x32x16 bf16 MFMA with fp32 accumulators.  Both operands are
// K-contiguous, so an operand register is one 16-byte LDS read.  Workgroup ids are remapped so
// that all M-tiles of one weight column-tile land on the same XCD (its L2 then serves the weight
// tile to every M-tile after one HBM read).
//
// fp32 path: plain SIMT tiling for the small fp32 configuration.
#include "sf_internal.h"

namespace sf {
namespace {

constexpr int BK = 64;
constexpr int LDK = 72;  // padded LDS row length in bf16 elements (144 B)
constexpr int XCDS = 8;

template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const bf16_t *__restrict__ A, const bf16_t *__restrict__ W,
                                                        const bf16_t *__restrict__ bias,
                                                        const bf16_t *residual, void *Y, int M, int N, int K,
                                                        int out_f32, int tiles_m, int tiles_n) {
  constexpr int WAVES_N = BN / WN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int A_CH = BM * 8 / 256, W_CH = BN * 8 / 256;  // 16-byte chunks per thread per slice
  static_assert((BM / WM) * (BN / WN) == 4, "4 waves");
  extern __shared__ __attribute__((aligned(16))) bf16_t smem[];
  bf16_t *sA = smem;                  // [2][BM][LDK]
  bf16_t *sW = smem + 2 * BM * LDK;   // [2][BN][LDK]

  // XCD-aware tile assignment: consecutive workgroup ids round-robin over the 8 XCDs
  const int id = blockIdx.x;
  const int xcd = id % XCDS, j = id / XCDS;
  const int tn = (j / tiles_m) * XCDS + xcd, tm = j % tiles_m;
  if (tn >= tiles_n) return;
  const int m0 = tm * BM, n0 = tn * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  const int ln = lane & 31, lh = lane >> 5;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  uint4 ra[A_CH], rw[W_CH];
  auto gload = [&](int k0) {
#pragma unroll
    for (int c = 0; c < A_CH; ++c) {
      const int cid = tid + 256 * c, row = cid >> 3, kc = (cid & 7) * 8;
      const int gr = m0 + row;
      ra[c] = (gr < M && k0 + kc < K) ? *reinterpret_cast<const uint4 *>(A + (size_t)gr * K + k0 + kc)
                                      : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int c = 0; c < W_CH; ++c) {
      const int cid = tid + 256 * c, row = cid >> 3, kc = (cid & 7) * 8;
      const int gr = n0 + row;
      rw[c] = (gr < N && k0 + kc < K) ? *reinterpret_cast<const uint4 *>(W + (size_t)gr * K + k0 + kc)
                                      : make_uint4(0, 0, 0, 0);
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int c = 0; c < A_CH; ++c) {
      const int cid = tid + 256 * c, row = cid >> 3, kc = (cid & 7) * 8;
      *reinterpret_cast<uint4 *>(sA + (buf * BM + row) * LDK + kc) = ra[c];
    }
#pragma unroll
    for (int c = 0; c < W_CH; ++c) {
      const int cid = tid + 256 * c, row = cid >> 3, kc = (cid & 7) * 8;
      *reinterpret_cast<uint4 *>(sW + (buf * BN + row) * LDK + kc) = rw[c];
    }
  };

  const int KT = (K + BK - 1) / BK;
  gload(0);
  sstore(0);
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < KT) gload((kt + 1) * BK);
    const bf16_t *pa = sA + (buf * BM + wm * WM + ln) * LDK + lh * 8;
    const bf16_t *pw = sW + (buf * BN + wn * WN + ln) * LDK + lh * 8;
#pragma unroll
    for (int s = 0; s < BK / 16; ++s) {
      bf16x8 fa[TM], fw[TN];
#pragma unroll
      for (int a = 0; a < TM; ++a)
        fa[a] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(pa + a * 32 * LDK + s * 16));
#pragma unroll
      for (int b = 0; b < TN; ++b)
        fw[b] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(pw + b * 32 * LDK + s * 16));
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fw[b], acc[a][b], 0, 0, 0);
    }
    if (kt + 1 < KT) sstore(buf ^ 1);
    __syncthreads();
  }

  // epilogue: lane holds column ln, rows c_row(v, lh) of every 32x32 tile
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b) {
      const int col = n0 + wn * WN + b * 32 + ln;
      if (col >= N) continue;
      const float bv = bias ? bf2f(bias[col]) : 0.f;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm * WM + a * 32 + c_row(v, lh);
        if (row >= M) continue;
        float r = acc[a][b][v] + bv;
        const size_t o = (size_t)row * N + col;
        if (residual) r += bf2f(residual[o]);
        if (out_f32) reinterpret_cast<float *>(Y)[o] = r;
        else reinterpret_cast<bf16_t *>(Y)[o] = f2bf(r);
      }
    }
}

template <int BM, int BN, int WM, int WN>
hipError_t run_bf16(const GemmArgs &a, hipStream_t s) {
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  const int groups = (tiles_n + XCDS - 1) / XCDS;
  const size_t lds = (size_t)2 * (BM + BN) * LDK * sizeof(bf16_t);
  auto kern = gemm_bf16_kernel<BM, BN, WM, WN>;
  static bool attr_done = false;
  if (!attr_done) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)lds);
    attr_done = true;
  }
  kern<<<dim3(groups * XCDS * tiles_m), dim3(256), lds, s>>>((const bf16_t *)a.x, (const bf16_t *)a.w,
                                                            (const bf16_t *)a.bias, (const bf16_t *)a.residual, a.y,
                                                            a.M, a.N, a.K, a.out_f32, tiles_m, tiles_n);
  return hipGetLastError();
}

// fp32: 64x64 tile, 16 wide k slices, each thread a 4x4 micro-tile
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float *__restrict__ A, const float *__restrict__ W,
                                                       const float *__restrict__ bias, const float *residual,
                                                       float *Y, int M, int N, int K) {
  __shared__ float sA[16][65], sW[16][65];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int x = tid; x < 64 * 16; x += 256) {
      const int r = x >> 4, kk = x & 15;
      sA[kk][r] = (m0 + r < M && k0 + kk < K) ? A[(size_t)(m0 + r) * K + k0 + kk] : 0.f;
      sW[kk][r] = (n0 + r < N && k0 + kk < K) ? W[(size_t)(n0 + r) * K + k0 + kk] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float av[4], wv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { av[i] = sA[kk][ty * 4 + i]; wv[i] = sW[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int jn = 0; jn < 4; ++jn) acc[i][jn] += av[i] * wv[jn];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int jn = 0; jn < 4; ++jn) {
      const int r = m0 + ty * 4 + i, c = n0 + tx * 4 + jn;
      if (r < M && c < N) {
        float v = acc[i][jn] + (bias ? bias[c] : 0.f);
        if (residual) v += residual[(size_t)r * N + c];
        Y[(size_t)r * N + c] = v;
      }
    }
}

}  // namespace

hipError_t launch_gemm_bf16(const GemmArgs &a, hipStream_t s) {
  // Tile choice: tall tiles once M fills them, otherwise 128x128.
  if (a.M > 384) return run_bf16<256, 128, 128, 64>(a, s);
  return run_bf16<128, 128, 64, 64>(a, s);
}

hipError_t launch_gemm_f32(const GemmArgs &a, hipStream_t s) {
  dim3 grid((a.N + 63) / 64, (a.M + 63) / 64);
  gemm_f32_kernel<<<grid, 256, 0, s>>>((const float *)a.x, (const float *)a.w, (const float *)a.bias,
                                       (const float *)a.residual, (float *)a.y, a.M, a.N, a.K);
  return hipGetLastError();
}

}  // namespace sf
